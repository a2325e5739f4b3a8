"""Pins of the sliced-decoding oracle (oracle/decoder_oracle.py): a scalar brute force of the whole decoder on a
tiny instance, an independent torch float64 build, the method's invariant (decoding slice by slice == decoding all
frames at once, for every slice size), and closed forms that fix the order of upsampling and convolution."""
import numpy as np
import pytest
import torch
import torch.nn.functional as TF

from oracle import decoder_oracle as do
from paper_2510_05367_amd import synth
from tests import brute

TINY = synth.DecoderConfig("t", N=3, H=4, W=6, C_lat=2, C_img=3, widths=(8, 8, 4), groups=2, heads=2, head_dim=4,
                           dtype="f32")


def w64(cfg, seed=0, scale=1.0):
    w = synth.make_decoder_weights(cfg, seed, sharp=6.0)
    return {k: (v.astype(np.float64) * (scale if k.endswith(".w") or k[-2:] in ("wq", "wk", "wv", "wo") else 1.0))
            for k, v in w.items()}


def test_weight_names_match_manifest():
    assert sorted(do.required_weights(TINY)) == sorted(n for n, _, _ in synth.decoder_weight_manifest(TINY))


def test_decoder_matches_brute_force():
    w = w64(TINY, scale=8.0)  # larger weights: every block contributes visibly
    z = synth.make_decoder_latents(TINY, 1).astype(np.float64)
    got = do.DecoderOracle(TINY, w).decode(z, 1)
    ref = np.array(brute.decoder(TINY, {k: v.tolist() for k, v in w.items()}, z.tolist()))
    assert got.shape == (3, 3, 16, 24)
    assert np.max(np.abs(got - ref)) < 1e-11 * max(1.0, np.max(np.abs(ref)))
    assert np.std(ref) > 1e-3


def torch_decoder(cfg, w, z):
    t = {k: torch.from_numpy(v) for k, v in w.items()}

    def res(h, p):
        g = TF.silu(TF.group_norm(h, cfg.groups, t[p + ".gn_g"], t[p + ".gn_b"], cfg.gn_eps))
        return h + TF.conv2d(g, t[p + ".w"], t[p + ".b"], padding=1)
    h = TF.conv2d(torch.from_numpy(z), t["conv_in.w"], t["conv_in.b"], padding=1)
    h = res(h, "mid.res0")
    n, C, H, W = h.shape
    g = TF.group_norm(h, cfg.groups, t["mid.attn.gn_g"], t["mid.attn.gn_b"], cfg.gn_eps).reshape(n, C, H * W).transpose(1, 2)
    q, k, v = (g @ t[f"mid.attn.{x}"].T for x in ("wq", "wk", "wv"))
    sp = lambda a: a.reshape(n, H * W, cfg.heads, cfg.head_dim).transpose(1, 2)
    o = TF.scaled_dot_product_attention(sp(q), sp(k), sp(v)).transpose(1, 2).reshape(n, H * W, C)
    h = h + (o @ t["mid.attn.wo"].T + t["mid.attn.bo"]).transpose(1, 2).reshape(n, C, H, W)
    h = res(h, "mid.res1")
    for l in range(cfg.levels):
        h = res(h, f"up{l}.res")
        h = TF.conv2d(TF.interpolate(h, scale_factor=2, mode="nearest"), t[f"up{l}.conv.w"], t[f"up{l}.conv.b"], padding=1)
    h = TF.silu(TF.group_norm(h, cfg.groups, t["out.gn_g"], t["out.gn_b"], cfg.gn_eps))
    return TF.conv2d(h, t["out.w"], t["out.b"], padding=1).numpy()


def test_decoder_matches_independent_torch_build():
    cfg = synth.DecoderConfig("m", N=2, H=6, W=4, C_lat=4, C_img=3, widths=(16, 8, 8, 4), groups=4, heads=2, head_dim=8,
                              dtype="f32")
    w = w64(cfg, scale=4.0)
    z = synth.make_decoder_latents(cfg, 2).astype(np.float64)
    got = do.DecoderOracle(cfg, w).decode(z, 0)
    ref = torch_decoder(cfg, w, z)
    assert got.shape == ref.shape == (2, 3, 48, 32)
    assert np.max(np.abs(got - ref)) < 1e-12 * max(1.0, np.max(np.abs(ref)))


@pytest.mark.parametrize("slice_frames", [1, 2, 3, 5, 0])
def test_sliced_equals_unsliced(slice_frames):
    cfg = TINY.with_(N=5)
    w = w64(cfg)
    z = synth.make_decoder_latents(cfg, 3).astype(np.float64)
    orc = do.DecoderOracle(cfg, w)
    whole = orc.decode(z, 0)
    assert np.array_equal(orc.decode(z, slice_frames), whole)  # every operator is per frame: the same sums
    # a frame's image does not depend on the other frames
    z2 = z.copy()
    z2[1] += 1.0
    d2 = orc.decode(z2, slice_frames)
    assert np.array_equal(d2[[0, 2, 3, 4]], whole[[0, 2, 3, 4]]) and not np.array_equal(d2[1], whole[1])


def test_upsampling_comes_before_the_level_convolution():
    """With every block switched off except one level's convolution (delta kernels elsewhere), the decoder is
    conv3x3(up2(.)): a horizontal-difference kernel applied AFTER nearest upsampling is zero inside each 2x2 block
    and non-zero across block borders; applied before it, it would be non-zero everywhere."""
    cfg = synth.DecoderConfig("u", N=1, H=4, W=4, C_lat=2, C_img=2, widths=(2, 2), groups=1, heads=1, head_dim=2, dtype="f32")
    w = {n: np.zeros(s) for n, s, _ in synth.decoder_weight_manifest(cfg)}
    for n in w:
        if n.endswith("gn_g"):
            w[n][:] = 1.0
    delta = np.zeros((2, 2, 3, 3)); delta[0, 0, 1, 1] = delta[1, 1, 1, 1] = 1.0
    w["conv_in.w"] = delta.copy()
    diff = np.zeros((2, 2, 3, 3)); diff[0, 0, 1, 1], diff[0, 0, 1, 0] = 1.0, -1.0; diff[1, 1, 1, 1] = 1.0
    w["up0.conv.w"] = diff
    orc = do.DecoderOracle(cfg, w)
    z = np.arange(32, dtype=np.float64).reshape(1, 2, 4, 4)
    h = orc.res_block(do.conv3x3(z, w["conv_in.w"], w["conv_in.b"]), "mid.res0")
    assert np.array_equal(h, z)  # zero conv weights: residual blocks and the attention block are the identity
    assert np.array_equal(orc.attn_block(z, "mid.attn"), z)
    # the part before the out block
    u = do.conv3x3(do.up2(z), w["up0.conv.w"], w["up0.conv.b"])
    assert np.all(u[0, 0, :, 1::2] == 0.0) and np.all(u[0, 0, :, 2::2] == 1.0)  # x[j] - x[j-1] on the upsampled row
    assert np.array_equal(u[0, 1], do.up2(z)[0, 1])
