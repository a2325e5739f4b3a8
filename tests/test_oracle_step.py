"""Pins for the oracle's full / cached steps: brute force on a tiny stage, the invariants the
method fixes (chunked == unchunked, cached == full on the same input, swap round trip is
byte-identical), special cases and symmetries, and an independent torch float64 build of
the same stage."""
import numpy as np
import pytest
import torch
import torch.nn.functional as TF

from oracle import lightcache_oracle as lo
from paper_2510_05367_amd import synth
from tests import brute

MICRO = synth.StageConfig("micro", B=2, F=3, H=4, W=4, C_lat=2, C=8, C_deep=16, groups=4,
                          n_res=2, heads=2, head_dim=4, dtype="f32")
SMALL = synth.StageConfig("small", B=2, F=4, H=8, W=6, C_lat=4, C=32, C_deep=64, groups=8,
                          n_res=2, heads=4, head_dim=8, dtype="f32")


def big_weights(cfg, seed=0):
    """Weights large enough (std 0.3) that every term matters in the comparison."""
    w = synth.make_weights(cfg, seed)
    out = {}
    for k, v in w.items():
        if k.endswith("gn_g"):
            out[k] = 1.0 + (v.astype(np.float64) - 1.0) * 15.0
        else:
            out[k] = v.astype(np.float64) * 15.0
    return out


def rel_l2(a, b):
    a, b = np.asarray(a, dtype=np.float64), np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def test_full_and_cached_step_match_brute_force():
    cfg = MICRO
    w = big_weights(cfg)
    x = synth.make_latents(cfg).astype(np.float64)
    o = lo.Oracle(cfg, w)
    eps = o.full_step(x, 0)
    wl = {k: v.tolist() for k, v in w.items()}
    eps_b, deep_b = brute.stage(cfg, wl, x.reshape(cfg.N, cfg.C_lat, cfg.H, cfg.W).tolist())
    assert np.max(np.abs(o.dev[0] - np.array(deep_b))) < 1e-10
    assert np.max(np.abs(eps.reshape(cfg.N, cfg.C_lat, cfg.H, cfg.W) - np.array(eps_b))) < 1e-10
    # cached step with a foreign deep feature
    deep = synth.make_deep(cfg).astype(np.float64)
    o.cache_write(1, deep)
    eps_c = o.cached_step(x, 1)
    eps_cb, _ = brute.stage(cfg, wl, x.reshape(cfg.N, cfg.C_lat, cfg.H, cfg.W).tolist(), deep.tolist())
    assert np.max(np.abs(eps_c.reshape(cfg.N, cfg.C_lat, cfg.H, cfg.W) - np.array(eps_cb))) < 1e-10
    assert rel_l2(eps_c, eps) > 1e-3  # the deep feature does matter


def torch_stage(cfg, w, x, deep=None):
    """The same stage built from torch float64 functionals (independent library routines)."""
    t = {k: torch.from_numpy(np.asarray(v, dtype=np.float64)) for k, v in w.items()}
    N, C, H, W, G = cfg.N, cfg.C, cfg.H, cfg.W, cfg.groups
    h = TF.conv2d(torch.from_numpy(x).reshape(N, cfg.C_lat, H, W), t["conv_in.w"], t["conv_in.b"], padding=1)
    for i in range(cfg.n_res):
        g = TF.silu(TF.group_norm(h, G, t[f"res{i}.gn_g"], t[f"res{i}.gn_b"], cfg.gn_eps))
        h = h + TF.conv2d(g, t[f"res{i}.w"], t[f"res{i}.b"], padding=1)

    def mha(X, p):  # X [batch, L, C]
        Bn, L, _ = X.shape
        sp = lambda m: (X @ t[p + m].T).reshape(Bn, L, cfg.heads, cfg.head_dim).transpose(1, 2)
        o = TF.scaled_dot_product_attention(sp(".wq"), sp(".wk"), sp(".wv"))
        return o.transpose(1, 2).reshape(Bn, L, C) @ t[p + ".wo"].T + t[p + ".bo"]

    g = TF.group_norm(h, G, t["sattn.gn_g"], t["sattn.gn_b"], cfg.gn_eps)
    h = h + mha(g.reshape(N, C, H * W).transpose(1, 2), "sattn").transpose(1, 2).reshape(N, C, H, W)
    g = TF.group_norm(h, G, t["tattn.gn_g"], t["tattn.gn_b"], cfg.gn_eps)
    X = g.reshape(cfg.B, cfg.F, C, H * W).permute(0, 3, 1, 2).reshape(cfg.B * H * W, cfg.F, C)
    Y = mha(X, "tattn").reshape(cfg.B, H * W, cfg.F, C).permute(0, 2, 3, 1).reshape(N, C, H, W)
    h = h + Y
    if deep is None:
        d0 = TF.conv2d(h, t["down.w"], t["down.b"], stride=2, padding=1)
        g = TF.silu(TF.group_norm(d0, G, t["dres.gn_g"], t["dres.gn_b"], cfg.gn_eps))
        dp = d0 + TF.conv2d(g, t["dres.w"], t["dres.b"], padding=1)
    else:
        dp = torch.from_numpy(deep)
    cat = torch.cat([h, TF.interpolate(dp, scale_factor=2, mode="nearest")], dim=1)
    u = TF.conv2d(TF.silu(TF.group_norm(cat, G, t["up.gn_g"], t["up.gn_b"], cfg.gn_eps)), t["up.w"], t["up.b"], padding=1)
    e = TF.conv2d(TF.silu(TF.group_norm(u, G, t["out.gn_g"], t["out.gn_b"], cfg.gn_eps)), t["out.w"], t["out.b"], padding=1)
    return e.numpy().reshape(cfg.B, cfg.F, cfg.C_lat, H, W), dp.numpy()


@pytest.mark.parametrize("cfg", [MICRO, SMALL])
def test_steps_match_torch_float64_build(cfg):
    w = big_weights(cfg, 3)
    x = synth.make_latents(cfg, 4).astype(np.float64)
    o = lo.Oracle(cfg, w)
    eps = o.full_step(x, 0)
    eps_t, deep_t = torch_stage(cfg, w, x)
    assert rel_l2(o.dev[0], deep_t) < 1e-11
    assert rel_l2(eps, eps_t) < 1e-11
    deep = synth.make_deep(cfg, 5).astype(np.float64)
    o.cache_write(0, deep)
    assert rel_l2(o.cached_step(x, 0), torch_stage(cfg, w, x, deep)[0]) < 1e-11


# ------------------------------------------------------------------ invariants of the method
@pytest.mark.parametrize("fc,tc", [(1, 0), (2, 0), (3, 0), (5, 0), (8, 0), (16, 0), (0, 1), (0, 7), (3, 5), (2, 48), (0, 1000)])
def test_chunked_equals_unchunked(fc, tc):
    cfg = SMALL
    w = big_weights(cfg, 1)
    x = synth.make_latents(cfg, 2).astype(np.float64)
    ref = lo.Oracle(cfg, w)
    e0 = ref.full_step(x, 0)
    c0 = ref.cached_step(x, 0)
    o = lo.Oracle(cfg, w)
    o.set_chunk(fc, tc)
    e1 = o.full_step(x, 0)
    c1 = o.cached_step(x, 0)
    # exact up to the summation blocking of the library matmul: far below any tolerance used
    assert rel_l2(e1, e0) < 1e-13 and rel_l2(c1, c0) < 1e-13
    assert rel_l2(o.dev[0], ref.dev[0]) < 1e-13


def test_cached_step_on_own_cache_equals_full_step():
    cfg = SMALL
    w = big_weights(cfg, 1)
    x = synth.make_latents(cfg, 2).astype(np.float64)
    o = lo.Oracle(cfg, w)
    e_full = o.full_step(x, 1)
    assert np.array_equal(o.cached_step(x, 1), e_full)


def test_swap_round_trip_is_byte_identical():
    cfg = SMALL
    w = big_weights(cfg, 1)
    x = synth.make_latents(cfg, 2).astype(np.float64)
    o = lo.Oracle(cfg, w, host_slots=3, dev_slots=2)
    e_full = o.full_step(x, 0)
    before = o.dev[0].tobytes()
    o.swap_out(0, 2)
    o.dev[0][...] = np.nan  # poison the device copy
    o.swap_in(2, 1)
    assert o.dev[1].tobytes() == before and o.host[2].tobytes() == before
    assert np.array_equal(o.cached_step(x, 1), e_full)


def test_state_errors():
    cfg = MICRO
    o = lo.Oracle(cfg, big_weights(cfg))
    x = synth.make_latents(cfg)
    with pytest.raises(RuntimeError):
        o.cached_step(x, 0)
    with pytest.raises(RuntimeError):
        o.swap_out(0, 0)
    with pytest.raises(RuntimeError):
        o.swap_in(0, 0)
    with pytest.raises(ValueError):
        o.set_chunk(-1, 0)
    with pytest.raises(ValueError):
        lo.Oracle(cfg.with_(heads=3), big_weights(cfg))


# ------------------------------------------------------------------ special cases / symmetries
def test_concat_order_skip_first_then_deep():
    # C = Cd = 8 and 2 groups: on the concatenated tensor group 0 is exactly the skip channels and
    # group 1 exactly the deep channels, so the two halves do not meet in the statistics. With the
    # up-conv weights zeroed on channels [C, C+Cd) the output must not depend on the deep feature.
    cfg = synth.StageConfig("m2", B=1, F=2, H=4, W=4, C_lat=2, C=8, C_deep=8, groups=2, n_res=1,
                            heads=2, head_dim=4, dtype="f32")
    w = big_weights(cfg)
    x = synth.make_latents(cfg).astype(np.float64)
    deep_a = synth.make_deep(cfg, 7).astype(np.float64)
    deep_b = synth.make_deep(cfg, 8).astype(np.float64)
    w0 = dict(w)
    w0["up.w"] = w["up.w"].copy()
    w0["up.w"][:, cfg.C:] = 0.0
    o = lo.Oracle(cfg, w0)
    o.cache_write(0, deep_a)
    o.cache_write(1, deep_b)
    assert np.allclose(o.cached_step(x, 0), o.cached_step(x, 1), atol=1e-13)
    # with the skip columns zeroed instead, the deep feature does change the result
    w1 = dict(w)
    w1["up.w"] = w["up.w"].copy()
    w1["up.w"][:, :cfg.C] = 0.0
    o = lo.Oracle(cfg, w1)
    o.cache_write(0, deep_a)
    o.cache_write(1, deep_b)
    assert rel_l2(o.cached_step(x, 0), o.cached_step(x, 1)) > 1e-3


def test_batch_halves_are_independent():
    cfg = SMALL
    w = big_weights(cfg, 1)
    x = synth.make_latents(cfg, 2).astype(np.float64)
    deep = synth.make_deep(cfg, 3).astype(np.float64)
    o = lo.Oracle(cfg, w)
    o.cache_write(0, deep)
    joint = o.cached_step(x, 0)
    half = cfg.with_(B=1)
    for b in range(2):
        oh = lo.Oracle(half, w)
        oh.cache_write(0, deep[b * cfg.F:(b + 1) * cfg.F])
        assert np.allclose(oh.cached_step(x[b:b + 1], 0), joint[b:b + 1], atol=1e-12)


def test_frame_permutation_equivariance():
    # no positional encoding on the frame axis: permuting frames permutes the output
    cfg = SMALL.with_(B=1)
    w = big_weights(cfg, 1)
    x = synth.make_latents(cfg, 2).astype(np.float64)
    deep = synth.make_deep(cfg, 3).astype(np.float64)
    perm = np.array([2, 0, 3, 1])
    o = lo.Oracle(cfg, w)
    o.cache_write(0, deep)
    e = o.cached_step(x, 0)
    o.cache_write(0, deep[perm])
    assert np.allclose(o.cached_step(x[:, perm], 0), e[:, perm], atol=1e-12)


def test_single_frame_temporal_block_is_linear():
    cfg = SMALL.with_(B=3, F=1)
    w = big_weights(cfg, 1)
    o = lo.Oracle(cfg, w)
    h = np.random.default_rng(0).standard_normal((3, cfg.C, cfg.H, cfg.W))
    g = lo.group_norm(h, w["tattn.gn_g"], w["tattn.gn_b"], cfg.groups, cfg.gn_eps)
    lin = np.einsum("oc,nchw->nohw", w["tattn.wo"] @ w["tattn.wv"], g) + w["tattn.bo"][None, :, None, None]
    assert np.allclose(o.temporal_block(h), h + lin, atol=1e-12)


def test_temporal_block_mixes_only_frames_of_one_position():
    cfg = SMALL
    w = big_weights(cfg, 1)
    o = lo.Oracle(cfg, w)
    h = np.random.default_rng(0).standard_normal((cfg.N, cfg.C, cfg.H, cfg.W))
    # identity GN statistics are per frame, so perturb in a statistics-preserving way: swap two
    # positions' channel vectors within one frame of batch 1
    h2 = h.copy()
    n = cfg.F + 1
    h2[n, :, 0, 0], h2[n, :, 3, 2] = h[n, :, 3, 2].copy(), h[n, :, 0, 0].copy()
    a, b = o.temporal_block(h), o.temporal_block(h2)
    diff = np.abs(a - b).max(axis=1)  # [N, H, W]
    touched = np.zeros_like(diff, dtype=bool)
    touched[cfg.F:, 0, 0] = True
    touched[cfg.F:, 3, 2] = True
    assert np.all(diff[~touched] < 1e-12) and np.all(diff[touched] > 1e-6)


def test_spatial_block_mixes_only_tokens_of_one_frame():
    cfg = SMALL
    w = big_weights(cfg, 1)
    o = lo.Oracle(cfg, w)
    h = np.random.default_rng(0).standard_normal((cfg.N, cfg.C, cfg.H, cfg.W))
    h2 = h.copy()
    h2[2] = h[2, :, ::-1, :]
    a, b = o.spatial_block(h), o.spatial_block(h2)
    for n in range(cfg.N):
        if n == 2:
            assert np.allclose(b[2], a[2][:, ::-1, :], atol=1e-12)  # token permutation within the frame
        else:
            assert np.array_equal(a[n], b[n])


def test_float32_build_agrees_with_float64():
    cfg = synth.CONFIGS["tiny"].with_(F=2, H=16, W=16)
    w = synth.make_weights(cfg)
    x = synth.make_latents(cfg)
    o64 = lo.Oracle(cfg, w)
    o32 = lo.Oracle(cfg, w, dtype=np.float32)
    e64, e32 = o64.full_step(x, 0), o32.full_step(x, 0)
    assert e32.dtype == np.float32
    assert rel_l2(e32, e64) < 2e-6
    assert rel_l2(o32.cached_step(x, 0), e64) < 2e-6


def test_schedule_counts_and_teacher_forcing():
    cfg = MICRO
    w = big_weights(cfg)
    x0 = synth.make_latents(cfg).astype(np.float64)
    o = lo.Oracle(cfg, w, host_slots=2, dev_slots=2)
    xs, eps = lo.run_schedule(o, x0, steps=7, interval=3)
    assert len(xs) == len(eps) == 7
    # steps 0, 3, 6 are normal steps: re-running a full step on the same latent reproduces them;
    # steps 1, 2 reuse the deep feature of step 0
    o2 = lo.Oracle(cfg, w)
    assert np.array_equal(o2.full_step(xs[0], 0), eps[0])
    assert np.array_equal(o2.cached_step(xs[1], 0), eps[1])
    assert np.array_equal(o2.cached_step(xs[2], 0), eps[2])
    assert np.array_equal(o2.full_step(xs[3], 0), eps[3])
    assert np.allclose(xs[1], xs[0] - eps[0] / 7.0, atol=1e-15)


# --------------------------------------------------------------------------- literal spatial chunk
SP = synth.StageConfig("sp", B=2, F=3, H=16, W=12, C_lat=4, C=32, C_deep=64, groups=8, n_res=2, heads=2, head_dim=16,
                       dtype="f32")


def test_conv_block_with_halo_is_a_slice_of_the_whole_convolution():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((2, 3, 8, 10))
    w = rng.standard_normal((4, 3, 3, 3))
    b = rng.standard_normal(4)
    whole = lo.conv3x3(x, w, b)  # (itself pinned by brute force and closed forms in test_oracle_ops.py)
    for (y0, y1, x0, x1) in [(0, 8, 0, 10), (0, 4, 0, 5), (4, 8, 5, 10), (2, 6, 3, 7), (0, 2, 8, 10), (7, 8, 0, 1)]:
        blk = lo.conv3x3_block(x, w, b, y0, y1, x0, x1)
        assert np.max(np.abs(blk - whole[:, :, y0:y1, x0:x1])) < 1e-13, (y0, y1, x0, x1)
    # the halo is what makes it so: the block convolved on its own (zeros around it) differs along its inner edges
    alone = lo.conv3x3(np.ascontiguousarray(x[:, :, 2:6, 3:7]), w, b)
    assert np.max(np.abs(alone - whole[:, :, 2:6, 3:7])) > 1e-2
    assert np.max(np.abs(alone[:, :, 1:3, 1:3] - whole[:, :, 3:5, 4:6])) < 1e-13  # its interior does not
    # against the scalar brute force directly, on a corner block
    bf = np.array(brute.conv3x3(x.tolist(), w.tolist(), b.tolist()))[:, :, 4:8, 5:10]
    assert np.max(np.abs(lo.conv3x3_block(x, w, b, 4, 8, 5, 10) - bf)) < 1e-12


def test_group_norm_in_two_passes_over_blocks():
    rng = np.random.default_rng(4)
    x = rng.standard_normal((2, 8, 6, 8)) * 2.0 + 0.7
    g, b = 1.0 + 0.1 * rng.standard_normal(8), 0.1 * rng.standard_normal(8)
    blocks = [(0, 3, 0, 4), (0, 3, 4, 8), (3, 6, 0, 4), (3, 6, 4, 8)]
    y = lo.group_norm_blocks(x, g, b, 4, 1e-5, blocks)
    assert np.max(np.abs(y - lo.group_norm(x, g, b, 4, 1e-5))) < 1e-13
    yb = np.array(brute.group_norm_silu(x.tolist(), g.tolist(), b.tolist(), 4, 1e-5, act=False))
    assert np.max(np.abs(y - yb)) < 1e-12
    with pytest.raises(AssertionError):  # blocks that do not tile the image
        lo.group_norm_blocks(x, g, b, 4, 1e-5, blocks[:3])


@pytest.mark.parametrize("eta,omega,fc", [(2, 1, 0), (1, 2, 0), (4, 3, 2), (8, 6, 0), (2, 2, 4)])
def test_spatially_chunked_steps_equal_unchunked(eta, omega, fc):
    w = {k: v.astype(np.float64) for k, v in synth.make_weights(SP, 0, sharp=4.0).items()}
    x = synth.make_latents(SP, 1)
    whole = lo.Oracle(SP, w)
    ref = whole.full_step(x, 0)
    o = lo.Oracle(SP, w)
    o.set_spatial_chunk(eta, omega)
    o.set_chunk(fc, 0)
    full = o.full_step(x, 0)
    assert np.max(np.abs(full - ref)) < 1e-12
    assert np.max(np.abs(o.dev[0] - whole.dev[0])) < 1e-12
    deep = synth.make_deep(SP, 2)
    o.cache_write(1, deep)
    whole.cache_write(1, deep)
    assert np.max(np.abs(o.cached_step(x, 1) - whole.cached_step(x, 1))) < 1e-12
    with pytest.raises(ValueError):
        o.set_spatial_chunk(3, 1)   # 16 / 3
    with pytest.raises(ValueError):
        o.set_spatial_chunk(16, 1)  # blocks of one row: the deep feature under them has no whole row
