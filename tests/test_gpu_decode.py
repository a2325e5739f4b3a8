"""GPU parity of sliced decoding: the decoder through the C ABI against the CPU oracle, the method's invariant
(decoding slice by slice == decoding all frames at once, bit for bit), the workspace sized by the slice, errors."""
import numpy as np
import pytest
import torch

from oracle import decoder_oracle as do
from paper_2510_05367_amd import binding as lcb
from paper_2510_05367_amd import synth
from tests.gpu_util import check, host

pytestmark = pytest.mark.gpu

DEC_F32 = synth.DecoderConfig("dec_f32", N=5, H=10, W=12, C_lat=4, C_img=3, widths=(64, 128, 64), groups=32, heads=1,
                              head_dim=64, dtype="f32")
DEC_BF16 = synth.DecoderConfig("dec_bf16", N=3, H=10, W=12, C_lat=4, C_img=3, widths=(320, 192, 128), groups=32, heads=8,
                               head_dim=40, dtype="bf16")
DEC_L0 = synth.DecoderConfig("dec_l0", N=2, H=6, W=10, C_lat=3, C_img=5, widths=(64,), groups=8, heads=4, head_dim=16,
                             dtype="f32")
AD = synth.DECODERS["animatediff"]


def w64_of(w):
    return {k: v.astype(np.float64) for k, v in w.items()}


@pytest.mark.parametrize("cfg", [DEC_F32, DEC_BF16, DEC_L0], ids=lambda c: c.name)
def test_decode_matches_oracle_and_slicing_is_exact(cfg):
    print(f"\n[case] {cfg.name} N={cfg.N} {cfg.H}x{cfg.W} widths={cfg.widths}", flush=True)
    w = synth.make_decoder_weights(cfg, 0, sharp=4.0)
    dec = lcb.Decoder(cfg, w, max_slice=cfg.N)
    try:
        z = synth.make_decoder_latents(cfg, 1)
        zd = dec.to_device(z)
        whole = dec.decode(zd, 0)
        dec.sync()
        ref = do.DecoderOracle(cfg, w64_of(w)).decode(z, 1)
        assert 1e-3 < float(np.std(ref)) < 1e2
        check("decoded video", host(whole), ref, cfg.dtype)
        for sl in (1, 2, cfg.N, cfg.N + 3):
            out = dec.decode(zd, sl)
            dec.sync()
            assert torch.equal(out, whole), sl
    finally:
        dec.close()


def test_workspace_is_sized_by_the_slice():
    c = lcb.make_decoder_config(AD)
    one = lcb.lc_decoder_workspace_bytes(c, 1)
    assert one > 0
    for n in (2, 4, 16):
        assert abs(lcb.lc_decoder_workspace_bytes(c, n) - n * one) <= 64 * 1024  # linear in the slice (alignment aside)
    assert lcb.lc_decoder_workspace_bytes(c, 0) == lcb.lc_decoder_workspace_bytes(c, 16) == lcb.lc_decoder_workspace_bytes(c, 99)
    # one frame: two fp32 maps of the largest stage (the 512 x 512 x 192 upsampled input of the last convolution)
    assert 2 * 512 * 512 * 192 * 4 <= one < 2 * 512 * 512 * 192 * 4 * 1.2


def test_decoder_errors():
    cfg = DEC_L0
    w = synth.make_decoder_weights(cfg, 0)
    dec = lcb.Decoder(cfg, w, max_slice=1)
    try:
        z = dec.to_device(synth.make_decoder_latents(cfg, 1))
        img = dec.decode(z, 1)
        dec.sync()
        assert bool(torch.isfinite(img.float()).all())
        with pytest.raises(lcb.LcError) as e:  # the workspace holds one frame, not two
            lcb.lc_decode(dec.dec, z.data_ptr(), img.data_ptr(), 2)
        assert e.value.status == lcb.LC_ERR_NOMEM and "slice" in str(e.value)
        with pytest.raises(lcb.LcError) as e:
            lcb.lc_decode(dec.dec, None, img.data_ptr(), 1)
        assert e.value.status == lcb.LC_ERR_ARG
        with pytest.raises(lcb.LcError) as e:
            lcb.lc_decode(dec.dec, z.data_ptr(), img.data_ptr(), -1)
        assert e.value.status == lcb.LC_ERR_ARG
    finally:
        dec.close()
    s = torch.cuda.Stream()
    d2 = lcb.lc_decoder_create(lcb.make_decoder_config(cfg), s.cuda_stream)
    try:
        with pytest.raises(lcb.LcError) as e:
            lcb.lc_decode(d2, 1, 1, 1)
        assert e.value.status == lcb.LC_ERR_STATE
    finally:
        lcb.lc_decoder_destroy(d2)


def test_decode_full_size_frame_by_frame():
    """512 x 512 frames from 64 x 64 latents (the AnimateDiff-sized decoder): four frames decoded one by one equal
    the same frames decoded two at a time and all at once, bit for bit; the first and last against the oracle."""
    cfg = AD.with_(N=4)
    print(f"\n[case] {cfg.name} N={cfg.N} {cfg.H}x{cfg.W} -> {cfg.H * 8}x{cfg.W * 8}", flush=True)
    w = synth.make_decoder_weights(cfg, 0)
    dec = lcb.Decoder(cfg, w, max_slice=cfg.N)
    try:
        z = synth.make_decoder_latents(cfg, 1)
        zd = dec.to_device(z)
        one = dec.decode(zd, 1)
        two = dec.decode(zd, 2)
        allf = dec.decode(zd, 0)
        dec.sync()
        assert torch.equal(one, two) and torch.equal(one, allf)
        orc = do.DecoderOracle(cfg.with_(N=1), w64_of(w))
        for f in (0, cfg.N - 1):
            print(f"[oracle] frame {f}", flush=True)
            check(f"decoded frame {f}", host(one[f:f + 1]), orc.decode(z[f:f + 1], 1), cfg.dtype)
    finally:
        dec.close()
