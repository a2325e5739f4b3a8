"""GPU parity of the U-Net stage with real block internals: normal and cache steps through the C ABI against the CPU
oracle (eps and the cached feature), the method's invariants (cache step on its own cache entry == normal step, bit
for bit; the cache bank byte-identical; every feature-chunk setting == all frames at once, bit for bit), a
refresh-interval schedule with swapping, errors."""
import numpy as np
import pytest
import torch

from oracle import unet_oracle as uo
from paper_2510_05367_amd import binding as lcb
from paper_2510_05367_amd import synth
from tests.gpu_util import check, host

pytestmark = pytest.mark.gpu

TINY = synth.UNETS["tiny"]                                   # fp32, 4 frames, 7 conditioning tokens
# bf16 with ragged pieces: 8 frames (the matrix-core temporal path), 24 x 16 latents, 77 conditioning tokens
SMALL_BF16 = synth.UnetConfig("small_bf16", B=2, F=8, H=24, W=16, C_lat=4, C=64, C1=128, C2=192, groups=32, head_dim=32,
                              ctx_len=77, ctx_dim=128, temb_dim=96, dtype="bf16")
# fp32 with 2 batch elements (per-element time embedding and conditioning) and head_dim 16
SMALL_F32 = synth.UnetConfig("small_f32", B=2, F=3, H=8, W=12, C_lat=3, C=64, C1=64, C2=128, groups=16, head_dim=16,
                             ctx_len=5, ctx_dim=64, temb_dim=40, dtype="f32", ff_mult=2)
MID = synth.UNETS["mid"]


def w64_of(w):
    return {k: v.astype(np.float64) for k, v in w.items()}


def to_planar(entry, cfg):
    """device entry [N, H*W, C1] -> numpy [N, C1, H, W]"""
    return host(entry).reshape(cfg.N, cfg.H, cfg.W, cfg.C1).transpose(0, 3, 1, 2)


def to_rows(deep, cfg):
    return np.ascontiguousarray(deep.transpose(0, 2, 3, 1)).reshape(cfg.N, cfg.H * cfg.W, cfg.C1)


def run_case(cfg, odtype=np.float64, sharp=4.0, chain=False, frame_chunk=None):
    print(f"\n[case] {cfg.name} chunk={frame_chunk} B={cfg.B} F={cfg.F} {cfg.H}x{cfg.W} C={cfg.C}/{cfg.C1}/{cfg.C2} d={cfg.head_dim} ctx {cfg.ctx_len}x{cfg.ctx_dim} {cfg.dtype}",
          flush=True)
    w = synth.make_unet_weights(cfg, 0, sharp=sharp)
    net = lcb.Unet(cfg, w, host_slots=1, dev_slots=2, frame_chunk=frame_chunk)
    try:
        x, temb, ctx = synth.make_unet_inputs(cfg, 1)
        xd, td, cd = net.to_device(x), net.to_device(temb), net.to_device(ctx)
        eps = net.empty(*x.shape)
        net.full_step(xd, td, cd, eps, 0)
        net.sync()
        print("[oracle] normal step ...", flush=True)
        orc = uo.UnetOracle(cfg, {k: v.astype(odtype) for k, v in w.items()}, dtype=odtype)
        ref = orc.full_step(x, temb, ctx, 0).astype(np.float64)
        assert float(np.std(ref)) > 1e-3
        check("normal step eps", host(eps), ref, cfg.dtype, chain=chain)
        check("cached feature", to_planar(net.dev_entry(0), cfg), orc.dev[0].astype(np.float64), cfg.dtype, chain=True)
        # cache step on a foreign entry and new inputs
        deep = synth.make_unet_deep(cfg, 7)
        x2, t2, c2 = synth.make_unet_inputs(cfg, 8)
        net.cache_write(1, net.to_device(to_rows(deep, cfg), f32=True))
        eps2 = net.empty(*x.shape)
        net.cached_step(net.to_device(x2), net.to_device(t2), net.to_device(c2), eps2, 1)
        net.sync()
        print("[oracle] cache step ...", flush=True)
        orc.cache_write(1, deep)
        check("cache step eps", host(eps2), orc.cached_step(x2, t2, c2, 1).astype(np.float64), cfg.dtype)
    finally:
        net.close()


@pytest.mark.parametrize("cfg", [TINY, SMALL_F32, SMALL_BF16], ids=lambda c: c.name)
def test_steps_match_oracle(cfg):
    run_case(cfg)


@pytest.mark.parametrize("cfg,frame_chunk", [(SMALL_F32, 2), (SMALL_BF16, 3)], ids=["small_f32-2", "small_bf16-3"])
def test_chunked_steps_match_oracle(cfg, frame_chunk):
    """The same comparison with the feature chunk on, in a workspace sized for the chunk: 2 of 6 frames (every chunk
    inside one batch element), and 3 of 16 (a ragged last chunk, chunks that straddle the two batch elements, position
    chunks of the temporal blocks that end inside an image row)."""
    run_case(cfg, frame_chunk=frame_chunk)


@pytest.mark.parametrize("cfg", [SMALL_F32, SMALL_BF16], ids=lambda c: c.name)
def test_chunked_equals_unchunked_bitwise(cfg):
    """Every chunk setting gives the normal step's eps, the cached feature and the cache step's eps of the run over all
    frames at once, bit for bit; the cached entries survive a change of the setting."""
    w = synth.make_unet_weights(cfg, 0, sharp=4.0)
    net = lcb.Unet(cfg, w, host_slots=1, dev_slots=2)
    try:
        x, temb, ctx = synth.make_unet_inputs(cfg, 1)
        xd, td, cd = net.to_device(x), net.to_device(temb), net.to_device(ctx)
        x2, t2, c2 = (net.to_device(a) for a in synth.make_unet_inputs(cfg, 8))
        ref, ref2 = net.empty(*x.shape), net.empty(*x.shape)
        net.full_step(xd, td, cd, ref, 0)
        net.cached_step(x2, t2, c2, ref2, 0)
        net.sync()
        d0 = net.dev_entry(0)
        assert bool(torch.isfinite(ref).all()) and not torch.equal(ref, ref2)
        whole = lcb.lc_unet_workspace_bytes(net.ccfg)
        for fc in (1, 2, 3, cfg.F, cfg.N - 1, cfg.N, cfg.N + 5):
            print(f"[chunk] {cfg.name} frame_chunk {fc}", flush=True)
            net.set_chunk(fc)
            assert lcb.lc_unet_chunk_workspace_bytes(net.ccfg, fc) <= whole
            out2 = net.empty(*x.shape)
            net.cached_step(x2, t2, c2, out2, 0)  # on the entry the unchunked normal step left
            net.sync()
            assert torch.equal(out2, ref2), fc
            out, out3 = net.empty(*x.shape), net.empty(*x.shape)
            net.full_step(xd, td, cd, out, 1)
            net.cached_step(x2, t2, c2, out3, 1)
            net.sync()
            assert torch.equal(out, ref), fc
            assert torch.equal(net.dev_entry(1), d0), fc
            assert torch.equal(out3, ref2), fc
        net.set_chunk(0)
        again = net.empty(*x.shape)
        net.full_step(xd, td, cd, again, 0)
        net.sync()
        assert torch.equal(again, ref)
    finally:
        net.close()


def test_benchmark_size_chunked_equals_unchunked():
    """The benchmark's configuration with a feature chunk of 4 of its 32 frames, in a workspace sized for that chunk,
    against the run over all frames at once in a workspace of its own: eps of the normal step, the cached feature and
    eps of a cache step agree bit for bit."""
    cfg = synth.UNETS["sd15_video"]
    w = synth.make_unet_weights(cfg, 0)
    x, temb, ctx = synth.make_unet_inputs(cfg, 1)
    results = []
    for fc in (None, 4):
        net = lcb.Unet(cfg, w, host_slots=0, dev_slots=1, frame_chunk=fc)
        try:
            print(f"[chunk] sd15_video frame_chunk {fc}: workspace {net.arena.numel() / 1e9:.3f} GB", flush=True)
            xd, td, cd = net.to_device(x), net.to_device(temb), net.to_device(ctx)
            full, cached = net.empty(*x.shape), net.empty(*x.shape)
            net.full_step(xd, td, cd, full, 0)
            net.cached_step(xd, td, cd, cached, 0)
            net.sync()
            results.append((full.clone(), cached.clone(), net.dev_entry(0), net.arena.numel()))
        finally:
            net.close()
            del net
    (f0, c0, d0, b0), (f1, c1, d1, b1) = results
    assert bool(torch.isfinite(f0).all())
    assert torch.equal(f1, f0) and torch.equal(c1, c0) and torch.equal(d1, d0)
    assert b1 < 0.6 * b0


@pytest.mark.slow
def test_full_width_steps_match_oracle():
    """Widths, conditioning and time embedding of the benchmark's U-Net (320 / 640 / 1280, 77 x 768, 1280) on 32 x 32
    latents, 2 x 8 frames; the oracle in float32 to keep it within a minute. The normal step's eps comes out of some
    eighty bf16 contractions in a row (the three-level deep branch and both shallow halves), twice the depth of
    anything the 2e-2 bound was stated for: it is held to rel-L2 <= 1e-2 and the element-wise bound that tolerance
    implies (gpu_util, `chain`); the cache step's eps, the shallow halves only, to the plain bounds."""
    run_case(MID, odtype=np.float32, sharp=1.0, chain=True)


@pytest.mark.slow
def test_full_resolution_steps_match_oracle():
    """The benchmark's U-Net at its full widths and full 64 x 64 latents (4096 tokens per frame: the tile and token
    geometry of the timed configuration), one batch element of 2 frames so that the float32 oracle stays under a
    minute (8 frames pass too, in three minutes; the 8-frame temporal path is what the half-resolution case covers)."""
    run_case(synth.UNETS["sd15_video"].with_(name="sd15_video_b1_f2", B=1, F=2), odtype=np.float32, sharp=1.0, chain=True)


@pytest.mark.parametrize("cfg", [SMALL_F32, SMALL_BF16], ids=lambda c: c.name)
def test_invariants_bitwise(cfg):
    w = synth.make_unet_weights(cfg, 0, sharp=4.0)
    net = lcb.Unet(cfg, w, host_slots=2, dev_slots=2)
    try:
        x, temb, ctx = synth.make_unet_inputs(cfg, 1)
        xd, td, cd = net.to_device(x), net.to_device(temb), net.to_device(ctx)
        full, cached, swapped, again = (net.empty(*x.shape) for _ in range(4))
        net.full_step(xd, td, cd, full, 0)
        net.cached_step(xd, td, cd, cached, 0)
        net.swap_out(0, 1)
        net.sync()
        assert bool(torch.isfinite(full).all())
        assert torch.equal(cached, full)  # cache step on its own entry == normal step
        d0 = net.dev_entry(0)
        assert net.host_entry_bytes(1) == d0.cpu().numpy().tobytes()
        net.cache_write(1, torch.full_like(d0, float("nan")))  # poison the other slot, then bring the entry back
        net.swap_in(1, 1)
        net.cached_step(xd, td, cd, swapped, 1)  # must wait for the copy on the GPU
        net.full_step(xd, td, cd, again, 0)      # and a second normal step reproduces the first
        net.sync()
        assert torch.equal(net.dev_entry(1), d0) and torch.equal(swapped, full)
        assert torch.equal(again, full) and torch.equal(net.dev_entry(0), d0)
        # a stale entry gives a different (finite) result
        x2, t2, c2 = synth.make_unet_inputs(cfg, 5)
        stale = net.empty(*x.shape)
        net.cached_step(net.to_device(x2), net.to_device(t2), net.to_device(c2), stale, 0)
        net.sync()
        assert bool(torch.isfinite(stale).all()) and not torch.equal(stale, full)
    finally:
        net.close()


def test_benchmark_size_invariants():
    """The benchmark's configuration (2 x 16 frames of 64 x 64, widths 320 / 640 / 1280), which the oracle cannot run in a
    test's time: the properties that hold at any size. A cache step on the entry its own normal step left reproduces
    that step bit for bit, a second normal step reproduces the first, the entry survives a swap round trip byte for
    byte, and eps has the scale the smaller cases have against the oracle (finite, std within 0.3 .. 1.5)."""
    cfg = synth.UNETS["sd15_video"]
    w = synth.make_unet_weights(cfg, 0)
    net = lcb.Unet(cfg, w, host_slots=1, dev_slots=2)
    try:
        x, temb, ctx = synth.make_unet_inputs(cfg, 1)
        xd, td, cd = net.to_device(x), net.to_device(temb), net.to_device(ctx)
        full, cached, again, swapped = (net.empty(*x.shape) for _ in range(4))
        net.full_step(xd, td, cd, full, 0)
        net.cached_step(xd, td, cd, cached, 0)
        net.swap_out(0, 0)
        net.full_step(xd, td, cd, again, 1)
        net.sync()
        assert bool(torch.isfinite(full).all()) and 0.3 < float(full.float().std()) < 1.5
        assert torch.equal(cached, full) and torch.equal(again, full)
        d0 = net.dev_entry(0)
        assert torch.equal(net.dev_entry(1), d0)
        assert net.host_entry_bytes(0) == d0.cpu().numpy().tobytes()
        net.cache_write(1, torch.zeros_like(d0))
        net.swap_in(0, 1)
        net.cached_step(xd, td, cd, swapped, 1)
        net.sync()
        assert torch.equal(swapped, full)
    finally:
        net.close()


def test_schedule_with_prefetch_matches_resident():
    """9 steps, a normal step every 3rd, the entry swapped out after it and prefetched one step ahead into the other
    device slot; free-running (x <- x - 0.1 * eps). Bit-identical to the run that keeps the entry resident."""
    cfg = SMALL_BF16
    w = synth.make_unet_weights(cfg, 0)
    net = lcb.Unet(cfg, w, host_slots=3, dev_slots=2)
    try:
        x, temb, ctx = synth.make_unet_inputs(cfg, 1)
        x0, td, cd = net.to_device(x), net.to_device(temb), net.to_device(ctx)

        def run(swapping, steps=9, interval=3):
            xx, outs, refresh, prefetched = x0.clone(), [], -1, None
            for t in range(steps):
                slot = t % 2 if swapping else 0
                out = net.empty(*x.shape)
                if t % interval == 0:
                    refresh += 1
                    net.full_step(xx, td, cd, out, slot)
                    if swapping:
                        net.swap_out(slot, refresh)
                else:
                    if swapping and prefetched != (t, slot):
                        net.swap_in(refresh, slot)
                    net.cached_step(xx, td, cd, out, slot)
                if swapping and t + 1 < steps and (t + 1) % interval != 0:
                    net.swap_in(refresh, (t + 1) % 2)
                    prefetched = (t + 1, (t + 1) % 2)
                outs.append(out)
                xx = xx - 0.1 * out
            net.sync()
            return outs
        with torch.cuda.stream(net.compute):  # torch's own update of x must be ordered with the library's kernels
            ref, got = run(False), run(True)
        for t, (a, b) in enumerate(zip(got, ref)):
            assert torch.equal(a, b), t
        assert not torch.equal(ref[1], ref[0])
    finally:
        net.close()


def test_unet_errors():
    cfg = SMALL_F32
    w = synth.make_unet_weights(cfg, 0)
    net = lcb.Unet(cfg, w, host_slots=1, dev_slots=2)
    try:
        x, temb, ctx = synth.make_unet_inputs(cfg, 1)
        xd, td, cd = net.to_device(x), net.to_device(temb), net.to_device(ctx)
        out = net.empty(*x.shape)

        def status(fn, *a):
            with pytest.raises(lcb.LcError) as e:
                fn(*a)
            return e.value.status
        assert status(net.cached_step, xd, td, cd, out, 0) == lcb.LC_ERR_STATE
        assert status(net.swap_out, 0, 0) == lcb.LC_ERR_STATE
        assert status(net.swap_in, 0, 0) == lcb.LC_ERR_STATE
        assert status(net.full_step, xd, td, cd, out, 2) == lcb.LC_ERR_ARG
        assert status(net.swap_out, 0, 1) == lcb.LC_ERR_ARG
        small = torch.empty(1 << 16, dtype=torch.uint8, device=net.device)
        assert status(lcb.lc_unet_set_workspace, net.ctx, small.data_ptr(), small.numel()) == lcb.LC_ERR_NOMEM
        assert status(lcb.lc_unet_set_workspace, net.ctx, small.data_ptr() + 8, small.numel()) == lcb.LC_ERR_ARG
        assert status(net.set_chunk, -1) == lcb.LC_ERR_ARG
        assert status(lcb.lc_unet_full_step, net.ctx, None, td.data_ptr(), cd.data_ptr(), out.data_ptr(), 0) == lcb.LC_ERR_ARG
        assert status(lcb.lc_unet_load_weights, net.ctx, lcb.lc_unet_weights()) == lcb.LC_ERR_ARG
        net.full_step(xd, td, cd, out, 0)
        net.sync()
        assert bool(torch.isfinite(out).all())
    finally:
        net.close()
