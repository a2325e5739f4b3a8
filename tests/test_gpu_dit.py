"""GPU parity of the diffusion-transformer variant: normal and cache steps through the C ABI against the CPU oracle,
the method's invariants (cache step on its own Delta == normal step and chunked == unchunked, bit for bit; the cache
bank byte-identical), the schedule with swapping, errors."""
import numpy as np
import pytest
import torch

from oracle import dit_oracle as dito
from paper_2510_05367_amd import binding as lcb
from paper_2510_05367_amd import synth
from tests.gpu_util import check, host

pytestmark = pytest.mark.gpu

DIT_F32 = synth.DitConfig("dit_f32", B=2, T=150, D=128, heads=2, head_dim=64, L=4, cache_a=1, cache_b=3, dtype="f32")
DIT_BF16 = synth.DitConfig("dit_bf16", B=1, T=200, D=320, heads=8, head_dim=40, L=3, cache_a=1, cache_b=2, dtype="bf16")
DIT_BF16_W = synth.DitConfig("dit_bf16_w", B=2, T=96, D=256, heads=4, head_dim=64, L=5, cache_a=0, cache_b=3, dtype="bf16",
                             mlp_ratio=2)
BIG = synth.DITS["video_dit"]


def w64_of(w):
    return {k: v.astype(np.float64) for k, v in w.items()}


@pytest.mark.parametrize("cfg,chunk", [(DIT_F32, 0), (DIT_F32, 64), (DIT_BF16, 70), (DIT_BF16, 33), (DIT_BF16_W, 32)], ids=lambda v: getattr(v, "name", str(v)))
def test_steps_match_oracle(cfg, chunk):
    print(f"\n[case] {cfg.name} B={cfg.B} T={cfg.T} D={cfg.D} L={cfg.L} cached [{cfg.cache_a},{cfg.cache_b}) chunk {chunk}", flush=True)
    w = synth.make_dit_weights(cfg, 0, sharp=8.0)  # logit std of about 8: a peaked softmax
    dit = lcb.Dit(cfg, w, host_slots=1, dev_slots=2, token_chunk=chunk)
    try:
        x = synth.make_dit_hidden(cfg, 1)
        mod = synth.make_dit_modulation(cfg, 2)
        xd, md = dit.to_device(x), dit.to_device(mod)
        out = dit.empty(*x.shape)
        dit.full_step(xd, md, out, 0)
        dit.sync()
        orc = dito.DitOracle(cfg, w64_of(w))
        ref = orc.full_step(x, mod, 0)
        assert float(np.std(ref - x)) > 1e-2
        check("normal step", host(out), ref, cfg.dtype, wide_range=True)
        check("Delta", host(dit.dev_entry(0)), orc.dev[0], cfg.dtype)
        # cache step on a foreign Delta and a new input
        delta = (synth.make_dit_hidden(cfg, 5) * np.float32(0.5)).astype(np.float32)
        x2 = synth.make_dit_hidden(cfg, 6)
        dit.cache_write(1, dit.to_device(delta))
        out2 = dit.empty(*x.shape)
        dit.cached_step(dit.to_device(x2), md, out2, 1)
        dit.sync()
        orc.cache_write(1, delta)
        check("cache step", host(out2), orc.cached_step(x2, mod, 1), cfg.dtype, wide_range=True)
    finally:
        dit.close()


@pytest.mark.parametrize("cfg", [DIT_F32, DIT_BF16], ids=lambda c: c.name)
def test_invariants_bitwise(cfg):
    w = synth.make_dit_weights(cfg, 0, sharp=10.0)
    dit = lcb.Dit(cfg, w, host_slots=2, dev_slots=2, token_chunk=0)
    try:
        xd = dit.to_device(synth.make_dit_hidden(cfg, 1))
        md = dit.to_device(synth.make_dit_modulation(cfg, 2))
        full, cached, swapped = (dit.empty(cfg.B, cfg.T, cfg.D) for _ in range(3))
        dit.full_step(xd, md, full, 0)
        dit.cached_step(xd, md, cached, 0)
        dit.swap_out(0, 1)
        dit.sync()
        assert bool(torch.isfinite(full).all())
        assert torch.equal(cached, full)  # cache step on its own Delta == normal step
        d0 = dit.dev_entry(0)
        assert dit.host_entry_bytes(1) == d0.cpu().numpy().tobytes()
        dit.cache_write(1, torch.full_like(d0, float("nan")))  # poison the other slot, then bring the entry back
        dit.swap_in(1, 1)
        dit.cached_step(xd, md, swapped, 1)  # must wait for the copy on the GPU
        dit.sync()
        assert torch.equal(dit.dev_entry(1), d0) and torch.equal(swapped, full)
        assert lcb.lc_dit_get_counts(dit.ctx) == (1, 2, 1, 1)
        for chunk in (1, 37, 64, cfg.T - 1, cfg.T + 5):  # token chunks never change a bit
            print(f"[chunk] {cfg.name} {chunk}", flush=True)
            dit.set_chunk(chunk)
            a, b = dit.empty(cfg.B, cfg.T, cfg.D), dit.empty(cfg.B, cfg.T, cfg.D)
            dit.full_step(xd, md, a, 0)
            dit.cached_step(xd, md, b, 0)
            dit.sync()
            assert torch.equal(a, full) and torch.equal(b, full), chunk
            assert torch.equal(dit.dev_entry(0), d0), chunk
    finally:
        dit.close()


def test_schedule_with_prefetch_matches_resident():
    """12 steps, a normal step every 4th, Delta swapped out after it and prefetched one step ahead into the other
    device slot; free-running (x <- x - 0.05 * (out - x)). Bit-identical to the run that keeps Delta resident."""
    cfg = DIT_BF16_W
    w = synth.make_dit_weights(cfg, 0)
    dit = lcb.Dit(cfg, w, host_slots=3, dev_slots=2, token_chunk=32)
    try:
        x0 = dit.to_device(synth.make_dit_hidden(cfg, 1))
        md = dit.to_device(synth.make_dit_modulation(cfg, 2))

        def run(swapping, steps=12, interval=4):
            x, outs, refresh, prefetched = x0.clone(), [], -1, None
            for t in range(steps):
                slot = t % 2 if swapping else 0
                out = dit.empty(cfg.B, cfg.T, cfg.D)
                if t % interval == 0:
                    refresh += 1
                    dit.full_step(x, md, out, slot)
                    if swapping:
                        dit.swap_out(slot, refresh)
                else:
                    if swapping and prefetched != (t, slot):
                        dit.swap_in(refresh, slot)
                    dit.cached_step(x, md, out, slot)
                if swapping and t + 1 < steps and (t + 1) % interval != 0:
                    dit.swap_in(refresh, (t + 1) % 2)
                    prefetched = (t + 1, (t + 1) % 2)
                outs.append(out)
                x = x - 0.05 * (out - x)
            dit.sync()
            return outs
        with torch.cuda.stream(dit.compute):  # torch's own update of x must be ordered with the library's kernels
            ref, got = run(False), run(True)
        for t, (a, b) in enumerate(zip(got, ref)):
            assert torch.equal(a, b), t
    finally:
        dit.close()


def test_dit_errors_and_footprint():
    cfg = DIT_F32
    c = lcb.make_dit_config(cfg)
    assert lcb.lc_dit_entry_bytes(c) == cfg.B * cfg.T * cfg.D * 4
    assert lcb.lc_dit_workspace_bytes(c, 16) < lcb.lc_dit_workspace_bytes(c, 64) < lcb.lc_dit_workspace_bytes(c, 0)
    w = synth.make_dit_weights(cfg, 0)
    dit = lcb.Dit(cfg, w, host_slots=1, dev_slots=2, token_chunk=16)
    try:
        xd = dit.to_device(synth.make_dit_hidden(cfg, 1))
        md = dit.to_device(synth.make_dit_modulation(cfg, 2))
        out = dit.empty(cfg.B, cfg.T, cfg.D)

        def status(fn, *a):
            with pytest.raises(lcb.LcError) as e:
                fn(*a)
            return e.value.status
        assert status(dit.cached_step, xd, md, out, 0) == lcb.LC_ERR_STATE
        assert status(dit.swap_out, 0, 0) == lcb.LC_ERR_STATE
        assert status(dit.swap_in, 0, 0) == lcb.LC_ERR_STATE
        assert status(dit.full_step, xd, md, out, 2) == lcb.LC_ERR_ARG
        assert status(lcb.lc_dit_set_chunk, dit.ctx, -1) == lcb.LC_ERR_ARG
        small = torch.empty(1 << 16, dtype=torch.uint8, device=dit.device)
        assert status(lcb.lc_dit_set_workspace, dit.ctx, small.data_ptr(), small.numel()) == lcb.LC_ERR_NOMEM
        assert status(lcb.lc_dit_set_workspace, dit.ctx, small.data_ptr() + 8, small.numel()) == lcb.LC_ERR_ARG
        assert status(lcb.lc_dit_full_step, dit.ctx, None, md.data_ptr(), out.data_ptr(), 0) == lcb.LC_ERR_ARG
        dit.full_step(xd, md, out, 0)
        dit.sync()
        assert bool(torch.isfinite(out).all())
    finally:
        dit.close()


@pytest.mark.slow
def test_video_dit_full_size_one_batch_element():
    """The benchmark's video DiT (4096 tokens, width 1024, 16 heads of 64) with one batch element and 4 blocks (2
    of them cached), in the workload's token chunks: normal and cache step against the oracle."""
    cfg = BIG.with_(B=1, L=4, cache_a=1, cache_b=3)
    print(f"\n[case] {cfg.name} B=1 T={cfg.T} D={cfg.D} L={cfg.L} chunk {cfg.token_chunk}", flush=True)
    w = synth.make_dit_weights(cfg, 0)
    dit = lcb.Dit(cfg, w, host_slots=1, dev_slots=2)
    try:
        x = synth.make_dit_hidden(cfg, 1)
        mod = synth.make_dit_modulation(cfg, 2)
        xd, md = dit.to_device(x), dit.to_device(mod)
        full, cached = dit.empty(*x.shape), dit.empty(*x.shape)
        dit.full_step(xd, md, full, 0)
        dit.cached_step(xd, md, cached, 0)
        dit.sync()
        assert torch.equal(full, cached)
        orc = dito.DitOracle(cfg, w64_of(w))
        orc.set_chunk(cfg.token_chunk)
        print("[oracle] normal step ...", flush=True)
        check("normal step", host(full), orc.full_step(x, mod, 0), cfg.dtype, wide_range=True)
    finally:
        dit.close()
