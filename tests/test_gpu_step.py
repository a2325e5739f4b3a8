"""GPU parity of the whole path through the C ABI: full and cached steps against the float64
oracle, the method's invariants on the device (chunked == unchunked bit for bit, cached == full
on the same input, swap round trip byte-identical), the double-buffered schedule, and the error
behaviour of the state machine."""
import numpy as np
import pytest
import torch

from oracle import lightcache_oracle as lo
from paper_2510_05367_amd import binding as lcb
from paper_2510_05367_amd import synth
from tests.gpu_util import check, dev, host, make_stage

pytestmark = pytest.mark.gpu

TINY = synth.CONFIGS["tiny"]
# ragged little stages (image not a multiple of the 8 x 16 pixel tile, frames not a multiple of the chunk)
RAG_F32 = synth.StageConfig("rag_f32", B=2, F=3, H=10, W=12, C_lat=4, C=64, C_deep=128, groups=32, n_res=1,
                            heads=1, head_dim=64, dtype="f32")
RAG_BF16 = synth.StageConfig("rag_bf16", B=2, F=3, H=10, W=12, C_lat=4, C=320, C_deep=640, groups=32, n_res=2,
                             heads=8, head_dim=40, dtype="bf16")
RAG_BF16_D64 = synth.StageConfig("rag_bf16_d64", B=1, F=5, H=12, W=18, C_lat=4, C=320, C_deep=640, groups=32,
                                 n_res=2, heads=5, head_dim=64, dtype="bf16")
# image rows of whole 32-pixel segments: conv_in runs in its tile kernel, every linear layer on whole 32-row tiles
W32_BF16 = synth.StageConfig("w32_bf16", B=1, F=3, H=6, W=32, C_lat=4, C=320, C_deep=640, groups=32, n_res=1,
                             heads=8, head_dim=40, dtype="bf16")


def oracle_for(cfg, w, **kw):
    return lo.Oracle(cfg, {k: v.astype(np.float64) for k, v in w.items()}, **kw)


@pytest.mark.parametrize("cfg,sharp,fc,tc", [
    (TINY, 1.0, 2, 0), (TINY, 8.0, 0, 0), (RAG_F32, 1.0, 4, 50), (RAG_F32, 8.0, 0, 0),
    (RAG_BF16, 1.0, 4, 0), (RAG_BF16, 8.0, 0, 33), (RAG_BF16_D64, 1.0, 2, 100), (RAG_BF16_D64, 8.0, 0, 0),
    (W32_BF16, 1.0, 2, 0), (W32_BF16, 8.0, 0, 64),
], ids=lambda v: getattr(v, "name", str(v)))
def test_full_and_cached_step_match_oracle(cfg, sharp, fc, tc):
    print(f"\n[case] {cfg.name} sharp={sharp} chunk=({fc},{tc})", flush=True)
    stage, w = make_stage(cfg, seed=0, sharp=sharp, frame_chunk=fc, token_chunk=tc)
    try:
        x = synth.make_latents(cfg, 1)
        xd = dev(stage, x)
        eps = stage.empty(*x.shape)
        orc = oracle_for(cfg, w)
        # normal step: fills slot 0
        stage.full_step(xd, eps, 0)
        stage.sync()
        ref = orc.full_step(x, 0)
        check("full_step eps", host(eps), ref, cfg.dtype)
        check("full_step deep", host(stage.cache_read(0)), orc.dev[0], cfg.dtype, cache_entry=True)
        # cache step on a foreign deep feature in slot 1
        deep = synth.make_deep(cfg, 2)
        stage.cache_write(1, dev(stage, deep))
        x2 = synth.make_latents(cfg, 3)
        x2d = dev(stage, x2)
        eps2 = stage.empty(*x.shape)
        stage.cached_step(x2d, eps2, 1)
        stage.sync()
        orc.cache_write(1, deep)
        check("cached_step eps", host(eps2), orc.cached_step(x2, 1), cfg.dtype)
        # injected deep feature is stored exactly
        assert np.array_equal(host(stage.cache_read(1)), deep.astype(np.float64))
    finally:
        stage.close()


@pytest.mark.parametrize("cfg", [RAG_F32, RAG_BF16, W32_BF16], ids=lambda c: c.name)
def test_chunked_equals_unchunked_bitwise(cfg):
    stage, w = make_stage(cfg, seed=0, sharp=4.0, frame_chunk=0, token_chunk=0)
    try:
        x = dev(stage, synth.make_latents(cfg, 1))
        ref_full, ref_cached = stage.empty(*x.shape), stage.empty(*x.shape)
        stage.full_step(x, ref_full, 0)
        stage.cached_step(x, ref_cached, 0)
        stage.sync()
        deep_ref = stage.dev_entry_bytes(0)
        for fc, tc in [(1, 0), (2, 0), (4, 0), (5, 0), (16, 0), (0, 1), (0, 50), (3, 64), (2, 1000)]:
            print(f"[chunk] {cfg.name} ({fc},{tc})", flush=True)
            stage.set_chunk(fc, tc)
            a, b = stage.empty(*x.shape), stage.empty(*x.shape)
            stage.full_step(x, a, 1)
            stage.cached_step(x, b, 1)
            stage.sync()
            assert torch.equal(a, ref_full), (fc, tc)
            assert torch.equal(b, ref_cached), (fc, tc)
            assert stage.dev_entry_bytes(1) == deep_ref, (fc, tc)
        # the chunks above ran on two lanes (alternate chunks on two streams); on one lane: the same bits
        stage.set_lanes(1)
        for fc, tc in [(2, 0), (3, 64)]:
            print(f"[chunk] {cfg.name} ({fc},{tc}) one lane", flush=True)
            stage.set_chunk(fc, tc)
            a, b = stage.empty(*x.shape), stage.empty(*x.shape)
            stage.full_step(x, a, 1)
            stage.cached_step(x, b, 1)
            stage.sync()
            assert torch.equal(a, ref_full), (fc, tc)
            assert torch.equal(b, ref_cached), (fc, tc)
        with pytest.raises(lcb.LcError):
            stage.set_lanes(3)
    finally:
        stage.close()


@pytest.mark.parametrize("cfg", [TINY, RAG_BF16], ids=lambda c: c.name)
def test_cached_equals_full_and_swap_round_trip(cfg):
    stage, w = make_stage(cfg, seed=0, host_slots=3, dev_slots=2)
    try:
        x = dev(stage, synth.make_latents(cfg, 1))
        e_full, e_c0, e_c1 = (stage.empty(*x.shape) for _ in range(3))
        stage.full_step(x, e_full, 0)
        stage.cached_step(x, e_c0, 0)
        stage.swap_out(0, 2)
        stage.sync()
        assert torch.equal(e_c0, e_full)  # cached step fed its own cache == full step
        dev_bytes = stage.dev_entry_bytes(0)
        assert stage.host_entry_bytes(2) == dev_bytes
        # poison the other device slot, then bring the entry back into it
        poison = torch.full((cfg.N, cfg.C_deep, cfg.H // 2, cfg.W // 2), float("nan"), dtype=stage.tdtype,
                            device=stage.device)
        stage.cache_write(1, poison)
        stage.swap_in(2, 1)
        stage.cached_step(x, e_c1, 1)  # must wait for the copy on the GPU
        stage.sync()
        assert stage.dev_entry_bytes(1) == dev_bytes
        assert torch.equal(e_c1, e_full)
        st = lcb.lc_get_stats(stage.ctx)
        assert (st.swaps_out, st.swaps_in) == (1, 1)
        assert st.bytes_out == st.bytes_in == len(dev_bytes)
        assert st.ms_out > 0 and st.ms_in > 0
    finally:
        stage.close()


def test_schedule_double_buffered_teacher_forced():
    """25 steps on the tiny stage, a normal step every 3rd; after each normal step the deep feature
    is swapped out; each cache step reads a device slot refilled one step ahead from the host bank
    (alternating slots). Every step is fed the oracle's latent and compared with the oracle."""
    cfg = TINY
    steps, interval = 25, 3
    stage, w = make_stage(cfg, seed=0, host_slots=2, dev_slots=2)
    try:
        orc = oracle_for(cfg, w, host_slots=2, dev_slots=2)
        xs, refs = lo.run_schedule(orc, synth.make_latents(cfg, 1), steps, interval)
        outs = [stage.empty(*xs[0].shape) for _ in range(steps)]
        xd = [dev(stage, x.astype(np.float32)) for x in xs]
        refresh = -1
        prefetched = None  # (step, dev slot) whose swap-in is already enqueued
        for t in range(steps):
            slot = t % 2
            if t % interval == 0:
                refresh += 1
                stage.full_step(xd[t], outs[t], slot)
                stage.swap_out(slot, refresh % 2)
            else:
                if prefetched != (t, slot):
                    stage.swap_in(refresh % 2, slot)
                stage.cached_step(xd[t], outs[t], slot)
            nxt = t + 1
            if nxt < steps and nxt % interval != 0:
                stage.swap_in(refresh % 2, nxt % 2)  # one step ahead, into the other buffer
                prefetched = (nxt, nxt % 2)
        stage.sync()
        worst = 0.0
        for t in range(steps):
            g = host(outs[t])
            r = float(np.linalg.norm(g - refs[t]) / np.linalg.norm(refs[t]))
            worst = max(worst, r)
            assert r <= 1e-4, (t, r)
        print(f"schedule: worst teacher-forced rel-L2 over {steps} steps = {worst:.3e}", flush=True)
        st = lcb.lc_get_stats(stage.ctx)
        assert st.full_steps == 9 and st.cached_steps == 16 and st.swaps_out == 9
    finally:
        stage.close()


def test_state_machine_errors():
    cfg = RAG_F32
    stage, w = make_stage(cfg, seed=0, host_slots=1, dev_slots=2)
    try:
        x = dev(stage, synth.make_latents(cfg, 1))
        eps = stage.empty(*x.shape)

        def status(fn, *a):
            with pytest.raises(lcb.LcError) as e:
                fn(*a)
            return e.value.status

        assert status(stage.cached_step, x, eps, 0) == lcb.LC_ERR_STATE
        assert status(stage.swap_out, 0, 0) == lcb.LC_ERR_STATE
        assert status(stage.swap_in, 0, 0) == lcb.LC_ERR_STATE
        assert status(stage.full_step, x, eps, 2) == lcb.LC_ERR_ARG
        assert status(stage.swap_out, 0, 1) == lcb.LC_ERR_ARG
        assert status(lcb.lc_set_chunk, stage.ctx, -1, 0) == lcb.LC_ERR_ARG
        assert status(lcb.lc_full_step, stage.ctx, None, eps.data_ptr(), 0) == lcb.LC_ERR_ARG
        assert status(lcb.lc_cache_peek, stage.ctx, 0) == lcb.LC_ERR_STATE
        assert "empty" in lcb.lc_last_error(stage.ctx)
        # a workspace that is too small is refused and the old one stays in force
        small = torch.empty(1 << 20, dtype=torch.uint8, device=stage.device)
        assert status(lcb.lc_set_workspace, stage.ctx, small.data_ptr(), small.numel()) == lcb.LC_ERR_NOMEM
        assert status(lcb.lc_set_workspace, stage.ctx, small.data_ptr() + 8, small.numel()) == lcb.LC_ERR_ARG
        stage.full_step(x, eps, 0)
        stage.sync()
        assert bool(torch.isfinite(eps.float()).all())
    finally:
        stage.close()
    # a context without weights / workspace
    ccfg = lcb.make_config(cfg)
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    ctx = lcb.lc_create(ccfg, s1.cuda_stream, s2.cuda_stream)
    try:
        with pytest.raises(lcb.LcError) as e:
            lcb.lc_full_step(ctx, 1, 1, 0)
        assert e.value.status == lcb.LC_ERR_STATE
        with pytest.raises(lcb.LcError) as e:
            lcb.lc_create(ccfg, s1.cuda_stream, s1.cuda_stream)
        assert e.value.status == lcb.LC_ERR_ARG
    finally:
        lcb.lc_destroy(ctx)


# stages whose frames are whole tiles of every kernel: 16 image rows (two 8-row conv tiles) of 64 / 32 pixels
SP_BF16 = synth.StageConfig("sp_bf16", B=1, F=3, H=16, W=64, C_lat=4, C=320, C_deep=640, groups=32, n_res=2,
                            heads=8, head_dim=40, dtype="bf16")
SP_F32 = synth.StageConfig("sp_f32", B=2, F=2, H=16, W=32, C_lat=4, C=64, C_deep=128, groups=32, n_res=1,
                           heads=1, head_dim=64, dtype="f32")


@pytest.mark.parametrize("cfg", [SP_BF16, SP_F32], ids=lambda c: c.name)
def test_spatial_chunk_equals_whole_frame_bitwise_and_matches_oracle(cfg):
    """The literal spatial feature chunk (H/eta x W/omega blocks, one-pixel halo from the neighbouring blocks, split
    GroupNorm sums, a block's queries against the whole frame's keys): bit-identical to the unchunked step for every
    factor pair the stage admits, alone and inside frame chunks, on one lane and two; and equal to the oracle's own
    block loops within the tolerance."""
    stage, w = make_stage(cfg, seed=0, sharp=4.0, frame_chunk=0, token_chunk=0)
    try:
        x = synth.make_latents(cfg, 1)
        xd = dev(stage, x)
        ref_full, ref_cached = stage.empty(*x.shape), stage.empty(*x.shape)
        stage.full_step(xd, ref_full, 0)
        deep = synth.make_deep(cfg, 2)
        stage.cache_write(1, dev(stage, deep))
        stage.cached_step(xd, ref_cached, 1)
        stage.sync()
        deep_ref = stage.dev_entry_bytes(0)
        pairs = [(2, 1), (1, 2), (2, 2)] if cfg.W == 64 else [(2, 1)]
        for eta, omega in pairs:
            for fc, lanes in [(0, 2), (2, 2), (1, 1)]:
                print(f"[spatial] {cfg.name} eta={eta} omega={omega} frame chunk {fc} lanes {lanes}", flush=True)
                stage.set_chunk(fc, 0)
                stage.set_spatial_chunk(eta, omega)
                stage.set_lanes(lanes)
                stage.cache_write(1, dev(stage, deep))  # (a larger workspace, once it is needed, starts with empty slots)
                a, b = stage.empty(*x.shape), stage.empty(*x.shape)
                stage.full_step(xd, a, 0)
                stage.cached_step(xd, b, 1)
                stage.sync()
                assert torch.equal(a, ref_full), (eta, omega, fc)
                assert torch.equal(b, ref_cached), (eta, omega, fc)
                assert stage.dev_entry_bytes(0) == deep_ref
        orc = oracle_for(cfg, w)
        orc.set_spatial_chunk(*pairs[-1])
        orc.cache_write(1, deep)
        check("cached_step eps (spatial chunk)", host(b), orc.cached_step(x, 1), cfg.dtype)
        # factors that do not give whole tiles are refused and leave the setting as it was
        for eta, omega, code in [(3, 1, lcb.LC_ERR_SHAPE), (4, 1, lcb.LC_ERR_SHAPE), (1, 4, lcb.LC_ERR_SHAPE),
                                 (0, 1, lcb.LC_ERR_ARG)]:
            with pytest.raises(lcb.LcError) as e:
                lcb.lc_set_spatial_chunk(stage.ctx, eta, omega)
            assert e.value.status == code, (eta, omega)
        c2 = stage.empty(*x.shape)
        stage.cached_step(xd, c2, 1)
        stage.sync()
        assert torch.equal(c2, ref_cached)
        stage.set_spatial_chunk(1, 1)
    finally:
        stage.close()


def test_double_destroy_and_failed_pinned_allocation():
    cfg = RAG_F32
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    ccfg = lcb.make_config(cfg, host_slots=3, dev_slots=2)
    ctx = lcb.lc_create(ccfg, s1.cuda_stream, s2.cuda_stream)
    lcb.lc_destroy(ctx)
    with pytest.raises(lcb.LcError) as e:  # the second time the pointer is unknown: an error, not a crash
        lcb.lc_destroy(ctx)
    assert e.value.status == lcb.LC_ERR_ARG
    # the second of three pinned allocations fails: LC_ERR_NOMEM, nothing left behind, the next create works
    free0 = torch.cuda.mem_get_info()[0]
    lcb.lc_test_fail_host_alloc(2)
    with pytest.raises(lcb.LcError) as e:
        lcb.lc_create(ccfg, s1.cuda_stream, s2.cuda_stream)
    assert e.value.status == lcb.LC_ERR_NOMEM and "pinned" in str(e.value)
    ctx = lcb.lc_create(ccfg, s1.cuda_stream, s2.cuda_stream)  # the hook fires once
    lcb.lc_destroy(ctx)
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] >= free0 - (8 << 20)


def test_profile_reports_dropped_brackets_and_untimed_copies():
    cfg = RAG_F32
    stage, w = make_stage(cfg, seed=0, frame_chunk=1, host_slots=1)
    try:
        x = dev(stage, synth.make_latents(cfg, 1))
        eps = stage.empty(*x.shape)
        stage.full_step(x, eps, 0)
        stage.swap_out(0, 0)
        lcb.lc_set_profiling(stage.ctx, 1 << lcb.LC_K["gn_final"])
        stage.cached_step(x, eps, 0)
        per_step = lcb.lc_get_profile(stage.ctx)["gn_final"]["launches"]
        assert per_step >= 6
        n = 4096 // per_step + 10  # more finalize launches than the 4096 brackets
        for i in range(n):
            stage.cached_step(x, eps, 0)
        prof = lcb.lc_get_profile(stage.ctx)
        assert prof["gn_final"]["launches"] == 4096 and prof["dropped"] == per_step * n - 4096
        assert lcb.lc_get_profile(stage.ctx)["dropped"] == 0
        lcb.lc_set_profiling(stage.ctx, 0)
        # more swaps than timing event pairs between two lc_get_stats: completed pairs are recycled on the way
        lcb.lc_reset_stats(stage.ctx)
        for i in range(600):
            stage.swap_in(0, 1)
        st = lcb.lc_get_stats(stage.ctx)
        assert st.swaps_in == 600 and 256 <= st.timed_in <= 600 and st.ms_in > 0
    finally:
        stage.close()


def test_profiling_brackets_count_launches():
    cfg = RAG_F32
    stage, w = make_stage(cfg, seed=0, frame_chunk=2)
    try:
        x = dev(stage, synth.make_latents(cfg, 1))
        eps = stage.empty(*x.shape)
        stage.cache_write(0, dev(stage, synth.make_deep(cfg, 2)))
        lcb.lc_set_profiling(stage.ctx, (1 << lcb.LC_K["conv_up"]) | (1 << lcb.LC_K["sattn"]))
        stage.cached_step(x, eps, 0)
        prof = lcb.lc_get_profile(stage.ctx)
        assert prof["conv_up"]["launches"] == 3 and prof["sattn"]["launches"] == 3  # 6 frames / chunk 2
        assert prof["conv_up"]["ms"] > 0 and prof["conv_res"]["launches"] == 0
        lcb.lc_set_profiling(stage.ctx, 0)
    finally:
        stage.close()
