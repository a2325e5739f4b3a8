"""The entry point for callers that cannot allocate (lc_cached_step_static): the cache step on the library's
static device array. Through the C ABI, against lc_cached_step on a caller-owned workspace: the same kernels on the
same data, so the outputs must agree bit for bit. Two calls in a row, the second with a smaller stage (the array
still holds the first call's contents); then the size limit."""
import numpy as np
import pytest
import torch

from paper_2510_05367_amd import binding as lcb
from paper_2510_05367_amd import synth
from tests.gpu_util import dev, make_stage

pytestmark = pytest.mark.gpu

BIG = synth.CONFIGS["tiny"].with_(name="static_a", F=6)                       # fp32, 32 x 32, frame chunk 2
SMALL = synth.StageConfig("static_b", B=1, F=3, H=10, W=12, C_lat=4, C=320, C_deep=640, groups=32, n_res=2,
                          heads=8, head_dim=40, dtype="bf16", frame_chunk=2)  # bf16, ragged, smaller footprint


def test_static_scratch_matches_workspace_path():
    assert lcb.lc_workspace_bytes(lcb.make_config(BIG), BIG.frame_chunk, 0) <= lcb.lc_static_scratch_bytes()
    assert (lcb.lc_workspace_bytes(lcb.make_config(SMALL), SMALL.frame_chunk, 0)
            < lcb.lc_workspace_bytes(lcb.make_config(BIG), BIG.frame_chunk, 0))
    stages = []
    try:
        for cfg in (BIG, SMALL):
            print(f"\n[case] {cfg.name} {cfg.dtype} N={cfg.N} {cfg.H}x{cfg.W} C={cfg.C}", flush=True)
            stage, w = make_stage(cfg, seed=3)
            stages.append(stage)
            x = dev(stage, synth.make_latents(cfg, 4))
            deep = dev(stage, synth.make_deep(cfg, 5))
            ref, got = stage.empty(*x.shape), stage.empty(*x.shape)
            got.fill_(float("nan"))
            stage.cache_write(0, deep)
            stage.cached_step(x, ref, 0)
            stage.sync()
            free0 = torch.cuda.mem_get_info()[0]
            steps0 = lcb.lc_get_stats(stage.ctx).cached_steps
            lcb.lc_cached_step_static(stage.ctx, x.data_ptr(), deep.data_ptr(), got.data_ptr())
            stage.sync()
            assert torch.cuda.mem_get_info()[0] == free0          # nothing was allocated or freed
            assert bool(torch.isfinite(ref.float()).all())
            assert torch.equal(got, ref), cfg.name
            assert lcb.lc_get_stats(stage.ctx).cached_steps == steps0 + 1
            # the context's own workspace and slot are as they were: the ordinary step still gives the same
            again = stage.empty(*x.shape)
            stage.cached_step(x, again, 0)
            stage.sync()
            assert torch.equal(again, ref)
        # the first stage once more, after the smaller one has used the array
        stage, cfg = stages[0], BIG
        x = dev(stage, synth.make_latents(cfg, 4))
        deep = dev(stage, synth.make_deep(cfg, 5))
        ref, got = stage.empty(*x.shape), stage.empty(*x.shape)
        stage.cached_step(x, ref, 0)
        lcb.lc_cached_step_static(stage.ctx, x.data_ptr(), deep.data_ptr(), got.data_ptr())
        stage.sync()
        assert torch.equal(got, ref)
    finally:
        for s in stages:
            s.close()


def test_static_scratch_rejects_what_does_not_fit():
    cfg = synth.CONFIGS["animatediff"].with_(B=1, F=4)
    assert lcb.lc_workspace_bytes(lcb.make_config(cfg), cfg.frame_chunk, 0) > lcb.lc_static_scratch_bytes()
    stage, w = make_stage(cfg, seed=3)
    try:
        x = dev(stage, synth.make_latents(cfg, 4))
        deep = dev(stage, synth.make_deep(cfg, 5))
        eps = stage.empty(*x.shape)
        with pytest.raises(lcb.LcError) as e:
            lcb.lc_cached_step_static(stage.ctx, x.data_ptr(), deep.data_ptr(), eps.data_ptr())
        assert e.value.status == lcb.LC_ERR_NOMEM and "static scratch" in str(e.value)
        with pytest.raises(lcb.LcError) as e:
            lcb.lc_cached_step_static(stage.ctx, x.data_ptr(), None, eps.data_ptr())
        assert e.value.status == lcb.LC_ERR_ARG
    finally:
        stage.close()
