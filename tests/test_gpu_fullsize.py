"""GPU parity at the workloads' real shapes. The float64 oracle cannot run a whole 32- or 50-frame
stage in a test's time, so the full sizes are covered three ways:
  * whole steps at the full image size, channel widths, head layout and chunk sizes, with one
    chunk's worth of frames (every launch then has the shape the timed configuration uses),
    compared element by element with the oracle; for the benchmark workload also with all 16 frames of
    one batch element (four frame chunks on two lanes, the temporal block over 16 frames);
  * single operators over all B*F frames, compared with the oracle on sampled frames, sampled
    query tokens and sampled spatial positions (each of which the oracle can compute on its own);
  * the method's invariants on the whole stage at full size: chunked == unchunked bit for bit,
    and a cached step fed the cache of the same input == the full step."""
import numpy as np
import pytest
import torch

from oracle import lightcache_oracle as lo
from paper_2510_05367_amd import binding as lcb
from paper_2510_05367_amd import synth
from tests.gpu_util import check, dev, dev32, empty32, host, make_stage, planar_to_rows, rows_to_planar

pytestmark = pytest.mark.gpu

AD = synth.CONFIGS["animatediff"]
SVD = synth.CONFIGS["svdxt"]
STRESS = synth.CONFIGS["stress"]


def w64_of(w):
    return {k: v.astype(np.float64) for k, v in w.items()}


# ------------------------------------------------------------------------------------------
# whole steps, one chunk of frames at the full image size
# ------------------------------------------------------------------------------------------
# (AD, 16): one batch element with all 16 frames, frame chunk 4 on two lanes - every launch of the cached step as
# bench.py times it, the 16-frame temporal attention on its MFMA tiles included; the oracle takes about 15 s for it.
# (SVD, 25) and (STRESS, 32): one batch element with all its frames in the workload's own chunking (frame chunk 5 +
# token chunk 2304: query windows of the spatial attention, position chunks of the temporal block over 25 frames on
# the 32 x 32 MFMA tiles; frame chunk 8 over 32 frames of 96 x 96); the oracle takes one to two minutes for each.
@pytest.mark.parametrize("base,F,full_too", [(AD, 4, True), (SVD, 2, False), (AD, 16, False),
                                             pytest.param(SVD, 25, False, marks=pytest.mark.slow),
                                             pytest.param(STRESS, 32, False, marks=pytest.mark.slow)],
                         ids=lambda v: getattr(v, "name", str(v)))
def test_step_one_chunk_full_image(base, F, full_too):
    cfg = base.with_(B=1, F=F)
    fc, tc = min(base.frame_chunk, F), base.token_chunk
    print(f"\n[case] {cfg.name} B=1 F={F} {cfg.H}x{cfg.W} chunk=({fc},{tc})", flush=True)
    stage, w = make_stage(cfg, seed=0, frame_chunk=fc, token_chunk=tc)
    try:
        orc = lo.Oracle(cfg, w64_of(w))
        orc.set_chunk(fc, tc)  # (the oracle's chunked loops give what its unchunked ones give: CPU tests)
        orc.progress = lambda what: print(f"[oracle] {what}", flush=True)
        x = synth.make_latents(cfg, 1)
        xd = dev(stage, x)
        deep = synth.make_deep(cfg, 2)
        stage.cache_write(1, dev(stage, deep))
        eps = stage.empty(*x.shape)
        stage.cached_step(xd, eps, 1)
        stage.sync()
        orc.cache_write(1, deep)
        print("[oracle] cached step ...", flush=True)
        check("cached_step eps", host(eps), orc.cached_step(x, 1), cfg.dtype)
        if full_too:
            eps2 = stage.empty(*x.shape)
            stage.full_step(xd, eps2, 0)
            stage.sync()
            print("[oracle] full step ...", flush=True)
            ref = orc.full_step(x, 0)
            check("full_step eps", host(eps2), ref, cfg.dtype)
            check("full_step deep", host(stage.cache_read(0)), orc.dev[0], cfg.dtype, cache_entry=True)
    finally:
        stage.close()


# ------------------------------------------------------------------------------------------
# single operators over all frames of the stage, oracle on samples
# ------------------------------------------------------------------------------------------
@pytest.fixture(scope="module", params=[AD, SVD], ids=lambda c: c.name)
def big(request):
    cfg = request.param
    print(f"\n[stage] {cfg.name} N={cfg.N} {cfg.H}x{cfg.W}", flush=True)
    stage, w = make_stage(cfg, seed=5, frame_chunk=0, token_chunk=0)  # scratch for all frames at once
    yield stage, cfg, w64_of(w)
    stage.close()


def sample_frames(cfg, seed):
    rng = np.random.default_rng(seed)
    return sorted({0, cfg.N - 1, int(rng.integers(1, cfg.N - 1))})


def test_res_block_all_frames(big):
    stage, cfg, w = big
    N, C, H, W, T = cfg.N, cfg.C, cfg.H, cfg.W, cfg.T
    x = synth.make_activation((N, C, H, W), 21, cfg.dtype, 1.5) + np.float32(0.5)
    xd = dev32(stage, planar_to_rows(x))
    y = empty32(stage, N * T, C)
    lcb.lc_op_res_block(stage.ctx, lcb.LC_L_RES0, xd.data_ptr(), y.data_ptr(), N)
    # the same frames in launches of one frame chunk give the same bits
    yc = empty32(stage, N * T, C)
    fc = cfg.frame_chunk
    for f0 in range(0, N, fc):
        n = min(fc, N - f0)
        lcb.lc_op_res_block(stage.ctx, lcb.LC_L_RES0, xd[f0 * T:].data_ptr(), yc[f0 * T:].data_ptr(), n)
    stage.sync()
    assert torch.equal(y, yc)
    for f in sample_frames(cfg, 1):
        x64 = x[f:f + 1].astype(np.float64)
        g = lo.silu(lo.group_norm(x64, w["res0.gn_g"], w["res0.gn_b"], cfg.groups, cfg.gn_eps))
        ref = x64 + lo.conv3x3(g, w["res0.w"], w["res0.b"])
        check(f"res_block frame {f}", rows_to_planar(host(y[f * T:(f + 1) * T]), 1, C, H, W), ref, cfg.dtype)


def test_up_conv_and_conv_out_all_frames(big):
    stage, cfg, w = big
    N, C, Cd, H, W, T = cfg.N, cfg.C, cfg.C_deep, cfg.H, cfg.W, cfg.T
    s = synth.make_activation((N, C, H, W), 81, cfg.dtype, 1.3)
    d = synth.make_activation((N, Cd, H // 2, W // 2), 82, cfg.dtype, 0.7) + np.float32(0.25)
    if cfg.dtype == "bf16":
        d = synth.round_to_bf16(d)
    sd, dd = dev32(stage, planar_to_rows(s)), dev(stage, planar_to_rows(d))
    u = empty32(stage, N * T, C)
    lcb.lc_op_up_conv(stage.ctx, sd.data_ptr(), dd.data_ptr(), u.data_ptr(), N)
    eps = stage.empty(N, cfg.C_lat, H, W)
    lcb.lc_op_conv_out(stage.ctx, sd.data_ptr(), eps.data_ptr(), N)
    stage.sync()
    for f in sample_frames(cfg, 2):
        s64 = s[f:f + 1].astype(np.float64)
        cat = np.concatenate([s64, lo.up2(d[f:f + 1].astype(np.float64))], axis=1)
        g = lo.silu(lo.group_norm(cat, w["up.gn_g"], w["up.gn_b"], cfg.groups, cfg.gn_eps))
        check(f"up_conv frame {f}", rows_to_planar(host(u[f * T:(f + 1) * T]), 1, C, H, W),
              lo.conv3x3(g, w["up.w"], w["up.b"]), cfg.dtype)
        g = lo.silu(lo.group_norm(s64, w["out.gn_g"], w["out.gn_b"], cfg.groups, cfg.gn_eps))
        check(f"conv_out frame {f}", host(eps[f:f + 1]), lo.conv3x3(g, w["out.w"], w["out.b"]), cfg.dtype)


def test_conv_in_and_down_all_frames(big):
    stage, cfg, w = big
    N, C, Cd, H, W, T = cfg.N, cfg.C, cfg.C_deep, cfg.H, cfg.W, cfg.T
    x = synth.make_activation((N, cfg.C_lat, H, W), 71, cfg.dtype)
    h = empty32(stage, N * T, C)
    lcb.lc_op_conv_in(stage.ctx, dev(stage, x).data_ptr(), h.data_ptr(), N)
    a = synth.make_activation((N, C, H, W), 23, cfg.dtype, 1.2)
    d0 = empty32(stage, N * (T // 4), Cd)
    lcb.lc_op_down_conv(stage.ctx, dev32(stage, planar_to_rows(a)).data_ptr(), d0.data_ptr(), N)
    stage.sync()
    for f in sample_frames(cfg, 3):
        check(f"conv_in frame {f}", rows_to_planar(host(h[f * T:(f + 1) * T]), 1, C, H, W),
              lo.conv3x3(x[f:f + 1].astype(np.float64), w["conv_in.w"], w["conv_in.b"]), cfg.dtype)
        check(f"down_conv frame {f}", rows_to_planar(host(d0[f * (T // 4):(f + 1) * (T // 4)]), 1, Cd, H // 2, W // 2),
              lo.conv3x3(a[f:f + 1].astype(np.float64), w["down.w"], w["down.b"], stride=2), cfg.dtype)


def test_spatial_attention_all_frames_sampled_queries(big):
    stage, cfg, w = big
    N, T, C = cfg.N, cfg.T, cfg.C
    qkv = synth.make_activation((N * T, 3 * C), 51, cfg.dtype)
    qkv[:, :2 * C] *= np.float32(1.5)
    # as in the steps: the q third holds q * log2(e)/sqrt(d); its stored (rounded) value defines q
    qs = np.float32(np.log2(np.e) / np.sqrt(cfg.head_dim))
    qkv[:, :C] *= qs
    if cfg.dtype == "bf16":
        qkv = synth.round_to_bf16(qkv)
    qd = dev(stage, qkv)
    qkv[:, :C] /= qs  # (float32 division of the stored values: close enough to exact for the tolerance)
    out = stage.empty(N * T, C)
    # query windows as the step cuts them: the stage's token chunk (whole frame if 0)
    tc = cfg.token_chunk if cfg.token_chunk else T
    for q0 in range(0, T, tc):
        lcb.lc_op_spatial_attention(stage.ctx, qd.data_ptr(), out.data_ptr(), N, q0, min(T, q0 + tc), 1)
    stage.sync()
    rng = np.random.default_rng(7)
    a = qkv.reshape(N, T, 3 * C)
    o = host(out).reshape(N, T, C)
    for f in sample_frames(cfg, 4):
        qi = np.unique(np.concatenate([[0, T - 1, tc - 1, min(tc, T - 1)], rng.integers(0, T, 252)]))
        fr = a[f].astype(np.float64)
        ref = lo.attention_core(fr[qi, :C], fr[:, C:2 * C], fr[:, 2 * C:], cfg.heads)
        check(f"spatial attention frame {f}, {len(qi)} queries", o[f][qi], ref, cfg.dtype)


def test_temporal_attention_all_positions_sampled(big):
    stage, cfg, w = big
    B, F, T, C = cfg.B, cfg.F, cfg.T, cfg.C
    qkv = synth.make_activation((B * F * T, 3 * C), 61, cfg.dtype)
    qkv[:, :2 * C] *= np.float32(2.0)
    if cfg.dtype == "bf16":
        qkv = synth.round_to_bf16(qkv)
    qd = dev(stage, qkv)
    out = stage.empty(B * F * T, C)
    lcb.lc_op_temporal_attention(stage.ctx, qd.data_ptr(), out.data_ptr(), T)
    stage.sync()
    rng = np.random.default_rng(8)
    pi = np.unique(np.concatenate([[0, T - 1], rng.integers(0, T, 510)]))
    a = qkv.reshape(B, F, T, 3 * C)[:, :, pi].astype(np.float64).transpose(0, 2, 1, 3)  # [B, P, F, 3C]
    ref = lo.attention_core(a[..., :C], a[..., C:2 * C], a[..., 2 * C:], cfg.heads).transpose(0, 2, 1, 3)
    got = host(out).reshape(B, F, T, C)[:, :, pi]
    check(f"temporal attention, {len(pi)} positions", got, ref, cfg.dtype)


def test_qkv_and_proj_all_frames(big):
    stage, cfg, w = big
    N, C, H, W, T = cfg.N, cfg.C, cfg.H, cfg.W, cfg.T
    x = synth.make_activation((N, C, H, W), 41, cfg.dtype, 1.4) - np.float32(0.3)
    xr = planar_to_rows(x)
    xd = dev32(stage, xr)
    qkv = stage.empty(N * T, 3 * C)
    lcb.lc_op_qkv(stage.ctx, lcb.LC_L_SATTN, xd.data_ptr(), qkv.data_ptr(), N)
    a_in = synth.make_activation((N * T, C), 43, cfg.dtype)
    ad, rd = dev(stage, a_in), xd.clone()
    lcb.lc_op_proj(stage.ctx, lcb.LC_L_SATTN, ad.data_ptr(), rd.data_ptr(), rd.data_ptr(), N * T)
    stage.sync()
    for f in sample_frames(cfg, 5):
        g = planar_to_rows(lo.group_norm(x[f:f + 1].astype(np.float64), w["sattn.gn_g"], w["sattn.gn_b"], cfg.groups,
                                         cfg.gn_eps))
        qs = np.log2(np.e) / np.sqrt(cfg.head_dim)  # the spatial q is stored with the softmax scale applied
        ref = np.concatenate([(g @ w["sattn.wq"].T) * qs, g @ w["sattn.wk"].T, g @ w["sattn.wv"].T], axis=1)
        check(f"qkv frame {f}", host(qkv[f * T:(f + 1) * T]), ref, cfg.dtype)
        sl = slice(f * T, (f + 1) * T)
        ref = xr[sl].astype(np.float64) + a_in[sl].astype(np.float64) @ w["sattn.wo"].T + w["sattn.bo"]
        check(f"proj frame {f}", host(rd[sl]), ref, cfg.dtype)


# ------------------------------------------------------------------------------------------
# invariants of the method on the whole stage
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("cfg,chunks", [
    (AD, [(4, 0), (16, 0), (8, 1024), (2, 0)]),
    (SVD, [(5, 2304), (25, 0)]),
    (STRESS, [(4, 2304), (8, 0)]),
], ids=lambda v: getattr(v, "name", ""))
def test_invariants_whole_stage(cfg, chunks):
    print(f"\n[case] {cfg.name} N={cfg.N} {cfg.H}x{cfg.W}", flush=True)
    stage, w = make_stage(cfg, seed=0, sharp=2.0, frame_chunk=0, token_chunk=0)
    try:
        x = dev(stage, synth.make_latents(cfg, 1))
        e_full, e_cached = stage.empty(*x.shape), stage.empty(*x.shape)
        stage.full_step(x, e_full, 0)
        stage.cached_step(x, e_cached, 0)
        stage.sync()
        assert bool(torch.isfinite(e_full.float()).all())
        assert torch.equal(e_full, e_cached)
        # eps of a denoiser on N(0,1) latents with these weights is O(1), not degenerate
        assert 1e-3 < float(e_full.float().std()) < 1e2
        deep_ref = stage.dev_entry_bytes(0)
        for fc, tc in chunks:
            print(f"[chunk] ({fc},{tc})", flush=True)
            stage.set_chunk(fc, tc)
            a, b = stage.empty(*x.shape), stage.empty(*x.shape)
            stage.full_step(x, a, 1)
            stage.cached_step(x, b, 1)
            stage.sync()
            assert torch.equal(a, e_full), (fc, tc)
            assert torch.equal(b, e_full), (fc, tc)
            assert stage.dev_entry_bytes(1) == deep_ref, (fc, tc)
        # the literal spatial chunk, inside the workload's frame chunks: blocks of H/eta x W/omega
        for eta, omega in {"animatediff": [(2, 2), (8, 1)], "svdxt": [(3, 4)], "stress": [(4, 3)]}[cfg.name]:
            print(f"[spatial chunk] {eta} x {omega}", flush=True)
            stage.set_chunk(cfg.frame_chunk, 0)
            stage.set_spatial_chunk(eta, omega)
            a, b = stage.empty(*x.shape), stage.empty(*x.shape)
            stage.full_step(x, a, 1)
            stage.cached_step(x, b, 1)
            stage.sync()
            assert torch.equal(a, e_full), (eta, omega)
            assert torch.equal(b, e_full), (eta, omega)
            assert stage.dev_entry_bytes(1) == deep_ref, (eta, omega)
        stage.set_spatial_chunk(1, 1)
    finally:
        stage.close()


# ------------------------------------------------------------------------------------------
# the stress schedule: 50 steps, a normal step every 5th, a bank of 10 host entries, two device buffers
# ------------------------------------------------------------------------------------------
def test_stress_schedule_bank_of_ten():
    """The whole 50-step schedule at the stress shape (batch 2 x 32 frames of 96 x 96), free-running (x <- x - eps/50
    on the device between steps). With swapping - each refresh swapped out to its own host entry, every cache step
    reading a device buffer refilled one step ahead - every eps must equal, bit for bit, the eps of the same
    schedule with the deep feature left resident in one device slot; each of the 10 host entries must hold the
    bytes its normal step produced. (Values against the oracle at this shape: test_step_one_chunk_full_image.)"""
    cfg = STRESS
    steps, interval, bank = 50, 5, 10
    stage, w = make_stage(cfg, seed=0, host_slots=bank, dev_slots=2)
    try:
        x0 = dev(stage, synth.make_latents(cfg, 1))

        def run(swapping):
            x = x0.clone()
            outs, entries = [], []
            eps = stage.empty(*x.shape)
            refresh, prefetched = -1, None
            for t in range(steps):
                slot = t % 2 if swapping else 0
                if t % interval == 0:
                    refresh += 1
                    stage.full_step(x, eps, slot)
                    if swapping:
                        stage.swap_out(slot, refresh)
                    else:
                        entries.append(stage.dev_entry_bytes(slot))
                else:
                    if swapping and prefetched != (t, slot):
                        stage.swap_in(refresh, slot)
                    stage.cached_step(x, eps, slot)
                nxt = t + 1
                if swapping and nxt < steps and nxt % interval != 0:
                    stage.swap_in(refresh, nxt % 2)
                    prefetched = (nxt, nxt % 2)
                outs.append(eps.clone())
                x = (x.float() - eps.float() / steps).to(x.dtype)  # (torch, on the compute stream)
            stage.sync()
            return outs, entries

        print("[schedule] resident", flush=True)
        ref, entries = run(False)
        print("[schedule] swapping, bank of 10", flush=True)
        got, _ = run(True)
        for t in range(steps):
            assert torch.equal(got[t], ref[t]), t
        assert bool(torch.isfinite(ref[-1].float()).all())
        for k in range(bank):
            assert stage.host_entry_bytes(k) == entries[k], k
        assert len({e[:4096] for e in entries}) == bank  # ten different features, not one written ten times
        st = lcb.lc_get_stats(stage.ctx)
        assert (st.full_steps, st.cached_steps, st.swaps_out, st.swaps_in) == (20, 80, 10, 40)
        assert st.host_bank_bytes == bank * lcb.lc_cache_entry_bytes(stage.ccfg)
    finally:
        stage.close()
