"""GPU parity, operator by operator: every kernel family the steps launch is called through the
C ABI on seeded inputs and compared element by element with the float64 oracle. Shapes are small
enough for the oracle to finish in seconds but span several tiles and ragged tails (10 x 12 images
against 8 x 16 pixel tiles and 64-row statistic splits; 120 tokens against 64-key stages)."""
import numpy as np
import pytest
import torch

from oracle import lightcache_oracle as lo
from paper_2510_05367_amd import binding as lcb
from paper_2510_05367_amd import synth
from tests.gpu_util import check, dev, dev32, empty32, host, make_stage, planar_to_rows, rows_to_planar

pytestmark = pytest.mark.gpu

# ragged little stages: fp32 with C=64 (narrow tiles) and bf16 with C=320 (wide tiles, d=40)
OPS_F32 = synth.StageConfig("ops_f32", B=2, F=3, H=10, W=12, C_lat=4, C=64, C_deep=128, groups=32, n_res=1,
                            heads=1, head_dim=64, dtype="f32")
OPS_BF16 = synth.StageConfig("ops_bf16", B=1, F=3, H=10, W=12, C_lat=4, C=320, C_deep=640, groups=32, n_res=2,
                             heads=8, head_dim=40, dtype="bf16")
OPS_BF16_D64 = synth.StageConfig("ops_bf16_d64", B=1, F=2, H=18, W=16, C_lat=4, C=320, C_deep=640, groups=32,
                                 n_res=1, heads=5, head_dim=64, dtype="bf16")
CFGS = [OPS_F32, OPS_BF16, OPS_BF16_D64]


@pytest.fixture(scope="module", params=CFGS, ids=lambda c: c.name)
def st(request):
    cfg = request.param
    print(f"\n[stage] {cfg.name}", flush=True)
    stage, w = make_stage(cfg, seed=11)
    w64 = {k: v.astype(np.float64) for k, v in w.items()}
    yield stage, cfg, w64
    stage.close()


def act(cfg, shape, seed, scale=1.0):
    return synth.make_activation(shape, seed, cfg.dtype, scale)


def test_res_block(st):
    stage, cfg, w = st
    N, C, H, W = cfg.N, cfg.C, cfg.H, cfg.W
    x = act(cfg, (N, C, H, W), 21, 1.5) + np.float32(0.5)
    xd = dev32(stage, planar_to_rows(x))
    for i in range(cfg.n_res):
        pre = f"res{i}"
        y = empty32(stage, *xd.shape)
        lcb.lc_op_res_block(stage.ctx, lcb.LC_L_RES0 + i, xd.data_ptr(), y.data_ptr(), N)
        stage.sync()
        x64 = x.astype(np.float64)
        g = lo.silu(lo.group_norm(x64, w[pre + ".gn_g"], w[pre + ".gn_b"], cfg.groups, cfg.gn_eps))
        ref = x64 + lo.conv3x3(g, w[pre + ".w"], w[pre + ".b"])
        check(f"res_block[{pre}]", rows_to_planar(host(y), N, C, H, W), ref, cfg.dtype)
    # fewer frames than the stage holds
    y = empty32(stage, *xd.shape)
    y.fill_(7.0)
    lcb.lc_op_res_block(stage.ctx, lcb.LC_L_RES0, xd.data_ptr(), y.data_ptr(), 1)
    stage.sync()
    x64 = x[:1].astype(np.float64)
    g = lo.silu(lo.group_norm(x64, w["res0.gn_g"], w["res0.gn_b"], cfg.groups, cfg.gn_eps))
    check("res_block 1 frame", rows_to_planar(host(y[:H * W]), 1, C, H, W),
          x64 + lo.conv3x3(g, w["res0.w"], w["res0.b"]), cfg.dtype)
    assert bool((y[H * W:] == 7.0).all())


def test_deep_stand_in(st):
    stage, cfg, w = st
    N, C, Cd, H, W = cfg.N, cfg.C, cfg.C_deep, cfg.H, cfg.W
    x = act(cfg, (N, C, H, W), 23, 1.2)
    xd = dev32(stage, planar_to_rows(x))
    d0 = empty32(stage, N * (H // 2) * (W // 2), Cd)
    lcb.lc_op_down_conv(stage.ctx, xd.data_ptr(), d0.data_ptr(), N)
    stage.sync()
    ref0 = lo.conv3x3(x.astype(np.float64), w["down.w"], w["down.b"], stride=2)
    check("down_conv", rows_to_planar(host(d0), N, Cd, H // 2, W // 2), ref0, cfg.dtype)
    # residual block at C_deep on an independent input; output has the cache-entry type
    z = act(cfg, (N, Cd, H // 2, W // 2), 24, 1.5)
    zd = dev32(stage, planar_to_rows(z))
    y = stage.empty(*zd.shape)
    lcb.lc_op_res_block(stage.ctx, lcb.LC_L_DRES, zd.data_ptr(), y.data_ptr(), N)
    stage.sync()
    z64 = z.astype(np.float64)
    g = lo.silu(lo.group_norm(z64, w["dres.gn_g"], w["dres.gn_b"], cfg.groups, cfg.gn_eps))
    check("res_block[dres]", rows_to_planar(host(y), N, Cd, H // 2, W // 2),
          z64 + lo.conv3x3(g, w["dres.w"], w["dres.b"]), cfg.dtype, cache_entry=True)


@pytest.mark.parametrize("layer,pre", [(lcb.LC_L_SATTN, "sattn"), (lcb.LC_L_TATTN, "tattn")])
def test_qkv_and_proj(st, layer, pre):
    stage, cfg, w = st
    N, C, H, W = cfg.N, cfg.C, cfg.H, cfg.W
    x = act(cfg, (N, C, H, W), 41, 1.4) - np.float32(0.3)
    xd = dev32(stage, planar_to_rows(x))
    rows = N * H * W
    qkv = stage.empty(rows, 3 * C)
    lcb.lc_op_qkv(stage.ctx, layer, xd.data_ptr(), qkv.data_ptr(), N)
    stage.sync()
    g = planar_to_rows(lo.group_norm(x.astype(np.float64), w[pre + ".gn_g"], w[pre + ".gn_b"], cfg.groups, cfg.gn_eps))
    # the spatial block's q is stored multiplied by the softmax scale in base 2 (applied before rounding)
    qs = np.log2(np.e) / np.sqrt(cfg.head_dim) if pre == "sattn" else 1.0
    ref = np.concatenate([(g @ w[pre + ".wq"].T) * qs, g @ w[pre + ".wk"].T, g @ w[pre + ".wv"].T], axis=1)
    check(f"qkv[{pre}]", host(qkv), ref, cfg.dtype)
    rows = 333  # not a multiple of the 128-row tile
    a_in = act(cfg, (rows, C), 43)
    res = act(cfg, (rows, C), 42)
    ad, rd = dev(stage, a_in), dev32(stage, res)
    lcb.lc_op_proj(stage.ctx, layer, ad.data_ptr(), rd.data_ptr(), rd.data_ptr(), rows)
    stage.sync()
    ref = res.astype(np.float64) + a_in.astype(np.float64) @ w[pre + ".wo"].T + w[pre + ".bo"]
    check(f"proj[{pre}]", host(rd), ref, cfg.dtype)


@pytest.mark.parametrize("prescaled", [0, 1])
@pytest.mark.parametrize("logit_scale", [1.0, 6.0])
def test_spatial_attention_core(st, logit_scale, prescaled):
    stage, cfg, w = st
    N, T, C = cfg.N, cfg.T, cfg.C
    qkv = act(cfg, (N * T, 3 * C), 51)
    qkv[:, :2 * C] *= np.float32(np.sqrt(logit_scale))  # logit std ~ logit_scale * sqrt(d)/sqrt(d)
    if cfg.dtype == "bf16":
        qkv = synth.round_to_bf16(qkv)
    # prescaled: the kernel is handed q' = q * log2(e)/sqrt(d); whatever q' holds (after rounding to
    # the storage type) defines the queries the oracle attends with, q = q' / that factor
    qs = np.log2(np.e) / np.sqrt(cfg.head_dim)
    a = qkv.astype(np.float64).reshape(N, T, 3 * C)
    if prescaled:
        qp = (qkv[:, :C].astype(np.float64) * qs).astype(np.float32)
        qkv[:, :C] = synth.round_to_bf16(qp) if cfg.dtype == "bf16" else qp
        a = qkv.astype(np.float64).reshape(N, T, 3 * C)
        a[..., :C] /= qs
    qd = dev(stage, qkv)
    out = stage.empty(N * T, C)
    out.zero_()
    q0, q1 = 0, T
    lcb.lc_op_spatial_attention(stage.ctx, qd.data_ptr(), out.data_ptr(), N, q0, q1, prescaled)
    stage.sync()
    ref = lo.attention_core(a[..., :C], a[..., C:2 * C], a[..., 2 * C:], cfg.heads).reshape(N * T, C)
    check(f"spatial core x{logit_scale} prescaled={prescaled}", host(out), ref, cfg.dtype)
    # a ragged query window must only write its own rows and reproduce them bit for bit
    out2 = stage.empty(N * T, C)
    out2.fill_(7.0)
    lcb.lc_op_spatial_attention(stage.ctx, qd.data_ptr(), out2.data_ptr(), N, 37, 101, prescaled)
    stage.sync()
    o1 = out.view(N, T, C)
    o2 = out2.view(N, T, C)
    assert torch.equal(o2[:, 37:101], o1[:, 37:101])
    assert bool((o2[:, :37] == 7.0).all()) and bool((o2[:, 101:] == 7.0).all())


def test_attention_blocks_in_place(st):
    """The two attention blocks as a step issues them (statistics, q,k,v projection with V^T written by its
    epilogue, attention core, output projection + residual) against the oracle's block functions."""
    stage, cfg, w = st
    N, C, H, W, T = cfg.N, cfg.C, cfg.H, cfg.W, cfg.T
    orc = lo.Oracle(cfg, w)
    x = act(cfg, (N, C, H, W), 141, 1.3) + np.float32(0.2)
    hd = dev32(stage, planar_to_rows(x))
    lcb.lc_op_spatial_block(stage.ctx, hd.data_ptr(), N)
    stage.sync()
    check("spatial block", rows_to_planar(host(hd), N, C, H, W), orc.spatial_block(x.astype(np.float64)), cfg.dtype)
    hd = dev32(stage, planar_to_rows(x))
    lcb.lc_op_temporal_block(stage.ctx, hd.data_ptr())
    stage.sync()
    check("temporal block", rows_to_planar(host(hd), N, C, H, W), orc.temporal_block(x.astype(np.float64)), cfg.dtype)
    # chunked: frames one at a time with query windows of 50 tokens, positions 40 at a time: the same bits
    h1, h2 = dev32(stage, planar_to_rows(x)), dev32(stage, planar_to_rows(x))
    lcb.lc_op_spatial_block(stage.ctx, h1.data_ptr(), N)
    lcb.lc_op_temporal_block(stage.ctx, h1.data_ptr())
    stage.set_chunk(1, 40)
    try:
        for f in range(N):
            lcb.lc_op_spatial_block(stage.ctx, h2[f * T:].data_ptr(), 1)
        with pytest.raises(lcb.LcError) as e:
            lcb.lc_op_spatial_block(stage.ctx, h2.data_ptr(), 2)
        assert e.value.status == lcb.LC_ERR_NOMEM
        lcb.lc_op_temporal_block(stage.ctx, h2.data_ptr())
        stage.sync()
        assert torch.equal(h1, h2)
    finally:
        stage.set_chunk(cfg.frame_chunk, cfg.token_chunk)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("heads,head_dim", [(8, 8), (4, 16), (2, 32), (8, 40), (1, 64)])
def test_spatial_attention_every_head_size(heads, head_dim, dtype):
    """Every head size the library accepts takes a different path through the spatial kernel (rows of V^T that
    deliver the softmax denominators or not, the running maximum folded into a spare contraction slot or not):
    each against the definition, unit and sharp logits, 140 tokens = two full key stages and a ragged third."""
    C = heads * head_dim
    cfg = synth.StageConfig(f"s_{heads}x{head_dim}_{dtype}", B=1, F=2, H=10, W=14, C_lat=4, C=C, C_deep=64, groups=8,
                            n_res=1, heads=heads, head_dim=head_dim, dtype=dtype)
    stage, _ = make_stage(cfg, seed=5)
    try:
        N, T = cfg.N, cfg.T
        for logit_scale in (1.0, 8.0):
            qkv = act(cfg, (N * T, 3 * C), 251)
            qkv[:, :2 * C] *= np.float32(np.sqrt(logit_scale) * 1.2)
            if dtype == "bf16":
                qkv = synth.round_to_bf16(qkv)
            out = stage.empty(N * T, C)
            lcb.lc_op_spatial_attention(stage.ctx, dev(stage, qkv).data_ptr(), out.data_ptr(), N, 0, T, 0)
            stage.sync()
            a = qkv.astype(np.float64).reshape(N, T, 3 * C)
            ref = lo.attention_core(a[..., :C], a[..., C:2 * C], a[..., 2 * C:], heads).reshape(N * T, C)
            check(f"spatial core {heads}x{head_dim} {dtype} x{logit_scale}", host(out), ref, dtype)
    finally:
        stage.close()


def test_temporal_attention_core(st):
    stage, cfg, w = st
    B, F, C = cfg.B, cfg.F, cfg.C
    P = 37
    qkv = act(cfg, (B * F * P, 3 * C), 61)
    qkv[:, :2 * C] *= np.float32(2.0)
    if cfg.dtype == "bf16":
        qkv = synth.round_to_bf16(qkv)
    qd = dev(stage, qkv)
    out = stage.empty(B * F * P, C)
    lcb.lc_op_temporal_attention(stage.ctx, qd.data_ptr(), out.data_ptr(), P)
    stage.sync()
    a = qkv.astype(np.float64).reshape(B, F, P, 3 * C).transpose(0, 2, 1, 3)  # [B, P, F, 3C]
    ref = lo.attention_core(a[..., :C], a[..., C:2 * C], a[..., 2 * C:], cfg.heads)
    ref = ref.transpose(0, 2, 1, 3).reshape(B * F * P, C)
    check("temporal core", host(out), ref, cfg.dtype)


def test_conv_in(st):
    stage, cfg, w = st
    N, H, W = cfg.N, cfg.H, cfg.W
    x = act(cfg, (N, cfg.C_lat, H, W), 71)
    xd = dev(stage, x)
    h = empty32(stage, N * H * W, cfg.C)
    lcb.lc_op_conv_in(stage.ctx, xd.data_ptr(), h.data_ptr(), N)
    stage.sync()
    ref = lo.conv3x3(x.astype(np.float64), w["conv_in.w"], w["conv_in.b"])
    check("conv_in", rows_to_planar(host(h), N, cfg.C, H, W), ref, cfg.dtype)


def test_up_conv(st):
    stage, cfg, w = st
    N, H, W, C, Cd = cfg.N, cfg.H, cfg.W, cfg.C, cfg.C_deep
    s = act(cfg, (N, C, H, W), 81, 1.3)
    d = act(cfg, (N, Cd, H // 2, W // 2), 82, 0.7) + np.float32(0.25)
    if cfg.dtype == "bf16":
        d = synth.round_to_bf16(d)
    sd, dd = dev32(stage, planar_to_rows(s)), dev(stage, planar_to_rows(d))
    u = empty32(stage, N * H * W, C)
    lcb.lc_op_up_conv(stage.ctx, sd.data_ptr(), dd.data_ptr(), u.data_ptr(), N)
    stage.sync()
    cat = np.concatenate([s.astype(np.float64), lo.up2(d.astype(np.float64))], axis=1)
    g = lo.silu(lo.group_norm(cat, w["up.gn_g"], w["up.gn_b"], cfg.groups, cfg.gn_eps))
    ref = lo.conv3x3(g, w["up.w"], w["up.b"])
    check("up_conv", rows_to_planar(host(u), N, C, H, W), ref, cfg.dtype)


def test_conv_out(st):
    stage, cfg, w = st
    N, H, W, C = cfg.N, cfg.H, cfg.W, cfg.C
    u = act(cfg, (N, C, H, W), 91, 2.0)
    ud = dev32(stage, planar_to_rows(u))
    eps = stage.empty(N, cfg.C_lat, H, W)
    lcb.lc_op_conv_out(stage.ctx, ud.data_ptr(), eps.data_ptr(), N)
    stage.sync()
    g = lo.silu(lo.group_norm(u.astype(np.float64), w["out.gn_g"], w["out.gn_b"], cfg.groups, cfg.gn_eps))
    ref = lo.conv3x3(g, w["out.w"], w["out.b"])
    check("conv_out", host(eps), ref, cfg.dtype)


def test_specialised_conv_equals_general_bitwise(st):
    """The 3x3 convolutions of a bf16 stage with C % 160 == 0 run in the kernel with specialised wavefronts;
    it accumulates the same products in the same order as the general kernel, so the two must agree bit for
    bit (output and the GroupNorm partial sums it writes, seen through the next operator)."""
    stage, cfg, w = st
    N, C, Cd, H, W = cfg.N, cfg.C, cfg.C_deep, cfg.H, cfg.W
    x = act(cfg, (N, C, H, W), 131, 1.5) + np.float32(0.25)
    d = act(cfg, (N, Cd, H // 2, W // 2), 132, 0.7)
    if cfg.dtype == "bf16":
        d = synth.round_to_bf16(d)
    xd, dd = dev32(stage, planar_to_rows(x)), dev(stage, planar_to_rows(d))
    outs = []
    for general in (0, 1):
        lcb.lc_set_conv_general(stage.ctx, general)
        y = empty32(stage, *xd.shape)
        u = empty32(stage, N * H * W, C)
        lcb.lc_op_res_block(stage.ctx, lcb.LC_L_RES0, xd.data_ptr(), y.data_ptr(), N)
        lcb.lc_op_up_conv(stage.ctx, xd.data_ptr(), dd.data_ptr(), u.data_ptr(), N)
        # a whole cached step as well: its GroupNorms read the partial sums the convolutions write
        lat = synth.make_latents(cfg, 133)
        eps = stage.empty(*lat.shape)
        stage.cache_write(0, dev(stage, synth.make_deep(cfg, 134)))
        stage.cached_step(dev(stage, lat), eps, 0)
        stage.sync()
        outs.append((y.clone(), u.clone(), eps.clone()))
    lcb.lc_set_conv_general(stage.ctx, 0)
    for a, b, name in zip(outs[0], outs[1], ("res_block", "up_conv", "cached_step")):
        assert torch.equal(a, b), name
    with pytest.raises(lcb.LcError):
        lcb.lc_set_conv_general(stage.ctx, 2)


@pytest.mark.parametrize("heads,head_dim,B", [(8, 40, 2), (5, 64, 1), (8, 8, 1), (4, 16, 1), (2, 32, 2)])
@pytest.mark.parametrize("logit_scale", [1.0, 8.0])
@pytest.mark.parametrize("F", [16, 11, 8, 32, 25, 17])
def test_temporal_attention_on_matrix_cores(heads, head_dim, B, logit_scale, F):
    """bf16 stages with 8 <= F <= 32 run the temporal attention on 16 x 16 or 32 x 32 MFMA tiles (one tile = the
    scores of one position and head, padded beyond F); every head size the library accepts, position counts that leave a
    ragged last workgroup, unit and sharp logits. Against the definition in float64."""
    C = heads * head_dim
    if C % 64:
        pytest.skip("C must be a multiple of 64")
    cfg = synth.StageConfig(f"t{F}_{heads}x{head_dim}", B=B, F=F, H=4, W=4, C_lat=4, C=C, C_deep=64, groups=8, n_res=1,
                            heads=heads, head_dim=head_dim, dtype="bf16")
    stage, _ = make_stage(cfg, seed=5)
    try:
        for P in (37, 1, 64):
            qkv = act(cfg, (B * F * P, 3 * C), 61 + P)
            qkv[:, :2 * C] *= np.float32(np.sqrt(logit_scale) * 1.4)
            qkv = synth.round_to_bf16(qkv)
            qd = dev(stage, qkv)
            out = stage.empty(B * F * P, C)
            out.fill_(7.0)
            lcb.lc_op_temporal_attention(stage.ctx, qd.data_ptr(), out.data_ptr(), P)
            stage.sync()
            a = qkv.astype(np.float64).reshape(B, F, P, 3 * C).transpose(0, 2, 1, 3)  # [B, P, F, 3C]
            ref = lo.attention_core(a[..., :C], a[..., C:2 * C], a[..., 2 * C:], heads)
            ref = ref.transpose(0, 2, 1, 3).reshape(B * F * P, C)
            check(f"temporal core F={F} {heads}x{head_dim} P={P} x{logit_scale}", host(out), ref, cfg.dtype)
    finally:
        stage.close()


@pytest.mark.parametrize("C,heads,head_dim,C_lat,H,W", [(320, 8, 40, 4, 6, 64), (64, 1, 64, 4, 4, 32), (128, 2, 64, 5, 2, 96),
                                                       (320, 5, 64, 2, 8, 32), (384, 6, 64, 1, 2, 32)])
def test_conv_in_tile_kernel(C, heads, head_dim, C_lat, H, W):
    """bf16 stages whose image rows are whole 32-pixel segments run conv_in in a kernel of its own (one workgroup
    per segment, all channels): widths that leave wavefronts without a channel tile (C = 64) or give them three
    (C = 320, 384), 1 to 5 latent planes, one and several segments per row; borders on all four sides."""
    cfg = synth.StageConfig(f"cin_{C}_{C_lat}_{H}x{W}", B=1, F=2, H=H, W=W, C_lat=C_lat, C=C, C_deep=64, groups=32, n_res=1,
                            heads=heads, head_dim=head_dim, dtype="bf16")
    stage, w = make_stage(cfg, seed=9)
    try:
        N = cfg.N
        x = act(cfg, (N, C_lat, H, W), 171, 1.3) - np.float32(0.2)
        xd = dev(stage, x)
        h = empty32(stage, N * H * W, C)
        h.fill_(7.0)
        lcb.lc_op_conv_in(stage.ctx, xd.data_ptr(), h.data_ptr(), 1)  # one frame of the two: the rest stays untouched
        stage.sync()
        assert bool((h[H * W:] == 7.0).all())
        lcb.lc_op_conv_in(stage.ctx, xd.data_ptr(), h.data_ptr(), N)
        stage.sync()
        ref = lo.conv3x3(x.astype(np.float64), w["conv_in.w"].astype(np.float64), w["conv_in.b"].astype(np.float64))
        check(f"conv_in tile {cfg.name}", rows_to_planar(host(h), N, C, H, W), ref, cfg.dtype)
    finally:
        stage.close()
