"""Pins of the diffusion-transformer oracle (oracle/dit_oracle.py): a scalar brute force of the block stack, an
independent torch float64 build, closed forms of LayerNorm / modulation / GELU, and the method's invariants (cache
step on its own cache == normal step, exactly; chunked == unchunked; swap round trip)."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as TF

from oracle import dit_oracle as dito
from paper_2510_05367_amd import synth
from tests import brute

SMALL = synth.DitConfig("s", B=2, T=7, D=8, heads=2, head_dim=4, L=4, cache_a=1, cache_b=3, dtype="f32")


def w64(cfg, seed=0, scale=8.0):
    return {k: v.astype(np.float64) * scale for k, v in synth.make_dit_weights(cfg, seed, sharp=3.0).items()}


def test_weight_names_match_manifest():
    assert dito.required_weights(SMALL) == [n for n, _, _ in synth.dit_weight_manifest(SMALL)]


def test_layer_norm_gelu_closed_forms():
    x = np.array([[1.0, 2.0, 3.0, 6.0]])
    y = dito.layer_norm(x, 0.0)
    assert abs(y.mean()) < 1e-15 and abs((y ** 2).mean() - 1.0) < 1e-14  # biased variance: E[y^2] = 1 exactly
    assert np.allclose(y, (x - 3.0) / math.sqrt(3.5))
    assert np.allclose(dito.layer_norm(x, 1e-6), TF.layer_norm(torch.from_numpy(x), (4,), eps=1e-6).numpy(), atol=1e-15)
    z = np.linspace(-4, 4, 33)
    assert np.allclose(dito.gelu_tanh(z), TF.gelu(torch.from_numpy(z), approximate="tanh").numpy(), atol=1e-15)
    assert dito.gelu_tanh(np.array([0.0]))[0] == 0.0 and abs(dito.gelu_tanh(np.array([10.0]))[0] - 10.0) < 1e-12


def test_block_stack_matches_brute_force():
    cfg = SMALL
    w = w64(cfg)
    x = synth.make_dit_hidden(cfg, 1).astype(np.float64)
    mod = synth.make_dit_modulation(cfg, 2).astype(np.float64)
    orc = dito.DitOracle(cfg, w)
    got = orc.full_step(x, mod, 0)
    wl = {k: v.tolist() for k, v in w.items()}
    for b in range(cfg.B):
        ref = np.array(brute.dit_blocks(cfg, wl, [[m.tolist() for m in mod[i, b]] for i in range(cfg.L)], x[b].tolist(), 0, cfg.L))
        assert np.max(np.abs(got[b] - ref)) < 1e-11
        # the stored Delta is what the deep blocks [a, b) add
        xa = np.array(brute.dit_blocks(cfg, wl, [[m.tolist() for m in mod[i, b]] for i in range(cfg.L)], x[b].tolist(), 0, cfg.cache_a))
        xb = np.array(brute.dit_blocks(cfg, wl, [[m.tolist() for m in mod[i, b]] for i in range(cfg.L)], xa.tolist(), cfg.cache_a, cfg.cache_b))
        assert np.max(np.abs(orc.dev[0][b] - (xb - xa))) < 1e-11
    assert np.std(got - x) > 1e-2  # the blocks do something


def torch_stack(cfg, w, mod, x):
    t = {k: torch.from_numpy(v) for k, v in w.items()}
    x = torch.from_numpy(x).clone()
    m = torch.from_numpy(mod)
    for i in range(cfg.L):
        sh1, sc1, g1, sh2, sc2, g2 = (m[i, :, j].unsqueeze(1) for j in range(6))
        h = TF.layer_norm(x, (cfg.D,), eps=cfg.ln_eps) * (1 + sc1) + sh1
        qkv = h @ t[f"blk{i}.wqkv"].T + t[f"blk{i}.bqkv"]
        sp = lambda a: a.reshape(cfg.B, cfg.T, cfg.heads, cfg.head_dim).transpose(1, 2)
        q, k, v = qkv.split(cfg.D, dim=-1)
        o = TF.scaled_dot_product_attention(sp(q), sp(k), sp(v)).transpose(1, 2).reshape(cfg.B, cfg.T, cfg.D)
        x = x + g1 * (o @ t[f"blk{i}.wo"].T + t[f"blk{i}.bo"])
        h = TF.layer_norm(x, (cfg.D,), eps=cfg.ln_eps) * (1 + sc2) + sh2
        u = TF.gelu(h @ t[f"blk{i}.w1"].T + t[f"blk{i}.b1"], approximate="tanh")
        x = x + g2 * (u @ t[f"blk{i}.w2"].T + t[f"blk{i}.b2"])
    return x.numpy()


def test_block_stack_matches_independent_torch_build():
    cfg = synth.DitConfig("m", B=2, T=19, D=24, heads=3, head_dim=8, L=3, cache_a=1, cache_b=2, dtype="f32")
    w = w64(cfg, scale=4.0)
    x = synth.make_dit_hidden(cfg, 3).astype(np.float64)
    mod = synth.make_dit_modulation(cfg, 4).astype(np.float64)
    got = dito.DitOracle(cfg, w).full_step(x, mod, 0)
    assert np.max(np.abs(got - torch_stack(cfg, w, mod, x))) < 1e-12


@pytest.mark.parametrize("a,b", [(1, 3), (0, 4), (2, 2), (0, 0), (4, 4)])
def test_cache_step_on_own_cache_equals_normal_step_exactly(a, b):
    cfg = SMALL.with_(cache_a=a, cache_b=b)
    w = w64(cfg)
    x = synth.make_dit_hidden(cfg, 1).astype(np.float64)
    mod = synth.make_dit_modulation(cfg, 2).astype(np.float64)
    orc = dito.DitOracle(cfg, w, host_slots=1, dev_slots=2)
    full = orc.full_step(x, mod, 0)
    assert np.array_equal(orc.cached_step(x, mod, 0), full)
    orc.swap_out(0, 0)
    orc.dev[1] = np.full_like(orc.dev[0], np.nan)
    orc.swap_in(0, 1)
    assert orc.dev[1].tobytes() == orc.dev[0].tobytes()
    assert np.array_equal(orc.cached_step(x, mod, 1), full)
    # with no block cached Delta is zero, and a foreign Delta shows in the result
    assert (a != b) or not np.any(orc.dev[0])
    orc.cache_write(1, orc.dev[0] + 0.5)
    assert not np.array_equal(orc.cached_step(x, mod, 1), full)
    with pytest.raises(RuntimeError):
        dito.DitOracle(cfg, w).cached_step(x, mod, 0)


@pytest.mark.parametrize("chunk", [1, 3, 7, 100])
def test_token_chunks_do_not_change_the_result(chunk):
    cfg = SMALL
    w = w64(cfg)
    x = synth.make_dit_hidden(cfg, 1).astype(np.float64)
    mod = synth.make_dit_modulation(cfg, 2).astype(np.float64)
    whole = dito.DitOracle(cfg, w).full_step(x, mod, 0)
    orc = dito.DitOracle(cfg, w)
    orc.set_chunk(chunk)
    assert np.max(np.abs(orc.full_step(x, mod, 0) - whole)) < 1e-13
    with pytest.raises(ValueError):
        orc.set_chunk(-1)


def test_modulation_and_gates_enter_where_they_should():
    cfg = SMALL.with_(L=1, cache_a=0, cache_b=0, B=1)
    w = w64(cfg)
    x = synth.make_dit_hidden(cfg, 1).astype(np.float64)
    mod = np.zeros((1, 1, 6, cfg.D))
    orc = dito.DitOracle(cfg, w)
    assert np.array_equal(orc.full_step(x, mod, 0), x)  # zero gates: the block is the identity
    mod[0, 0, 2] = 1.0  # attention gate only
    y_attn = orc.full_step(x, mod, 0)
    mod[0, 0, 2], mod[0, 0, 5] = 0.0, 1.0  # MLP gate only
    y_mlp = orc.full_step(x, mod, 0)
    h = dito.layer_norm(x[0], cfg.ln_eps)
    ref = x[0] + dito.gelu_tanh(h @ w["blk0.w1"].T + w["blk0.b1"]) @ w["blk0.w2"].T + w["blk0.b2"]
    assert np.max(np.abs(y_mlp[0] - ref)) < 1e-13
    assert not np.allclose(y_attn, y_mlp)
    mod[0, 0, 4], mod[0, 0, 3] = 0.5, 0.25  # scale_mlp, shift_mlp
    ref = x[0] + dito.gelu_tanh((h * 1.5 + 0.25) @ w["blk0.w1"].T + w["blk0.b1"]) @ w["blk0.w2"].T + w["blk0.b2"]
    assert np.max(np.abs(orc.full_step(x, mod, 0)[0] - ref)) < 1e-13
