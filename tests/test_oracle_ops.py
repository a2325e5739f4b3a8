"""Pins for the oracle's operators: closed forms, brute force, symmetries and independent
library routines (torch CPU float64 functionals used only as a second opinion)."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as TF

from oracle import lightcache_oracle as lo
from tests import brute

rng = np.random.default_rng(1234)


def rnd(*shape):
    return rng.standard_normal(shape)


def rel_l2(a, b):
    a, b = np.asarray(a, dtype=np.float64), np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


# ----------------------------------------------------------------------------- conv3x3
@pytest.mark.parametrize("stride", [1, 2])
def test_conv_matches_brute_force(stride):
    x, w, b = rnd(2, 3, 6, 4), rnd(5, 3, 3, 3), rnd(5)
    y = lo.conv3x3(x, w, b, stride)
    yb = np.array(brute.conv3x3(x.tolist(), w.tolist(), b.tolist(), stride))
    assert y.shape == yb.shape == (2, 5, 6 // stride, 4 // stride)
    assert np.max(np.abs(y - yb)) < 1e-12


@pytest.mark.parametrize("stride", [1, 2])
def test_conv_matches_torch(stride):
    x, w, b = rnd(3, 7, 10, 12), rnd(6, 7, 3, 3), rnd(6)
    y = lo.conv3x3(x, w, b, stride)
    yt = TF.conv2d(torch.from_numpy(x), torch.from_numpy(w), torch.from_numpy(b), stride=stride, padding=1).numpy()
    assert rel_l2(y, yt) < 1e-13


def test_conv_delta_kernel_is_identity():
    x = rnd(2, 4, 5, 7)
    w = np.zeros((4, 4, 3, 3))
    for c in range(4):
        w[c, c, 1, 1] = 1.0
    assert np.array_equal(lo.conv3x3(x, w, np.zeros(4)), x)


def test_conv_shift_kernel_is_cross_correlation():
    # a single 1 at tap (a, e) reads x[i + a - 1, j + e - 1]: the image moves the other way
    x = rnd(1, 1, 6, 6)
    for a in range(3):
        for e in range(3):
            w = np.zeros((1, 1, 3, 3))
            w[0, 0, a, e] = 1.0
            y = lo.conv3x3(x, w, np.zeros(1))
            for i in range(6):
                for j in range(6):
                    ii, jj = i + a - 1, j + e - 1
                    want = x[0, 0, ii, jj] if 0 <= ii < 6 and 0 <= jj < 6 else 0.0
                    assert y[0, 0, i, j] == want


def test_conv_ones_kernel_counts_zero_padding():
    Cin = 3
    x = np.ones((1, Cin, 5, 6))
    y = lo.conv3x3(x, np.ones((2, Cin, 3, 3)), np.zeros(2))
    assert y[0, 0, 0, 0] == 4 * Cin and y[0, 1, 4, 5] == 4 * Cin  # corners
    assert y[0, 0, 0, 2] == 6 * Cin and y[0, 0, 3, 0] == 6 * Cin  # edges
    assert y[0, 0, 2, 3] == 9 * Cin  # interior


def test_conv_stride2_ones_kernel():
    # output (i, j) reads rows 2i-1..2i+1: the first row/column of outputs touches the padding
    Cin = 2
    x = np.ones((1, Cin, 6, 6))
    y = lo.conv3x3(x, np.ones((1, Cin, 3, 3)), np.zeros(1), stride=2)
    assert y.shape == (1, 1, 3, 3)
    assert y[0, 0, 0, 0] == 4 * Cin
    assert y[0, 0, 0, 1] == 6 * Cin and y[0, 0, 2, 0] == 6 * Cin
    assert y[0, 0, 1, 1] == 9 * Cin and y[0, 0, 2, 2] == 9 * Cin  # last rows are fully inside


def test_conv_bias_and_channel_roles():
    # w[o, c]: output channel first. One input channel lit, one weight set.
    x = np.zeros((1, 3, 4, 4))
    x[0, 2] = 1.0
    w = np.zeros((2, 3, 3, 3))
    w[1, 2, 1, 1] = 5.0
    y = lo.conv3x3(x, w, np.array([0.25, -0.5]))
    assert np.all(y[0, 0] == 0.25) and np.all(y[0, 1] == 4.5)


def test_conv_translation_equivariance_interior():
    x = np.zeros((1, 2, 12, 12))
    x[:, :, 4:7, 4:7] = rnd(1, 2, 3, 3)
    w, b = rnd(3, 2, 3, 3), np.zeros(3)
    y0 = lo.conv3x3(x, w, b)
    y1 = lo.conv3x3(np.roll(x, (2, 3), axis=(2, 3)), w, b)
    assert np.allclose(np.roll(y0, (2, 3), axis=(2, 3)), y1, atol=1e-14)


# -------------------------------------------------------------------------- group norm
def test_group_norm_moments():
    x = rnd(3, 8, 5, 6) * 3.0 + 2.0
    eps = 1e-5
    y = lo.group_norm(x, np.ones(8), np.zeros(8), 4, eps)
    yg = y.reshape(3, 4, -1)
    xg = x.reshape(3, 4, -1)
    assert np.max(np.abs(yg.mean(axis=2))) < 1e-13
    var = xg.var(axis=2)  # biased
    assert np.allclose(yg.var(axis=2), var / (var + eps), rtol=1e-12)


def test_group_norm_biased_variance_closed_form():
    # slab values {0, 2}: mean 1, biased variance 1 -> y = +-1/sqrt(1 + eps)
    x = np.zeros((1, 2, 1, 2))
    x[0, :, 0, 1] = 2.0
    y = lo.group_norm(x, np.ones(2), np.zeros(2), 1, 0.25)
    assert np.allclose(y.ravel(), np.array([-1, 1, -1, 1]) / math.sqrt(1.25))


def test_group_norm_matches_torch_and_brute():
    x, g, b = rnd(2, 12, 4, 5), rnd(12), rnd(12)
    y = lo.group_norm(x, g, b, 3, 1e-5)
    yt = TF.group_norm(torch.from_numpy(x), 3, torch.from_numpy(g), torch.from_numpy(b), 1e-5).numpy()
    assert rel_l2(y, yt) < 1e-13
    yb = np.array(brute.group_norm_silu(x.tolist(), g.tolist(), b.tolist(), 3, 1e-5, act=False))
    assert np.max(np.abs(y - yb)) < 1e-12


def test_group_norm_is_per_frame_and_per_group():
    x = rnd(2, 8, 3, 3)
    y = lo.group_norm(x, np.ones(8), np.zeros(8), 4, 1e-5)
    x2 = x.copy()
    x2[1] *= 7.0  # other frame
    x2[0, 2:4] += 3.0  # other group of frame 0
    y2 = lo.group_norm(x2, np.ones(8), np.zeros(8), 4, 1e-5)
    assert np.allclose(y[0, 0:2], y2[0, 0:2], atol=1e-14)
    assert np.allclose(y[0, 4:], y2[0, 4:], atol=1e-14)


# -------------------------------------------------------------------------------- silu
def test_silu_closed_forms():
    x = np.array([0.0, 1.0, -1.0, 30.0, -30.0])
    y = lo.silu(x)
    assert y[0] == 0.0
    assert abs(y[1] - 1.0 / (1.0 + math.exp(-1.0))) < 1e-15
    assert abs(y[3] - 30.0) < 1e-11 and abs(y[4]) < 1e-11
    z = rnd(100)
    assert np.allclose(lo.silu(z) - lo.silu(-z), z, atol=1e-14)  # x*s(x) + x*s(-x) = x
    assert rel_l2(lo.silu(z), TF.silu(torch.from_numpy(z)).numpy()) < 1e-14


# --------------------------------------------------------------------------- attention
def _attn_weights(C):
    return [rnd(C, C) * 0.3 for _ in range(4)] + [rnd(C) * 0.3]


def test_attention_matches_brute_force():
    C, L, heads = 6, 5, 2
    X = rnd(L, C)
    ws = _attn_weights(C)
    y = lo.attention(X, X, *ws, heads)
    yb = np.array(brute.attn_rows(X.tolist(), *[w.tolist() for w in ws], heads))
    assert np.max(np.abs(y - yb)) < 1e-12


def test_attention_core_matches_brute_force():
    # distinct q, k, v with fewer queries than keys (a query chunk), three heads
    C, Lq, L, heads = 6, 3, 7, 3
    q, k, v = rnd(Lq, C) * 2.0, rnd(L, C) * 2.0, rnd(L, C)
    o = lo.attention_core(q, k, v, heads)
    ob = np.array(brute.attn_core(q.tolist(), k.tolist(), v.tolist(), heads))
    assert o.shape == (Lq, C)
    assert np.max(np.abs(o - ob)) < 1e-13


def test_attention_core_batched_matches_torch_sdpa_and_closed_forms():
    C, Lq, L, heads = 16, 4, 9, 4
    d = C // heads
    q, k, v = rnd(2, 3, Lq, C), rnd(2, 3, L, C), rnd(2, 3, L, C)
    o = lo.attention_core(q, k, v, heads)
    split = lambda t: torch.from_numpy(t).reshape(2, 3, t.shape[2], heads, d).transpose(2, 3)
    ot = TF.scaled_dot_product_attention(split(q), split(k), split(v)).transpose(2, 3).reshape(2, 3, Lq, C).numpy()
    assert np.max(np.abs(o - ot)) < 1e-13
    # zero queries: every key weighs the same, the output is the mean of the values
    assert np.allclose(lo.attention_core(np.zeros_like(q), k, v, heads), v.mean(axis=2, keepdims=True).repeat(Lq, 2), atol=1e-14)
    # one key: the softmax is 1 and the output is that value whatever the scores are
    assert np.allclose(lo.attention_core(q, k[:, :, :1], v[:, :, :1], heads), v[:, :, :1].repeat(Lq, 2), atol=0)
    # two keys, one head of size 4, q.k = 4 and 0: weights e^{4/2} : 1 (the 1/sqrt(d) scale)
    qq = np.array([[1.0, 1.0, 1.0, 1.0]]); kk = np.array([[1.0, 1.0, 1.0, 1.0], [0.0, 0.0, 0.0, 0.0]])
    vv = np.array([[1.0, 0, 0, 0], [0, 1.0, 0, 0]])
    w0 = math.exp(2.0) / (math.exp(2.0) + 1.0)
    assert np.allclose(lo.attention_core(qq, kk, vv, 1), [[w0, 1 - w0, 0, 0]], atol=1e-15)
    # transposed-operand mistake (scores of k against q) would change a non-square case
    assert o.shape == q.shape


def test_attention_is_projections_around_the_core():
    C, L, heads = 8, 6, 2
    X = rnd(L, C)
    wq, wk, wv, wo, bo = _attn_weights(C)
    y = lo.attention(X[1:4], X, wq, wk, wv, wo, bo, heads)
    o = np.array(brute.attn_core((X[1:4] @ wq.T).tolist(), (X @ wk.T).tolist(), (X @ wv.T).tolist(), heads))
    assert np.max(np.abs(y - (o @ wo.T + bo))) < 1e-13


def test_attention_matches_torch_sdpa():
    C, L, heads = 16, 9, 4
    X = rnd(3, L, C)
    wq, wk, wv, wo, bo = _attn_weights(C)
    y = lo.attention(X, X, wq, wk, wv, wo, bo, heads)
    t = torch.from_numpy(X)
    d = C // heads

    def split(w):
        return (t @ torch.from_numpy(w).T).reshape(3, L, heads, d).transpose(1, 2)

    o = TF.scaled_dot_product_attention(split(wq), split(wk), split(wv))  # scale = 1/sqrt(d)
    o = o.transpose(1, 2).reshape(3, L, C) @ torch.from_numpy(wo).T + torch.from_numpy(bo)
    assert rel_l2(y, o.numpy()) < 1e-12


def test_attention_single_token_is_linear():
    # L = 1: softmax of one logit is 1, so Y = X Wv^T Wo^T + bo
    C = 8
    X = rnd(4, 1, C)
    wq, wk, wv, wo, bo = _attn_weights(C)
    y = lo.attention(X, X, wq, wk, wv, wo, bo, 2)
    assert np.allclose(y, X @ wv.T @ wo.T + bo, atol=1e-13)


def test_attention_zero_query_is_mean_of_values():
    C, L = 8, 7
    X = rnd(L, C)
    _, wk, wv, wo, bo = _attn_weights(C)
    y = lo.attention(X, X, np.zeros((C, C)), wk, wv, wo, bo, 4)
    want = (X @ wv.T).mean(axis=0) @ wo.T + bo
    assert np.allclose(y, np.broadcast_to(want, (L, C)), atol=1e-13)


def test_attention_scale_is_inverse_sqrt_head_dim():
    # two keys, d = 4, one head: logits q.k/2. Choose q.k = 2*ln(3) vs 0 -> weights 3/4, 1/4.
    C = 4
    I = np.eye(C)
    X = np.zeros((2, C))
    X[0, 0] = math.sqrt(2 * math.log(3.0))
    y = lo.attention(X[:1], X, I, I, I, I, np.zeros(C), 1)
    assert np.allclose(y[0], 0.75 * X[0] + 0.25 * X[1], atol=1e-13)


def test_attention_heads_do_not_mix():
    # with Wo = I, output channels of head 0 do not depend on head-1 channels of V
    C, L, heads = 8, 5, 2
    X = rnd(L, C)
    wq, wk, wv = rnd(C, C), rnd(C, C), rnd(C, C)
    y0 = lo.attention(X, X, wq, wk, wv, np.eye(C), np.zeros(C), heads)
    wv2 = wv.copy()
    wv2[4:] = rnd(4, C)
    y1 = lo.attention(X, X, wq, wk, wv2, np.eye(C), np.zeros(C), heads)
    assert np.allclose(y0[:, :4], y1[:, :4], atol=1e-14) and not np.allclose(y0[:, 4:], y1[:, 4:])


def test_attention_token_permutation_equivariance():
    C, L = 8, 11
    X = rnd(L, C)
    ws = _attn_weights(C)
    perm = rng.permutation(L)
    assert np.allclose(lo.attention(X, X, *ws, 2)[perm], lo.attention(X[perm], X[perm], *ws, 2), atol=1e-13)


def test_attention_query_chunk_is_row_slice():
    C, L = 8, 10
    X = rnd(L, C)
    ws = _attn_weights(C)
    full = lo.attention(X, X, *ws, 2)
    assert np.allclose(lo.attention(X[3:7], X, *ws, 2), full[3:7], atol=1e-14)


def test_softmax_rows_sum_to_one_and_shift_invariant():
    s = rnd(4, 9) * 20
    a = lo.softmax_rows(s)
    assert np.allclose(a.sum(axis=-1), 1.0, atol=1e-14)
    assert np.allclose(a, lo.softmax_rows(s + 1000.0), atol=1e-12)
    assert np.all(np.isfinite(lo.softmax_rows(np.array([[1e4, -1e4]]))))


# --------------------------------------------------------------------------------- up2
def test_up2_blocks_and_torch():
    z = rnd(2, 3, 4, 5)
    u = lo.up2(z)
    assert u.shape == (2, 3, 8, 10)
    for di in range(2):
        for dj in range(2):
            assert np.array_equal(u[:, :, di::2, dj::2], z)
    ut = TF.interpolate(torch.from_numpy(z), scale_factor=2, mode="nearest").numpy()
    assert np.array_equal(u, ut)


def test_chunk_ranges():
    assert list(lo._chunks(10, 0)) == [(0, 10)]
    assert list(lo._chunks(10, 16)) == [(0, 10)]
    assert list(lo._chunks(10, 4)) == [(0, 4), (4, 8), (8, 10)]
    assert list(lo._chunks(8, 2)) == [(0, 2), (2, 4), (4, 6), (6, 8)]
