"""CPU oracle for the cache-hit step of a video diffusion transformer (DiT), the variant of the method that the
paper's EasyAnimate rows measure and its conclusion names as the extension.

TEST INFRASTRUCTURE ONLY. Only the test-suite and the benchmark's CPU-baseline leg may import it; the product
path never does, and nothing here imports the product.

What is computed. A DiT has no down/up branches; the reuse rule of the "Asynchronous Swapping" section (features
computed at a normal step are stored and reused at the following cache steps, only the shallow part being
recomputed) is applied to its stack of L blocks: blocks [0, a) and [b, L) play the shallow part, blocks [a, b) the
deep part. What the deep part contributes to the hidden states is the sum of its blocks' gated branch outputs,
Delta = x_b - x_a. A *normal* step runs all blocks and stores Delta; a *cache* step runs blocks [0, a), adds the
stored Delta, and runs blocks [b, L). In both kinds of step the deep part enters as x_a + Delta, with Delta held in
an accumulator of its own, so a cache step fed the Delta of the same input reproduces the normal step exactly. The
cache entry is kept in host memory and brought back when required (a pure copy), as in the U-Net case. The paper
does not say which blocks are cached for a DiT; this split is the reading taken.

One block (adaLN-modulated, as in DiT; the conditioning vectors are inputs):
    h  = LN(x) * (1 + scale_msa) + shift_msa              LN: per token over D, biased variance, no affine
    x += gate_msa * (Attn(h) )                            Attn: q,k,v = h W^T + b per head, softmax(q k^T / sqrt(d)) v,
                                                          output projection with bias; tokens = ALL tokens of the
                                                          video (full 3-D attention), per batch element
    h  = LN(x) * (1 + scale_mlp) + shift_mlp
    x += gate_mlp * (W2 gelu_tanh(W1 h + b1) + b2)
Feature chunk: LN, projections and MLP run over token chunks, attention over query chunks against all keys;
the chunked variants really loop over slices and give the same result.

Pins: tests/test_oracle_dit.py (scalar brute force, an independent torch float64 build, closed forms, the method's
invariants). The paper prints no values for this path.
"""
from __future__ import annotations

import math
from typing import Dict, List, Optional

import numpy as np

from .lightcache_oracle import _chunks, attention_core

Weights = Dict[str, np.ndarray]
MOD_NAMES = ("shift_msa", "scale_msa", "gate_msa", "shift_mlp", "scale_mlp", "gate_mlp")


def layer_norm(x: np.ndarray, eps: float) -> np.ndarray:
    """Per row over the last axis: (x - mean) / sqrt(biased variance + eps); no scale, no shift."""
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + x.dtype.type(eps))


def gelu_tanh(x: np.ndarray) -> np.ndarray:
    """0.5 x (1 + tanh(sqrt(2/pi) (x + 0.044715 x^3)))."""
    return 0.5 * x * (1.0 + np.tanh(math.sqrt(2.0 / math.pi) * (x + 0.044715 * x ** 3)))


def required_weights(cfg) -> List[str]:
    return [f"blk{i}.{k}" for i in range(cfg.L) for k in ("wqkv", "bqkv", "wo", "bo", "w1", "b1", "w2", "b2")]


class DitOracle:
    """``cfg``: B, T (tokens per batch element), D, heads, head_dim (heads * head_dim == D), L, cache_a, cache_b,
    mlp_ratio, ln_eps. ``weights``: name -> array, PyTorch order ([out, in]); wqkv stacks q, k, v rows.
    ``mod`` arguments: array [L, B, 6, D] in the order of MOD_NAMES."""

    def __init__(self, cfg, weights: Weights, dtype=np.float64, host_slots: int = 1, dev_slots: int = 2):
        self.cfg = cfg
        self.dtype = np.dtype(dtype)
        self.w = {k: np.asarray(v, dtype=self.dtype) for k, v in weights.items()}
        self.token_chunk = 0
        self.dev: List[Optional[np.ndarray]] = [None] * dev_slots
        self.host: List[Optional[np.ndarray]] = [None] * host_slots
        if cfg.heads * cfg.head_dim != cfg.D:
            raise ValueError("heads * head_dim must equal D")
        if not (0 <= cfg.cache_a <= cfg.cache_b <= cfg.L):
            raise ValueError("need 0 <= cache_a <= cache_b <= L")

    def set_chunk(self, token_chunk: int) -> None:
        if token_chunk < 0:
            raise ValueError("chunk size must be >= 0")
        self.token_chunk = token_chunk

    # ---- one block's two branches, for one batch element: x [T, D] -> what is added to x --------------------
    def attn_branch(self, x, i, m):
        c, w = self.cfg, self.w
        D = c.D
        h = np.empty_like(x)
        for t0, t1 in _chunks(c.T, self.token_chunk):
            h[t0:t1] = layer_norm(x[t0:t1], c.ln_eps) * (1.0 + m[1]) + m[0]
        qkv = np.empty((c.T, 3 * D), dtype=self.dtype)
        for t0, t1 in _chunks(c.T, self.token_chunk):
            qkv[t0:t1] = h[t0:t1] @ w[f"blk{i}.wqkv"].T + w[f"blk{i}.bqkv"]
        out = np.empty_like(x)
        for t0, t1 in _chunks(c.T, self.token_chunk):  # queries in chunks, keys and values of all tokens
            o = attention_core(qkv[t0:t1, :D], qkv[:, D:2 * D], qkv[:, 2 * D:], c.heads)
            out[t0:t1] = m[2] * (o @ w[f"blk{i}.wo"].T + w[f"blk{i}.bo"])
        return out

    def mlp_branch(self, x, i, m):
        c, w = self.cfg, self.w
        out = np.empty_like(x)
        for t0, t1 in _chunks(c.T, self.token_chunk):
            h = layer_norm(x[t0:t1], c.ln_eps) * (1.0 + m[4]) + m[3]
            u = gelu_tanh(h @ w[f"blk{i}.w1"].T + w[f"blk{i}.b1"])
            out[t0:t1] = m[5] * (u @ w[f"blk{i}.w2"].T + w[f"blk{i}.b2"])
        return out

    def _blocks(self, x, mod, i0, i1):
        """Blocks [i0, i1) applied to x [B, T, D] in place of a copy."""
        x = x.copy()
        for i in range(i0, i1):
            for b in range(self.cfg.B):
                x[b] += self.attn_branch(x[b], i, mod[i, b])
                x[b] += self.mlp_branch(x[b], i, mod[i, b])
        return x

    def _deep(self, xa, mod):
        """Delta = what blocks [a, b) add to xa, accumulated apart from xa."""
        c = self.cfg
        delta = np.zeros_like(xa)
        for i in range(c.cache_a, c.cache_b):
            for b in range(c.B):
                delta[b] += self.attn_branch(xa[b] + delta[b], i, mod[i, b])
                delta[b] += self.mlp_branch(xa[b] + delta[b], i, mod[i, b])
        return delta

    def _check(self, x, mod):
        c = self.cfg
        x = np.asarray(x, dtype=self.dtype)
        mod = np.asarray(mod, dtype=self.dtype)
        assert x.shape == (c.B, c.T, c.D), x.shape
        assert mod.shape == (c.L, c.B, 6, c.D), mod.shape
        return x, mod

    def full_step(self, x, mod, dev_slot: int = 0):
        """Normal step: all blocks; Delta of the deep blocks goes into device slot `dev_slot`."""
        c = self.cfg
        x, mod = self._check(x, mod)
        xa = self._blocks(x, mod, 0, c.cache_a)
        delta = self._deep(xa, mod)
        self.dev[dev_slot] = delta
        return self._blocks(xa + delta, mod, c.cache_b, c.L)

    def cached_step(self, x, mod, dev_slot: int = 0):
        """Cache step: blocks [0, a), the stored Delta, blocks [b, L)."""
        c = self.cfg
        if self.dev[dev_slot] is None:
            raise RuntimeError("cached step on an empty device slot")
        x, mod = self._check(x, mod)
        xa = self._blocks(x, mod, 0, c.cache_a)
        return self._blocks(xa + self.dev[dev_slot], mod, c.cache_b, c.L)

    # ---- cache bank ---------------------------------------------------------------------------------------
    def cache_write(self, dev_slot: int, delta) -> None:
        c = self.cfg
        delta = np.asarray(delta, dtype=self.dtype)
        assert delta.shape == (c.B, c.T, c.D)
        self.dev[dev_slot] = delta.copy()

    def swap_out(self, dev_slot: int, host_slot: int) -> None:
        if self.dev[dev_slot] is None:
            raise RuntimeError("swap-out of an empty device slot")
        self.host[host_slot] = self.dev[dev_slot].copy()

    def swap_in(self, host_slot: int, dev_slot: int) -> None:
        if self.host[host_slot] is None:
            raise RuntimeError("swap-in from an empty host slot")
        self.dev[dev_slot] = self.host[host_slot].copy()
