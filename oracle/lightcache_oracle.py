"""CPU oracle for the cache-hit denoising step of a DeepCache-style video UNet.

TEST INFRASTRUCTURE ONLY. This file is the slow, plain reference that the HIP path is
checked against. Only the test-suite, the smoke check and the benchmark's CPU-baseline
leg may import it; the product path never does, and nothing here imports the product.

Everything is the plain definition of the operation, in float64 by default (pass
``dtype=np.float32`` to ``Oracle`` for a single-precision run). Tensors are in the
paper's order ("Feature chunk" section): a feature map is [B, F, C, H, W]; internally
the batch and frame axes are flattened to N = B*F, i.e. arrays are [N, C, H, W].
numpy ``matmul`` is used as a step where the definition is a contraction; there is no
blocking, fusion or re-ordering beyond what the definitions below state.

What is computed (citations are to the paper's sections / equations):

* U-Net skip structure, "Feature Calculation" paragraph, eq. U_i = Concat(D_i, U_{i+1}):
  the shallowest up block consumes the channel-concatenation of the shallow skip feature
  D_m and the deep feature U_{m+1} (skip channels first).
* DeepCache reuse rule, "Asynchronous Swapping" section, cache equation and the text
  after it: the deep feature U_{m+1} computed at a *normal* step t is stored and, at the
  *cache* steps t+1 .. t+n-1, only D_m and U_m are recomputed and the stored feature is
  used in the concatenation. ``full_step`` is the normal step, ``cached_step`` the cache
  step.
* Cache swapping, same section: the stored feature lives in host memory and is brought
  back when required; it is a pure copy ("does not affect generation quality").
* Feature chunk, "Feature chunk and Sliced Decoding" section, eq. Chunk(F): feature maps
  are processed in pieces. Here every operator is chunked only along an axis it is
  independent over (frames for per-frame operators, spatial positions for temporal
  attention, query tokens for spatial attention), so chunking is exact; the chunked
  variants below really loop over slices.
* The same equation taken literally, F_i of size H/eta x W/omega (``set_spatial_chunk``):
  every operator of the shallow branch loops over the eta x omega spatial blocks of a
  frame. A 3x3 convolution computes a block from the block plus a one-pixel halo taken
  from the neighbouring blocks (zeros beyond the image); GroupNorm is two passes over the
  blocks (split sums of x and x^2 first, then the normalisation block by block); spatial
  attention takes a block's tokens as queries against all tokens of the frame; temporal
  attention takes a block's positions. The results are those of the unchunked operators
  up to the rounding of the split sums.

The operators inside the shallow blocks (the paper does not spell them out; these are
the standard definitions):
  conv3x3      cross-correlation, zero padding 1, stride 1 or 2, plus bias
  group_norm   per frame and per group of C/G consecutive channels, biased variance
  silu         x / (1 + exp(-x))
  attention    bias-free Q/K/V projections, h heads of size d, softmax(QK^T/sqrt(d))V,
               output projection with bias
  up2          nearest-neighbour 2x upsampling

Pins: tests/test_oracle_ops.py, tests/test_oracle_step.py (brute force on tiny inputs,
closed forms, library second opinions, the method's invariants). Output *values* of a
whole step are not printed anywhere in the paper; they are pinned by those tests only.
"""
from __future__ import annotations

import math
from typing import Dict, List, Optional

import numpy as np

Weights = Dict[str, np.ndarray]


# --------------------------------------------------------------------------------------
# Operators
# --------------------------------------------------------------------------------------

def conv3x3(x: np.ndarray, w: np.ndarray, b: np.ndarray, stride: int = 1) -> np.ndarray:
    """y[n,o,i,j] = b[o] + sum_{c,a,e} w[o,c,a,e] * x[n,c,stride*i+a-1,stride*j+e-1], zero outside.

    x [N,Cin,H,W], w [Cout,Cin,3,3], b [Cout] -> y [N,Cout,H/stride,W/stride].
    """
    N, Cin, H, W = x.shape
    Cout = w.shape[0]
    assert w.shape == (Cout, Cin, 3, 3) and b.shape == (Cout,)
    assert stride in (1, 2) and H % stride == 0 and W % stride == 0
    Ho, Wo = H // stride, W // stride
    xp = np.zeros((N, Cin, H + 2, W + 2), dtype=x.dtype)
    xp[:, :, 1:H + 1, 1:W + 1] = x
    y = np.empty((N, Cout, Ho, Wo), dtype=x.dtype)
    y[...] = b[None, :, None, None]
    for a in range(3):
        for e in range(3):
            # padded index of input row for output row i is stride*i + a
            patch = xp[:, :, a:a + stride * Ho:stride, e:e + stride * Wo:stride]
            patch = np.ascontiguousarray(patch).reshape(N, Cin, Ho * Wo)
            w_tap = np.ascontiguousarray(w[:, :, a, e])  # [Cout, Cin]
            y += np.matmul(w_tap[None], patch).reshape(N, Cout, Ho, Wo)
    return y


def conv3x3_block(x: np.ndarray, w: np.ndarray, b: np.ndarray, y0: int, y1: int, x0: int, x1: int) -> np.ndarray:
    """Rows [y0, y1) x columns [x0, x1) of conv3x3(x, w, b) (stride 1), computed from that block of x and its
    one-pixel halo only: the halo comes from the neighbouring blocks of x, zeros where it leaves the image."""
    N, Cin, H, W = x.shape
    Cout = w.shape[0]
    bh, bw = y1 - y0, x1 - x0
    assert 0 <= y0 < y1 <= H and 0 <= x0 < x1 <= W
    patch = np.zeros((N, Cin, bh + 2, bw + 2), dtype=x.dtype)   # patch[i, j] = x[y0 - 1 + i, x0 - 1 + j]
    ys0, ys1 = max(y0 - 1, 0), min(y1 + 1, H)
    xs0, xs1 = max(x0 - 1, 0), min(x1 + 1, W)
    patch[:, :, ys0 - (y0 - 1):ys1 - (y0 - 1), xs0 - (x0 - 1):xs1 - (x0 - 1)] = x[:, :, ys0:ys1, xs0:xs1]
    y = np.empty((N, Cout, bh, bw), dtype=x.dtype)
    y[...] = b[None, :, None, None]
    for a in range(3):
        for e in range(3):
            tap = np.ascontiguousarray(patch[:, :, a:a + bh, e:e + bw]).reshape(N, Cin, bh * bw)
            y += np.matmul(np.ascontiguousarray(w[:, :, a, e])[None], tap).reshape(N, Cout, bh, bw)
    return y


def group_norm_blocks(x: np.ndarray, gamma: np.ndarray, beta: np.ndarray, groups: int, eps: float, blocks) -> np.ndarray:
    """GroupNorm in two passes over spatial blocks [(y0, y1, x0, x1), ...] that tile the image: pass 1 adds up, per
    frame and group, the count, the sum and the sum of squares block by block (mean = S1 / n, biased variance =
    S2 / n - mean^2); pass 2 normalises each block with those statistics."""
    N, C, H, W = x.shape
    cg = C // groups
    assert C % groups == 0
    n = 0
    s1 = np.zeros((N, groups), dtype=x.dtype)
    s2 = np.zeros((N, groups), dtype=x.dtype)
    for (y0, y1, x0, x1) in blocks:
        blk = x[:, :, y0:y1, x0:x1].reshape(N, groups, -1)
        n += blk.shape[2]
        s1 += blk.sum(axis=2)
        s2 += (blk * blk).sum(axis=2)
    assert n == cg * H * W, "the blocks must tile the image"
    mu = s1 / n
    rstd = 1.0 / np.sqrt(s2 / n - mu * mu + x.dtype.type(eps))
    mu_c, rstd_c = np.repeat(mu, cg, axis=1), np.repeat(rstd, cg, axis=1)  # per channel
    y = np.empty_like(x)
    for (y0, y1, x0, x1) in blocks:
        blk = (x[:, :, y0:y1, x0:x1] - mu_c[:, :, None, None]) * rstd_c[:, :, None, None]
        y[:, :, y0:y1, x0:x1] = blk * gamma[None, :, None, None] + beta[None, :, None, None]
    return y


def group_norm(x: np.ndarray, gamma: np.ndarray, beta: np.ndarray, groups: int, eps: float) -> np.ndarray:
    """Per (frame, group): mean and biased variance over (C/G)*H*W elements, then affine."""
    N, C, H, W = x.shape
    assert C % groups == 0
    xg = x.reshape(N, groups, (C // groups) * H * W)
    mu = xg.mean(axis=2, keepdims=True)
    var = ((xg - mu) ** 2).mean(axis=2, keepdims=True)
    y = ((xg - mu) / np.sqrt(var + x.dtype.type(eps))).reshape(N, C, H, W)
    return y * gamma[None, :, None, None] + beta[None, :, None, None]


def silu(x: np.ndarray) -> np.ndarray:
    return x / (1.0 + np.exp(-x))


def softmax_rows(s: np.ndarray) -> np.ndarray:
    e = s - s.max(axis=-1, keepdims=True)
    np.exp(e, out=e)
    e /= e.sum(axis=-1, keepdims=True)
    return e


def attention_core(q: np.ndarray, k: np.ndarray, v: np.ndarray, heads: int) -> np.ndarray:
    """Per head: softmax(Q_h K_h^T / sqrt(d)) V_h, heads merged again on the channel axis.

    q [.., Lq, C]; k, v [.., L, C]; head h owns channels [h*d, (h+1)*d), d = C / heads. No mask, no
    dropout. This is the part of the attention block between the q/k/v projections and the output
    projection."""
    C = q.shape[-1]
    d = C // heads
    assert heads * d == C and k.shape[-1] == C and v.shape[-1] == C
    o = np.empty(q.shape, dtype=q.dtype)
    scale = 1.0 / math.sqrt(d)
    for hd in range(heads):
        sl = slice(hd * d, (hd + 1) * d)
        qh, kh, vh = (np.ascontiguousarray(t[..., sl]) for t in (q, k, v))
        s = (qh @ np.swapaxes(kh, -1, -2)) * q.dtype.type(scale)
        o[..., sl] = softmax_rows(s) @ vh
    return o


def attention(xq: np.ndarray, xkv: np.ndarray, wq, wk, wv, wo, bo, heads: int) -> np.ndarray:
    """Multi-head self-attention of query rows xq [.., Lq, C] against rows xkv [.., L, C].

    Q = xq Wq^T, K = xkv Wk^T, V = xkv Wv^T; per head softmax(Q K^T / sqrt(d)) V; heads merged;
    Y = O Wo^T + bo. (xq is xkv itself, or a slice of its rows when queries are chunked.)
    """
    C = xq.shape[-1]
    assert C % heads == 0
    o = attention_core(_project(xq, wq), _project(xkv, wk), _project(xkv, wv), heads)
    return _project(o, wo) + bo


def _project(x: np.ndarray, w: np.ndarray) -> np.ndarray:
    """x W^T over the last axis. All leading axes are flattened into one row axis first, so a stack
    of many short sequences (temporal attention: one per spatial position) is one matrix product."""
    y = x.reshape(-1, x.shape[-1]) @ np.ascontiguousarray(w.T)
    return y.reshape(x.shape[:-1] + (w.shape[0],))


def up2(z: np.ndarray) -> np.ndarray:
    """Nearest-neighbour 2x: out[n,c,i,j] = z[n,c,i//2,j//2]."""
    return np.repeat(np.repeat(z, 2, axis=2), 2, axis=3)


def _chunks(total: int, size: int):
    """Consecutive [start, stop) ranges of at most `size`; size <= 0 or >= total means one range."""
    if size <= 0 or size >= total:
        yield 0, total
        return
    for s in range(0, total, size):
        yield s, min(s + size, total)


# --------------------------------------------------------------------------------------
# The stage
# --------------------------------------------------------------------------------------

class Oracle:
    """Full (normal) and cached steps of one shallow stage, plus a host/device cache bank.

    ``cfg`` is any object with attributes B, F, H, W, C_lat, C, C_deep, groups, n_res,
    heads, head_dim, gn_eps. ``weights`` maps names ("conv_in.w", "res0.gn_g", ...,
    see ``required_weights``) to arrays in PyTorch order ([Cout, Cin, 3, 3] / [Cout, Cin]).
    """

    def __init__(self, cfg, weights: Weights, dtype=np.float64, host_slots: int = 1, dev_slots: int = 2):
        self.cfg = cfg
        self.dtype = np.dtype(dtype)
        self.w = {k: np.asarray(v, dtype=self.dtype) for k, v in weights.items()}
        self.frame_chunk = 0
        self.token_chunk = 0
        self.eta = 1    # spatial chunk: eta x omega blocks per frame (1, 1 = off)
        self.omega = 1
        self.progress = None  # optional callable(str): told after every chunk of a step (long runs report where they are)
        self.dev: List[Optional[np.ndarray]] = [None] * dev_slots
        self.host: List[Optional[np.ndarray]] = [None] * host_slots
        c = cfg
        if c.C % c.groups or c.C_deep % c.groups or (c.C + c.C_deep) % c.groups:
            raise ValueError("channel counts must be divisible by the number of groups")
        if c.heads * c.head_dim != c.C:
            raise ValueError("heads * head_dim must equal C")
        if c.H % 2 or c.W % 2:
            raise ValueError("H and W must be even")

    # ---- chunk control --------------------------------------------------------------
    def set_chunk(self, frame_chunk: int, token_chunk: int) -> None:
        if frame_chunk < 0 or token_chunk < 0:
            raise ValueError("chunk sizes must be >= 0")
        self.frame_chunk, self.token_chunk = frame_chunk, token_chunk

    def set_spatial_chunk(self, eta: int, omega: int) -> None:
        """Literal spatial feature chunk: every frame is processed in eta x omega blocks of H/eta x W/omega."""
        c = self.cfg
        if eta < 1 or omega < 1 or c.H % eta or c.W % omega or (c.H // eta) % 2 or (c.W // omega) % 2:
            raise ValueError("eta must divide H and omega must divide W into blocks of even size")
        self.eta, self.omega = eta, omega

    def _spatial(self) -> bool:
        return self.eta * self.omega > 1

    def _blocks(self, H: int, W: int):
        """(y0, y1, x0, x1) of the spatial blocks of an H x W map, row-major."""
        bh, bw = H // self.eta, W // self.omega
        return [(i * bh, (i + 1) * bh, j * bw, (j + 1) * bw) for i in range(self.eta) for j in range(self.omega)]

    def _conv(self, x, w, b):
        """conv3x3, block by block (each from its block and halo) under a spatial chunk."""
        if not self._spatial():
            return conv3x3(x, w, b)
        N, _, H, W = x.shape
        y = np.empty((N, w.shape[0], H, W), dtype=self.dtype)
        for (y0, y1, x0, x1) in self._blocks(H, W):
            y[:, :, y0:y1, x0:x1] = conv3x3_block(x, w, b, y0, y1, x0, x1)
        return y

    def _token_chunk(self) -> int:
        c = self.cfg
        if self.token_chunk > 0:
            return self.token_chunk
        if self.frame_chunk > 0 and self.frame_chunk < c.B * c.F:
            # same number of (frame, position) rows per pass as a frame chunk has
            return -(-(self.frame_chunk * c.H * c.W) // (c.B * c.F))
        return 0

    def _tick(self, what: str) -> None:
        if self.progress is not None:
            self.progress(what)

    # ---- blocks ---------------------------------------------------------------------
    def _gn(self, x, prefix):
        g, b = self.w[prefix + ".gn_g"], self.w[prefix + ".gn_b"]
        if self._spatial() and x.shape[2:] == (self.cfg.H, self.cfg.W):
            return group_norm_blocks(x, g, b, self.cfg.groups, self.cfg.gn_eps, self._blocks(*x.shape[2:]))
        return group_norm(x, g, b, self.cfg.groups, self.cfg.gn_eps)

    def res_block(self, h, prefix):
        """h + conv3x3(SiLU(GN(h))). (The residual block of the deep stand-in, at half resolution, is never
        chunked spatially.)"""
        if h.shape[2:] != (self.cfg.H, self.cfg.W):
            return h + conv3x3(silu(self._gn(h, prefix)), self.w[prefix + ".w"], self.w[prefix + ".b"])
        return h + self._conv(silu(self._gn(h, prefix)), self.w[prefix + ".w"], self.w[prefix + ".b"])

    def _attn_w(self, prefix):
        w = self.w
        return (w[prefix + ".wq"], w[prefix + ".wk"], w[prefix + ".wv"], w[prefix + ".wo"], w[prefix + ".bo"])

    def spatial_block(self, h):
        """Per frame: tokens = spatial positions (t = i*W + j); h += Attn(GN(h)). Queries chunked."""
        N, C, H, W = h.shape
        g = self._gn(h, "sattn")
        out = h.copy()
        for n in range(N):
            X = g[n].reshape(C, H * W).T  # [T, C]
            if self._spatial():
                # queries = the tokens of one spatial block, keys and values = all tokens of the frame
                for (y0, y1, x0, x1) in self._blocks(H, W):
                    tok = (np.arange(y0, y1)[:, None] * W + np.arange(x0, x1)[None, :]).ravel()
                    Y = attention(X[tok], X, *self._attn_w("sattn"), self.cfg.heads)
                    out[n].reshape(C, H * W)[:, tok] += Y.T
                continue
            for t0, t1 in _chunks(H * W, self._token_chunk()):
                Y = attention(X[t0:t1], X, *self._attn_w("sattn"), self.cfg.heads)  # [tq, C]
                out[n].reshape(C, H * W)[:, t0:t1] += Y.T
        return out

    def temporal_block(self, h):
        """Per batch element and spatial position: tokens = the F frames; h += Attn(GN(h)).
        GroupNorm statistics are per frame over the whole frame; positions are chunked."""
        c = self.cfg
        N, C, H, W = h.shape
        B, F = c.B, N // c.B
        g = self._gn(h, "tattn").reshape(B, F, C, H * W)
        out = h.copy().reshape(B, F, C, H * W)
        if self._spatial():
            pos_sets = [(np.arange(y0, y1)[:, None] * W + np.arange(x0, x1)[None, :]).ravel()
                        for (y0, y1, x0, x1) in self._blocks(H, W)]  # the positions of one spatial block at a time
        else:
            pos_sets = [np.arange(p0, p1) for p0, p1 in _chunks(H * W, self._token_chunk())]
        for pos in pos_sets:
            X = np.transpose(g[:, :, :, pos], (0, 3, 1, 2))  # [B, positions, F, C]
            Y = attention(X, X, *self._attn_w("tattn"), c.heads)  # [B, positions, F, C]
            out[:, :, :, pos] += np.transpose(Y, (0, 2, 3, 1))
        return out.reshape(N, C, H, W)

    def shallow_down(self, x):
        """D_m: conv_in, n_res residual blocks, spatial block; per-frame work in frame chunks."""
        c = self.cfg
        N = x.shape[0]
        h = np.empty((N, c.C, c.H, c.W), dtype=self.dtype)
        for n0, n1 in _chunks(N, self.frame_chunk):
            t = self._conv(x[n0:n1], self.w["conv_in.w"], self.w["conv_in.b"])
            for i in range(c.n_res):
                t = self.res_block(t, f"res{i}")
            h[n0:n1] = self.spatial_block(t)
            self._tick(f"shallow down: frames {n0}..{n1 - 1} of {N}")
        h = self.temporal_block(h)
        self._tick("temporal block")
        return h

    def deep_branch(self, s):
        """Stand-in for everything below the shallow stage: stride-2 conv then one residual block."""
        N = s.shape[0]
        c = self.cfg
        deep = np.empty((N, c.C_deep, c.H // 2, c.W // 2), dtype=self.dtype)
        for n0, n1 in _chunks(N, self.frame_chunk):
            d0 = conv3x3(s[n0:n1], self.w["down.w"], self.w["down.b"], stride=2)
            deep[n0:n1] = self.res_block(d0, "dres")
        return deep

    def shallow_up(self, s, deep):
        """U_m: Concat(skip, up2(deep)) -> GN -> SiLU -> conv3x3 -> GN -> SiLU -> conv_out."""
        c = self.cfg
        N = s.shape[0]
        eps = np.empty((N, c.C_lat, c.H, c.W), dtype=self.dtype)
        for n0, n1 in _chunks(N, self.frame_chunk):
            if self._spatial():
                # the concatenated map block by block: a block of the skip feature with the 2x upsampled block of
                # the deep feature that lies under it
                cat = np.empty((n1 - n0, c.C + c.C_deep, c.H, c.W), dtype=self.dtype)
                for (y0, y1, x0, x1) in self._blocks(c.H, c.W):
                    cat[:, :, y0:y1, x0:x1] = np.concatenate(
                        [s[n0:n1, :, y0:y1, x0:x1], up2(deep[n0:n1, :, y0 // 2:y1 // 2, x0 // 2:x1 // 2])], axis=1)
            else:
                cat = np.concatenate([s[n0:n1], up2(deep[n0:n1])], axis=1)
            u = self._conv(silu(self._gn(cat, "up")), self.w["up.w"], self.w["up.b"])
            eps[n0:n1] = self._conv(silu(self._gn(u, "out")), self.w["out.w"], self.w["out.b"])
            self._tick(f"shallow up: frames {n0}..{n1 - 1} of {N}")
        return eps

    # ---- steps ----------------------------------------------------------------------
    def _flat(self, x):
        c = self.cfg
        x = np.asarray(x, dtype=self.dtype)
        assert x.shape == (c.B, c.F, c.C_lat, c.H, c.W), x.shape
        return x.reshape(c.B * c.F, c.C_lat, c.H, c.W)

    def full_step(self, x, dev_slot: int = 0):
        """Normal step: recompute everything; the deep feature goes into device slot `dev_slot`."""
        c = self.cfg
        s = self.shallow_down(self._flat(x))
        deep = self.deep_branch(s)
        self.dev[dev_slot] = deep
        return self.shallow_up(s, deep).reshape(c.B, c.F, c.C_lat, c.H, c.W)

    def cached_step(self, x, dev_slot: int = 0):
        """Cache step: only the shallow branch is recomputed; the deep feature is read from the slot."""
        c = self.cfg
        if self.dev[dev_slot] is None:
            raise RuntimeError("cached step on an empty device slot")
        s = self.shallow_down(self._flat(x))
        return self.shallow_up(s, self.dev[dev_slot]).reshape(c.B, c.F, c.C_lat, c.H, c.W)

    # ---- cache bank -----------------------------------------------------------------
    def cache_write(self, dev_slot: int, deep) -> None:
        c = self.cfg
        deep = np.asarray(deep, dtype=self.dtype)
        assert deep.shape == (c.B * c.F, c.C_deep, c.H // 2, c.W // 2)
        self.dev[dev_slot] = deep.copy()

    def swap_out(self, dev_slot: int, host_slot: int) -> None:
        if self.dev[dev_slot] is None:
            raise RuntimeError("swap-out of an empty device slot")
        buf = np.empty_like(self.dev[dev_slot])
        np.copyto(buf, self.dev[dev_slot])
        self.host[host_slot] = buf

    def swap_in(self, host_slot: int, dev_slot: int) -> None:
        if self.host[host_slot] is None:
            raise RuntimeError("swap-in from an empty host slot")
        buf = np.empty_like(self.host[host_slot])
        np.copyto(buf, self.host[host_slot])
        self.dev[dev_slot] = buf


def required_weights(cfg) -> List[str]:
    names = ["conv_in.w", "conv_in.b"]
    for i in range(cfg.n_res):
        names += [f"res{i}.{k}" for k in ("gn_g", "gn_b", "w", "b")]
    for blk in ("sattn", "tattn"):
        names += [f"{blk}.{k}" for k in ("gn_g", "gn_b", "wq", "wk", "wv", "wo", "bo")]
    names += ["down.w", "down.b", "dres.gn_g", "dres.gn_b", "dres.w", "dres.b",
              "up.gn_g", "up.gn_b", "up.w", "up.b", "out.gn_g", "out.gn_b", "out.w", "out.b"]
    return names


def run_schedule(oracle: Oracle, x0, steps: int, interval: int, dt: Optional[float] = None):
    """Denoising loop of the "Asynchronous Swapping" section: a normal step when t is a multiple
    of `interval`, a cache step otherwise. After each normal step the deep feature is swapped out
    to host slot (refresh index mod host slots); every cache step reads a device slot that was
    refilled from the host bank (alternating device slots). The latent update between steps is
    the fixed rule x <- x - dt * eps (dt = 1/steps), a stand-in for the sampler.
    Returns (list of x_t fed to each step, list of eps_t)."""
    dt = 1.0 / steps if dt is None else dt
    x = np.asarray(x0, dtype=oracle.dtype)
    xs, outs = [], []
    refresh = -1
    n_dev, n_host = len(oracle.dev), len(oracle.host)
    for t in range(steps):
        xs.append(x.copy())
        if t % interval == 0:
            refresh += 1
            slot = t % n_dev
            eps = oracle.full_step(x, slot)
            oracle.swap_out(slot, refresh % n_host)
        else:
            slot = t % n_dev
            oracle.swap_in(refresh % n_host, slot)
            eps = oracle.cached_step(x, slot)
        outs.append(eps)
        x = x - oracle.dtype.type(dt) * eps
    return xs, outs
