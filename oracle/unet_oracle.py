"""CPU oracle for the U-Net stage with real block internals: the normal and the cache step with the blocks of the
video U-Nets the paper ran (AnimateDiff / Stable-Video-Diffusion style) and a three-level deep branch, so that the
refresh interval n of the "Asynchronous Swapping" section can be swept on synthetic weights.

TEST INFRASTRUCTURE ONLY. Only the test-suite and the benchmark's CPU-baseline leg may import it; the product
path never does, and nothing here imports the product.

The method is the same as in ``lightcache_oracle``: a normal step runs everything and stores the deep feature
U_{m+1} entering the shallowest up block; a cache step recomputes only the shallow down / up blocks and
concatenates the stored feature ("Feature Calculation" paragraph, U_i = Concat(D_i, U_{i+1})). What differs are the
blocks, which the paper takes from its pretrained models and does not describe; they are the usual ones:

  RB(x; temb)   residual block with two convolutions and a time-embedding add:
                  h = conv1(SiLU(GN(x))) + (W_t SiLU(temb) + b_t)[channel];  y = short(x) + conv2(SiLU(GN(h)))
                  short = identity, or a 1x1 convolution when the channel count changes
  ST(x; ctx)    spatial transformer block, tokens = the positions of one frame:
                  z = pin(GN(x));  z += SelfAttn(LN(z));  z += CrossAttn(LN(z), ctx);  z += FF(LN(z));  y = x + pout(z)
                  FF(h) = W2 (a * gelu(g)) + b2 with [a, g] = W1 h + b1 (GEGLU; gelu in its tanh form)
  TT(x)         temporal transformer block, tokens = the F frames of one (batch element, position):
                  z = pin(GN(x));  z += SelfAttn(LN(z) + PE);  z += FF(LN(z));  y = x + pout(z)
                  PE[f, 2i] = sin(f / 10000^(2i/C)), PE[f, 2i+1] = cos(f / 10000^(2i/C))
  Down(x)       conv3x3, stride 2;   UpC(x) = conv3x3(nearest2x(x))

  shallow down  h = conv_in(x);  s = TT(ST(RB(h)))                                  at C,  H x W
  deep          d = TT(ST(RB(Down(s))))                                             at C1, H/2 x W/2
                e = UpC(RB(RB(Down(d))))                                            at C2, H/4 x W/4 (and back to H/2)
                d = TT(ST(RB(Concat(d, e))));  deep = UpC(d)                        at C1, H x W: the cached feature
  shallow up    u = TT(ST(RB(Concat(s, deep))));  eps = conv_out(SiLU(GN(u)))

Attention: bias-free q/k/v, heads of `head_dim` channels, scale 1/sqrt(head_dim), output projection with bias;
LayerNorm with affine (eps ln_eps), GroupNorm with `groups` groups per frame (eps gn_eps).

Pins: tests/test_oracle_unet.py (scalar brute force of each block kind, an independent torch float64 build of
the whole stage, closed forms, cache step on own cache == normal step). The paper prints no values for this path.
"""
from __future__ import annotations

import math
from typing import Dict, List, Optional

import numpy as np

from .dit_oracle import gelu_tanh, layer_norm
from .lightcache_oracle import attention_core, conv3x3, group_norm, silu, up2

Weights = Dict[str, np.ndarray]


def positional_encoding(F: int, C: int, dtype=np.float64) -> np.ndarray:
    """Sinusoidal encoding of the frame index, [F, C] (C even)."""
    pe = np.zeros((F, C), dtype=dtype)
    f = np.arange(F, dtype=dtype)[:, None]
    div = np.exp(-math.log(10000.0) * np.arange(0, C, 2, dtype=dtype) / C)[None, :]
    pe[:, 0::2] = np.sin(f * div)
    pe[:, 1::2] = np.cos(f * div)
    return pe


class UnetOracle:
    """``cfg``: B, F, H, W (multiples of 4), C_lat, C, C1, C2, groups, head_dim, ctx_len, ctx_dim, temb_dim, ff_mult,
    gn_eps, ln_eps. Step inputs: x [B, F, C_lat, H, W], temb [B, temb_dim], ctx [B, ctx_len, ctx_dim]."""

    def __init__(self, cfg, weights: Weights, dtype=np.float64, dev_slots: int = 2, host_slots: int = 1):
        self.cfg = cfg
        self.dtype = np.dtype(dtype)
        self.w = {k: np.asarray(v, dtype=self.dtype) for k, v in weights.items()}
        self.dev: List[Optional[np.ndarray]] = [None] * dev_slots
        self.host: List[Optional[np.ndarray]] = [None] * host_slots
        for c in (cfg.C, cfg.C1, cfg.C2, cfg.C + cfg.C1, cfg.C1 + cfg.C2):
            if c % cfg.groups:
                raise ValueError("channel counts must be divisible by groups")
        for c in (cfg.C, cfg.C1):
            if c % cfg.head_dim:
                raise ValueError("transformer widths must be multiples of head_dim")
        if cfg.H % 4 or cfg.W % 4:
            raise ValueError("H and W must be multiples of 4")

    # ---- blocks -----------------------------------------------------------------------------------------------
    def _gn(self, x, g, b):
        return group_norm(x, self.w[g], self.w[b], self.cfg.groups, self.cfg.gn_eps)

    def _ln(self, z, p):
        return layer_norm(z, self.cfg.ln_eps) * self.w[p + "_g"] + self.w[p + "_b"]

    def _attn(self, q_in, kv_in, p):
        w = self.w
        heads = q_in.shape[-1] // self.cfg.head_dim
        o = attention_core(q_in @ w[p + ".wq"].T, kv_in @ w[p + ".wk"].T, kv_in @ w[p + ".wv"].T, heads)
        return o @ w[p + ".wo"].T + w[p + ".bo"]

    def _ff(self, h, p):
        w = self.w
        u = h @ w[p + ".ff1.w"].T + w[p + ".ff1.b"]
        half = u.shape[-1] // 2
        return (u[..., :half] * gelu_tanh(u[..., half:])) @ w[p + ".ff2.w"].T + w[p + ".ff2.b"]

    def rb(self, x, temb, p):
        """x [N, Cin, H, W]; temb [B, temb_dim] (frame n belongs to batch element n // F)."""
        w = self.w
        N = x.shape[0]
        t = silu(temb) @ w[p + ".temb.w"].T + w[p + ".temb.b"]          # [B, Cout]
        t = np.repeat(t, N // temb.shape[0], axis=0)                     # per frame
        h = conv3x3(silu(self._gn(x, p + ".gn1_g", p + ".gn1_b")), w[p + ".conv1.w"], w[p + ".conv1.b"]) + t[:, :, None, None]
        y = conv3x3(silu(self._gn(h, p + ".gn2_g", p + ".gn2_b")), w[p + ".conv2.w"], w[p + ".conv2.b"])
        if p + ".short.w" in w:
            sc = np.einsum("oc,nchw->nohw", w[p + ".short.w"], x) + w[p + ".short.b"][None, :, None, None]
        else:
            sc = x
        return sc + y

    def st(self, x, ctx, p):
        """Spatial transformer block; x [N, C, H, W], ctx [B, L, ctx_dim]."""
        w = self.w
        N, C, H, W = x.shape
        g = self._gn(x, p + ".gn_g", p + ".gn_b").reshape(N, C, H * W).transpose(0, 2, 1)   # [N, T, C]
        z = g @ w[p + ".pin.w"].T + w[p + ".pin.b"]
        cx = np.repeat(ctx, N // ctx.shape[0], axis=0)                                        # [N, L, ctx_dim]
        z = z + self._attn(self._ln(z, p + ".ln1"), self._ln(z, p + ".ln1"), p + ".attn1")
        z = z + self._attn(self._ln(z, p + ".ln2"), cx, p + ".attn2")
        z = z + self._ff(self._ln(z, p + ".ln3"), p)
        y = z @ w[p + ".pout.w"].T + w[p + ".pout.b"]
        return x + y.transpose(0, 2, 1).reshape(N, C, H, W)

    def tt(self, x, p):
        """Temporal transformer block; x [N = B*F, C, H, W]."""
        w, c = self.w, self.cfg
        N, C, H, W = x.shape
        B, F = c.B, N // c.B
        g = self._gn(x, p + ".gn_g", p + ".gn_b").reshape(B, F, C, H * W).transpose(0, 3, 1, 2)  # [B, P, F, C]
        z = g @ w[p + ".pin.w"].T + w[p + ".pin.b"]
        a = self._ln(z, p + ".ln1") + positional_encoding(F, C, self.dtype)
        z = z + self._attn(a, a, p + ".attn1")
        z = z + self._ff(self._ln(z, p + ".ln3"), p)
        y = z @ w[p + ".pout.w"].T + w[p + ".pout.b"]
        return x + y.transpose(0, 2, 3, 1).reshape(N, C, H, W)

    def upc(self, x, p):
        return conv3x3(up2(x), self.w[p + ".w"], self.w[p + ".b"])

    # ---- the stage --------------------------------------------------------------------------------------------
    def shallow_down(self, x, temb, ctx):
        h = conv3x3(x, self.w["conv_in.w"], self.w["conv_in.b"])
        return self.tt(self.st(self.rb(h, temb, "d0.rb"), ctx, "d0.st"), "d0.tt")

    def deep_branch(self, s, temb, ctx):
        w = self.w
        d = conv3x3(s, w["d0.down.w"], w["d0.down.b"], stride=2)
        d = self.tt(self.st(self.rb(d, temb, "d1.rb"), ctx, "d1.st"), "d1.tt")
        e = conv3x3(d, w["d1.down.w"], w["d1.down.b"], stride=2)
        e = self.rb(self.rb(e, temb, "mid.rb0"), temb, "mid.rb1")
        e = self.upc(e, "u2.up")
        d = self.rb(np.concatenate([d, e], axis=1), temb, "u1.rb")
        d = self.tt(self.st(d, ctx, "u1.st"), "u1.tt")
        return self.upc(d, "u1.up")

    def shallow_up(self, s, deep, temb, ctx):
        u = self.rb(np.concatenate([s, deep], axis=1), temb, "u0.rb")
        u = self.tt(self.st(u, ctx, "u0.st"), "u0.tt")
        return conv3x3(silu(self._gn(u, "out.gn_g", "out.gn_b")), self.w["out.w"], self.w["out.b"])

    def _in(self, x, temb, ctx):
        c = self.cfg
        x = np.asarray(x, dtype=self.dtype)
        assert x.shape == (c.B, c.F, c.C_lat, c.H, c.W), x.shape
        temb, ctx = np.asarray(temb, dtype=self.dtype), np.asarray(ctx, dtype=self.dtype)
        assert temb.shape == (c.B, c.temb_dim) and ctx.shape == (c.B, c.ctx_len, c.ctx_dim)
        return x.reshape(c.B * c.F, c.C_lat, c.H, c.W), temb, ctx

    def full_step(self, x, temb, ctx, dev_slot: int = 0):
        c = self.cfg
        x, temb, ctx = self._in(x, temb, ctx)
        s = self.shallow_down(x, temb, ctx)
        deep = self.deep_branch(s, temb, ctx)
        self.dev[dev_slot] = deep
        return self.shallow_up(s, deep, temb, ctx).reshape(c.B, c.F, c.C_lat, c.H, c.W)

    def cached_step(self, x, temb, ctx, dev_slot: int = 0):
        c = self.cfg
        if self.dev[dev_slot] is None:
            raise RuntimeError("cached step on an empty device slot")
        x, temb, ctx = self._in(x, temb, ctx)
        s = self.shallow_down(x, temb, ctx)
        return self.shallow_up(s, self.dev[dev_slot], temb, ctx).reshape(c.B, c.F, c.C_lat, c.H, c.W)

    def cache_write(self, dev_slot: int, deep) -> None:
        c = self.cfg
        deep = np.asarray(deep, dtype=self.dtype)
        assert deep.shape == (c.B * c.F, c.C1, c.H, c.W)
        self.dev[dev_slot] = deep.copy()

    def swap_out(self, dev_slot: int, host_slot: int) -> None:
        if self.dev[dev_slot] is None:
            raise RuntimeError("swap-out of an empty device slot")
        self.host[host_slot] = self.dev[dev_slot].copy()

    def swap_in(self, host_slot: int, dev_slot: int) -> None:
        if self.host[host_slot] is None:
            raise RuntimeError("swap-in from an empty host slot")
        self.dev[dev_slot] = self.host[host_slot].copy()
