"""Seeded synthetic inputs for the cached-step stage of a DeepCache-style video UNet.

This module only *describes shapes and draws random numbers*. It holds none of the
method's arithmetic (no convolution, normalisation, attention, caching): both the CPU
oracle's tests and the HIP path's tests import it so that the two sides receive
bit-identical arrays.

Shapes follow the 5-D feature-map convention of the paper's "Feature chunk" section,
{batch, frames, channels, height, width}, with batch = 2 standing for the conditional
and unconditional halves of classifier-free guidance.

Recipe
------
* One ``numpy.random.default_rng(seed)`` stream per tensor family (weights / latents /
  injected deep feature), drawn in the fixed order of :func:`weight_manifest`.
* Convolution and projection weights and all biases ~ N(0, 0.02).
* GroupNorm scale = 1 + N(0, 0.02), GroupNorm shift ~ N(0, 0.02) (a literal N(0, 0.02)
  scale would shrink every activation fifty-fold and make absolute tolerances vacuous).
* Latents and injected deep features ~ N(0, 1).
* Everything is drawn as float32. For bf16 workloads the arrays are then rounded once to
  the nearest bf16-representable value (ties to even) and still *stored* as float32, so
  that a float64 consumer and a bf16 consumer see exactly the same numbers.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, List, Tuple

import numpy as np


@dataclass(frozen=True)
class StageConfig:
    """Shape of one shallow UNet stage plus its chunking / schedule parameters."""

    name: str
    B: int
    F: int
    H: int
    W: int
    C_lat: int
    C: int
    C_deep: int
    groups: int
    n_res: int
    heads: int
    head_dim: int
    dtype: str  # "f32" or "bf16"
    frame_chunk: int = 0  # 0 = unchunked
    token_chunk: int = 0  # 0 = derived from frame_chunk / unchunked
    gn_eps: float = 1e-5

    @property
    def N(self) -> int:  # frames of the flattened (batch, frame) axis
        return self.B * self.F

    @property
    def T(self) -> int:  # tokens (spatial positions) per frame
        return self.H * self.W

    def with_(self, **kw) -> "StageConfig":
        return replace(self, **kw)

    def cached_step_flops(self) -> float:
        """Algorithmic FLOPs of one cached step (unpadded head_dim, no recompute)."""
        N, T, P = self.N, self.T, self.N * self.T
        C, Cd, Cl = self.C, self.C_deep, self.C_lat

        def conv(ci, co):
            return 2.0 * 9 * ci * co * P

        f = conv(Cl, C) + self.n_res * conv(C, C)
        proj = 8.0 * C * C * P
        f += proj + 4.0 * T * T * self.head_dim * self.heads * N
        f += proj + 4.0 * self.F * self.F * self.head_dim * self.heads * self.B * T
        f += conv(C + Cd, C) + conv(C, Cl)
        return f


# The workloads: a tiny fp32 stage, an AnimateDiff-like stage (512x512 video -> 64x64
# latents, 16 frames), an SVD-XT-like stage (576x1024 -> 72x128 latents, 25 frames) and a
# stress instance. They are shape-faithful stand-ins for the pretrained models the paper
# measured, which are not available here.
CONFIGS: Dict[str, StageConfig] = {
    "tiny": StageConfig("tiny", B=1, F=8, H=32, W=32, C_lat=4, C=64, C_deep=128, groups=32,
                        n_res=1, heads=1, head_dim=64, dtype="f32", frame_chunk=2),
    "animatediff": StageConfig("animatediff", B=2, F=16, H=64, W=64, C_lat=4, C=320, C_deep=640,
                               groups=32, n_res=2, heads=8, head_dim=40, dtype="bf16",
                               frame_chunk=4),
    "svdxt": StageConfig("svdxt", B=2, F=25, H=72, W=128, C_lat=4, C=320, C_deep=640,
                         groups=32, n_res=2, heads=5, head_dim=64, dtype="bf16",
                         frame_chunk=5, token_chunk=2304),
    "stress": StageConfig("stress", B=2, F=32, H=96, W=96, C_lat=4, C=320, C_deep=640,
                          groups=32, n_res=2, heads=8, head_dim=40, dtype="bf16",
                          frame_chunk=8),
}


def weight_manifest(cfg: StageConfig) -> List[Tuple[str, Tuple[int, ...], str]]:
    """(name, shape, kind) in generation order. kind: 'w' weight/bias, 'g' GN scale, 'b' GN shift."""
    C, Cd, Cl = cfg.C, cfg.C_deep, cfg.C_lat
    m: List[Tuple[str, Tuple[int, ...], str]] = []
    m += [("conv_in.w", (C, Cl, 3, 3), "w"), ("conv_in.b", (C,), "w")]
    for i in range(cfg.n_res):
        m += [(f"res{i}.gn_g", (C,), "g"), (f"res{i}.gn_b", (C,), "b"),
              (f"res{i}.w", (C, C, 3, 3), "w"), (f"res{i}.b", (C,), "w")]
    for blk in ("sattn", "tattn"):
        m += [(f"{blk}.gn_g", (C,), "g"), (f"{blk}.gn_b", (C,), "b"),
              (f"{blk}.wq", (C, C), "w"), (f"{blk}.wk", (C, C), "w"),
              (f"{blk}.wv", (C, C), "w"), (f"{blk}.wo", (C, C), "w"),
              (f"{blk}.bo", (C,), "w")]
    m += [("down.w", (Cd, C, 3, 3), "w"), ("down.b", (Cd,), "w")]
    m += [("dres.gn_g", (Cd,), "g"), ("dres.gn_b", (Cd,), "b"),
          ("dres.w", (Cd, Cd, 3, 3), "w"), ("dres.b", (Cd,), "w")]
    m += [("up.gn_g", (C + Cd,), "g"), ("up.gn_b", (C + Cd,), "b"),
          ("up.w", (C, C + Cd, 3, 3), "w"), ("up.b", (C,), "w")]
    m += [("out.gn_g", (C,), "g"), ("out.gn_b", (C,), "b"),
          ("out.w", (Cl, C, 3, 3), "w"), ("out.b", (Cl,), "w")]
    return m


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16-representable float32 (ties to even)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    u = (u + 0x7FFF + lsb) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(a.shape)


def _finish(a: np.ndarray, cfg: StageConfig) -> np.ndarray:
    a = a.astype(np.float32)
    return round_to_bf16(a) if cfg.dtype == "bf16" else a


def make_weights(cfg: StageConfig, seed: int = 0, sharp: float = 1.0) -> Dict[str, np.ndarray]:
    """Draw every weight of the stage. ``sharp`` multiplies the query/key projections so that
    attention logits get a standard deviation well above 1 (a peaked softmax)."""
    rng = np.random.default_rng(seed)
    out: Dict[str, np.ndarray] = {}
    for name, shape, kind in weight_manifest(cfg):
        a = rng.standard_normal(shape, dtype=np.float32) * np.float32(0.02)
        if kind == "g":
            a = a + np.float32(1.0)
        if sharp != 1.0 and (name.endswith(".wq") or name.endswith(".wk")):
            a = a * np.float32(sharp)
        out[name] = _finish(a, cfg)
    return out


def make_latents(cfg: StageConfig, seed: int = 1) -> np.ndarray:
    """Noisy latents x, shape [B, F, C_lat, H, W], ~N(0,1)."""
    rng = np.random.default_rng(seed)
    return _finish(rng.standard_normal((cfg.B, cfg.F, cfg.C_lat, cfg.H, cfg.W), dtype=np.float32), cfg)


def make_deep(cfg: StageConfig, seed: int = 2) -> np.ndarray:
    """A stand-in cached deep feature, shape [B*F, C_deep, H/2, W/2], ~N(0,1)."""
    rng = np.random.default_rng(seed)
    return _finish(rng.standard_normal((cfg.N, cfg.C_deep, cfg.H // 2, cfg.W // 2), dtype=np.float32), cfg)


def make_activation(shape, seed: int, dtype: str = "f32", scale: float = 1.0) -> np.ndarray:
    """A generic ~N(0, scale^2) activation tensor for single-operator tests."""
    rng = np.random.default_rng(seed)
    a = rng.standard_normal(shape, dtype=np.float32) * np.float32(scale)
    return round_to_bf16(a) if dtype == "bf16" else a


# --------------------------------------------------------------------------------------
# Sliced decoding: a convolutional latent decoder (stand-in for the pretrained one)
# --------------------------------------------------------------------------------------
@dataclass(frozen=True)
class DecoderConfig:
    """Shape of the decoder of the sliced-decoding stage. N = frames (batch and frame axes merged), H x W the
    latent size; widths = (C_0, ..., C_L): mid width and the width after each of the L 2x upsampling levels."""

    name: str
    N: int
    H: int
    W: int
    C_lat: int
    C_img: int
    widths: Tuple[int, ...]
    groups: int
    heads: int
    head_dim: int
    dtype: str
    slice_frames: int = 1
    gn_eps: float = 1e-5

    @property
    def levels(self) -> int:
        return len(self.widths) - 1

    def with_(self, **kw) -> "DecoderConfig":
        return replace(self, **kw)

    def decode_flops(self) -> float:
        """Algorithmic FLOPs of decoding all N frames."""
        P = self.H * self.W
        C0 = self.widths[0]
        f = 2.0 * 9 * self.C_lat * C0 * P + 2 * 2.0 * 9 * C0 * C0 * P       # conv_in, two mid residual blocks
        f += 8.0 * C0 * C0 * P + 4.0 * P * P * C0                            # attention block
        for l in range(self.levels):
            f += 2.0 * 9 * self.widths[l] ** 2 * P                            # residual block of the level
            P *= 4
            f += 2.0 * 9 * self.widths[l] * self.widths[l + 1] * P            # convolution after the upsampling
        f += 2.0 * 9 * self.widths[-1] * self.C_img * P
        return f * self.N


DECODERS: Dict[str, DecoderConfig] = {
    # tiny fp32 decoder on the latents of the tiny stage
    "tiny": DecoderConfig("tiny", N=8, H=32, W=32, C_lat=4, C_img=3, widths=(64, 64, 64), groups=32, heads=1,
                          head_dim=64, dtype="f32"),
    # 512 x 512 video frames from 64 x 64 latents, 16 frames (the guidance halves are already combined)
    "animatediff": DecoderConfig("animatediff", N=16, H=64, W=64, C_lat=4, C_img=3, widths=(320, 320, 192, 128),
                                 groups=32, heads=8, head_dim=40, dtype="bf16"),
}


def decoder_weight_manifest(cfg: DecoderConfig) -> List[Tuple[str, Tuple[int, ...], str]]:
    C0 = cfg.widths[0]
    m: List[Tuple[str, Tuple[int, ...], str]] = [("conv_in.w", (C0, cfg.C_lat, 3, 3), "w"), ("conv_in.b", (C0,), "w")]

    def res(prefix, C):
        return [(f"{prefix}.gn_g", (C,), "g"), (f"{prefix}.gn_b", (C,), "b"), (f"{prefix}.w", (C, C, 3, 3), "w"),
                (f"{prefix}.b", (C,), "w")]
    m += res("mid.res0", C0)
    m += [("mid.attn.gn_g", (C0,), "g"), ("mid.attn.gn_b", (C0,), "b")]
    m += [(f"mid.attn.{k}", (C0, C0), "w") for k in ("wq", "wk", "wv", "wo")] + [("mid.attn.bo", (C0,), "w")]
    m += res("mid.res1", C0)
    for l in range(cfg.levels):
        m += res(f"up{l}.res", cfg.widths[l])
        m += [(f"up{l}.conv.w", (cfg.widths[l + 1], cfg.widths[l], 3, 3), "w"), (f"up{l}.conv.b", (cfg.widths[l + 1],), "w")]
    CL = cfg.widths[-1]
    m += [("out.gn_g", (CL,), "g"), ("out.gn_b", (CL,), "b"), ("out.w", (cfg.C_img, CL, 3, 3), "w"), ("out.b", (cfg.C_img,), "w")]
    return m


def make_decoder_weights(cfg: DecoderConfig, seed: int = 0, sharp: float = 1.0) -> Dict[str, np.ndarray]:
    """Same recipe as make_weights: weights and biases ~N(0, 0.02), GroupNorm scale 1 + N(0, 0.02), shift N(0, 0.02)."""
    rng = np.random.default_rng(seed)
    out: Dict[str, np.ndarray] = {}
    for name, shape, kind in decoder_weight_manifest(cfg):
        a = rng.standard_normal(shape, dtype=np.float32) * np.float32(0.02)
        if kind == "g":
            a = a + np.float32(1.0)
        if sharp != 1.0 and (name.endswith(".wq") or name.endswith(".wk")):
            a = a * np.float32(sharp)
        out[name] = round_to_bf16(a) if cfg.dtype == "bf16" else a
    return out


def make_decoder_latents(cfg: DecoderConfig, seed: int = 1) -> np.ndarray:
    """Denoised latents z, shape [N, C_lat, H, W], ~N(0,1)."""
    rng = np.random.default_rng(seed)
    a = rng.standard_normal((cfg.N, cfg.C_lat, cfg.H, cfg.W), dtype=np.float32)
    return round_to_bf16(a) if cfg.dtype == "bf16" else a


# --------------------------------------------------------------------------------------
# Diffusion-transformer variant: a stack of adaLN-modulated blocks with a cached block range
# --------------------------------------------------------------------------------------
@dataclass(frozen=True)
class DitConfig:
    """B batch elements (2 with classifier-free guidance) of T tokens (all patches of all latent frames: the
    attention is over the whole video) and width D; L blocks of which [cache_a, cache_b) are the cached deep part."""

    name: str
    B: int
    T: int
    D: int
    heads: int
    head_dim: int
    L: int
    cache_a: int
    cache_b: int
    dtype: str
    mlp_ratio: int = 4
    token_chunk: int = 0
    ln_eps: float = 1e-6

    def with_(self, **kw) -> "DitConfig":
        return replace(self, **kw)

    def block_flops(self) -> float:
        """Algorithmic FLOPs of one block over all B * T tokens."""
        P = self.B * self.T
        return 8.0 * self.D * self.D * P + 4.0 * self.T * self.T * self.D * self.B + 4.0 * self.mlp_ratio * self.D * self.D * P

    def cached_step_flops(self) -> float:
        return (self.L - (self.cache_b - self.cache_a)) * self.block_flops()

    def full_step_flops(self) -> float:
        return self.L * self.block_flops()


DITS: Dict[str, DitConfig] = {
    "tiny": DitConfig("tiny", B=1, T=256, D=128, heads=2, head_dim=64, L=4, cache_a=1, cache_b=3, dtype="f32", token_chunk=64),
    # a video DiT in the size class of the paper's DiT rows: 4 latent frames of 32 x 32 patches attended jointly
    "video_dit": DitConfig("video_dit", B=2, T=4096, D=1024, heads=16, head_dim=64, L=12, cache_a=2, cache_b=10,
                           dtype="bf16", token_chunk=1024),
}


def dit_weight_manifest(cfg: DitConfig) -> List[Tuple[str, Tuple[int, ...], str]]:
    D, H = cfg.D, cfg.mlp_ratio * cfg.D
    m: List[Tuple[str, Tuple[int, ...], str]] = []
    for i in range(cfg.L):
        m += [(f"blk{i}.wqkv", (3 * D, D), "w"), (f"blk{i}.bqkv", (3 * D,), "w"), (f"blk{i}.wo", (D, D), "w"),
              (f"blk{i}.bo", (D,), "w"), (f"blk{i}.w1", (H, D), "w"), (f"blk{i}.b1", (H,), "w"),
              (f"blk{i}.w2", (D, H), "w"), (f"blk{i}.b2", (D,), "w")]
    return m


def make_dit_weights(cfg: DitConfig, seed: int = 0, sharp: float = 1.0) -> Dict[str, np.ndarray]:
    """All weights and biases ~N(0, 0.02); `sharp` multiplies the q and k rows of wqkv (peaked softmax)."""
    rng = np.random.default_rng(seed)
    out: Dict[str, np.ndarray] = {}
    for name, shape, _ in dit_weight_manifest(cfg):
        a = rng.standard_normal(shape, dtype=np.float32) * np.float32(0.02)
        if sharp != 1.0 and name.endswith(".wqkv"):
            a[:2 * cfg.D] *= np.float32(sharp)
        out[name] = round_to_bf16(a) if cfg.dtype == "bf16" else a
    return out


def make_dit_hidden(cfg: DitConfig, seed: int = 1) -> np.ndarray:
    """Hidden states entering the block stack, [B, T, D] float32, ~N(0,1)."""
    return np.random.default_rng(seed).standard_normal((cfg.B, cfg.T, cfg.D), dtype=np.float32)


def make_dit_modulation(cfg: DitConfig, seed: int = 2) -> np.ndarray:
    """The adaLN vectors of every block, [L, B, 6, D] float32 in the order shift_msa, scale_msa, gate_msa,
    shift_mlp, scale_mlp, gate_mlp: shifts and scales ~N(0, 0.1), gates 1 + N(0, 0.1)."""
    a = np.random.default_rng(seed).standard_normal((cfg.L, cfg.B, 6, cfg.D), dtype=np.float32) * np.float32(0.1)
    a[:, :, 2] += np.float32(1.0)
    a[:, :, 5] += np.float32(1.0)
    return a


# --------------------------------------------------------------------------------------
# U-Net stage with the block internals of the video U-Nets the paper ran (time-embedding residual blocks,
# transformer blocks with cross-attention and a GEGLU feed-forward, frame positional encoding) and a
# three-level deep branch
# --------------------------------------------------------------------------------------
@dataclass(frozen=True)
class UnetConfig:
    """B batch elements of F frames of H x W latents; widths C (H x W), C1 (H/2 x W/2), C2 (H/4 x W/4); heads of
    head_dim channels; ctx_len conditioning tokens of ctx_dim channels; a time embedding of temb_dim channels."""

    name: str
    B: int
    F: int
    H: int
    W: int
    C_lat: int
    C: int
    C1: int
    C2: int
    groups: int
    head_dim: int
    ctx_len: int
    ctx_dim: int
    temb_dim: int
    dtype: str
    ff_mult: int = 4
    gn_eps: float = 1e-5
    ln_eps: float = 1e-5

    @property
    def N(self) -> int:
        return self.B * self.F

    def with_(self, **kw) -> "UnetConfig":
        return replace(self, **kw)

    # ---- algorithmic FLOPs (2 per multiply-add; norms, activations and softmax not counted) ----
    def _rb(self, cin, cout, P):
        f = 2.0 * 9 * cin * cout * P + 2.0 * 9 * cout * cout * P
        return f + (2.0 * cin * cout * P if cin != cout else 0.0)

    def _st(self, C, P):
        lin = 2.0 * C * C * P * (2 + 4 + 2 + 3 * self.ff_mult)      # pin, pout; q,k,v,o; cross q,o; GEGLU feed-forward
        return lin + 4.0 * P * P * C + 4.0 * P * self.ctx_len * C

    def _tt(self, C, P):
        return 2.0 * C * C * P * (2 + 4 + 3 * self.ff_mult) + 4.0 * P * self.F * C

    def shallow_flops(self) -> float:
        P = self.H * self.W
        per = 2.0 * 9 * self.C_lat * self.C * P * 2 + self._rb(self.C, self.C, P) + self._rb(self.C + self.C1, self.C, P)
        per += 2 * (self._st(self.C, P) + self._tt(self.C, P))
        return per * self.N

    def deep_flops(self) -> float:
        P, P1, P2 = self.H * self.W, self.H * self.W // 4, self.H * self.W // 16
        C, C1, C2 = self.C, self.C1, self.C2
        per = 2.0 * 9 * C * C * P1 + self._rb(C, C1, P1) + self._st(C1, P1) + self._tt(C1, P1)
        per += 2.0 * 9 * C1 * C1 * P2 + self._rb(C1, C2, P2) + self._rb(C2, C2, P2) + 2.0 * 9 * C2 * C2 * P1
        per += self._rb(C1 + C2, C1, P1) + self._st(C1, P1) + self._tt(C1, P1) + 2.0 * 9 * C1 * C1 * P
        return per * self.N

    def cached_step_flops(self) -> float:
        return self.shallow_flops()

    def full_step_flops(self) -> float:
        return self.shallow_flops() + self.deep_flops()


UNETS: Dict[str, UnetConfig] = {
    "tiny": UnetConfig("tiny", B=1, F=4, H=32, W=32, C_lat=4, C=64, C1=128, C2=128, groups=32, head_dim=32, ctx_len=7,
                       ctx_dim=64, temb_dim=64, dtype="f32"),
    # full widths at a quarter of the positions: the parity case of the bf16 path
    "mid": UnetConfig("mid", B=2, F=8, H=32, W=32, C_lat=4, C=320, C1=640, C2=1280, groups=32, head_dim=40, ctx_len=77,
                      ctx_dim=768, temb_dim=1280, dtype="bf16"),
    # 512 x 512 video, 16 frames, guidance pair: widths, text tokens and time embedding of the SD-1.5 family
    "sd15_video": UnetConfig("sd15_video", B=2, F=16, H=64, W=64, C_lat=4, C=320, C1=640, C2=1280, groups=32, head_dim=40,
                             ctx_len=77, ctx_dim=768, temb_dim=1280, dtype="bf16"),
}


def _unet_rb(p, cin, cout, td):
    m = [(f"{p}.gn1_g", (cin,), "g"), (f"{p}.gn1_b", (cin,), "b"), (f"{p}.conv1.w", (cout, cin, 3, 3), "w"), (f"{p}.conv1.b", (cout,), "w"),
         (f"{p}.temb.w", (cout, td), "w"), (f"{p}.temb.b", (cout,), "w"), (f"{p}.gn2_g", (cout,), "g"), (f"{p}.gn2_b", (cout,), "b"),
         (f"{p}.conv2.w", (cout, cout, 3, 3), "w"), (f"{p}.conv2.b", (cout,), "w")]
    if cin != cout:
        m += [(f"{p}.short.w", (cout, cin), "w"), (f"{p}.short.b", (cout,), "w")]
    return m


def _unet_tf(p, C, ctx_dim, fm):
    """A transformer block; ctx_dim == 0: no cross-attention (the temporal block)."""
    m = [(f"{p}.gn_g", (C,), "g"), (f"{p}.gn_b", (C,), "b"), (f"{p}.pin.w", (C, C), "w"), (f"{p}.pin.b", (C,), "w"),
         (f"{p}.ln1_g", (C,), "g"), (f"{p}.ln1_b", (C,), "b")]
    m += [(f"{p}.attn1.{k}", (C, C), "w") for k in ("wq", "wk", "wv", "wo")] + [(f"{p}.attn1.bo", (C,), "w")]
    if ctx_dim:
        m += [(f"{p}.ln2_g", (C,), "g"), (f"{p}.ln2_b", (C,), "b"), (f"{p}.attn2.wq", (C, C), "w"), (f"{p}.attn2.wk", (C, ctx_dim), "w"),
              (f"{p}.attn2.wv", (C, ctx_dim), "w"), (f"{p}.attn2.wo", (C, C), "w"), (f"{p}.attn2.bo", (C,), "w")]
    m += [(f"{p}.ln3_g", (C,), "g"), (f"{p}.ln3_b", (C,), "b"), (f"{p}.ff1.w", (2 * fm * C, C), "w"), (f"{p}.ff1.b", (2 * fm * C,), "w"),
          (f"{p}.ff2.w", (C, fm * C), "w"), (f"{p}.ff2.b", (C,), "w"), (f"{p}.pout.w", (C, C), "w"), (f"{p}.pout.b", (C,), "w")]
    return m


UNET_RB = ("d0.rb", "d1.rb", "mid.rb0", "mid.rb1", "u1.rb", "u0.rb")   # residual blocks, in the order of the C interface
UNET_ST = ("d0.st", "d1.st", "u1.st", "u0.st")                          # spatial transformer blocks
UNET_TT = ("d0.tt", "d1.tt", "u1.tt", "u0.tt")                          # temporal transformer blocks


def unet_weight_manifest(cfg: UnetConfig) -> List[Tuple[str, Tuple[int, ...], str]]:
    """(name, shape, kind) of every weight, in generation order; kind 'w' weight or bias, 'g' norm scale, 'b' norm shift."""
    C, C1, C2, Cl, td, cd, fm = cfg.C, cfg.C1, cfg.C2, cfg.C_lat, cfg.temb_dim, cfg.ctx_dim, cfg.ff_mult
    m: List[Tuple[str, Tuple[int, ...], str]] = [("conv_in.w", (C, Cl, 3, 3), "w"), ("conv_in.b", (C,), "w")]
    m += _unet_rb("d0.rb", C, C, td) + _unet_tf("d0.st", C, cd, fm) + _unet_tf("d0.tt", C, 0, fm)
    m += [("d0.down.w", (C, C, 3, 3), "w"), ("d0.down.b", (C,), "w")]
    m += _unet_rb("d1.rb", C, C1, td) + _unet_tf("d1.st", C1, cd, fm) + _unet_tf("d1.tt", C1, 0, fm)
    m += [("d1.down.w", (C1, C1, 3, 3), "w"), ("d1.down.b", (C1,), "w")]
    m += _unet_rb("mid.rb0", C1, C2, td) + _unet_rb("mid.rb1", C2, C2, td)
    m += [("u2.up.w", (C2, C2, 3, 3), "w"), ("u2.up.b", (C2,), "w")]
    m += _unet_rb("u1.rb", C1 + C2, C1, td) + _unet_tf("u1.st", C1, cd, fm) + _unet_tf("u1.tt", C1, 0, fm)
    m += [("u1.up.w", (C1, C1, 3, 3), "w"), ("u1.up.b", (C1,), "w")]
    m += _unet_rb("u0.rb", C + C1, C, td) + _unet_tf("u0.st", C, cd, fm) + _unet_tf("u0.tt", C, 0, fm)
    m += [("out.gn_g", (C,), "g"), ("out.gn_b", (C,), "b"), ("out.w", (Cl, C, 3, 3), "w"), ("out.b", (Cl,), "w")]
    return m


def make_unet_weights(cfg: UnetConfig, seed: int = 0, sharp: float = 1.0) -> Dict[str, np.ndarray]:
    """Weights and biases ~N(0, 0.02), norm scales 1 + N(0, 0.02), norm shifts N(0, 0.02); `sharp` multiplies the
    query and key projections (peaked softmax)."""
    rng = np.random.default_rng(seed)
    out: Dict[str, np.ndarray] = {}
    for name, shape, kind in unet_weight_manifest(cfg):
        a = rng.standard_normal(shape, dtype=np.float32) * np.float32(0.02)
        if kind == "g":
            a = a + np.float32(1.0)
        if sharp != 1.0 and (name.endswith(".wq") or name.endswith(".wk")):
            a = a * np.float32(sharp)
        out[name] = round_to_bf16(a) if cfg.dtype == "bf16" else a
    return out


def make_unet_inputs(cfg: UnetConfig, seed: int = 1):
    """(x [B, F, C_lat, H, W], temb [B, temb_dim], ctx [B, ctx_len, ctx_dim]), all ~N(0, 1), in the storage type's values."""
    rng = np.random.default_rng(seed)
    fin = (lambda a: round_to_bf16(a)) if cfg.dtype == "bf16" else (lambda a: a)
    x = fin(rng.standard_normal((cfg.B, cfg.F, cfg.C_lat, cfg.H, cfg.W), dtype=np.float32))
    temb = fin(rng.standard_normal((cfg.B, cfg.temb_dim), dtype=np.float32))
    ctx = fin(rng.standard_normal((cfg.B, cfg.ctx_len, cfg.ctx_dim), dtype=np.float32))
    return x, temb, ctx


def make_unet_deep(cfg: UnetConfig, seed: int = 2) -> np.ndarray:
    """A stand-in cached feature, [B*F, C1, H, W] float32, ~N(0, 1)."""
    return np.random.default_rng(seed).standard_normal((cfg.N, cfg.C1, cfg.H, cfg.W), dtype=np.float32)
