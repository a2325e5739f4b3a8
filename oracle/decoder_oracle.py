"""CPU oracle for sliced decoding: a convolutional latent decoder applied to a video frame by frame.

TEST INFRASTRUCTURE ONLY. Only the test-suite and the benchmark's CPU-baseline leg may import it; the
product path never does, and nothing here imports the product.

What is computed ("Feature chunk and Sliced Decoding" section): at the decoding stage the batch and
frame axes are merged, F in R^{(B x T) x C x H x W}, and the decoder would process all frames at once;
sliced decoding treats the video as a sequence of pictures, decodes the latent frame by frame (here:
`slice_frames` frames per pass, 1 = frame by frame) and merges the decoded images back into the video.
Every operator of the decoder works on one frame at a time (convolutions, per-frame GroupNorm, attention
over the positions of one frame, upsampling), so slicing is exact; ``decode`` really loops over slices.

The paper uses the pretrained decoder of its models and does not describe it. This stand-in has the
usual shape of such a decoder, with synthetic weights:

    conv_in  3x3, C_lat -> C_0
    mid      ResBlock(C_0), spatial self-attention block(C_0), ResBlock(C_0)
    level l = 0 .. L-1:  ResBlock(C_l), nearest 2x upsampling, conv3x3 C_l -> C_{l+1}
    out      GroupNorm -> SiLU -> conv3x3 C_L -> C_img

with ResBlock(h) = h + conv3x3(SiLU(GroupNorm(h))) and the attention block h + Attn(GroupNorm(h)) (bias-free
q/k/v projections, `heads` heads, scale 1/sqrt(d), output projection with bias), all taken from the operator
definitions of ``lightcache_oracle`` (float64 by default; no blocking or fusion of its own).

Pins: tests/test_oracle_decoder.py (scalar brute force on a tiny decoder, an independent torch float64
build, sliced == unsliced, closed forms). The paper prints no decoded values.
"""
from __future__ import annotations

from typing import Dict, List

import numpy as np

from .lightcache_oracle import _chunks, attention, conv3x3, group_norm, silu, up2

Weights = Dict[str, np.ndarray]


def required_weights(cfg) -> List[str]:
    names = ["conv_in.w", "conv_in.b"]
    for blk in ("mid.res0", "mid.res1"):
        names += [f"{blk}.{k}" for k in ("gn_g", "gn_b", "w", "b")]
    names += [f"mid.attn.{k}" for k in ("gn_g", "gn_b", "wq", "wk", "wv", "wo", "bo")]
    for l in range(len(cfg.widths) - 1):
        names += [f"up{l}.res.{k}" for k in ("gn_g", "gn_b", "w", "b")]
        names += [f"up{l}.conv.w", f"up{l}.conv.b"]
    names += ["out.gn_g", "out.gn_b", "out.w", "out.b"]
    return names


class DecoderOracle:
    """``cfg``: any object with N (frames, batch and frame axes merged), H, W (latent size), C_lat, C_img,
    widths (C_0 .. C_L), groups, heads, head_dim (heads * head_dim == C_0), gn_eps. ``weights``: name -> array in
    PyTorch order, names as in ``required_weights``."""

    def __init__(self, cfg, weights: Weights, dtype=np.float64):
        self.cfg = cfg
        self.dtype = np.dtype(dtype)
        self.w = {k: np.asarray(v, dtype=self.dtype) for k, v in weights.items()}
        if cfg.heads * cfg.head_dim != cfg.widths[0]:
            raise ValueError("heads * head_dim must equal the mid width")
        if any(c % cfg.groups for c in cfg.widths):
            raise ValueError("every width must be divisible by the number of groups")

    def _gn(self, x, prefix):
        return group_norm(x, self.w[prefix + ".gn_g"], self.w[prefix + ".gn_b"], self.cfg.groups, self.cfg.gn_eps)

    def res_block(self, h, prefix):
        return h + conv3x3(silu(self._gn(h, prefix)), self.w[prefix + ".w"], self.w[prefix + ".b"])

    def attn_block(self, h, prefix):
        """Per frame: tokens = the positions of the frame; h + Attn(GroupNorm(h))."""
        n, C, H, W = h.shape
        g = self._gn(h, prefix)
        w = self.w
        out = h.copy()
        for i in range(n):
            X = g[i].reshape(C, H * W).T
            Y = attention(X, X, w[prefix + ".wq"], w[prefix + ".wk"], w[prefix + ".wv"], w[prefix + ".wo"],
                          w[prefix + ".bo"], self.cfg.heads)
            out[i] += Y.T.reshape(C, H, W)
        return out

    def decode_frames(self, z):
        """The decoder on a stack of frames z [n, C_lat, H, W] -> images [n, C_img, H * 2^L, W * 2^L]."""
        w = self.w
        h = conv3x3(z, w["conv_in.w"], w["conv_in.b"])
        h = self.res_block(h, "mid.res0")
        h = self.attn_block(h, "mid.attn")
        h = self.res_block(h, "mid.res1")
        for l in range(len(self.cfg.widths) - 1):
            h = self.res_block(h, f"up{l}.res")
            h = conv3x3(up2(h), w[f"up{l}.conv.w"], w[f"up{l}.conv.b"])
        return conv3x3(silu(self._gn(h, "out")), w["out.w"], w["out.b"])

    def decode(self, z, slice_frames: int = 1):
        """Sliced decoding: the frames of z [N, C_lat, H, W] in passes of `slice_frames` (1 = frame by frame,
        0 or >= N = all at once), the decoded images merged back in frame order."""
        c = self.cfg
        z = np.asarray(z, dtype=self.dtype)
        assert z.shape == (c.N, c.C_lat, c.H, c.W), z.shape
        s = 2 ** (len(c.widths) - 1)
        out = np.empty((c.N, c.C_img, c.H * s, c.W * s), dtype=self.dtype)
        for n0, n1 in _chunks(c.N, slice_frames):
            out[n0:n1] = self.decode_frames(z[n0:n1])
        return out
