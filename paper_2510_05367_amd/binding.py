"""ctypes binding of liblightcache.so (the C ABI in include/lightcache.h).

Argument marshalling only: every function here has the name and argument order of the C entry
point it forwards to, and raises :class:`LcError` when the library returns a non-zero status.
:class:`Stage` is a small convenience holder that uses PyTorch for what it is here for, device
memory and streams, and calls the same entry points.

There is no fallback: if the shared library is missing, importing this module's functions
raises with the build command to run.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "liblightcache.so")

LC_OK, LC_ERR_ARG, LC_ERR_SHAPE, LC_ERR_STATE, LC_ERR_NOMEM, LC_ERR_HIP = range(6)
LC_F32, LC_BF16 = 0, 1
LC_MAX_RES = 4
KERNEL_FAMILIES = ["conv_in", "gn_stats", "gn_final", "gn_apply", "conv_res", "qkv", "sattn", "tattn",
                   "proj", "cat_apply", "conv_up", "conv_out", "deep"]
LC_K = {n: i for i, n in enumerate(KERNEL_FAMILIES)}
LC_L_RES0, LC_L_SATTN, LC_L_TATTN, LC_L_DRES = 0, 8, 9, 10
STATUS_NAMES = ["LC_OK", "LC_ERR_ARG", "LC_ERR_SHAPE", "LC_ERR_STATE", "LC_ERR_NOMEM", "LC_ERR_HIP"]


class LcError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{STATUS_NAMES[status] if 0 <= status < 6 else status}: {message}")
        self.status = status


class lc_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("B", "F", "H", "W", "C_lat", "C", "C_deep", "groups", "n_res",
                                         "heads", "head_dim", "dtype")] + \
               [("gn_eps", C.c_float), ("host_slots", C.c_int32), ("dev_slots", C.c_int32)]


class lc_gnconv_w(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("gn_g", "gn_b", "w", "b")]


class lc_attn_w(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("gn_g", "gn_b", "wq", "wk", "wv", "wo", "bo")]


class lc_weights(C.Structure):
    _fields_ = [("conv_in_w", C.c_void_p), ("conv_in_b", C.c_void_p), ("res", lc_gnconv_w * LC_MAX_RES),
                ("sattn", lc_attn_w), ("tattn", lc_attn_w), ("down_w", C.c_void_p), ("down_b", C.c_void_p),
                ("dres", lc_gnconv_w), ("up", lc_gnconv_w), ("out", lc_gnconv_w)]


class lc_stats(C.Structure):
    _fields_ = [("full_steps", C.c_int64), ("cached_steps", C.c_int64), ("swaps_out", C.c_int64),
                ("swaps_in", C.c_int64), ("bytes_out", C.c_int64), ("bytes_in", C.c_int64),
                ("ms_out", C.c_double), ("ms_in", C.c_double), ("timed_out", C.c_int64), ("timed_in", C.c_int64),
                ("workspace_bytes", C.c_size_t),
                ("weight_bytes", C.c_size_t), ("host_bank_bytes", C.c_size_t)]


class lc_profile(C.Structure):
    _fields_ = [("ms", C.c_double * len(KERNEL_FAMILIES)), ("launches", C.c_int64 * len(KERNEL_FAMILIES)),
                ("dropped", C.c_int64)]


LC_DEC_MAX_LEVELS = 3


class lc_decoder_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("N", "H", "W", "C_lat", "C_img", "levels")] + \
               [("widths", C.c_int32 * (LC_DEC_MAX_LEVELS + 1))] + \
               [(n, C.c_int32) for n in ("groups", "heads", "head_dim", "dtype")] + [("gn_eps", C.c_float)]


class lc_decoder_weights(C.Structure):
    _fields_ = [("conv_in_w", C.c_void_p), ("conv_in_b", C.c_void_p), ("mid_res", lc_gnconv_w * 2), ("mid_attn", lc_attn_w),
                ("up_res", lc_gnconv_w * LC_DEC_MAX_LEVELS), ("up_conv_w", C.c_void_p * LC_DEC_MAX_LEVELS),
                ("up_conv_b", C.c_void_p * LC_DEC_MAX_LEVELS), ("out", lc_gnconv_w)]


LC_DIT_MAX_BLOCKS = 64


class lc_dit_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("B", "T", "D", "heads", "head_dim", "L", "cache_a", "cache_b", "mlp_ratio", "dtype")] + \
               [("ln_eps", C.c_float), ("host_slots", C.c_int32), ("dev_slots", C.c_int32)]


class lc_dit_block_w(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("wqkv", "bqkv", "wo", "bo", "w1", "b1", "w2", "b2")]


class lc_dit_weights(C.Structure):
    _fields_ = [("blk", lc_dit_block_w * LC_DIT_MAX_BLOCKS)]


class lc_unet_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("B", "F", "H", "W", "C_lat", "C", "C1", "C2", "groups", "head_dim", "ctx_len", "ctx_dim",
                                         "temb_dim", "ff_mult", "dtype")] + \
               [("gn_eps", C.c_float), ("ln_eps", C.c_float), ("host_slots", C.c_int32), ("dev_slots", C.c_int32)]


class lc_unet_rb_w(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("gn1_g", "gn1_b", "conv1_w", "conv1_b", "temb_w", "temb_b", "gn2_g", "gn2_b", "conv2_w",
                                          "conv2_b", "short_w", "short_b")]


class lc_unet_attn_w(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("wq", "wk", "wv", "wo", "bo")]


class lc_unet_tf_w(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("gn_g", "gn_b", "pin_w", "pin_b", "ln1_g", "ln1_b")] + [("attn1", lc_unet_attn_w)] + \
               [(n, C.c_void_p) for n in ("ln2_g", "ln2_b")] + [("attn2", lc_unet_attn_w)] + \
               [(n, C.c_void_p) for n in ("ln3_g", "ln3_b", "ff1_w", "ff1_b", "ff2_w", "ff2_b", "pout_w", "pout_b")]


class lc_unet_conv_w(C.Structure):
    _fields_ = [("w", C.c_void_p), ("b", C.c_void_p)]


class lc_unet_weights(C.Structure):
    _fields_ = [("conv_in", lc_unet_conv_w), ("rb", lc_unet_rb_w * 6), ("st", lc_unet_tf_w * 4), ("tt", lc_unet_tf_w * 4),
                ("down", lc_unet_conv_w * 2), ("up", lc_unet_conv_w * 2), ("out_gn_g", C.c_void_p), ("out_gn_b", C.c_void_p),
                ("out", lc_unet_conv_w)]


# name -> (restype, argtypes). Every symbol include/lightcache.h declares is listed here.
_P, _I, _I64 = C.c_void_p, C.c_int, C.c_int64
PROTOTYPES = {
    "lc_check_config": (_I, [C.POINTER(lc_config)]),
    "lc_cache_entry_bytes": (C.c_size_t, [C.POINTER(lc_config)]),
    "lc_workspace_bytes": (C.c_size_t, [C.POINTER(lc_config), _I, _I]),
    "lc_last_error": (C.c_char_p, [_P]),
    "lc_create": (_I, [C.POINTER(lc_config), _P, _P, C.POINTER(_P)]),
    "lc_destroy": (_I, [_P]),
    "lc_load_weights": (_I, [_P, C.POINTER(lc_weights)]),
    "lc_set_workspace": (_I, [_P, _P, C.c_size_t]),
    "lc_set_chunk": (_I, [_P, _I, _I]),
    "lc_set_spatial_chunk": (_I, [_P, _I, _I]),
    "lc_workspace_bytes_spatial": (C.c_size_t, [C.POINTER(lc_config), _I, _I, _I, _I]),
    "lc_set_lanes": (_I, [_P, _I]),
    "lc_set_conv_general": (_I, [_P, _I]),
    "lc_full_step": (_I, [_P, _P, _P, _I]),
    "lc_cached_step": (_I, [_P, _P, _P, _I]),
    "lc_cached_step_static": (_I, [_P, _P, _P, _P]),
    "lc_static_scratch_bytes": (C.c_size_t, []),
    "lc_test_fail_host_alloc": (_I, [_I]),
    "lc_op_spatial_block": (_I, [_P, _P, _I]),
    "lc_op_temporal_block": (_I, [_P, _P]),
    "lc_swap_out": (_I, [_P, _I, _I]),
    "lc_swap_in": (_I, [_P, _I, _I]),
    "lc_sync": (_I, [_P]),
    "lc_cache_write": (_I, [_P, _I, _P]),
    "lc_cache_read": (_I, [_P, _I, _P]),
    "lc_cache_peek": (_I, [_P, _I, C.POINTER(_P), C.POINTER(C.c_size_t)]),
    "lc_cache_dev_peek": (_I, [_P, _I, C.POINTER(_P), C.POINTER(C.c_size_t)]),
    "lc_get_stats": (_I, [_P, C.POINTER(lc_stats)]),
    "lc_reset_stats": (_I, [_P]),
    "lc_set_profiling": (_I, [_P, C.c_uint32]),
    "lc_get_profile": (_I, [_P, C.POINTER(lc_profile)]),
    "lc_decoder_check_config": (_I, [C.POINTER(lc_decoder_config)]),
    "lc_decoder_workspace_bytes": (C.c_size_t, [C.POINTER(lc_decoder_config), _I]),
    "lc_decoder_last_error": (C.c_char_p, [_P]),
    "lc_decoder_create": (_I, [C.POINTER(lc_decoder_config), _P, C.POINTER(_P)]),
    "lc_decoder_destroy": (_I, [_P]),
    "lc_decoder_load_weights": (_I, [_P, C.POINTER(lc_decoder_weights)]),
    "lc_decoder_set_workspace": (_I, [_P, _P, C.c_size_t]),
    "lc_decode": (_I, [_P, _P, _P, _I]),
    "lc_decoder_sync": (_I, [_P]),
    "lc_dit_check_config": (_I, [C.POINTER(lc_dit_config)]),
    "lc_dit_entry_bytes": (C.c_size_t, [C.POINTER(lc_dit_config)]),
    "lc_dit_workspace_bytes": (C.c_size_t, [C.POINTER(lc_dit_config), _I]),
    "lc_dit_last_error": (C.c_char_p, [_P]),
    "lc_dit_create": (_I, [C.POINTER(lc_dit_config), _P, _P, C.POINTER(_P)]),
    "lc_dit_destroy": (_I, [_P]),
    "lc_dit_load_weights": (_I, [_P, C.POINTER(lc_dit_weights)]),
    "lc_dit_set_workspace": (_I, [_P, _P, C.c_size_t]),
    "lc_dit_set_chunk": (_I, [_P, _I]),
    "lc_dit_full_step": (_I, [_P, _P, _P, _P, _I]),
    "lc_dit_cached_step": (_I, [_P, _P, _P, _P, _I]),
    "lc_dit_swap_out": (_I, [_P, _I, _I]),
    "lc_dit_swap_in": (_I, [_P, _I, _I]),
    "lc_dit_sync": (_I, [_P]),
    "lc_dit_cache_write": (_I, [_P, _I, _P]),
    "lc_dit_cache_peek": (_I, [_P, _I, C.POINTER(_P), C.POINTER(C.c_size_t)]),
    "lc_dit_cache_dev_peek": (_I, [_P, _I, C.POINTER(_P), C.POINTER(C.c_size_t)]),
    "lc_dit_get_counts": (_I, [_P] + [C.POINTER(C.c_int64)] * 4),
    "lc_unet_check_config": (_I, [C.POINTER(lc_unet_config)]),
    "lc_unet_entry_bytes": (C.c_size_t, [C.POINTER(lc_unet_config)]),
    "lc_unet_workspace_bytes": (C.c_size_t, [C.POINTER(lc_unet_config)]),
    "lc_unet_chunk_workspace_bytes": (C.c_size_t, [C.POINTER(lc_unet_config), _I]),
    "lc_unet_set_chunk": (_I, [_P, _I]),
    "lc_unet_last_error": (C.c_char_p, [_P]),
    "lc_unet_create": (_I, [C.POINTER(lc_unet_config), _P, _P, C.POINTER(_P)]),
    "lc_unet_destroy": (_I, [_P]),
    "lc_unet_load_weights": (_I, [_P, C.POINTER(lc_unet_weights)]),
    "lc_unet_set_workspace": (_I, [_P, _P, C.c_size_t]),
    "lc_unet_full_step": (_I, [_P, _P, _P, _P, _P, _I]),
    "lc_unet_cached_step": (_I, [_P, _P, _P, _P, _P, _I]),
    "lc_unet_swap_out": (_I, [_P, _I, _I]),
    "lc_unet_swap_in": (_I, [_P, _I, _I]),
    "lc_unet_sync": (_I, [_P]),
    "lc_unet_cache_write": (_I, [_P, _I, _P]),
    "lc_unet_cache_peek": (_I, [_P, _I, C.POINTER(_P), C.POINTER(C.c_size_t)]),
    "lc_unet_cache_dev_peek": (_I, [_P, _I, C.POINTER(_P), C.POINTER(C.c_size_t)]),
    "lc_op_conv_in": (_I, [_P, _P, _P, _I]),
    "lc_op_res_block": (_I, [_P, _I, _P, _P, _I]),
    "lc_op_qkv": (_I, [_P, _I, _P, _P, _I]),
    "lc_op_spatial_attention": (_I, [_P, _P, _P, _I, _I, _I, _I]),
    "lc_op_temporal_attention": (_I, [_P, _P, _P, _I]),
    "lc_op_proj": (_I, [_P, _I, _P, _P, _P, _I64]),
    "lc_op_down_conv": (_I, [_P, _P, _P, _I]),
    "lc_op_up_conv": (_I, [_P, _P, _P, _P, _I]),
    "lc_op_conv_out": (_I, [_P, _P, _P, _I]),
}

_lib: Optional[C.CDLL] = None


def lib() -> C.CDLL:
    """Loads the shared library (once). Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with "
                               f"`python -m paper_2510_05367_amd.build` (needs hipcc)")
        _lib = C.CDLL(LIB_PATH)
        for name, (res, args) in PROTOTYPES.items():
            fn = getattr(_lib, name)
            fn.restype, fn.argtypes = res, args
    return _lib


def _check(status: int, ctx) -> None:
    if status != LC_OK:
        msg = lib().lc_last_error(ctx)
        raise LcError(status, msg.decode() if msg else "")


def make_config(cfg, host_slots: int = 1, dev_slots: int = 2) -> lc_config:
    """cfg: any object with the StageConfig attributes."""
    return lc_config(B=cfg.B, F=cfg.F, H=cfg.H, W=cfg.W, C_lat=cfg.C_lat, C=cfg.C, C_deep=cfg.C_deep,
                     groups=cfg.groups, n_res=cfg.n_res, heads=cfg.heads, head_dim=cfg.head_dim,
                     dtype=LC_BF16 if cfg.dtype == "bf16" else LC_F32, gn_eps=cfg.gn_eps,
                     host_slots=host_slots, dev_slots=dev_slots)


# ---- one thin function per entry point --------------------------------------------------------
def lc_check_config(cfg: lc_config) -> None:
    _check(lib().lc_check_config(C.byref(cfg)), None)


def lc_cache_entry_bytes(cfg: lc_config) -> int:
    return lib().lc_cache_entry_bytes(C.byref(cfg))


def lc_workspace_bytes(cfg: lc_config, frame_chunk: int, token_chunk: int) -> int:
    return lib().lc_workspace_bytes(C.byref(cfg), frame_chunk, token_chunk)


def lc_last_error(ctx=None) -> str:
    return lib().lc_last_error(ctx).decode()


def lc_create(cfg: lc_config, compute_stream: int, side_stream: int):
    out = C.c_void_p()
    _check(lib().lc_create(C.byref(cfg), compute_stream, side_stream, C.byref(out)), None)
    return out


def lc_destroy(ctx) -> None:
    _check(lib().lc_destroy(ctx), None)


def lc_load_weights(ctx, w: lc_weights) -> None:
    _check(lib().lc_load_weights(ctx, C.byref(w)), ctx)


def lc_set_workspace(ctx, arena_ptr: int, nbytes: int) -> None:
    _check(lib().lc_set_workspace(ctx, arena_ptr, nbytes), ctx)


def lc_set_chunk(ctx, frame_chunk: int, token_chunk: int) -> None:
    _check(lib().lc_set_chunk(ctx, frame_chunk, token_chunk), ctx)


def lc_set_spatial_chunk(ctx, eta: int, omega: int) -> None:
    _check(lib().lc_set_spatial_chunk(ctx, eta, omega), ctx)


def lc_workspace_bytes_spatial(cfg: lc_config, frame_chunk: int, token_chunk: int, eta: int, omega: int) -> int:
    return lib().lc_workspace_bytes_spatial(C.byref(cfg), frame_chunk, token_chunk, eta, omega)


def lc_set_lanes(ctx, lanes: int) -> None:
    _check(lib().lc_set_lanes(ctx, lanes), ctx)


def lc_set_conv_general(ctx, general: int) -> None:
    _check(lib().lc_set_conv_general(ctx, general), ctx)


def lc_full_step(ctx, x_ptr: int, eps_ptr: int, dev_slot: int) -> None:
    _check(lib().lc_full_step(ctx, x_ptr, eps_ptr, dev_slot), ctx)


def lc_cached_step(ctx, x_ptr: int, eps_ptr: int, dev_slot: int) -> None:
    _check(lib().lc_cached_step(ctx, x_ptr, eps_ptr, dev_slot), ctx)


def lc_cached_step_static(ctx, x_ptr: int, deep_ptr: int, eps_ptr: int) -> None:
    _check(lib().lc_cached_step_static(ctx, x_ptr, deep_ptr, eps_ptr), ctx)


def lc_static_scratch_bytes() -> int:
    return lib().lc_static_scratch_bytes()


def lc_test_fail_host_alloc(nth: int) -> None:
    _check(lib().lc_test_fail_host_alloc(nth), None)


def lc_swap_out(ctx, dev_slot: int, host_slot: int) -> None:
    _check(lib().lc_swap_out(ctx, dev_slot, host_slot), ctx)


def lc_swap_in(ctx, host_slot: int, dev_slot: int) -> None:
    _check(lib().lc_swap_in(ctx, host_slot, dev_slot), ctx)


def lc_sync(ctx) -> None:
    _check(lib().lc_sync(ctx), ctx)


def lc_cache_write(ctx, dev_slot: int, deep_ptr: int) -> None:
    _check(lib().lc_cache_write(ctx, dev_slot, deep_ptr), ctx)


def lc_cache_read(ctx, dev_slot: int, deep_ptr: int) -> None:
    _check(lib().lc_cache_read(ctx, dev_slot, deep_ptr), ctx)


def lc_cache_peek(ctx, host_slot: int):
    p, n = C.c_void_p(), C.c_size_t()
    _check(lib().lc_cache_peek(ctx, host_slot, C.byref(p), C.byref(n)), ctx)
    return p.value, n.value


def lc_cache_dev_peek(ctx, dev_slot: int):
    p, n = C.c_void_p(), C.c_size_t()
    _check(lib().lc_cache_dev_peek(ctx, dev_slot, C.byref(p), C.byref(n)), ctx)
    return p.value, n.value


def lc_get_stats(ctx) -> lc_stats:
    s = lc_stats()
    _check(lib().lc_get_stats(ctx, C.byref(s)), ctx)
    return s


def lc_reset_stats(ctx) -> None:
    _check(lib().lc_reset_stats(ctx), ctx)


def lc_set_profiling(ctx, mask: int) -> None:
    _check(lib().lc_set_profiling(ctx, mask), ctx)


def lc_get_profile(ctx) -> Dict[str, Dict[str, float]]:
    """Per family {"ms", "launches"}; the key "dropped" holds lc_profile.dropped (an int)."""
    p = lc_profile()
    _check(lib().lc_get_profile(ctx, C.byref(p)), ctx)
    out = {n: {"ms": p.ms[i], "launches": int(p.launches[i])} for i, n in enumerate(KERNEL_FAMILIES)}
    out["dropped"] = int(p.dropped)
    return out


def lc_op_conv_in(ctx, x_ptr, h_ptr, frames) -> None:
    _check(lib().lc_op_conv_in(ctx, x_ptr, h_ptr, frames), ctx)


def lc_op_res_block(ctx, layer, x_ptr, y_ptr, frames) -> None:
    _check(lib().lc_op_res_block(ctx, layer, x_ptr, y_ptr, frames), ctx)


def lc_op_qkv(ctx, layer, x_ptr, qkv_ptr, frames) -> None:
    _check(lib().lc_op_qkv(ctx, layer, x_ptr, qkv_ptr, frames), ctx)


def lc_op_spatial_attention(ctx, qkv_ptr, out_ptr, frames, q0, q1, q_prescaled=0) -> None:
    _check(lib().lc_op_spatial_attention(ctx, qkv_ptr, out_ptr, frames, q0, q1, q_prescaled), ctx)


def lc_op_spatial_block(ctx, h_ptr, frames) -> None:
    _check(lib().lc_op_spatial_block(ctx, h_ptr, frames), ctx)


def lc_op_temporal_block(ctx, h_ptr) -> None:
    _check(lib().lc_op_temporal_block(ctx, h_ptr), ctx)


def lc_op_temporal_attention(ctx, qkv_ptr, out_ptr, positions) -> None:
    _check(lib().lc_op_temporal_attention(ctx, qkv_ptr, out_ptr, positions), ctx)


def lc_op_proj(ctx, layer, a_ptr, res_ptr, y_ptr, rows) -> None:
    _check(lib().lc_op_proj(ctx, layer, a_ptr, res_ptr, y_ptr, rows), ctx)


def lc_op_down_conv(ctx, x_ptr, d0_ptr, frames) -> None:
    _check(lib().lc_op_down_conv(ctx, x_ptr, d0_ptr, frames), ctx)


def lc_op_up_conv(ctx, skip_ptr, deep_ptr, u_ptr, frames) -> None:
    _check(lib().lc_op_up_conv(ctx, skip_ptr, deep_ptr, u_ptr, frames), ctx)


def lc_op_conv_out(ctx, u_ptr, eps_ptr, frames) -> None:
    _check(lib().lc_op_conv_out(ctx, u_ptr, eps_ptr, frames), ctx)


# ---- sliced decoding ---------------------------------------------------------------------------
def _dcheck(status: int, dec) -> None:
    if status != LC_OK:
        msg = lib().lc_decoder_last_error(dec)
        raise LcError(status, msg.decode() if msg else "")


def make_decoder_config(cfg) -> lc_decoder_config:
    """cfg: any object with the synth.DecoderConfig attributes."""
    c = lc_decoder_config(N=cfg.N, H=cfg.H, W=cfg.W, C_lat=cfg.C_lat, C_img=cfg.C_img, levels=len(cfg.widths) - 1,
                          groups=cfg.groups, heads=cfg.heads, head_dim=cfg.head_dim,
                          dtype=LC_BF16 if cfg.dtype == "bf16" else LC_F32, gn_eps=cfg.gn_eps)
    for i, wd in enumerate(cfg.widths):
        c.widths[i] = wd
    return c


def lc_decoder_check_config(cfg: lc_decoder_config) -> None:
    _dcheck(lib().lc_decoder_check_config(C.byref(cfg)), None)


def lc_decoder_workspace_bytes(cfg: lc_decoder_config, slice_frames: int) -> int:
    return lib().lc_decoder_workspace_bytes(C.byref(cfg), slice_frames)


def lc_decoder_last_error(dec=None) -> str:
    return lib().lc_decoder_last_error(dec).decode()


def lc_decoder_create(cfg: lc_decoder_config, stream: int):
    out = C.c_void_p()
    _dcheck(lib().lc_decoder_create(C.byref(cfg), stream, C.byref(out)), None)
    return out


def lc_decoder_destroy(dec) -> None:
    _dcheck(lib().lc_decoder_destroy(dec), None)


def lc_decoder_load_weights(dec, w: lc_decoder_weights) -> None:
    _dcheck(lib().lc_decoder_load_weights(dec, C.byref(w)), dec)


def lc_decoder_set_workspace(dec, arena_ptr: int, nbytes: int) -> None:
    _dcheck(lib().lc_decoder_set_workspace(dec, arena_ptr, nbytes), dec)


def lc_decode(dec, z_ptr: int, img_ptr: int, slice_frames: int) -> None:
    _dcheck(lib().lc_decode(dec, z_ptr, img_ptr, slice_frames), dec)


def lc_decoder_sync(dec) -> None:
    _dcheck(lib().lc_decoder_sync(dec), dec)


class Decoder:
    """The decoder of the sliced-decoding stage on the current GPU; torch owns memory and the stream.
    `weights`: name -> numpy float32 array, names as in synth.decoder_weight_manifest."""

    def __init__(self, cfg, weights, max_slice: int = 1, device: str = "cuda:0"):
        import torch
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU visible: the HIP path cannot run (there is no CPU fallback)")
        self.torch, self.cfg = torch, cfg
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self.tdtype = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
        self.ccfg = make_decoder_config(cfg)
        lc_decoder_check_config(self.ccfg)
        self.stream = torch.cuda.Stream(device=self.device)
        self.dec = lc_decoder_create(self.ccfg, self.stream.cuda_stream)
        t = {k: self.to_device(v) for k, v in weights.items()}
        self.stream.synchronize()
        p = lambda n: t[n].data_ptr()
        gc = lambda pre: lc_gnconv_w(p(pre + ".gn_g"), p(pre + ".gn_b"), p(pre + ".w"), p(pre + ".b"))
        w = lc_decoder_weights()
        w.conv_in_w, w.conv_in_b = p("conv_in.w"), p("conv_in.b")
        w.mid_res[0], w.mid_res[1] = gc("mid.res0"), gc("mid.res1")
        w.mid_attn = lc_attn_w(*[p(f"mid.attn.{k}") for k in ("gn_g", "gn_b", "wq", "wk", "wv", "wo", "bo")])
        for l in range(len(cfg.widths) - 1):
            w.up_res[l] = gc(f"up{l}.res")
            w.up_conv_w[l], w.up_conv_b[l] = p(f"up{l}.conv.w"), p(f"up{l}.conv.b")
        w.out = gc("out")
        lc_decoder_load_weights(self.dec, w)
        del t
        self.arena = None
        self.ensure_workspace(max_slice)

    def to_device(self, a):
        with self.torch.cuda.stream(self.stream):
            return self.torch.from_numpy(a).to(self.device).to(self.tdtype).contiguous()

    def ensure_workspace(self, slice_frames: int) -> int:
        need = lc_decoder_workspace_bytes(self.ccfg, slice_frames)
        if self.arena is None or self.arena.numel() < need:
            lc_decoder_sync(self.dec)
            self.arena = None
            self.arena = self.torch.empty(need, dtype=self.torch.uint8, device=self.device)
            self.torch.cuda.synchronize(self.device)
            lc_decoder_set_workspace(self.dec, self.arena.data_ptr(), self.arena.numel())
        return need

    def decode(self, z, slice_frames: int = 1):
        c = self.cfg
        s = 2 ** (len(c.widths) - 1)
        with self.torch.cuda.stream(self.stream):
            img = self.torch.empty(c.N, c.C_img, c.H * s, c.W * s, dtype=self.tdtype, device=self.device)
        lc_decode(self.dec, z.data_ptr(), img.data_ptr(), slice_frames)
        return img

    def sync(self):
        lc_decoder_sync(self.dec)

    def close(self):
        if self.dec is not None:
            lc_decoder_destroy(self.dec)
            self.dec = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


# ---- diffusion-transformer variant -----------------------------------------------------------------
def _tcheck(status: int, ctx) -> None:
    if status != LC_OK:
        msg = lib().lc_dit_last_error(ctx)
        raise LcError(status, msg.decode() if msg else "")


def make_dit_config(cfg, host_slots: int = 1, dev_slots: int = 2) -> lc_dit_config:
    """cfg: any object with the synth.DitConfig attributes."""
    return lc_dit_config(B=cfg.B, T=cfg.T, D=cfg.D, heads=cfg.heads, head_dim=cfg.head_dim, L=cfg.L, cache_a=cfg.cache_a,
                         cache_b=cfg.cache_b, mlp_ratio=cfg.mlp_ratio, dtype=LC_BF16 if cfg.dtype == "bf16" else LC_F32,
                         ln_eps=cfg.ln_eps, host_slots=host_slots, dev_slots=dev_slots)


def lc_dit_check_config(cfg: lc_dit_config) -> None:
    _tcheck(lib().lc_dit_check_config(C.byref(cfg)), None)


def lc_dit_entry_bytes(cfg: lc_dit_config) -> int:
    return lib().lc_dit_entry_bytes(C.byref(cfg))


def lc_dit_workspace_bytes(cfg: lc_dit_config, token_chunk: int) -> int:
    return lib().lc_dit_workspace_bytes(C.byref(cfg), token_chunk)


def lc_dit_last_error(ctx=None) -> str:
    return lib().lc_dit_last_error(ctx).decode()


def lc_dit_create(cfg: lc_dit_config, compute_stream: int, side_stream: int):
    out = C.c_void_p()
    _tcheck(lib().lc_dit_create(C.byref(cfg), compute_stream, side_stream, C.byref(out)), None)
    return out


def lc_dit_destroy(ctx) -> None:
    _tcheck(lib().lc_dit_destroy(ctx), None)


def lc_dit_load_weights(ctx, w: lc_dit_weights) -> None:
    _tcheck(lib().lc_dit_load_weights(ctx, C.byref(w)), ctx)


def lc_dit_set_workspace(ctx, arena_ptr: int, nbytes: int) -> None:
    _tcheck(lib().lc_dit_set_workspace(ctx, arena_ptr, nbytes), ctx)


def lc_dit_set_chunk(ctx, token_chunk: int) -> None:
    _tcheck(lib().lc_dit_set_chunk(ctx, token_chunk), ctx)


def lc_dit_full_step(ctx, x_in_ptr: int, mod_ptr: int, x_out_ptr: int, dev_slot: int) -> None:
    _tcheck(lib().lc_dit_full_step(ctx, x_in_ptr, mod_ptr, x_out_ptr, dev_slot), ctx)


def lc_dit_cached_step(ctx, x_in_ptr: int, mod_ptr: int, x_out_ptr: int, dev_slot: int) -> None:
    _tcheck(lib().lc_dit_cached_step(ctx, x_in_ptr, mod_ptr, x_out_ptr, dev_slot), ctx)


def lc_dit_swap_out(ctx, dev_slot: int, host_slot: int) -> None:
    _tcheck(lib().lc_dit_swap_out(ctx, dev_slot, host_slot), ctx)


def lc_dit_swap_in(ctx, host_slot: int, dev_slot: int) -> None:
    _tcheck(lib().lc_dit_swap_in(ctx, host_slot, dev_slot), ctx)


def lc_dit_sync(ctx) -> None:
    _tcheck(lib().lc_dit_sync(ctx), ctx)


def lc_dit_cache_write(ctx, dev_slot: int, delta_ptr: int) -> None:
    _tcheck(lib().lc_dit_cache_write(ctx, dev_slot, delta_ptr), ctx)


def lc_dit_cache_peek(ctx, host_slot: int):
    p, n = C.c_void_p(), C.c_size_t()
    _tcheck(lib().lc_dit_cache_peek(ctx, host_slot, C.byref(p), C.byref(n)), ctx)
    return p.value, n.value


def lc_dit_cache_dev_peek(ctx, dev_slot: int):
    p, n = C.c_void_p(), C.c_size_t()
    _tcheck(lib().lc_dit_cache_dev_peek(ctx, dev_slot, C.byref(p), C.byref(n)), ctx)
    return p.value, n.value


def lc_dit_get_counts(ctx):
    v = [C.c_int64() for _ in range(4)]
    _tcheck(lib().lc_dit_get_counts(ctx, *[C.byref(x) for x in v]), ctx)
    return tuple(x.value for x in v)


class Dit:
    """The block stack of the diffusion-transformer variant on the current GPU; torch owns memory and streams.
    `weights`: name -> numpy float32 array, names as in synth.dit_weight_manifest."""

    def __init__(self, cfg, weights, host_slots: int = 1, dev_slots: int = 2, token_chunk: Optional[int] = None,
                 device: str = "cuda:0"):
        import torch
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU visible: the HIP path cannot run (there is no CPU fallback)")
        self.torch, self.cfg = torch, cfg
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self.tdtype = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
        self.ccfg = make_dit_config(cfg, host_slots, dev_slots)
        lc_dit_check_config(self.ccfg)
        self.compute = torch.cuda.Stream(device=self.device)
        self.side = torch.cuda.Stream(device=self.device)
        self.ctx = lc_dit_create(self.ccfg, self.compute.cuda_stream, self.side.cuda_stream)
        with torch.cuda.stream(self.compute):
            t = {k: torch.from_numpy(v).to(self.device).to(self.tdtype).contiguous() for k, v in weights.items()}
        self.compute.synchronize()
        w = lc_dit_weights()
        for i in range(cfg.L):
            w.blk[i] = lc_dit_block_w(*[t[f"blk{i}.{k}"].data_ptr() for k in ("wqkv", "bqkv", "wo", "bo", "w1", "b1", "w2", "b2")])
        lc_dit_load_weights(self.ctx, w)
        del t
        self.arena = None
        self._chunk = 0  # what a fresh context plans for: unchunked
        self.set_chunk(cfg.token_chunk if token_chunk is None else token_chunk)

    def to_device(self, a):
        """numpy -> float32 device tensor (hidden states, modulation, Delta), on the compute stream."""
        with self.torch.cuda.stream(self.compute):
            return self.torch.from_numpy(a).to(self.device).float().contiguous()

    def empty(self, *shape):
        with self.torch.cuda.stream(self.compute):
            return self.torch.empty(*shape, dtype=self.torch.float32, device=self.device)

    def set_chunk(self, token_chunk: int) -> None:
        need = max(lc_dit_workspace_bytes(self.ccfg, token_chunk), lc_dit_workspace_bytes(self.ccfg, self._chunk))
        if self.arena is None or self.arena.numel() < need:
            # an arena that covers the plan in force and the new one (a new workspace starts with empty slots)
            lc_dit_sync(self.ctx)
            self.arena = None
            self.arena = self.torch.empty(need, dtype=self.torch.uint8, device=self.device)
            self.torch.cuda.synchronize(self.device)
            lc_dit_set_workspace(self.ctx, self.arena.data_ptr(), self.arena.numel())
        lc_dit_set_chunk(self.ctx, token_chunk)
        self._chunk = token_chunk

    def full_step(self, x, mod, out, dev_slot: int = 0):
        lc_dit_full_step(self.ctx, x.data_ptr(), mod.data_ptr(), out.data_ptr(), dev_slot)

    def cached_step(self, x, mod, out, dev_slot: int = 0):
        lc_dit_cached_step(self.ctx, x.data_ptr(), mod.data_ptr(), out.data_ptr(), dev_slot)

    def swap_out(self, dev_slot: int, host_slot: int):
        lc_dit_swap_out(self.ctx, dev_slot, host_slot)

    def swap_in(self, host_slot: int, dev_slot: int):
        lc_dit_swap_in(self.ctx, host_slot, dev_slot)

    def cache_write(self, dev_slot: int, delta):
        lc_dit_cache_write(self.ctx, dev_slot, delta.data_ptr())

    def sync(self):
        lc_dit_sync(self.ctx)

    def host_entry_bytes(self, host_slot: int) -> bytes:
        ptr, n = lc_dit_cache_peek(self.ctx, host_slot)
        return C.string_at(ptr, n)

    def dev_entry(self, dev_slot: int):
        """The Delta in a device slot as a float32 tensor [B, T, D] (a copy)."""
        ptr, n = lc_dit_cache_dev_peek(self.ctx, dev_slot)
        self.sync()
        off = ptr - self.arena.data_ptr()
        c = self.cfg
        return self.arena[off:off + n].view(self.torch.float32).reshape(c.B, c.T, c.D).clone()

    def close(self):
        if self.ctx is not None:
            lc_dit_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


# ---- U-Net stage with real block internals ------------------------------------------------------------
def _ucheck(status: int, ctx) -> None:
    if status != LC_OK:
        msg = lib().lc_unet_last_error(ctx)
        raise LcError(status, msg.decode() if msg else "")


def make_unet_config(cfg, host_slots: int = 1, dev_slots: int = 2) -> lc_unet_config:
    """cfg: any object with the synth.UnetConfig attributes."""
    return lc_unet_config(B=cfg.B, F=cfg.F, H=cfg.H, W=cfg.W, C_lat=cfg.C_lat, C=cfg.C, C1=cfg.C1, C2=cfg.C2, groups=cfg.groups,
                          head_dim=cfg.head_dim, ctx_len=cfg.ctx_len, ctx_dim=cfg.ctx_dim, temb_dim=cfg.temb_dim, ff_mult=cfg.ff_mult,
                          dtype=LC_BF16 if cfg.dtype == "bf16" else LC_F32, gn_eps=cfg.gn_eps, ln_eps=cfg.ln_eps,
                          host_slots=host_slots, dev_slots=dev_slots)


def lc_unet_check_config(cfg: lc_unet_config) -> None:
    _ucheck(lib().lc_unet_check_config(C.byref(cfg)), None)


def lc_unet_entry_bytes(cfg: lc_unet_config) -> int:
    return lib().lc_unet_entry_bytes(C.byref(cfg))


def lc_unet_workspace_bytes(cfg: lc_unet_config) -> int:
    return lib().lc_unet_workspace_bytes(C.byref(cfg))


def lc_unet_chunk_workspace_bytes(cfg: lc_unet_config, frame_chunk: int) -> int:
    return lib().lc_unet_chunk_workspace_bytes(C.byref(cfg), frame_chunk)


def lc_unet_set_chunk(ctx, frame_chunk: int) -> None:
    _ucheck(lib().lc_unet_set_chunk(ctx, frame_chunk), ctx)


def lc_unet_last_error(ctx=None) -> str:
    return lib().lc_unet_last_error(ctx).decode()


def lc_unet_create(cfg: lc_unet_config, compute_stream: int, side_stream: int):
    out = C.c_void_p()
    _ucheck(lib().lc_unet_create(C.byref(cfg), compute_stream, side_stream, C.byref(out)), None)
    return out


def lc_unet_destroy(ctx) -> None:
    _ucheck(lib().lc_unet_destroy(ctx), None)


def lc_unet_load_weights(ctx, w: lc_unet_weights) -> None:
    _ucheck(lib().lc_unet_load_weights(ctx, C.byref(w)), ctx)


def lc_unet_set_workspace(ctx, arena_ptr: int, nbytes: int) -> None:
    _ucheck(lib().lc_unet_set_workspace(ctx, arena_ptr, nbytes), ctx)


def lc_unet_full_step(ctx, x_ptr: int, temb_ptr: int, cond_ptr: int, eps_ptr: int, dev_slot: int) -> None:
    _ucheck(lib().lc_unet_full_step(ctx, x_ptr, temb_ptr, cond_ptr, eps_ptr, dev_slot), ctx)


def lc_unet_cached_step(ctx, x_ptr: int, temb_ptr: int, cond_ptr: int, eps_ptr: int, dev_slot: int) -> None:
    _ucheck(lib().lc_unet_cached_step(ctx, x_ptr, temb_ptr, cond_ptr, eps_ptr, dev_slot), ctx)


def lc_unet_swap_out(ctx, dev_slot: int, host_slot: int) -> None:
    _ucheck(lib().lc_unet_swap_out(ctx, dev_slot, host_slot), ctx)


def lc_unet_swap_in(ctx, host_slot: int, dev_slot: int) -> None:
    _ucheck(lib().lc_unet_swap_in(ctx, host_slot, dev_slot), ctx)


def lc_unet_sync(ctx) -> None:
    _ucheck(lib().lc_unet_sync(ctx), ctx)


def lc_unet_cache_write(ctx, dev_slot: int, deep_ptr: int) -> None:
    _ucheck(lib().lc_unet_cache_write(ctx, dev_slot, deep_ptr), ctx)


def lc_unet_cache_peek(ctx, host_slot: int):
    p, n = C.c_void_p(), C.c_size_t()
    _ucheck(lib().lc_unet_cache_peek(ctx, host_slot, C.byref(p), C.byref(n)), ctx)
    return p.value, n.value


def lc_unet_cache_dev_peek(ctx, dev_slot: int):
    p, n = C.c_void_p(), C.c_size_t()
    _ucheck(lib().lc_unet_cache_dev_peek(ctx, dev_slot, C.byref(p), C.byref(n)), ctx)
    return p.value, n.value


UNET_RB = ("d0.rb", "d1.rb", "mid.rb0", "mid.rb1", "u1.rb", "u0.rb")
UNET_TF = ("d0", "d1", "u1", "u0")


class Unet:
    """The U-Net stage with real block internals on the current GPU; torch owns memory and streams.
    `weights`: name -> numpy float32 array, names as in synth.unet_weight_manifest. `frame_chunk`: the feature chunk
    the workspace is sized for (None: all frames at once, which every later set_chunk fits)."""

    def __init__(self, cfg, weights, host_slots: int = 1, dev_slots: int = 2, device: str = "cuda:0",
                 frame_chunk: Optional[int] = None):
        import torch
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU visible: the HIP path cannot run (there is no CPU fallback)")
        self.torch, self.cfg = torch, cfg
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self.tdtype = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
        self.ccfg = make_unet_config(cfg, host_slots, dev_slots)
        lc_unet_check_config(self.ccfg)
        self.compute = torch.cuda.Stream(device=self.device)
        self.side = torch.cuda.Stream(device=self.device)
        self.ctx = lc_unet_create(self.ccfg, self.compute.cuda_stream, self.side.cuda_stream)
        with torch.cuda.stream(self.compute):
            t = {k: torch.from_numpy(v).to(self.device).to(self.tdtype).contiguous() for k, v in weights.items()}
        self.compute.synchronize()
        ptr = lambda name: t[name].data_ptr() if name in t else None
        w = lc_unet_weights()
        w.conv_in = lc_unet_conv_w(ptr("conv_in.w"), ptr("conv_in.b"))
        for i, p in enumerate(UNET_RB):
            w.rb[i] = lc_unet_rb_w(*[ptr(f"{p}.{k}") for k in ("gn1_g", "gn1_b", "conv1.w", "conv1.b", "temb.w", "temb.b", "gn2_g",
                                                             "gn2_b", "conv2.w", "conv2.b", "short.w", "short.b")])
        for kind, arr in (("st", w.st), ("tt", w.tt)):
            for i, lvl in enumerate(UNET_TF):
                p = f"{lvl}.{kind}"
                q = lc_unet_tf_w()
                for k in ("gn_g", "gn_b", "ln1_g", "ln1_b", "ln2_g", "ln2_b", "ln3_g", "ln3_b"):
                    setattr(q, k, ptr(f"{p}.{k}"))
                for k in ("pin", "ff1", "ff2", "pout"):
                    setattr(q, k + "_w", ptr(f"{p}.{k}.w"))
                    setattr(q, k + "_b", ptr(f"{p}.{k}.b"))
                q.attn1 = lc_unet_attn_w(*[ptr(f"{p}.attn1.{k}") for k in ("wq", "wk", "wv", "wo", "bo")])
                q.attn2 = lc_unet_attn_w(*[ptr(f"{p}.attn2.{k}") for k in ("wq", "wk", "wv", "wo", "bo")])
                arr[i] = q
        w.down[0] = lc_unet_conv_w(ptr("d0.down.w"), ptr("d0.down.b"))
        w.down[1] = lc_unet_conv_w(ptr("d1.down.w"), ptr("d1.down.b"))
        w.up[0] = lc_unet_conv_w(ptr("u2.up.w"), ptr("u2.up.b"))
        w.up[1] = lc_unet_conv_w(ptr("u1.up.w"), ptr("u1.up.b"))
        w.out_gn_g, w.out_gn_b = ptr("out.gn_g"), ptr("out.gn_b")
        w.out = lc_unet_conv_w(ptr("out.w"), ptr("out.b"))
        lc_unet_load_weights(self.ctx, w)
        del t
        if frame_chunk:
            lc_unet_set_chunk(self.ctx, frame_chunk)
        need = lc_unet_chunk_workspace_bytes(self.ccfg, frame_chunk or 0)
        with torch.cuda.stream(self.compute):
            self.arena = torch.empty(need, dtype=torch.uint8, device=self.device)
        self.compute.synchronize()
        lc_unet_set_workspace(self.ctx, self.arena.data_ptr(), self.arena.numel())

    def set_chunk(self, frame_chunk: int):
        """Frames per chunk from the next step on (0: all frames at once); the cached entries stay where they are."""
        self.sync()
        lc_unet_set_chunk(self.ctx, frame_chunk)

    def to_device(self, a, f32: bool = False):
        """numpy -> device tensor of the stage's dtype (f32: float32, for cache entries), on the compute stream."""
        with self.torch.cuda.stream(self.compute):
            return self.torch.from_numpy(a).to(self.device).to(self.torch.float32 if f32 else self.tdtype).contiguous()

    def empty(self, *shape):
        with self.torch.cuda.stream(self.compute):
            return self.torch.empty(*shape, dtype=self.tdtype, device=self.device)

    def full_step(self, x, temb, ctx, eps, dev_slot: int = 0):
        lc_unet_full_step(self.ctx, x.data_ptr(), temb.data_ptr(), ctx.data_ptr(), eps.data_ptr(), dev_slot)

    def cached_step(self, x, temb, ctx, eps, dev_slot: int = 0):
        lc_unet_cached_step(self.ctx, x.data_ptr(), temb.data_ptr(), ctx.data_ptr(), eps.data_ptr(), dev_slot)

    def swap_out(self, dev_slot: int, host_slot: int):
        lc_unet_swap_out(self.ctx, dev_slot, host_slot)

    def swap_in(self, host_slot: int, dev_slot: int):
        lc_unet_swap_in(self.ctx, host_slot, dev_slot)

    def cache_write(self, dev_slot: int, deep):
        """deep: float32 device tensor [B*F, H*W, C1] (channels last)."""
        lc_unet_cache_write(self.ctx, dev_slot, deep.data_ptr())

    def sync(self):
        lc_unet_sync(self.ctx)

    def host_entry_bytes(self, host_slot: int) -> bytes:
        ptr, n = lc_unet_cache_peek(self.ctx, host_slot)
        return C.string_at(ptr, n)

    def dev_entry(self, dev_slot: int):
        """The cached feature in a device slot as a float32 tensor [B*F, H*W, C1] (a copy)."""
        ptr, n = lc_unet_cache_dev_peek(self.ctx, dev_slot)
        self.sync()
        off = ptr - self.arena.data_ptr()
        c = self.cfg
        return self.arena[off:off + n].view(self.torch.float32).reshape(c.B * c.F, c.H * c.W, c.C1).clone()

    def close(self):
        if self.ctx is not None:
            lc_unet_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


# ---- convenience holder: torch owns memory and streams, the library does the work ---------------
class Stage:
    """One shallow stage on the current GPU. `weights`: name -> numpy float32 array (PyTorch layouts,
    names as in synth.weight_manifest)."""

    def __init__(self, cfg, weights, host_slots: int = 1, dev_slots: int = 2, frame_chunk: Optional[int] = None,
                 token_chunk: Optional[int] = None, device: str = "cuda:0"):
        import torch
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU visible: the HIP path cannot run (there is no CPU fallback)")
        self.torch = torch
        self.cfg = cfg
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self.tdtype = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
        self.ccfg = make_config(cfg, host_slots, dev_slots)
        lc_check_config(self.ccfg)
        self.compute = torch.cuda.Stream(device=self.device)
        self.side = torch.cuda.Stream(device=self.device)
        self.ctx = lc_create(self.ccfg, self.compute.cuda_stream, self.side.cuda_stream)
        fc = cfg.frame_chunk if frame_chunk is None else frame_chunk
        tc = cfg.token_chunk if token_chunk is None else token_chunk
        self._wt = {k: self.to_device(v) for k, v in weights.items()}
        torch.cuda.synchronize(self.device)
        lc_load_weights(self.ctx, self._weights_struct())
        self._wt = None  # the library keeps packed private copies
        lc_set_chunk(self.ctx, fc, tc)
        self.arena = None
        self._fc, self._tc, self._eta, self._omega = fc, tc, 1, 1
        self._ensure_arena(fc, tc)

    # -- memory helpers
    # Tensors the library reads or writes are allocated, filled and converted on the compute stream: torch's
    # caching allocator then hands a freed block only to later work of that same stream, so a temporary that
    # the caller drops right after an (asynchronous) library call is not reused under a kernel that still
    # reads it, and torch's own copies are ordered with the library's kernels.
    def to_device(self, a):
        with self.torch.cuda.stream(self.compute):
            t = self.torch.from_numpy(a).to(self.device)
            return t.to(self.tdtype).contiguous()

    def empty(self, *shape):
        with self.torch.cuda.stream(self.compute):
            return self.torch.empty(*shape, dtype=self.tdtype, device=self.device)

    def _ensure_arena(self, fc, tc, eta=None, omega=None):
        eta = self._eta if eta is None else eta
        omega = self._omega if omega is None else omega
        need = lc_workspace_bytes_spatial(self.ccfg, fc, tc, eta, omega) or lc_workspace_bytes(self.ccfg, fc, tc)
        if self.arena is None or self.arena.numel() < need:
            lc_sync(self.ctx)
            self.arena = self.torch.empty(need, dtype=self.torch.uint8, device=self.device)
            self.torch.cuda.synchronize(self.device)
            lc_set_workspace(self.ctx, self.arena.data_ptr(), self.arena.numel())

    def _weights_struct(self) -> lc_weights:
        t = self._wt
        p = lambda n: t[n].data_ptr()
        w = lc_weights()
        w.conv_in_w, w.conv_in_b = p("conv_in.w"), p("conv_in.b")
        for i in range(self.cfg.n_res):
            w.res[i] = lc_gnconv_w(p(f"res{i}.gn_g"), p(f"res{i}.gn_b"), p(f"res{i}.w"), p(f"res{i}.b"))
        for name in ("sattn", "tattn"):
            setattr(w, name, lc_attn_w(*[p(f"{name}.{k}") for k in ("gn_g", "gn_b", "wq", "wk", "wv", "wo", "bo")]))
        w.down_w, w.down_b = p("down.w"), p("down.b")
        for name in ("dres", "up", "out"):
            setattr(w, name, lc_gnconv_w(*[p(f"{name}.{k}") for k in ("gn_g", "gn_b", "w", "b")]))
        return w

    # -- the method
    def set_chunk(self, frame_chunk: int, token_chunk: int) -> None:
        self._ensure_arena(frame_chunk, token_chunk)
        lc_set_chunk(self.ctx, frame_chunk, token_chunk)
        self._fc, self._tc = frame_chunk, token_chunk

    def set_spatial_chunk(self, eta: int, omega: int) -> None:
        self._ensure_arena(self._fc, self._tc, eta, omega)
        lc_set_spatial_chunk(self.ctx, eta, omega)
        self._eta, self._omega = eta, omega

    def set_lanes(self, lanes: int) -> None:
        lc_set_lanes(self.ctx, lanes)

    def set_conv_general(self, general: bool) -> None:
        lc_set_conv_general(self.ctx, 1 if general else 0)

    def full_step(self, x, eps, dev_slot: int = 0):
        lc_full_step(self.ctx, x.data_ptr(), eps.data_ptr(), dev_slot)

    def cached_step(self, x, eps, dev_slot: int = 0):
        lc_cached_step(self.ctx, x.data_ptr(), eps.data_ptr(), dev_slot)

    def swap_out(self, dev_slot: int, host_slot: int):
        lc_swap_out(self.ctx, dev_slot, host_slot)

    def swap_in(self, host_slot: int, dev_slot: int):
        lc_swap_in(self.ctx, host_slot, dev_slot)

    def cache_write(self, dev_slot: int, deep):
        lc_cache_write(self.ctx, dev_slot, deep.data_ptr())

    def cache_read(self, dev_slot: int):
        """The slot in public layout; lc_sync (or a wait on the compute stream) before it is read elsewhere."""
        c = self.cfg
        out = self.empty(c.N, c.C_deep, c.H // 2, c.W // 2)
        lc_cache_read(self.ctx, dev_slot, out.data_ptr())
        return out

    def sync(self):
        lc_sync(self.ctx)

    def host_entry_bytes(self, host_slot: int) -> bytes:
        ptr, n = lc_cache_peek(self.ctx, host_slot)
        return C.string_at(ptr, n)

    def dev_entry_bytes(self, dev_slot: int) -> bytes:
        """Raw bytes of a device slot (the slots live inside the torch-owned arena)."""
        ptr, n = lc_cache_dev_peek(self.ctx, dev_slot)
        self.sync()
        off = ptr - self.arena.data_ptr()
        assert 0 <= off and off + n <= self.arena.numel()
        return self.arena[off:off + n].cpu().numpy().tobytes()

    def close(self):
        if self.ctx is not None:
            lc_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
