"""CPU-side checks of the boundary: the shared library loads without a GPU, exports every symbol
the header declares, and its host-only entry points validate their arguments."""
import ctypes
import os
import re

import pytest

from paper_2510_05367_amd import binding as lcb
from paper_2510_05367_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_symbols():
    text = open(os.path.join(ROOT, "include", "lightcache.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lc_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = header_symbols()
    assert len(names) >= 25
    lib = lcb.lib()
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in lightcache.h but not exported"
    # and the binding knows a prototype for each of them
    assert sorted(lcb.PROTOTYPES) == names


def test_struct_sizes_match_header_layout():
    assert ctypes.sizeof(lcb.lc_config) == 15 * 4
    assert ctypes.sizeof(lcb.lc_weights) == 8 * (2 + 4 * lcb.LC_MAX_RES + 7 + 7 + 2 + 4 + 4 + 4)
    assert ctypes.sizeof(lcb.lc_profile) == 16 * len(lcb.KERNEL_FAMILIES) + 8
    assert ctypes.sizeof(lcb.lc_stats) == 8 * 13
    assert lcb.lc_static_scratch_bytes() == 64 << 20


def test_destroy_rejects_pointers_it_did_not_hand_out():
    # NULL is a no-op; any other pointer that lc_create never returned (or that was destroyed before) must be
    # refused without being dereferenced
    lcb.lc_destroy(None)
    junk = ctypes.create_string_buffer(4096)
    with pytest.raises(lcb.LcError) as e:
        lcb.lc_destroy(ctypes.c_void_p(ctypes.addressof(junk)))
    assert e.value.status == lcb.LC_ERR_ARG
    assert "destroyed" in lcb.lc_last_error()
    assert junk.raw == bytes(4096)


def test_host_alloc_failure_hook_validates():
    with pytest.raises(lcb.LcError) as e:
        lcb.lc_test_fail_host_alloc(-1)
    assert e.value.status == lcb.LC_ERR_ARG
    lcb.lc_test_fail_host_alloc(0)


@pytest.mark.parametrize("name", list(synth.CONFIGS))
def test_named_configs_are_valid(name):
    c = lcb.make_config(synth.CONFIGS[name], host_slots=2, dev_slots=2)
    lcb.lc_check_config(c)
    cfg = synth.CONFIGS[name]
    es = 2 if cfg.dtype == "bf16" else 4
    assert lcb.lc_cache_entry_bytes(c) == cfg.N * cfg.C_deep * (cfg.H // 2) * (cfg.W // 2) * es


@pytest.mark.parametrize("field,value", [("H", 31), ("W", 7), ("C", 100), ("C_deep", 96), ("groups", 7),
                                         ("heads", 3), ("head_dim", 24), ("C_lat", 17), ("n_res", 5),
                                         ("dev_slots", 0), ("host_slots", 65), ("B", 0), ("gn_eps", 0.0)])
def test_bad_configs_are_rejected(field, value):
    c = lcb.make_config(synth.CONFIGS["tiny"])
    setattr(c, field, value)
    with pytest.raises(lcb.LcError) as e:
        lcb.lc_check_config(c)
    assert e.value.status == lcb.LC_ERR_SHAPE
    assert lcb.lc_workspace_bytes(c, 0, 0) == 0 and lcb.lc_cache_entry_bytes(c) == 0


def test_bad_dtype_and_null():
    c = lcb.make_config(synth.CONFIGS["tiny"])
    c.dtype = 7
    with pytest.raises(lcb.LcError) as e:
        lcb.lc_check_config(c)
    assert e.value.status == lcb.LC_ERR_ARG
    assert lcb.lib().lc_check_config(None) == lcb.LC_ERR_ARG
    assert "NULL" in lcb.lc_last_error()


def test_footprint_model_scales_with_chunk_not_with_frames():
    cfg = synth.CONFIGS["animatediff"]
    c = lcb.make_config(cfg)
    full = lcb.lc_workspace_bytes(c, 0, 0)
    # a chunked step keeps two chunks in flight (one per lane), so halving the axis saves nothing yet
    sizes = [lcb.lc_workspace_bytes(c, fc, 0) for fc in (8, 4, 2, 1)]
    assert all(a > b for a, b in zip([full] + sizes, sizes))
    # persistent part: fp32 skip feature + dev_slots cache entries + GroupNorm partial sums (three tensors
    # of [N][T/32][C][2] floats written by the kernels that produce the normalised tensors, and the
    # much smaller ones of the cached deep feature, per slot)
    es = 2
    persistent = cfg.N * cfg.T * cfg.C * 4 + 2 * lcb.lc_cache_entry_bytes(c) + 3 * cfg.N * (cfg.T // 32) * cfg.C * 8
    # one frame of scratch: fp32 ping-pong copy of the stream + q,k,v + attention output
    chunk1 = cfg.T * (4 * cfg.C + 4 * cfg.C * es)
    assert sizes[-1] - persistent < 2 * chunk1 + 32e6
    # chunk scratch is linear in the frame chunk (fc = 8 -> 4, two lanes each)
    assert abs((sizes[0] - sizes[1]) - 2 * 4 * chunk1) < 1e6
    # negative chunk
    assert lcb.lc_workspace_bytes(c, -1, 0) == 0
    # clamping: a chunk above the axis length equals unchunked
    assert lcb.lc_workspace_bytes(c, 1000, 0) == full
    # no score matrix is ever materialised: the stress instance stays far below 64 GB even unchunked
    s = lcb.make_config(synth.CONFIGS["stress"], host_slots=10)
    assert lcb.lc_workspace_bytes(s, 0, 0) < 4e9


def test_token_chunk_bounds_the_temporal_pass():
    cfg = synth.CONFIGS["svdxt"]
    c = lcb.make_config(cfg)
    a = lcb.lc_workspace_bytes(c, 5, 2304)
    b = lcb.lc_workspace_bytes(c, 5, 0)
    assert a > 0 and b > 0
    # 50 frames x 2304 positions = 115200 rows > 5 x 9216 = 46080 rows: the token chunk dominates
    assert a > b


def test_decoder_config_checks_and_footprint_without_a_gpu():
    cfg = synth.DECODERS["animatediff"]
    c = lcb.make_decoder_config(cfg)
    lcb.lc_decoder_check_config(c)
    assert ctypes.sizeof(lcb.lc_decoder_config) == 4 * (6 + 4 + 4) + 4
    one = lcb.lc_decoder_workspace_bytes(c, 1)
    assert 0 < one < lcb.lc_decoder_workspace_bytes(c, 2) < lcb.lc_decoder_workspace_bytes(c, 0)
    assert lcb.lc_decoder_workspace_bytes(c, -1) == 0
    for field, value in [("levels", 4), ("groups", 7), ("heads", 3), ("head_dim", 24), ("C_lat", 17), ("N", 0), ("gn_eps", 0.0)]:
        bad = lcb.make_decoder_config(cfg)
        setattr(bad, field, value)
        with pytest.raises(lcb.LcError) as e:
            lcb.lc_decoder_check_config(bad)
        assert e.value.status == lcb.LC_ERR_SHAPE, field
        assert lcb.lc_decoder_workspace_bytes(bad, 1) == 0
    bad = lcb.make_decoder_config(cfg)
    bad.widths[1] = 100
    with pytest.raises(lcb.LcError):
        lcb.lc_decoder_check_config(bad)
    for name in synth.DECODERS:
        lcb.lc_decoder_check_config(lcb.make_decoder_config(synth.DECODERS[name]))


def test_unet_config_checks_and_footprint_without_a_gpu():
    cfg = synth.UNETS["sd15_video"]
    c = lcb.make_unet_config(cfg)
    lcb.lc_unet_check_config(c)
    assert ctypes.sizeof(lcb.lc_unet_config) == 4 * 19
    assert ctypes.sizeof(lcb.lc_unet_weights) == 8 * (2 + 6 * 12 + 8 * 26 + 4 + 4 + 2 + 2)
    assert lcb.lc_unet_entry_bytes(c) == cfg.N * cfg.H * cfg.W * cfg.C1 * 4
    ws = lcb.lc_unet_workspace_bytes(c)
    assert ws > 2 * lcb.lc_unet_entry_bytes(c)   # the device slots are part of it
    more = lcb.make_unet_config(cfg, dev_slots=3)
    assert lcb.lc_unet_workspace_bytes(more) - ws == lcb.lc_unet_entry_bytes(c)
    # feature chunk: what lives inside a block scales with the chunk, what passes between blocks does not
    by_chunk = {fc: lcb.lc_unet_chunk_workspace_bytes(c, fc) for fc in (0, 1, 2, 4, 8, 16, 32, 40)}
    assert by_chunk[0] == by_chunk[32] == by_chunk[40] == ws
    assert by_chunk[1] < by_chunk[2] < by_chunk[4] < by_chunk[8] < by_chunk[16] < by_chunk[32]
    inside = {fc: by_chunk[fc] - by_chunk[1] for fc in (2, 4, 8, 16, 32)}
    for fc in (4, 8, 16, 32):   # linear in the chunk, up to the 256-byte rounding of each buffer
        assert abs(inside[fc] - (fc - 1) * inside[2]) <= 1 << 14, fc
    assert by_chunk[4] < 0.6 * ws
    assert lcb.lc_unet_chunk_workspace_bytes(c, -1) == 0
    for field, value in [("H", 6), ("C", 100), ("C1", 4096), ("groups", 7), ("head_dim", 24), ("C_lat", 17), ("ff_mult", 5), ("F", 0),
                         ("F", 64), ("ctx_dim", 100), ("dev_slots", 0), ("host_slots", 65), ("gn_eps", 0.0), ("ln_eps", -1.0)]:
        bad = lcb.make_unet_config(cfg)
        setattr(bad, field, value)
        with pytest.raises(lcb.LcError) as e:
            lcb.lc_unet_check_config(bad)
        assert e.value.status == lcb.LC_ERR_SHAPE, field
        assert lcb.lc_unet_workspace_bytes(bad) == 0 and lcb.lc_unet_entry_bytes(bad) == 0
    bad = lcb.make_unet_config(cfg)
    bad.dtype = 7
    with pytest.raises(lcb.LcError) as e:
        lcb.lc_unet_check_config(bad)
    assert e.value.status == lcb.LC_ERR_ARG
    for name in synth.UNETS:
        lcb.lc_unet_check_config(lcb.make_unet_config(synth.UNETS[name]))
