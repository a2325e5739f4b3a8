"""Register budgets that the design counts on, read from the compiled gfx950 code objects' metadata:
  * the GroupNorm finalize kernel stays within 32 vector registers - the 3x3 convolution kernel runs two
    wavefronts of at most 240 registers per SIMD, which leaves exactly that many of the 512, so a finalize
    launched on one stream starts beside the other stream's convolution instead of behind it;
  * the convolution kernel itself stays within those 240;
  * the conv_in tile kernel and the MFMA temporal-attention kernels stay small enough for several workgroups
    per compute unit (their speed comes from workgroups overlapping each other's phases), and spill nothing."""
import re
import subprocess
from pathlib import Path

import pytest

from paper_2510_05367_amd import build as lcbuild

CSRC = Path(lcbuild.__file__).parent / "csrc"


def kernel_meta(tmp, src):
    out = tmp / (src + ".s")
    cmd = [lcbuild._hipcc(), *lcbuild.FLAGS, "-S", "--cuda-device-only", str(CSRC / src), "-o", str(out)]
    subprocess.run(cmd, check=True, capture_output=True)
    meta = {}
    for m in re.finditer(r"\.amdhsa_kernel (\S+)(.*?)\.end_amdhsa_kernel", out.read_text(), flags=re.S):
        body = m.group(2)
        vg = int(re.search(r"\.amdhsa_next_free_vgpr (\d+)", body).group(1))
        scratch = int(re.search(r"\.amdhsa_private_segment_fixed_size (\d+)", body).group(1))
        meta[m.group(1)] = (vg, scratch)
    return meta


@pytest.fixture(scope="module")
def tmp(tmp_path_factory):
    return tmp_path_factory.mktemp("asm")


def pick(meta, *needles):
    hits = {k: v for k, v in meta.items() if all(n in k for n in needles)}
    assert hits, needles
    return hits


def test_finalize_fits_beside_the_convolution(tmp):
    fin = pick(kernel_meta(tmp, "lc_norm.hip"), "gn_finalize_kernel")
    for name, (vg, scratch) in fin.items():
        assert vg <= 32 and scratch == 0, (name, vg, scratch)
    ws = pick(kernel_meta(tmp, "lc_convws.hip"), "conv_ws_kernel")
    assert len(ws) == 2
    for name, (vg, scratch) in ws.items():
        assert vg <= 240 and scratch == 0, (name, vg, scratch)


def test_small_kernels_stay_small(tmp):
    conv = kernel_meta(tmp, "lc_conv.hip")
    for name, (vg, scratch) in pick(conv, "conv_in_tile_kernel").items():
        assert vg <= 128 and scratch == 0, (name, vg, scratch)  # four workgroups of four wavefronts per compute unit
    attn = kernel_meta(tmp, "lc_attn.hip")
    for name, (vg, scratch) in pick(attn, "temporal_attn_mfma_kernel").items():
        assert vg <= 64 and scratch == 0, (name, vg, scratch)
    for name, (vg, scratch) in pick(attn, "temporal_attn_mfma32_kernel").items():
        assert vg <= 128 and scratch == 0, (name, vg, scratch)
