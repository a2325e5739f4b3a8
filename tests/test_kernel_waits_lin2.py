"""The dense-row linear kernel (lc_lin2.hip) streams both operands global -> LDS directly into a ring of two stages:
the loads of step s + 1 are issued right after the barrier of step s, and the wait before a barrier is for every load in
flight (the only ones are those the step needs). Two workgroups are budgeted per compute unit. This test compiles the
kernel to gfx950 assembly and checks, for every instantiation: every barrier is preceded by a full wait for memory and
for the LDS reads (the stage about to be overwritten was read before it), the loads come in whole stages, nothing
spills, and the registers leave room for two workgroups on a compute unit."""
import re
import subprocess
from pathlib import Path

import pytest

from paper_2510_05367_amd import build as lcbuild

CSRC = Path(lcbuild.__file__).parent / "csrc"


@pytest.fixture(scope="module")
def asm(tmp_path_factory):
    out = tmp_path_factory.mktemp("asm") / "lc_lin2.s"
    cmd = [lcbuild._hipcc(), *lcbuild.FLAGS, "-S", "--cuda-device-only", str(CSRC / "lc_lin2.hip"), "-o", str(out)]
    subprocess.run(cmd, check=True, capture_output=True)
    return out.read_text()


def kernels(asm):
    names = re.findall(r"^(_ZN2lc11lin2_kernelI(?:f|DF16b)Li(\d)ELb[01]EE[^:\n]*):", asm, flags=re.M)
    # {fp32, bf16 output} x {160, 128 channels} x {dense, mapped rows}
    assert len(names) == 8
    for name, nt in names:
        start = asm.index("\n" + name + ":")
        yield name, int(nt), asm[start:asm.index(".Lfunc_end", start)]


def test_ring_waits_match_emitted_loads(asm):
    for name, nt, body in kernels(asm):
        assert "scratch_" not in body, f"{name}: register spills"
        per_step = 4 + nt  # global -> LDS instructions per wavefront per stage: x tile, W tile
        lines = [l.strip() for l in body.splitlines() if l.strip() and not l.strip().startswith(";")]
        bars = [i for i, l in enumerate(lines) if l.startswith("s_barrier")]
        assert bars, name
        for i in bars:
            assert re.fullmatch(r"s_waitcnt vmcnt\(0\) lgkmcnt\(0\)", lines[i - 1]), (name, lines[i - 1])
        # prologue: one stage; loop body: one (the compiler may duplicate the loop body's group, never split it)
        dma = len(re.findall(r"\bglobal_load_lds_dwordx4\b", body))
        assert dma % per_step == 0 and dma >= 2 * per_step, (name, dma, per_step)
    # two workgroups per compute unit: 256 registers per lane at most, and the LDS of both fits
    counts = re.findall(r"\.name:\s+(_ZN2lc11lin2_kernel\S*)\n(?:.*\n)*?\s+\.vgpr_count:\s+(\d+)", asm)
    assert len(counts) == 8
    for name, n in counts:
        assert int(n) <= 256, name
