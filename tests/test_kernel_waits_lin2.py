"""The dense-row linear kernel (lc_lin2.hip) streams both operands global -> LDS directly into a ring of three
stages: the loads of step s + 2 are issued while step s is contracted, and the wait before the barrier of a step may
leave exactly the loads of step s + 1 in flight (none at the last step). A count that is too large would let a
wavefront contract a stage that is still on its way. This test compiles the kernel to gfx950 assembly and checks,
for every instantiation: every barrier is preceded by such a wait and by a wait for the LDS reads (the stage about to
be overwritten was read before it), the loads per step are what the wait assumes, nothing spills, stores come only
after the last barrier, and the epilogue's stores wait for memory at most once per half tile (the residual)."""
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
    names = re.findall(r"^(_ZN2lc11lin2_kernelI(?:f|DF16b)Li(\d)ELi(\d)ELb[01]ELi(\d)E[^:\n]*):", asm, flags=re.M)
    # {fp32, bf16 output} x {160, 128 channels} x {dense, mapped rows} x {256 rows / 3 stages, 128 / 3, 128 / 2}
    assert len(names) == 24
    for name, nt, mr, st in names:
        start = asm.index("\n" + name + ":")
        yield name, int(nt), int(mr), int(st), asm[start:asm.index(".Lfunc_end", start)]


def test_ring_waits_match_emitted_loads(asm):
    for name, nt, mr, st, body in kernels(asm):
        assert "scratch_" not in body, f"{name}: register spills"
        per_step = 4 * mr + nt  # global -> LDS instructions per wavefront per stage: x tile, W tile
        lines = [l.strip() for l in body.splitlines() if l.strip() and not l.strip().startswith(";")]
        bars = [i for i, l in enumerate(lines) if l.startswith("s_barrier")]
        assert bars, name
        waits = set()
        for i in bars:
            m = re.fullmatch(r"s_waitcnt vmcnt\((\d+)\) lgkmcnt\(0\)", lines[i - 1])
            assert m, (name, lines[i - 1])
            waits.add(int(m.group(1)))
        # three stages: the loads of the next step may stay in flight (none at the last step); two stages: the loads
        # awaited are the youngest, the wait is for everything
        assert waits == ({0, per_step} if st == 3 else {0}), (name, waits)
        # prologue: ST - 1 stages; loop body: one (the compiler may duplicate the loop body's group, never split it)
        dma = len(re.findall(r"\bglobal_load_lds_dwordx4\b", body))
        assert dma % per_step == 0 and dma >= st * per_step, (name, dma, per_step)
        # stores only behind the last barrier; there, at most one full wait per half tile (for its residual)
        # (text order follows execution order in the three-stage form only: the two-stage loop comes out rotated)
        if st == 3:
            head, tail = "\n".join(lines[:bars[-1]]), "\n".join(lines[bars[-1] + 1:])
            assert "global_store" not in head and "global_store" in tail, name
            assert "global_load_lds" not in tail, name
            assert len(re.findall(r"s_waitcnt vmcnt\(0\)", tail)) <= mr, (name, tail.count("vmcnt(0)"))
    # the two-stage form is budgeted for two workgroups per compute unit
    for m in re.finditer(r"\.name:\s+(_ZN2lc11lin2_kernel\S*ELi2EE\S*)\n(?:.*\n)*?\s+\.vgpr_count:\s+(\d+)", asm):
        assert int(m.group(2)) <= 256, m.group(1)
