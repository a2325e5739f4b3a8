"""The conv kernel's workgroup barriers leave a counted number of vector-memory loads in flight
(weights of later steps, which go to LDS directly, and the halo packets of the next slab) and rely on
the loads issued in a tap being exactly those the source spells out. The weights of step s + 1 are the
last loads of an earlier tap; before the barrier that ends tap s they must have landed, so the wait
may leave at most the loads of the taps since then outstanding. This test compiles the kernel file to
gfx950 assembly and checks that, for every 3x3 instantiation and every barrier interval of its main
loop, against the loads the compiler actually emitted."""
import re
import subprocess
from pathlib import Path

import pytest

from paper_2510_05367_amd import build as lcbuild

CSRC = Path(lcbuild.__file__).parent / "csrc"


@pytest.fixture(scope="module")
def gemm_asm(tmp_path_factory):
    out = tmp_path_factory.mktemp("asm") / "lc_gemm.s"
    cmd = [lcbuild._hipcc(), *lcbuild.FLAGS, "-S", "--cuda-device-only", str(CSRC / "lc_gemm.hip"), "-o", str(out)]
    subprocess.run(cmd, check=True, capture_output=True)
    return out.read_text()


def test_barrier_waits_match_emitted_loads(gemm_asm):
    names = [n for n in re.findall(r"^(_ZN2lc11gemm_kernel[^:\n]*):", gemm_asm, flags=re.M) if "Li9E" in n]
    assert len(names) >= 10
    for name in names:
        start = gemm_asm.index("\n" + name + ":")
        body = gemm_asm[start:gemm_asm.index("s_endpgm", start)]
        assert "scratch_" not in body, f"{name}: register spills"
        parts = body.split("s_barrier")[:-1]
        assert len(parts) >= 1 + 2 * 9  # prologue + at least two slab bodies of nine taps
        nloop = (len(parts) - 1) // 9 * 9  # what follows the main loop (the hand-over of the K halves) is not counted
        issued, waits = [], []
        for part in parts:
            issued.append(len(re.findall(r"global_load_lds_dwordx4", part)) + len(re.findall(r"global_load_dword", part)))
            waits.append([int(v) for v in re.findall(r"s_waitcnt vmcnt\((\d+)\)", part)])
        # the weight loads run kWBuf - 1 steps ahead: those of step s + 1 are kWBuf - 3 taps old at the end of tap s
        ahead = int(re.search(r"constexpr int kWBuf = (\d+);", (CSRC / "lc_gemm.hip").read_text()).group(1)) - 1
        exact = 0
        for k in range(1, nloop + 1):
            assert len(waits[k]) == 1, (name, k, waits[k])  # the explicit one before the barrier, nothing earlier
            younger = sum(issued[max(k - (ahead - 2), 0):k + 1])
            assert waits[k][0] <= younger, (name, k, issued[k - 1:k + 1], waits[k])
            exact += waits[k][0] == younger
        # and it does not wait for more than it must, except where the loop runs out of steps
        assert exact >= nloop - 5, (name, exact, nloop)
