"""The conv kernel's workgroup barriers leave a counted number of vector-memory loads in flight
(the weights of step s + 2 and the halo packet requested in the same tap) and rely on the loads
issued in a tap being exactly those the source spells out. This test compiles the kernel file to
gfx950 assembly and checks, for every 3x3 instantiation and every barrier interval of its main loop,
that the count in the wait before the barrier equals the loads the compiler actually emitted."""
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
        for k, part in enumerate(parts[1:1 + nloop], start=1):
            dma = len(re.findall(r"global_load_lds_dwordx4", part))
            loads = len(re.findall(r"global_load_dword", part))
            waits = [int(v) for v in re.findall(r"s_waitcnt vmcnt\((\d+)\)", part)]
            assert len(waits) == 1, (name, k, waits)  # the explicit one before the barrier, nothing earlier
            # either everything must have landed, or exactly this interval's loads may stay in flight
            assert waits[0] in (0, dma + loads), (name, k, dma, loads, waits)
            if dma == 0:
                assert waits[0] == 0, (name, k)
