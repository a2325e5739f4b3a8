"""The loader wavefronts of the specialised-wavefront conv kernel (lc_convws.hip) end every tap with a
wait that leaves a counted number of vector-memory loads in flight: the weights of step s + kwLead must
have landed, and they were the last loads of tap s + kwLead - kwAhead, so the wait may leave at most the
loads of the taps since then outstanding. A count that is too large would let the contracting wavefronts
read a weight tile that is still on its way. This test compiles the kernel to gfx950 assembly and checks
every such wait against the loads the compiler actually emitted, and that the contracting wavefronts'
main loop touches no global memory, spills nothing and waits for no LDS read before its barriers."""
import re
import subprocess
from pathlib import Path

import pytest

from paper_2510_05367_amd import build as lcbuild

CSRC = Path(lcbuild.__file__).parent / "csrc"
SRC = (CSRC / "lc_convws.hip").read_text()


def const(name):
    return int(re.search(rf"constexpr int {name} = (\d+);", SRC).group(1))


@pytest.fixture(scope="module")
def ws_asm(tmp_path_factory):
    out = tmp_path_factory.mktemp("asm") / "lc_convws.s"
    cmd = [lcbuild._hipcc(), *lcbuild.FLAGS, "-S", "--cuda-device-only", str(CSRC / "lc_convws.hip"), "-o", str(out)]
    subprocess.run(cmd, check=True, capture_output=True)
    return out.read_text()


def kernels(asm):
    names = re.findall(r"^(_ZN2lc14conv_ws_kernel[^:\n]*):", asm, flags=re.M)
    assert len(names) == 2  # plain and concat loader
    for name in names:
        start = asm.index("\n" + name + ":")
        yield name, asm[start:asm.index(".Lfunc_end", start)]


def n_loads(text):
    return len(re.findall(r"\bglobal_load_lds_dwordx4\b", text)) + len(re.findall(r"\bglobal_load_dword(x\d)?\b", text))


def test_no_spills_and_two_waves_per_simd(ws_asm):
    for name, body in kernels(ws_asm):
        assert "scratch_" not in body, f"{name}: register spills"
    for m in re.finditer(r"\.vgpr_count:\s+(\d+)", ws_asm):
        assert int(m.group(1)) <= 256  # eight wavefronts per workgroup: two per SIMD


def test_loader_waits_match_emitted_loads(ws_asm):
    span = const("kwBuf") - 1 - const("kwLead")  # taps whose loads are younger than the awaited weights, the current one included
    assert span >= 1
    for name, body in kernels(ws_asm):
        parts = body.split("s_barrier")[:-1]
        checked = exact = 0
        run = []  # loads of the loader taps that precede this one in the text without interruption
        for part in parts:
            lines = [l for l in part.rstrip().splitlines() if l.strip() and not l.strip().startswith(";")]
            waits = [int(v) for v in re.findall(r"s_waitcnt vmcnt\((\d+)\)", part)]
            # a tap of a loader main loop ends with its explicit wait, right before the barrier
            if "v_mfma" in part or not lines or "s_waitcnt vmcnt" not in lines[-1]:
                run = []
                continue
            run.append(n_loads(part))
            if len(run) < span:
                continue  # its predecessors are in another block: not checked here
            younger = sum(run[-span:])
            # never more loads left outstanding than were issued after the awaited weights
            assert waits[-1] <= younger, (name, waits[-1], run[-span:])
            exact += waits[-1] == younger
            checked += 1
        assert checked >= 16, (name, checked)
        # and it does not wait for more than it must (the prologue's wait is the exception)
        assert exact >= checked - 2, (name, exact, checked)


def test_contracting_loop_is_lds_and_mfma_only(ws_asm):
    for name, body in kernels(ws_asm):
        parts = body.split("s_barrier")
        loop = [p for p in parts if p.count("v_mfma") >= 20]
        assert len(loop) >= 9, name  # nine taps of the unrolled slab
        for p in loop:
            assert n_loads(p) == 0 and "global_store" not in p, name
            # the barrier that ends a tap is not preceded by a wait for all LDS reads: the requests for the
            # next step stay in flight across it
            last = [l for l in p.rstrip().splitlines() if l.strip() and not l.strip().startswith(";")][-1]
            assert "lgkmcnt(0)" not in last, (name, last)
