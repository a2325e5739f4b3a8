"""The contracting wavefronts of the specialised-wavefront conv kernel (lc_convws.hip) request the weight
tiles themselves (global -> LDS directly, kwAhead steps ahead) and end every step with a wait that leaves
a counted number of those requests in flight: the weights of step s + kwLead must have landed, and they
were requested kwAhead - kwLead steps ago, so the wait may leave at most the requests of the steps since
then outstanding. A count that is too large would let a wavefront read a weight tile that is still on its
way. This test compiles the kernel to gfx950 assembly and checks every such wait against the loads the
compiler actually emitted, that the contracting loop issues no other global-memory operation, spills
nothing and waits for no LDS read before its barriers."""
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


def test_step_waits_match_emitted_requests(ws_asm):
    assert const("kwBuf") - 1 - const("kwLead") == 1  # requests younger than the awaited weights: those of the current step
    per_step = 160 * 8 // 256  # instructions per contracting wavefront per step
    for name, body in kernels(ws_asm):
        parts = body.split("s_barrier")
        steps = [p for p in parts if p.count("v_mfma") >= 20]
        assert len(steps) >= 18, name  # nine unrolled taps of the main loop and of the last slab
        seen = set()
        for p in steps:
            lines = [l for l in p.rstrip().splitlines() if l.strip() and not l.strip().startswith(";")]
            dma = len(re.findall(r"\bglobal_load_lds_dwordx4\b", p))
            assert n_loads(p) == dma and "global_store" not in p, name  # weight requests only
            # the barrier that ends a step is preceded by the explicit wait for the weights, and by no wait for
            # all LDS reads: the fragment requests for the next step stay in flight across it
            m = re.fullmatch(r"\s*s_waitcnt vmcnt\((\d+)\)\s*", lines[-1])
            assert m, (name, lines[-1])
            wait = int(m.group(1))
            assert wait <= dma, (name, wait, dma)  # never more left outstanding than were issued after the awaited weights
            seen.add((wait, dma))
        assert seen == {(per_step, per_step), (0, 0)}, (name, seen)
        # the prologue: kwAhead steps requested, the last kwAhead - kwLead may stay in flight
        pro = next(p for p in parts if len(re.findall(r"\bglobal_load_lds_dwordx4\b", p)) == (const("kwBuf") - 1) * per_step)
        waits = [int(v) for v in re.findall(r"s_waitcnt vmcnt\((\d+)\)", pro)]
        assert waits and waits[-1] <= (const("kwBuf") - 1 - const("kwLead")) * per_step, (name, waits)
