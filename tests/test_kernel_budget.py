"""Register budget of the headline instantiations, checked on the compiler's own output (no GPU).

The 32-row K/V tile kernels at D = 128 are compiled for 168 registers per lane (three wavefronts per
SIMD) and sit at the edge of that budget: the prologue parks a few loop-invariant values in scratch
memory, which is fine, but a scratch access INSIDE the unmasked main loop (a spilled Q fragment
reloaded per tile) costs about a tenth of the throughput and nothing else shows it -- results stay
right, the resource summary barely moves.  Harmless-looking edits of the prologue have caused exactly
that, so the assembly is inspected here.
"""
import re
import shutil
import subprocess
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parents[1]
CSRC = ROOT / "paper_2603_01960_amd" / "csrc"
HIPCC = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"


def kernels_of(asm: str):
    """name -> lines, for every sdpa_fwd_kernel in an assembly listing."""
    out, name = {}, None
    for line in asm.split("\n"):
        m = re.match(r"^(_ZN5tsdpa15sdpa_fwd_kernel\S+):", line)
        if m:
            name = m.group(1)
            out[name] = []
        elif name is not None:
            out[name].append(line)
            if "s_endpgm" in line:
                name = None
    return out


def loops_of(lines):
    """[(header label, lines of the blocks of that loop)] for the depth-1 loops, in program order.  The
    compiler annotates every block label with the loop it belongs to."""
    loops, current = [], None
    for line in lines:
        if re.match(r"^(\.LBB\d+_\d+:|; %bb\.\d+:)", line) is not None:
            current = None
            if re.search(r"Loop Header: Depth=1", line):
                loops.append((re.match(r"^\.(LBB\d+_\d+):", line).group(1)[1:], []))      # "BB6_9"
                current = loops[-1][1]
            else:
                for header, body in loops:
                    if re.search(r"in Loop: Header=" + re.escape(header) + r"\b", line):
                        current = body
        elif current is not None:
            current.append(line)
    return loops


def scratch_ops_in_main_loop(lines):
    """Scratch loads/stores in the first loop that holds MFMAs (the unmasked main loop; a loop without any is
    the one in which a wavefront without query rows only keeps up the tile loads)."""
    for header, body in loops_of(lines):
        if any("v_mfma" in line for line in body):
            return sum("scratch_" in line for line in body)
    raise AssertionError("no loop with MFMAs found")


@pytest.mark.skipif(not Path(HIPCC).exists(), reason="hipcc not available")
@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_main_loop_of_the_headline_kernels_touches_no_scratch_memory(dtype, tmp_path):
    from paper_2603_01960_amd import build as lib_build

    kernels = {}
    # 32-row and 64-row K/V tiles are separate translation units, each with the flags the build gives it
    for src in (CSRC / f"sdpa_fwd_{dtype}_d128.hip", CSRC / f"sdpa_fwd_{dtype}_d128_tn64.hip",
                CSRC / f"sdpa_fwd_{dtype}_d160_tn64.hip"):
        asm = tmp_path / (src.stem + ".s")
        cmd = [HIPCC, *lib_build.FLAGS, *lib_build.extra_flags(src), "-S", "--cuda-device-only",
               str(src), "-o", str(asm)]
        subprocess.run(cmd, check=True, capture_output=True, timeout=600)
        kernels.update(kernels_of(asm.read_text()))
    # the square problem (last template argument 0) on 128- and 256-row query tiles: the configurations the bench times
    checked = 0
    for name, lines in kernels.items():
        m = re.search(r"Li128ELi(4|8)ELi(32|64|128)ELi\dELi0E", name)
        if not m:
            continue
        checked += 1
        n = scratch_ops_in_main_loop(lines)
        assert n == 0, f"{name}: {n} scratch accesses inside the main loop (T_M = {32 * int(m.group(1))}, T_N = {m.group(2)})"
    assert checked == 4, f"expected the 128x32, 128x64, 128x128 and 256x64 instantiations, found {checked}"
    # D = 160 on 64-row K/V tiles (the heuristic's tiles there from S = 512): no scratch access in the main loop
    checked = 0
    for name, lines in kernels.items():
        m = re.search(r"Li160ELi(4|8)ELi64ELi\dELi0E", name)
        if m:
            checked += 1
            n = scratch_ops_in_main_loop(lines)
            assert n == 0, f"{name}: {n} scratch accesses inside the main loop (D = 160, T_M = {32 * int(m.group(1))})"
    assert checked == 2, f"expected the 128x64 and 256x64 instantiations at D = 160, found {checked}"
    # every instantiation has two loops with MFMAs (unmasked tiles, masked tiles) and, in the square problem, at
    # most one without (wavefronts past the end of a ragged sequence): a buffer descriptor the compiler takes for
    # lane-dependent turns each of its loads into a loop over distinct descriptors (this happened to the
    # paged-cache variant and cost a quarter of its speed on short runs)
    for name, lines in kernels.items():
        loops = loops_of(lines)
        with_mfma = sum(any("v_mfma" in line for line in body) for _, body in loops)
        square = re.search(r"ELi0EEEv", name) is not None
        assert with_mfma <= 2 and len(loops) - with_mfma <= (1 if square else 0), \
            f"{name}: {len(loops)} loops in the assembly, {with_mfma} with MFMAs (a load wrapped in a descriptor loop?)"
