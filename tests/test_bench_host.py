"""Host-side logic of bench.py (no GPU): the HBM-traffic figure comes from the committed rocprofv3
summaries and only from the one that profiles the very instantiation that was timed; the roof that
bounds each configuration; the refusal of more than one GPU."""
import subprocess
import sys
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parent.parent
sys.path.insert(0, str(ROOT))
import bench  # noqa: E402
from paper_2603_01960_amd.workloads import WORKLOADS  # noqa: E402


def test_traffic_is_read_from_the_profile_of_the_same_instantiation():
    got, src = bench.profiled_traffic("C4", "bf16", 128, 256, 64)          # the heuristic's tile on C4
    assert src == "profiles/sdpa_fwd_C4_bf16.md" and 500e6 < got < 600e6
    text = (ROOT / src).read_text()
    assert f"| total | | {got / 1e6:.1f} MB |" in text          # the figure is the file's own "total" row
    got64, src64 = bench.profiled_traffic("C4", "bf16", 128, 128, 64)
    assert src64.endswith("_tile_128x64.md") and 500e6 < got64 < 600e6
    got32, src32 = bench.profiled_traffic("C4", "bf16", 128, 128, 32)
    assert src32.endswith("_tile_128x32.md") and got32 != got
    # no committed counter run for that tile, dtype or head dim: no figure, and the reason says which kernel
    for args in (("C4", "bf16", 128, 64, 32), ("C4", "f16", 128, 256, 64), ("C2", "bf16", 64, 128, 64), ("C9", "bf16", 128, 128, 64)):
        val, why = bench.profiled_traffic(*args)
        assert val is None and "no committed counter run" in why and f"T_M={args[3]},T_N={args[4]}" in why
    # a profile of another tile under the workload's plain name is not taken for this tile
    val, _ = bench.profiled_traffic("C3", "bf16", 64, 128, 64)
    assert val is None


def test_every_committed_forward_profile_parses():
    import re
    seen = 0
    for path in sorted((ROOT / "profiles").glob("sdpa_fwd_C*_*.md")):
        m = re.match(r"sdpa_fwd_(C\d)_(f16|bf16)(?:_tile_(\d+)x(\d+))?\.md$", path.name)
        if not m or "default_bench_command" in path.name or "linear_grid" in path.name:
            continue
        k = re.search(r"sdpa_fwd_kernelI(?:DF16_|DF16b)Li(\d+)ELi(\d+)ELi(\d+)E", path.read_text())
        assert k, path.name
        D, tm, tn = int(k.group(1)), 32 * int(k.group(2)), int(k.group(3))
        if m.group(3):
            assert (tm, tn) == (int(m.group(3)), int(m.group(4))), path.name      # the file name tells the truth
        val, src = bench.profiled_traffic(m.group(1), m.group(2), D, tm, tn)
        assert val is not None and src == "profiles/" + path.name, path.name
        assert val >= 0.99 * WORKLOADS[m.group(1)].compulsory_bytes(2)
        seen += 1
    assert seen >= 8


def test_the_roof_that_bounds_each_configuration():
    r = {n: bench.roofline_of(w, 1.0) for n, w in WORKLOADS.items()}
    assert r["C1"]["bound"] == "latency" and r["C1"]["frac"] is None
    assert r["C3"]["bound"] == "hbm" and r["C3"]["peak"] == 8000.0
    for n in ("C2", "C4", "C5"):
        assert r[n]["bound"] == "mfma" and r[n]["peak"] == 2500.0
    w = WORKLOADS["C4"]
    assert bench.roofline_of(w, w.flops / 2500e12 * 1e3)["frac"] == pytest.approx(1.0, abs=1e-4)
    assert bench.roofline_of(WORKLOADS["C3"], WORKLOADS["C3"].compulsory_bytes(2) / 8000e9 * 1e3)["frac"] == pytest.approx(1.0, abs=1e-4)


def test_more_than_one_gpu_is_refused_with_a_message():
    res = subprocess.run([sys.executable, str(ROOT / "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert res.returncode == 2 and "ONE GPU" in res.stderr and res.stdout.strip() == ""


def test_the_grid_mode_walks_the_eighty_points_of_the_papers_grid():
    """Section 4.3: S in {512 ... 8192} x D in {64, 96, 128, 160} x FP16/BF16 x causal / non-causal."""
    import bench

    assert len(bench.GRID_HEAD_DIMS) * len(bench.GRID_SEQ_LENS) * len(bench.GRID_DTYPES) * 2 == 80
    assert bench.GRID_HEAD_DIMS == (64, 96, 128, 160) and bench.GRID_SEQ_LENS == (512, 1024, 2048, 4096, 8192)
