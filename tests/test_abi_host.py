"""CPU-side checks of the C-ABI: the library loads, exports what include/tiled_sdpa.h declares,
and rejects bad arguments before anything reaches a GPU (no compute calls here)."""
import ctypes
import math
import re
from pathlib import Path

import pytest

from paper_2603_01960_amd import binding

ROOT = Path(__file__).resolve().parent.parent
HEADER = ROOT / "include" / "tiled_sdpa.h"


@pytest.fixture(scope="module")
def lib():
    if not binding.library_path().exists():
        from paper_2603_01960_amd import build
        build.build(force=True)
    return binding.load_library()


def declared_functions():
    text = re.sub(r"/\*.*?\*/", "", HEADER.read_text(), flags=re.S)
    return sorted(set(re.findall(r"\b(tiled_sdpa_\w+)\s*\(", text)))


def test_header_and_binding_agree_on_the_entry_points():
    assert declared_functions() == sorted(binding.EXPORTS)


def test_library_exports_every_declared_symbol(lib):
    for name in declared_functions():
        assert hasattr(lib, name), name


def test_version_and_status_strings(lib):
    assert binding.version() >= 100
    seen = set()
    for code in range(0, 12):
        s = binding.status_string(code)
        assert s and s != "unknown status"
        seen.add(s)
    assert len(seen) == 12
    assert binding.status_string(12345) == "unknown status"


OK, NULL, SHAPE, DTYPE, BAD_D, ALIGN, TILE, SCALE = 0, 1, 2, 3, 4, 5, 6, 7
P = 0x1000  # fake, aligned, never dereferenced: every case below fails validation before launch


@pytest.mark.parametrize("kwargs,expect", [
    (dict(dtype=2), DTYPE),
    (dict(dtype=-1), DTYPE),
    (dict(D=80), BAD_D),
    (dict(D=192), BAD_D),
    (dict(D=0), BAD_D),
    (dict(B=-1), SHAPE),
    (dict(S=-5), SHAPE),
    (dict(B=1 << 20, H=1 << 10, S=1 << 20), SHAPE),
    (dict(B=0), OK),
    (dict(S=0), OK),
    (dict(S=0, q=None, o=None), OK),
    (dict(q=None), NULL),
    (dict(k=None), NULL),
    (dict(v=None), NULL),
    (dict(o=None), NULL),
    (dict(q=P + 8), ALIGN),
    (dict(o=P + 2), ALIGN),
    (dict(lse=P + 2), ALIGN),
    (dict(tile_m=32, tile_n=64), TILE),
    (dict(tile_m=128, tile_n=0), TILE),
    (dict(tile_m=128, tile_n=256), TILE),
    (dict(tile_m=256, tile_n=32), TILE),           # 256 query rows come with 64-row K/V tiles only
    (dict(tile_m=256, tile_n=128), TILE),
    (dict(tile_m=512, tile_n=64), TILE),
    (dict(D=160, tile_m=128, tile_n=128), TILE),
    (dict(D=160, tile_m=64, tile_n=128), TILE),     # 128-row K/V tiles exist up to D = 128 (LDS)
    (dict(D=128, tile_m=64, tile_n=128, S=0), OK),
    (dict(D=96, tile_m=128, tile_n=128, S=0), OK),
    (dict(D=64, tile_m=64, tile_n=128, S=0), OK),
    (dict(D=160, tile_m=64, tile_n=64, S=0), OK),
    (dict(S=1 << 23, D=128), SHAPE),
    (dict(scale=math.inf), SCALE),
    (dict(scale=-math.inf), SCALE),
])
def test_validation_order_and_codes(lib, kwargs, expect):
    a = dict(q=P, k=P, v=P, o=P, lse=None, B=1, H=2, S=128, D=64, scale=0.125, dtype=0,
             stream=None, tile_m=0, tile_n=0, flags=0)
    a.update(kwargs)
    st = binding.tiled_sdpa_fwd_ex(a["q"], a["k"], a["v"], a["o"], a["lse"], a["B"], a["H"], a["S"],
                                   a["D"], a["scale"], a["dtype"], a["stream"], a["tile_m"],
                                   a["tile_n"], a["flags"])
    assert st == expect, binding.status_string(st)


def test_plain_entry_point_validates_too(lib):
    assert binding.tiled_sdpa_fwd(None, P, P, P, None, 1, 1, 16, 64, 0.125, 0, None) == NULL
    assert binding.tiled_sdpa_fwd(P, P, P, P, None, 1, 1, 16, 80, 0.125, 0, None) == BAD_D
    assert binding.tiled_sdpa_fwd(None, P, P, P, None, 1, 1, 16, 96, 0.125, 0, None) == NULL
    assert binding.tiled_sdpa_fwd(None, None, None, None, None, 0, 4, 16, 64, 0.125, 1, None) == OK


WORKSPACE, SPLITS = 9, 10


@pytest.mark.parametrize("kwargs,expect", [
    (dict(dtype=7), DTYPE),
    (dict(D=72), BAD_D),
    (dict(Sq=-1), SHAPE),
    (dict(Skv=-1), SHAPE),
    (dict(Skv=0), SHAPE),                          # a softmax over no keys
    (dict(Skv=0, Sq=0), OK),
    (dict(Sq=0, q=None, o=None), OK),
    (dict(Sq=300, Skv=299, flags=8), SHAPE),       # causal needs Skv >= Sq
    (dict(Sq=300, Skv=299, flags=0, q=None), NULL),
    (dict(Skv=1 << 23), SHAPE),
    (dict(B=1 << 12, H=1 << 12, Sq=64), SHAPE),    # grid with the maximum split count overflows
    (dict(k=None), NULL),
    (dict(v=P + 4), ALIGN),
    (dict(tile_m=128, tile_n=128), TILE),          # the general kernel has no 128-row K/V tile
    (dict(tile_m=256, tile_n=32), TILE),           # the 256-row query tile comes with 64-row K/V tiles only
    (dict(tile_m=0, tile_n=64), TILE),
    (dict(scale=math.inf), SCALE),
    (dict(splits=-1), SPLITS),
    (dict(splits=129), SPLITS),
    (dict(splits=2, ws=None), WORKSPACE),
    (dict(splits=2, ws=P + 8, ws_bytes=1 << 30), WORKSPACE),
    (dict(splits=4, ws=P, ws_bytes=4 * 2 * 4 * 5 * 66 * 4 - 1), WORKSPACE),
])
def test_kv_entry_point_validation_order_and_codes(lib, kwargs, expect):
    a = dict(q=P, k=P, v=P, o=P, lse=None, B=2, H=4, Sq=5, Skv=700, D=64, scale=0.125, dtype=1,
             stream=None, tile_m=0, tile_n=0, flags=0, splits=1, ws=None, ws_bytes=0)
    a.update(kwargs)
    st = binding.tiled_sdpa_fwd_kv(a["q"], a["k"], a["v"], a["o"], a["lse"], a["B"], a["H"], a["Sq"], a["Skv"],
                                   a["D"], a["scale"], a["dtype"], a["stream"], a["tile_m"], a["tile_n"],
                                   a["flags"], a["splits"], a["ws"], a["ws_bytes"])
    assert st == expect, binding.status_string(st)


@pytest.mark.parametrize("kwargs,expect", [
    (dict(), NULL),                                 # q = None below: everything before the pointers passes
    (dict(Hkv=3), SHAPE),                           # 8 query heads over 3 key/value heads
    (dict(Hkv=0), SHAPE),
    (dict(Hkv=-2), SHAPE),
    (dict(Hkv=16), SHAPE),                          # more key/value heads than query heads
    (dict(H=0, Hkv=0), OK),                         # empty problem
    (dict(Hkv=8), NULL),                            # Hkv = H is tiled_sdpa_fwd_kv
    (dict(Hkv=1), NULL),                            # multi-query
    (dict(D=80, Hkv=3), BAD_D),                     # head dim is checked before the grouping
    (dict(Sq=800, flags=binding.FLAG_CAUSAL), SHAPE),   # causal needs Skv >= Sq per query head ...
    (dict(Sq=350, flags=binding.FLAG_CAUSAL), NULL),    # ... not per folded group of 4 * 350 rows
    (dict(B=1 << 12, H=1 << 12, Hkv=1, Sq=1 << 9), SHAPE),
])
def test_gqa_entry_point_validation(lib, kwargs, expect):
    a = dict(B=2, H=8, Hkv=2, Sq=5, Skv=700, D=64, flags=0)
    a.update(kwargs)
    st = binding.tiled_sdpa_fwd_gqa(None, P, P, P, None, a["B"], a["H"], a["Hkv"], a["Sq"], a["Skv"], a["D"],
                                    0.125, 1, None, 0, 0, a["flags"], 1, None, 0)
    assert st == expect, binding.status_string(st)


def test_kvcache_entry_point_checks_the_length_array(lib):
    call = lambda lens, **kw: binding.tiled_sdpa_fwd_kvcache(P, P, P, P, None, lens, kw.get("B", 2), 8, 2, 1, 700, 64,
                                                             0.125, 1, None, 0, 0, 0, 1, None, 0)
    assert binding.tiled_sdpa_fwd_kvcache(None, P, P, P, None, P, 2, 8, 2, 1, 700, 64, 0.125, 1, None) == NULL
    assert binding.tiled_sdpa_fwd_kvcache(P, P, P, P, None, P + 2, 2, 8, 2, 1, 700, 64, 0.125, 1, None,
                                          0, 0, 0, 1, None, 0) == ALIGN
    assert call(P + 2, B=0) == OK                   # empty problem: nothing else is looked at
    assert binding.tiled_sdpa_fwd_kvcache(P, P, P, P, None, P, 2, 8, 3, 1, 700, 64, 0.125, 1, None) == SHAPE


@pytest.mark.parametrize("kwargs,expect", [
    (dict(), WORKSPACE),                           # everything passes up to the workspace (splits = 2, none given)
    (dict(block_rows=48), SHAPE),                   # not a power of two
    (dict(block_rows=32), SHAPE),                   # a 64-row K/V tile would straddle two pages
    (dict(block_rows=96), SHAPE),
    (dict(block_rows=0), SHAPE),
    (dict(max_blocks=-1), SHAPE),
    (dict(max_blocks=1 << 25, block_rows=1024), SHAPE),     # capacity overflows an int
    (dict(max_blocks=1 << 14, block_rows=1024), SHAPE),     # capacity beyond the 2^30-byte head range
    (dict(lens=None), NULL),
    (dict(table=None), NULL),
    (dict(table=P + 2), ALIGN),
    (dict(lens=P + 1), ALIGN),
    (dict(Hkv=3), SHAPE),
    (dict(B=0, lens=None, table=None), OK),
    (dict(D=72), BAD_D),
    (dict(Sq=5000, flags=binding.FLAG_CAUSAL), SHAPE),      # more query rows than the cache can hold
    (dict(splits=1), NULL),                        # q = None: reached only after every check above
])
def test_paged_entry_point_validation(lib, kwargs, expect):
    a = dict(q=P, lens=P, table=P, B=2, H=8, Hkv=2, Sq=1, max_blocks=16, block_rows=256, D=128, flags=0, splits=2)
    a.update(kwargs)
    if kwargs.get("splits") == 1:
        a["q"] = None
    st = binding.tiled_sdpa_fwd_paged(a["q"], P, P, P, None, a["lens"], a["table"], a["B"], a["H"], a["Hkv"], a["Sq"],
                                      a["max_blocks"], a["block_rows"], a["D"], 0.125, 1, None, 0, 0, a["flags"],
                                      a["splits"], None, 0)
    assert st == expect, binding.status_string(st)


def test_grouped_backward_entry_point_validation(lib):
    call = lambda **kw: lib.tiled_sdpa_bwd_gqa(kw.get("q", P), P, P, P, P, P, P, P, P, kw.get("B", 2), kw.get("H", 8),
                                               kw.get("Hkv", 2), 100, kw.get("D", 64), 0.125, 1, 0, kw.get("ws", P), 1 << 20, None)
    assert call(Hkv=3) == SHAPE and call(Hkv=0) == SHAPE and call(Hkv=-1) == SHAPE and call(Hkv=16) == SHAPE
    assert call(D=72) == BAD_D
    assert call(B=0) == OK and call(H=0, Hkv=0) == OK
    assert call(q=None) == NULL and call(ws=None) == WORKSPACE


def test_tune_entry_point_validation(lib):
    tm, tn = ctypes.c_int(-1), ctypes.c_int(-1)
    ms = (ctypes.c_float * len(binding.TILE_ORDER))(*([7.0] * len(binding.TILE_ORDER)))
    call = lambda **kw: lib.tiled_sdpa_tune_tile(kw.get("q", P), P, P, P, kw.get("B", 2), 4, kw.get("S", 300), kw.get("D", 64),
                                                 0.125, kw.get("dtype", 1), None, 0, kw.get("launches", 5),
                                                 kw.get("tm", ctypes.byref(tm)), ctypes.byref(tn), ms)
    assert call(tm=None) == NULL
    assert call(launches=0) == SHAPE and call(launches=1001) == SHAPE
    assert call(dtype=4) == DTYPE and call(D=72) == BAD_D and call(S=-1) == SHAPE
    # an empty problem measures nothing and reports the heuristic's tile
    assert call(B=0) == OK
    assert (tm.value, tn.value) == binding.default_tile(0, 4, 300, 64, binding.BF16)
    assert all(x == -1.0 for x in ms)
    assert call(q=None) == NULL                     # reached through the forward entry point's own checks


def test_kv_workspace_size_and_default_splits(lib):
    assert binding.kv_workspace_bytes(2, 4, 5, 64, 1) == 0
    assert binding.kv_workspace_bytes(2, 4, 5, 64, 0) == 0
    assert binding.kv_workspace_bytes(2, 4, 5, 64, 4) == 2 * 4 * 4 * 5 * (64 + 2) * 4
    assert binding.kv_workspace_bytes(-1, 4, 5, 64, 4) == 0
    # enough query tiles: no split; a single decoding query over a long cache: split, but never into
    # runs shorter than four tiles, never more than the maximum
    assert binding.kv_default_splits(4, 16, 4096, 4096, 128, binding.BF16) == 1
    n = binding.kv_default_splits(1, 8, 1, 16384, 128, binding.BF16)
    assert 2 <= n <= 64 and 16384 // 64 // n >= 4
    assert binding.kv_default_splits(1, 1, 1, 100, 64, binding.F16) == 1
    assert binding.kv_default_splits(1, 1, 1, 1 << 20, 64, binding.F16) <= 128
    with pytest.raises(binding.TiledSdpaError):
        binding.kv_default_splits(1, 1, 8, 4, 64, binding.F16, binding.FLAG_CAUSAL)


@pytest.mark.parametrize("kwargs,expect", [
    (dict(dtype=3), DTYPE),
    (dict(D=80), BAD_D),
    (dict(D=192), BAD_D),
    (dict(D=96, q=None), NULL),                    # 96 and 160 pass the head-dim check
    (dict(D=160, ws=None), WORKSPACE),
    (dict(S=-1), SHAPE),
    (dict(B=1 << 10, H=1 << 10, S=1 << 10), SHAPE),    # statistics arrays beyond a 32-bit byte range
    (dict(S=0, q=None, dq=None, ws=None), OK),
    (dict(dout=None), NULL),
    (dict(lse=None), NULL),
    (dict(dv=None), NULL),
    (dict(dk=P + 8), ALIGN),
    (dict(lse=P + 2), ALIGN),
    (dict(scale=-math.inf), SCALE),
    (dict(ws=None), WORKSPACE),
    (dict(ws=P + 4), WORKSPACE),
    (dict(ws_bytes=2 * (2 * 3 * 50 + 128) * 4 - 1), WORKSPACE),
])
def test_backward_entry_point_validation_order_and_codes(lib, kwargs, expect):
    a = dict(q=P, k=P, v=P, o=P, dout=P, lse=P, dq=P, dk=P, dv=P, B=2, H=3, S=50, D=128, scale=0.125,
             dtype=0, flags=0, ws=P, ws_bytes=1 << 20, stream=None)
    a.update(kwargs)
    st = binding.tiled_sdpa_bwd(a["q"], a["k"], a["v"], a["o"], a["dout"], a["lse"], a["dq"], a["dk"], a["dv"],
                                a["B"], a["H"], a["S"], a["D"], a["scale"], a["dtype"], a["flags"],
                                a["ws"], a["ws_bytes"], a["stream"])
    assert st == expect, binding.status_string(st)
    assert binding.bwd_workspace_bytes(2, 3, 50) == 2 * (2 * 3 * 50 + 128) * 4
    assert binding.bwd_workspace_bytes(-1, 3, 50) == 0


def test_probe_validates_before_touching_the_gpu(lib):
    import ctypes
    fl = ctypes.c_double(-1.0)
    assert lib.tiled_sdpa_probe_mfma(5, 0, 10, P, ctypes.byref(fl), None) == DTYPE
    assert lib.tiled_sdpa_probe_mfma(0, 0, -1, P, ctypes.byref(fl), None) == SHAPE
    assert lib.tiled_sdpa_probe_mfma(0, 0, 10, None, ctypes.byref(fl), None) == NULL
    assert lib.tiled_sdpa_probe_mfma(1, 1, 0, P, ctypes.byref(fl), None) == OK     # iters = 0: flops only
    assert fl.value == 0.0
    assert binding.probe_mfma(binding.BF16, True, 0) == 0.0
    # flops only needs no sink; a launch without one is refused on both sides of the boundary
    assert lib.tiled_sdpa_probe_mfma(1, 1, 0, None, ctypes.byref(fl), None) == OK
    with pytest.raises(ValueError):
        binding.probe_mfma(binding.BF16, True, 10)
    # the read stream: null pointers, alignment, and a buffer too small to give every workgroup a loop trip
    assert lib.tiled_sdpa_probe_hbm_read(None, 1 << 30, P, ctypes.byref(fl), None) == NULL
    assert lib.tiled_sdpa_probe_hbm_read(P, 1 << 30, None, ctypes.byref(fl), None) == NULL
    assert lib.tiled_sdpa_probe_hbm_read(P + 8, 1 << 30, P, ctypes.byref(fl), None) == ALIGN
    assert lib.tiled_sdpa_probe_hbm_read(P, (128 << 20) - 1, P, ctypes.byref(fl), None) == SHAPE
    assert lib.tiled_sdpa_probe_hbm_read(P, 0, P, ctypes.byref(fl), None) == SHAPE


def test_default_tile_is_a_legal_tile(lib):
    for S in (1, 32, 64, 197, 1024, 16384):
        for D in (64, 96, 128, 160):
            tm, tn = binding.default_tile(2, 4, S, D, binding.BF16)
            assert (tm, tn) in binding.TILE_ORDER and not (D != 64 and tn == 128)
            ctm, ctn = binding.default_tile(2, 4, S, D, binding.BF16, binding.FLAG_CAUSAL)
            assert ctm in (64, 128) and (ctm, ctn) in binding.TILE_ORDER        # never the 256-row tile under the mask
    # 256 query rows per workgroup: from D = 96, without the mask, once every CU gets a workgroup
    assert binding.default_tile(2, 32, 8192, 128, binding.BF16, binding.FLAG_CAUSAL) == (128, 64)
    assert binding.default_tile(2, 32, 8192, 128, binding.BF16) == (256, 64)
    assert binding.default_tile(2, 32, 8192, 160, binding.BF16) == (256, 64)
    assert binding.default_tile(2, 32, 8192, 64, binding.BF16) == (128, 64)
    assert binding.default_tile(1, 8, 4096, 128, binding.BF16) == (128, 64)     # 128 workgroups of 256 rows: too few
    # D = 96 takes it from S = 4096; D = 160 runs 64-row K/V tiles from S = 512 and 64 query rows on a few short heads
    assert binding.default_tile(4, 16, 2048, 96, binding.BF16) == (128, 64)
    assert binding.default_tile(4, 16, 4096, 96, binding.BF16) == (256, 64)
    assert binding.default_tile(2, 32, 8192, 160, binding.BF16, binding.FLAG_CAUSAL) == (128, 64)
    assert binding.default_tile(1, 16, 1024, 160, binding.BF16) == (128, 64)
    assert binding.default_tile(4, 16, 197, 160, binding.BF16) == (64, 32)
    assert binding.default_tile(16, 16, 197, 160, binding.BF16) == (128, 32)
    assert len(binding.TILE_ORDER) == 7
    with pytest.raises(binding.TiledSdpaError):
        binding.default_tile(1, 1, 16, 72, 0)


def test_python_front_end_rejects_host_tensors_and_causal():
    import torch
    x = torch.zeros(1, 1, 4, 64, dtype=torch.float16)
    with pytest.raises(ValueError):
        binding.sdpa(x, x, x)
    with pytest.raises(ValueError):
        binding.sdpa(x, x, x, causal=True)


def test_product_path_does_not_import_the_oracle():
    pkg = ROOT / "paper_2603_01960_amd"
    for path in list(pkg.glob("*.py")) + list((pkg / "csrc").glob("*")):
        text = path.read_text()
        assert "oracle" not in text.lower(), path


def test_header_is_plain_c_and_a_c_program_links_against_the_library(tmp_path):
    """The boundary is a C-ABI: the header must compile as C99 (and as C++), and a C program that only
    knows the header must link against the library and get answers from the calls that need no GPU."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None or not binding.library_path().exists():
        pytest.skip("gcc or the built library is missing")
    src = tmp_path / "use.c"
    src.write_text(
        '#include <stdio.h>\n#include "tiled_sdpa.h"\n'
        "int main(void) {\n"
        "    int tm = 0, tn = 0, splits = 0;\n"
        "    if (tiled_sdpa_version() < 100) return 1;\n"
        "    if (tiled_sdpa_default_tile(2, 32, 8192, 128, TSDPA_BF16, 0u, &tm, &tn) != TSDPA_OK) return 2;\n"
        "    if (tiled_sdpa_kv_default_splits(1, 8, 1, 16384, 128, TSDPA_BF16, 0u, &splits) != TSDPA_OK) return 3;\n"
        "    if (tiled_sdpa_fwd(0, 0, 0, 0, 0, 2, 4, 100, 64, 0.125f, TSDPA_F16, 0) != TSDPA_ERR_NULL_PTR) return 4;\n"
        "    if (tiled_sdpa_bwd_workspace_bytes(2, 4, 100) != 2ull * (2 * 4 * 100 + 128) * 4) return 5;\n"
        '    printf("%d %d %d %s\\n", tm, tn, splits, tiled_sdpa_status_string(TSDPA_ERR_BAD_TILE));\n'
        "    return 0;\n}\n")
    inc = str(ROOT / "include")
    subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", f"-I{inc}", "-fsyntax-only", str(src)],
                   check=True, capture_output=True)
    gxx = shutil.which("g++")
    if gxx:
        subprocess.run([gxx, "-std=c++11", "-Wall", "-Werror", f"-I{inc}", "-fsyntax-only", "-x", "c++", str(src)],
                       check=True, capture_output=True)
    lib = binding.library_path()
    exe = tmp_path / "use"
    subprocess.run([gcc, "-std=c99", f"-I{inc}", str(src), "-o", str(exe), f"-L{lib.parent}", "-l:" + lib.name,
                    f"-Wl,-rpath,{lib.parent}"], check=True, capture_output=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True, timeout=120).stdout.split(maxsplit=3)
    assert (int(out[0]), int(out[1])) == binding.default_tile(2, 32, 8192, 128, binding.BF16)
    assert int(out[2]) == binding.kv_default_splits(1, 8, 1, 16384, 128, binding.BF16)
    assert out[3].strip() == binding.status_string(6)


@pytest.mark.parametrize("S", [8192, 16384, 4096, 197, 1])
def test_sampled_rows_hold_both_sides_of_every_tile_boundary(S):
    """The row subset of the full-size parity tests: every multiple of 32 (one wavefront's rows), 64 and
    128 (the query tiles) has the row before it and the row at it, whatever the thinning limit."""
    from paper_2603_01960_amd.workloads import sample_rows
    for limit in (None, 0, 5):
        rows = sample_rows(S, limit=limit)
        assert rows == sorted(set(rows)) and rows[0] == 0 and rows[-1] == S - 1
        have = set(rows)
        for b in range(32, S, 32):
            assert b - 1 in have and b in have, (S, b)
        # every query tile of every tile size is therefore touched on its first and last row
        for tm in (64, 128):
            for t in range((S + tm - 1) // tm):
                assert t * tm in have and min(S, (t + 1) * tm) - 1 in have


def test_static_scratch_entry_point_validates_and_enforces_its_limit(lib):
    """tiled_sdpa_fwd_kvcache_static refuses, before anything is enqueued, a problem whose split states do
    not fit the library's 32 MiB buffer; the other checks come in the order of tiled_sdpa_fwd_kvcache."""
    STATIC = 11
    f = binding.tiled_sdpa_fwd_kvcache_static
    base = dict(q=P, k=P, v=P, o=P, lse=None, lens=None, B=2, H=8, Hkv=2, Sq=1, Skv=4096, D=128, scale=0.1,
                dtype=1, stream=None, tm=0, tn=0, flags=0, splits=4)

    def call(**kw):
        a = dict(base); a.update(kw)
        return f(a["q"], a["k"], a["v"], a["o"], a["lse"], a["lens"], a["B"], a["H"], a["Hkv"], a["Sq"], a["Skv"],
                 a["D"], a["scale"], a["dtype"], a["stream"], a["tm"], a["tn"], a["flags"], a["splits"])
    assert call(dtype=7) == DTYPE
    assert call(D=80) == BAD_D
    assert call(Skv=0) == SHAPE
    assert call(Hkv=3) == SHAPE
    assert call(B=0) == OK
    assert call(splits=129) == 10
    assert call(tm=32, tn=32, splits=0) == TILE
    # 8 * 32 heads x 64 splits x 128 rows x 130 floats = 1.09 GB of split states
    assert binding.kv_workspace_bytes(8, 32, 128, 128, 64) > binding.STATIC_SCRATCH_BYTES
    assert call(B=8, H=32, Hkv=32, Sq=128, splits=64) == STATIC
    # exactly at the limit passes the size check and goes on to the pointer checks
    assert binding.kv_workspace_bytes(1, 63, 8, 128, 128) <= binding.STATIC_SCRATCH_BYTES
    assert "static scratch" in binding.status_string(STATIC)


def test_static_scratch_buffer_is_a_symbol_the_runtime_can_look_up(tmp_path):
    """hipGetSymbolAddress finds a device variable through the code object's dynamic symbol table.  A
    file-scope static one gets there only because the compiler gives it external linkage when host code
    names it; kept local (as an `used` attribute once made it) the lookup aborts the process."""
    import shutil
    import subprocess
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    readelf = "/opt/rocm/llvm/bin/llvm-readelf"
    if not (Path(hipcc).exists() and Path(readelf).exists()):
        pytest.skip("hipcc / llvm-readelf not available")
    from paper_2603_01960_amd import build as lib_build
    co = tmp_path / "tiled_sdpa.co"
    subprocess.run([hipcc, *lib_build.FLAGS, "--cuda-device-only", "--no-gpu-bundle-output", "-c",
                    str(lib_build.CSRC / "tiled_sdpa.hip"), "-o", str(co)], check=True, capture_output=True, timeout=600)
    syms = subprocess.run([readelf, "--dyn-syms", "-W", str(co)], check=True, capture_output=True, text=True).stdout
    rows = [l.split() for l in syms.splitlines() if l.strip().endswith("scratch")]
    assert len(rows) == 1, syms
    assert rows[0][2] == str(binding.STATIC_SCRATCH_BYTES) and rows[0][3] == "OBJECT" and rows[0][4] == "GLOBAL"
