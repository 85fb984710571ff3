"""Parity of the HIP path (through the C-ABI) against the float64 CPU oracle.

Tolerances (max-abs over every compared element, stated by the benchmark spec):
FP16 2e-3, BF16 1.6e-2; the output must be finite.  LSE (an extra the paper does not
define; parity otherwise unpinned by the paper) is held to 1e-4 absolute: it is an FP32
quantity of magnitude <= ~40 built from FP32-accumulated dot products.
"""
import math
import sys

import numpy as np
import pytest
import torch

from oracle import sdpa_oracle as orc
from paper_2603_01960_amd import binding
from paper_2603_01960_amd.workloads import make_qkv, make_workload, sample_rows

pytestmark = pytest.mark.gpu

TOL = {"f16": 2e-3, "bf16": 1.6e-2}
LSE_TOL = 1e-4
TILES = [(64, 32), (64, 64), (64, 128), (128, 32), (128, 64), (128, 128), (256, 64)]


def legal(tile, D):
    """128-row K/V tiles exist up to D = 128 (at D = 160 four such slots exceed the LDS)."""
    return tile[1] != 128 or D <= 128


def expect_bad_tile(D, dtype, tile):
    q, k, v = make_qkv(1, 1, 64, D, dtype, seed=1)
    with pytest.raises(binding.TiledSdpaError) as e:
        binding.sdpa(q.cuda(), k.cuda(), v.cuda(), tile=tile)
    assert e.value.status == 6


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module", autouse=True)
def _device():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    binding.load_library()   # fails loudly if the HIP library is not built
    yield
    torch.cuda.synchronize()


def gpu_sdpa(q, k, v, scale=None, tile=None, flags=0, return_lse=True, causal=False):
    qd, kd, vd = (t.cuda() for t in (q, k, v))
    o, lse = binding.sdpa(qd, kd, vd, causal=causal, scale=scale, return_lse=True, tile=tile, flags=flags)
    torch.cuda.synchronize()
    return o.cpu(), lse.cpu()


def check(q, k, v, dtype, scale=None, tile=None, rows=None, flags=0, tag="", causal=False):
    say(f"[case] {tag} shape={tuple(q.shape)} dtype={dtype} scale={scale} tile={tile} causal={causal} "
        f"rows={'all' if rows is None else len(rows)}")
    o, lse = gpu_sdpa(q, k, v, scale=scale, tile=tile, flags=flags, causal=causal)
    assert torch.isfinite(o.float()).all(), "non-finite output"
    assert torch.isfinite(lse).all(), "non-finite lse"
    ref_o, ref_lse = orc.sdpa(q.float().numpy(), k.float().numpy(), v.float().numpy(),
                              scale=scale, rows=rows, return_lse=True, causal=causal)
    got_o = o.double().numpy()
    got_lse = lse.double().numpy()
    if rows is not None:
        got_o, got_lse = got_o[:, :, rows], got_lse[:, :, rows]
    err = float(np.abs(got_o - ref_o).max()) if got_o.size else 0.0
    lerr = float(np.abs(got_lse - ref_lse).max()) if got_lse.size else 0.0
    say(f"        max|dO|={err:.3e} (tol {TOL[dtype]:.1e})  max|dLSE|={lerr:.3e}")
    assert err <= TOL[dtype], f"{tag}: output error {err}"
    assert lerr <= LSE_TOL * max(1.0, float(np.abs(ref_lse).max()) / 16.0), f"{tag}: lse error {lerr}"
    return err


# ------------------------------------------------------------------ small shapes, every tile
@pytest.mark.parametrize("tile", TILES)
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("D", [64, 128])
def test_small_shapes_all_tiles(D, dtype, tile):
    if not legal(tile, D):
        return expect_bad_tile(D, dtype, tile)
    # lengths around every tile edge, a prime, one key, several tiles plus a ragged tail
    for S in (1, 2, 31, 32, 33, 63, 64, 65, 127, 129, 197, 257, 300):
        q, k, v = make_qkv(2, 3, S, D, dtype, seed=7000 + S)
        check(q, k, v, dtype, tile=tile, tag=f"small S={S}")


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_default_tile_and_plain_entry_point(dtype):
    q, k, v = make_qkv(2, 2, 333, 128, dtype, seed=11)
    check(q, k, v, dtype, tag="heuristic tile")
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    o = torch.empty_like(qd)
    st = binding.tiled_sdpa_fwd(qd.data_ptr(), kd.data_ptr(), vd.data_ptr(), o.data_ptr(), None,
                                2, 2, 333, 128, math.nan, binding.F16 if dtype == "f16" else binding.BF16,
                                torch.cuda.current_stream().cuda_stream)
    assert st == 0
    torch.cuda.synchronize()
    o2 = binding.sdpa(qd, kd, vd)
    assert torch.equal(o, o2)


@pytest.mark.parametrize("scale", [0.0, -0.125, 0.5, -1.0, 1e-3])
def test_scale_variants(scale):
    q, k, v = make_qkv(1, 2, 200, 64, "f16", seed=21)
    check(q, k, v, "f16", scale=scale, tag=f"scale={scale}")
    q, k, v = make_qkv(1, 2, 150, 128, "bf16", seed=22)
    check(q, k, v, "bf16", scale=scale, tile=(64, 32), tag=f"scale={scale}")


def test_rising_maxima_exercise_the_rescale():
    """Keys sorted so each streamed tile raises the running maximum (Eqs. 3-4 rescale every tile)."""
    S, D = 512, 64
    q, k, v = make_qkv(1, 1, S, D, "f16", seed=31)
    q = torch.ones_like(q)
    ramp = torch.linspace(-2.0, 2.0, S).view(1, 1, S, 1)
    k = (torch.ones(1, 1, S, D) * ramp).to(torch.float16)
    check(q, k, v, "f16", tile=(128, 32), tag="rising maxima")
    check(q, k.flip(2).contiguous(), v, "f16", tile=(64, 64), tag="falling maxima")


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("causal", [False, True])
def test_wide_logit_ranges_exercise_the_lazy_reference(dtype, causal):
    """The reference of the exponentials is raised only when a tile's weights sum past 2^8: drive it
    with logits whose spread is far beyond that (near one-hot softmax rows, weights that overflow FP32
    against a stale reference) and with logits that creep up by less than the threshold per tile."""
    D, S = 128, 700
    for std in (3.0, 6.0):                         # logits of standard deviation 9 and 36
        # (value rows of standard deviation 1/2: a near one-hot row returns a value row, and one rounding
        # of an FP16 output of magnitude >= 4 would by itself use up the tolerance of 2e-3)
        q, k, v = make_qkv(1, 3, S, D, dtype, seed=41, qk_std=std, v_std=0.5)
        for tile in ((128, 32), (128, 64), (64, 32)):
            check(q, k, v, dtype, tile=tile, causal=causal, tag=f"wide logits std={std}")
    # one query direction, keys along it with a slope of ~5 log2 units per 32-key tile (below the
    # threshold of 8) and then a jump of 400 units: weights against the stale reference overflow
    q = torch.zeros(1, 1, S, D)
    q[..., 0] = 1.0
    ramp = torch.arange(S, dtype=torch.float32) * (5.0 / 32.0) * math.log(2.0) * math.sqrt(D)
    ramp[500:] += 400.0 * math.log(2.0) * math.sqrt(D)
    k = torch.zeros(1, 1, S, D)
    k[..., 0] = ramp.view(1, 1, S)
    tdt = torch.float16 if dtype == "f16" else torch.bfloat16
    _, _, v = make_qkv(1, 1, S, D, dtype, seed=42, v_std=0.5)
    check(q.to(tdt), k.to(tdt), v, dtype, tile=(128, 32), causal=causal, tag="creeping then jumping logits")
    check(q.to(tdt), k.to(tdt).flip(2).contiguous(), v, dtype, tile=(128, 64), causal=causal, tag="falling logits")


def test_closed_forms_on_device():
    S, D = 197, 64
    _, k, v = make_qkv(1, 2, S, D, "bf16", seed=41)
    q = torch.zeros_like(k)
    o, lse = gpu_sdpa(q, k, v)
    mean = v.double().mean(dim=2, keepdim=True)
    assert (o.double() - mean).abs().max() <= TOL["bf16"]
    assert (lse.double() - math.log(S)).abs().max() <= 1e-5
    # one key: the output is the value row, exactly
    q1, k1, v1 = make_qkv(2, 2, 1, 128, "f16", seed=42)
    o1, _ = gpu_sdpa(q1, k1, v1)
    assert torch.equal(o1, v1)
    # constant value rows
    row = v[:, :, :1].expand_as(v).contiguous()
    q2, k2, _ = make_qkv(1, 2, S, D, "bf16", seed=43)
    o2, _ = gpu_sdpa(q2, k2, row)
    assert (o2.double() - row.double()).abs().max() <= 2 ** -8 * row.double().abs().max()


def test_no_write_outside_the_output_and_no_read_dependence_past_S():
    """Ragged S: guard bands around o and lse stay untouched; the result ignores memory after K/V."""
    B, H, S, D = 1, 3, 197, 64
    q, k, v = make_qkv(B, H, S, D, "bf16", seed=51)
    n = B * H * S * D
    pad = 4096
    buf = torch.full((n + 2 * pad,), 7.0, dtype=torch.bfloat16, device="cuda")
    lbuf = torch.full((B * H * S + 2 * pad,), -3.0, dtype=torch.float32, device="cuda")
    o = buf[pad:pad + n].view(B, H, S, D)
    lse = lbuf[pad:pad + B * H * S].view(B, H, S)
    binding.sdpa(q.cuda(), k.cuda(), v.cuda(), out=o, lse_out=lse, return_lse=True, tile=(128, 64))
    torch.cuda.synchronize()
    assert (buf[:pad] == 7.0).all() and (buf[pad + n:] == 7.0).all()
    assert (lbuf[:pad] == -3.0).all() and (lbuf[pad + B * H * S:] == -3.0).all()
    ref = orc.sdpa(q.float().numpy(), k.float().numpy(), v.float().numpy())
    assert np.abs(o.cpu().double().numpy() - ref).max() <= TOL["bf16"]


@pytest.mark.parametrize("S,D,tile", [(197, 64, (128, 32)), (197, 64, (64, 128)), (130, 128, (128, 64)),
                                      (64, 128, (64, 32)), (256, 64, (128, 64)), (33, 128, (128, 64)), (200, 64, (128, 128)),
                                      (197, 96, (128, 64)), (130, 160, (128, 32)), (70, 160, (64, 64))])
@pytest.mark.parametrize("causal", [False, True])
def test_nothing_is_read_past_the_end_of_k_and_v(S, D, tile, causal):
    """K and V end exactly where a NaN-filled region starts.  A row index >= S of the LAST head that
    was fetched from memory (ragged tail, or a tile prefetched past the end) would bring NaN into the
    V operand, and 0 * NaN = NaN would reach the output."""
    B, H = 1, 2
    q, k, v = make_qkv(B, H, S, D, "bf16", seed=55)
    n = B * H * S * D
    guard = 1 << 17
    bufs = []
    for t in (k, v):
        buf = torch.full((n + guard,), float("nan"), dtype=torch.bfloat16, device="cuda")
        buf[:n] = t.flatten().cuda()
        bufs.append(buf)
    kd, vd = (b[:n].view(B, H, S, D) for b in bufs)
    o, lse = binding.sdpa(q.cuda(), kd, vd, causal=causal, return_lse=True, tile=tile)
    torch.cuda.synchronize()
    assert torch.isfinite(o.float()).all() and torch.isfinite(lse).all()
    ref = orc.sdpa(q.float().numpy(), k.float().numpy(), v.float().numpy(), causal=causal)
    assert np.abs(o.cpu().double().numpy() - ref).max() <= TOL["bf16"]


def test_non_default_stream_and_repeatability():
    q, k, v = make_qkv(2, 4, 777, 128, "f16", seed=61)
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    ref = binding.sdpa(qd, kd, vd)
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        outs = [binding.sdpa(qd, kd, vd) for _ in range(5)]
    s.synchronize()
    for o in outs:
        assert torch.equal(o, ref)     # same schedule, same rounding order: bit-identical


def test_linear_grid_flag_gives_identical_bits():
    q, k, v = make_qkv(3, 5, 300, 64, "bf16", seed=71)
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    a = binding.sdpa(qd, kd, vd, tile=(64, 64))
    b = binding.sdpa(qd, kd, vd, tile=(64, 64), flags=binding.FLAG_LINEAR_GRID)
    torch.cuda.synchronize()
    assert torch.equal(a, b)


def test_exact_max_flag_matches_the_oracle_and_the_default():
    """tau = 0 (Eq. 2 literally) and the lazy reference give the same result up to rounding."""
    for dtype, D in (("f16", 64), ("bf16", 128)):
        q, k, v = make_qkv(1, 3, 700, D, dtype, seed=81, qk_std=1.5)
        a = check(q, k, v, dtype, flags=binding.FLAG_EXACT_MAX, tag="exact max")
        b = check(q, k, v, dtype, tag="lazy reference")
        assert abs(a - b) <= TOL[dtype]


def test_mfma_probe_runs_and_reports_its_flops():
    sink = torch.zeros(512 * 256, dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    for dt in (binding.F16, binding.BF16):
        for rnd in (0, 1, 2):       # constant, random, random + the loop's LDS-read / vector-ALU mix
            flops = binding.probe_mfma(dt, rnd, 10, sink.data_ptr(), stream)
            torch.cuda.synchronize()
            assert flops == 512 * 4 * 10 * 64 * 32768
            assert torch.isfinite(sink).all()
    # constant operands: every accumulator element is 16 (ones . ones over k = 16) per MFMA
    binding.probe_mfma(binding.BF16, False, 1, sink.data_ptr(), stream)
    torch.cuda.synchronize()
    assert float(sink[0]) == 64 * 16 * 16      # 64 MFMAs x 16 accumulator elements summed x 16


def test_read_stream_probe_reads_what_it_reports_and_checks_every_word():
    """Every lane keeps an XOR of the words it read and the first lane of a workgroup leaves its own in the
    sink: zeros give zero, and a byte changed in a word that lane reads changes that workgroup's entry only."""
    nbytes = (128 << 20) + 4096 + 16                  # one loop trip per workgroup, plus a tail that is not read
    src = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
    sink = torch.full((512 * 256,), -1.0, dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    done = binding.probe_hbm_read(src.data_ptr(), nbytes, sink.data_ptr(), stream)
    torch.cuda.synchronize()
    assert done == 128 << 20
    assert torch.all(sink[:8192] == 0) and torch.all(sink[8192:] == -1)
    per_group = (128 << 20) // 8192
    assert per_group == 1024 * 16                      # one loop trip: 256 lanes x 4 loads of 16 bytes
    src[5 * per_group + 512 * 16 + 1] = 7              # workgroup 5, third load of lane 0
    src[(128 << 20) + 100] = 9                         # in the tail: must not be read
    binding.probe_hbm_read(src.data_ptr(), nbytes, sink.data_ptr(), stream)
    torch.cuda.synchronize()
    changed = torch.nonzero(sink[:8192]).flatten().tolist()
    assert changed == [5], changed


# ------------------------------------------------------------------ head dims 96 and 160 (Section 4.3 grid)
@pytest.mark.parametrize("tile", TILES)
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("D", [96, 160])
@pytest.mark.parametrize("causal", [False, True])
def test_head_dims_96_and_160(D, dtype, tile, causal):
    if not legal(tile, D):
        return expect_bad_tile(D, dtype, tile)
    for S in (1, 33, 64, 127, 197, 256, 300, 513):
        q, k, v = make_qkv(2, 2, S, D, dtype, seed=9500 + S + D)
        check(q, k, v, dtype, tile=tile, causal=causal, tag=f"D={D} S={S}")


@pytest.mark.parametrize("D", [96, 160])
def test_head_dims_96_and_160_mid_size_default_tile_and_guards(D):
    q, k, v = make_qkv(2, 4, 1024, D, "bf16", seed=9600 + D)
    check(q, k, v, "bf16", tag=f"D={D} S=1024")
    check(q, k, v, "bf16", causal=True, tag=f"D={D} S=1024 causal")
    # output rows are D wide in memory: nothing may be written between or after them
    B, H, S = 1, 2, 197
    q, k, v = make_qkv(B, H, S, D, "f16", seed=9700 + D)
    n, pad = B * H * S * D, 4096
    buf = torch.full((n + 2 * pad,), 7.0, dtype=torch.float16, device="cuda")
    o = buf[pad:pad + n].view(B, H, S, D)
    binding.sdpa(q.cuda(), k.cuda(), v.cuda(), out=o)
    torch.cuda.synchronize()
    assert (buf[:pad] == 7.0).all() and (buf[pad + n:] == 7.0).all()
    ref = orc.sdpa(q.float().numpy(), k.float().numpy(), v.float().numpy())
    assert np.abs(o.cpu().double().numpy() - ref).max() <= TOL["f16"]


@pytest.mark.parametrize("D", [96, 160])
def test_head_dims_96_and_160_long_sequences_sampled_rows(D):
    """S = 8192 (the longest length of the grid of Section 4.3) on the tiles the heuristic takes there: the
    256-row query tile without the mask, 128 x 64 under it; rows on both sides of every tile edge plus a stride."""
    B, H, S = 1, 8, 8192
    dtype = "bf16" if D == 160 else "f16"
    q, k, v = make_qkv(B, H, S, D, dtype, seed=9800 + D)
    assert binding.default_tile(B, H, S, D, binding.BF16) == (256, 64)
    assert binding.default_tile(B, H, S, D, binding.BF16, binding.FLAG_CAUSAL) == (128, 64)
    rows = sample_rows(S, limit=8)
    check(q, k, v, dtype, rows=rows, tag=f"D={D} S={S} sampled rows")
    check(q, k, v, dtype, rows=rows, causal=True, tag=f"D={D} S={S} causal, sampled rows")
    check(q, k, v, dtype, rows=rows, tile=(128, 32), tag=f"D={D} S={S} sampled rows")


# ------------------------------------------------------------------ causal mask (Section 4.1.3)
@pytest.mark.parametrize("tile", TILES)
@pytest.mark.parametrize("dtype,D", [("f16", 64), ("bf16", 128), ("bf16", 64), ("f16", 128)])
def test_causal_small_shapes_all_tiles(dtype, D, tile):
    if not legal(tile, D):
        return expect_bad_tile(D, dtype, tile)
    for S in (1, 2, 31, 33, 64, 65, 127, 128, 129, 197, 256, 300, 513):
        q, k, v = make_qkv(2, 2, S, D, dtype, seed=9000 + S)
        check(q, k, v, dtype, tile=tile, causal=True, tag=f"causal S={S}")


def test_causal_scale_variants_and_first_row():
    q, k, v = make_qkv(1, 2, 260, 64, "f16", seed=91)
    for scale in (0.0, -0.3, 1.0):
        check(q, k, v, "f16", scale=scale, causal=True, tag=f"causal scale={scale}")
    o, _ = gpu_sdpa(q, k, v, causal=True)
    assert torch.equal(o[:, :, 0], v[:, :, 0])          # row 0 sees key 0 only


def test_causal_rows_do_not_depend_on_later_keys_or_values():
    q, k, v = make_qkv(1, 2, 700, 128, "bf16", seed=92)
    o1, l1 = gpu_sdpa(q, k, v, causal=True)
    k2, v2 = k.clone(), v.clone()
    k2[:, :, 400:] = 7.0
    v2[:, :, 400:] = -9.0
    o2, l2 = gpu_sdpa(q, k2, v2, causal=True)
    assert torch.equal(o1[:, :, :400], o2[:, :, :400]) and torch.equal(l1[:, :, :400], l2[:, :, :400])
    assert not torch.equal(o1[:, :, 400:], o2[:, :, 400:])


def test_causal_text_regime_full_and_long_context_sampled():
    w, q, k, v = make_workload("C2", "bf16")
    check(q, k, v, "bf16", causal=True, tag="C2 causal")
    w, q, k, v = make_workload("C4")
    rows = sample_rows(w.S)
    check(q, k, v, "bf16", causal=True, rows=rows, tag="C4 causal, sampled rows")
    check(q, k, v, "bf16", causal=True, rows=rows, tile=(64, 64), tag="C4 causal, sampled rows")


# ------------------------------------------------------------------ the five configurations
def test_config_C1_full():
    w, q, k, v = make_workload("C1")
    check(q, k, v, "f16", tag="C1")


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_config_C2_full(dtype):
    w, q, k, v = make_workload("C2", dtype)
    check(q, k, v, dtype, tag="C2")


def test_config_C3_full():
    w, q, k, v = make_workload("C3")
    check(q, k, v, "bf16", tag="C3")
    for tile in [(64, 64), (128, 128)]:
        check(q[:4], k[:4], v[:4], "bf16", tile=tile, tag="C3 slice")


def _long_config(name, tiles):
    w, q, k, v = make_workload(name)
    dtype = w.dtypes[0]
    rows = sample_rows(w.S)
    say(f"[{name}] oracle on {len(rows)} sampled query rows x {w.BH} heads")
    qn, kn, vn = q.float().numpy(), k.float().numpy(), v.float().numpy()
    ref_o, ref_lse = orc.sdpa(qn, kn, vn, rows=rows, return_lse=True)
    # ... and EVERY row of the first and the last head (each lies in another XCD's share of the grid)
    whole = [(0, 0), (w.B - 1, w.H - 1)]
    ref_whole = [orc.sdpa(qn[b:b + 1, h:h + 1], kn[b:b + 1, h:h + 1], vn[b:b + 1, h:h + 1], return_lse=True) for b, h in whole]
    vmax = v.float().amax(dim=2, keepdim=True)
    vmin = v.float().amin(dim=2, keepdim=True)
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    for tile in tiles:
        say(f"[case] {name} tile={tile}")
        o, lse = binding.sdpa(qd, kd, vd, return_lse=True, tile=tile)
        torch.cuda.synchronize()
        o, lse = o.cpu(), lse.cpu()
        assert torch.isfinite(o.float()).all() and torch.isfinite(lse).all()
        err = float(np.abs(o[:, :, rows].double().numpy() - ref_o).max())
        lerr = float(np.abs(lse[:, :, rows].double().numpy() - ref_lse).max())
        for (b, h), (ro, rl) in zip(whole, ref_whole):
            err = max(err, float(np.abs(o[b:b + 1, h:h + 1].double().numpy() - ro).max()))
            lerr = max(lerr, float(np.abs(lse[b:b + 1, h:h + 1].double().numpy() - rl).max()))
        say(f"        max|dO|={err:.3e} (tol {TOL[dtype]:.1e}) max|dLSE|={lerr:.3e}")
        assert err <= TOL[dtype]
        assert lerr <= 5 * LSE_TOL
        # property that holds at any size: every output is a convex combination of value rows
        slack = TOL[dtype]
        assert (o.float() <= vmax + slack).all() and (o.float() >= vmin - slack).all()


def test_config_C4_sampled_rows_tile_sweep():
    _long_config("C4", [None] + [t for t in TILES if legal(t, 128)])


def test_config_C5_sampled_rows():
    _long_config("C5", [None, (64, 32), (128, 64)])


def test_schedule_search_returns_a_legal_tile_and_its_timings():
    for D, dtype, n_tiles in ((128, "bf16", 7), (64, "f16", 7), (160, "bf16", 5)):
        q, k, v = (t.cuda() for t in make_qkv(2, 4, 700, D, dtype, seed=33))
        tile, times = binding.tune_tile(q, k, v, causal=(D == 64), launches=3)
        say(f"[case] tune D={D} {dtype}: {tile} {times}")
        assert tile in times and len(times) == n_tiles
        assert all(0 < t < 100 for t in times.values())
        assert times[tile] == min(times.values())
        assert legal(tile, D)
        # the tile it reports gives the same result as any other
        a = binding.sdpa(q, k, v, causal=(D == 64), tile=tile)
        b = binding.sdpa(q, k, v, causal=(D == 64))
        torch.cuda.synchronize()
        assert float((a.float() - b.float()).abs().max()) <= TOL[dtype]
