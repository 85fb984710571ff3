"""Parity of the Sq x Skv / split-KV entry point (through the C-ABI) against the float64 CPU oracle.

Same tolerances as the square problem: max-abs FP16 2e-3, BF16 1.6e-2, finite output; LSE 1e-4.
The split count must not change the result beyond rounding: the merged states of Eqs. 2-4 over
disjoint key ranges are the same sums in another order.
"""
import math
import sys

import numpy as np
import pytest
import torch

from oracle import sdpa_oracle as orc
from paper_2603_01960_amd import binding
from paper_2603_01960_amd.workloads import make_qkv, sample_rows

pytestmark = pytest.mark.gpu

TOL = {"f16": 2e-3, "bf16": 1.6e-2}
LSE_TOL = 1e-4
KV_TILES = [(64, 32), (64, 64), (128, 32), (128, 64), (256, 64)]      # the last one on dense caches only


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module", autouse=True)
def _device():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    binding.load_library()
    yield
    torch.cuda.synchronize()


def make_q_kv(B, H, Sq, Skv, D, dtype, seed, std=1.0):
    q = make_qkv(B, H, Sq, D, dtype, seed=seed, qk_std=std)[0]
    _, k, v = make_qkv(B, H, Skv, D, dtype, seed=seed + 1, qk_std=std)
    return q, k, v


def check_kv(q, k, v, dtype, *, causal=False, splits=0, tile=None, scale=None, rows=None, flags=0, tag=""):
    say(f"[case] {tag} q={tuple(q.shape)} kv={tuple(k.shape)} dtype={dtype} causal={causal} splits={splits} "
        f"tile={tile} scale={scale} rows={'all' if rows is None else len(rows)}")
    o, lse = binding.sdpa_kv(q.cuda(), k.cuda(), v.cuda(), causal=causal, scale=scale, splits=splits,
                             return_lse=True, tile=tile, flags=flags)
    torch.cuda.synchronize()
    o, lse = o.cpu(), lse.cpu()
    assert torch.isfinite(o.float()).all(), "non-finite output"
    assert torch.isfinite(lse).all(), "non-finite lse"
    ref_o, ref_lse = orc.sdpa(q.float().numpy(), k.float().numpy(), v.float().numpy(),
                              scale=scale, rows=rows, return_lse=True, causal=causal)
    got_o, got_lse = o.double().numpy(), lse.double().numpy()
    if rows is not None:
        got_o, got_lse = got_o[:, :, rows], got_lse[:, :, rows]
    err = float(np.abs(got_o - ref_o).max()) if got_o.size else 0.0
    lerr = float(np.abs(got_lse - ref_lse).max()) if got_lse.size else 0.0
    say(f"        max|dO|={err:.3e} (tol {TOL[dtype]:.1e})  max|dLSE|={lerr:.3e}")
    assert err <= TOL[dtype], f"{tag}: output error {err}"
    assert lerr <= LSE_TOL * max(1.0, float(np.abs(ref_lse).max()) / 16.0), f"{tag}: lse error {lerr}"
    return o, lse


# ------------------------------------------------------------------ shapes x splits x tiles
@pytest.mark.parametrize("tile", KV_TILES)
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("D", [64, 128])
def test_decode_and_chunk_shapes_every_tile(D, dtype, tile):
    # one query, a few, a ragged tile of them, more queries than keys; key lengths around tile edges
    for Sq, Skv in ((1, 1), (1, 65), (1, 700), (3, 257), (17, 130), (64, 64), (100, 333), (130, 97), (200, 1000)):
        q, k, v = make_q_kv(2, 2, Sq, Skv, D, dtype, seed=9000 + Sq + Skv)
        for splits in (1, 3):
            check_kv(q, k, v, dtype, splits=splits, tile=tile, tag="kv shapes")
            if Skv >= Sq:
                check_kv(q, k, v, dtype, causal=True, splits=splits, tile=tile, tag="kv shapes causal")


@pytest.mark.parametrize("splits", [0, 1, 2, 5, 8, 16, 37, 128])
def test_split_counts_including_more_splits_than_tiles(splits):
    q, k, v = make_q_kv(1, 3, 5, 1237, 128, "bf16", seed=9100)          # 20 tiles of 64, ragged tail
    check_kv(q, k, v, "bf16", splits=splits, tag="split count")
    check_kv(q, k, v, "bf16", splits=splits, causal=True, tag="split count causal")
    q, k, v = make_q_kv(1, 2, 300, 300, 64, "f16", seed=9101)           # square: splits past the diagonal are empty
    check_kv(q, k, v, "f16", splits=splits, causal=True, tile=(128, 32), tag="square causal split")


@pytest.mark.parametrize("D", [96, 160])
def test_other_head_dims(D):
    q, k, v = make_q_kv(1, 2, 9, 777, D, "bf16", seed=9200 + D)
    check_kv(q, k, v, "bf16", splits=4, tag=f"D={D}")
    check_kv(q, k, v, "bf16", splits=4, causal=True, tile=(64, 64), tag=f"D={D} causal")
    q, k, v = make_q_kv(1, 2, 150, 400, D, "f16", seed=9210 + D)
    check_kv(q, k, v, "f16", splits=3, causal=True, tag=f"D={D} chunk")


def test_square_problem_agrees_with_the_plain_entry_point():
    """Sq = Skv, one split: the general kernel computes what tiled_sdpa_fwd_ex computes, bit for bit."""
    for causal in (False, True):
        q, k, v = make_qkv(2, 2, 500, 128, "bf16", seed=9300)
        qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
        o1, l1 = binding.sdpa(qd, kd, vd, causal=causal, return_lse=True, tile=(128, 64))
        o2, l2 = binding.sdpa_kv(qd, kd, vd, causal=causal, return_lse=True, tile=(128, 64), splits=1)
        torch.cuda.synchronize()
        assert torch.equal(o1, o2) and torch.equal(l1, l2)


def test_split_count_changes_the_result_only_by_rounding():
    q, k, v = make_q_kv(2, 4, 4, 4096, 128, "f16", seed=9400)
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    base = binding.sdpa_kv(qd, kd, vd, splits=1).float()
    for n in (2, 4, 16):
        o = binding.sdpa_kv(qd, kd, vd, splits=n).float()
        torch.cuda.synchronize()
        assert (o - base).abs().max().item() <= 2 * 2.0 ** -11 * max(1.0, base.abs().max().item())


def test_decode_step_equals_last_rows_of_square_causal_attention():
    """The device's own consistency: the last rows of square causal attention = those rows as a
    chunk against the whole cache (oracle-checked separately above)."""
    q, k, v = make_qkv(1, 4, 1000, 128, "bf16", seed=9500)
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    full = binding.sdpa(qd, kd, vd, causal=True)
    tail = binding.sdpa_kv(qd[:, :, -7:].contiguous(), kd, vd, causal=True, splits=4)
    torch.cuda.synchronize()
    assert (full[:, :, -7:].float() - tail.float()).abs().max().item() <= 1.6e-2
    check_kv(q[:, :, -7:].contiguous(), k, v, "bf16", causal=True, splits=4, tag="decode tail")


def test_scale_flags_and_caller_owned_buffers():
    q, k, v = make_q_kv(1, 2, 33, 900, 64, "f16", seed=9600)
    for scale in (0.0, -0.25, 0.5):
        check_kv(q, k, v, "f16", scale=scale, splits=3, tag=f"scale={scale}")
    check_kv(q, k, v, "f16", splits=3, flags=binding.FLAG_EXACT_MAX, tag="exact max")
    check_kv(q, k, v, "f16", splits=3, flags=binding.FLAG_LINEAR_GRID, causal=True, tag="linear grid")
    # caller-owned workspace, larger than needed and pre-filled with NaN: every read slot is written first
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    need = binding.kv_workspace_bytes(1, 2, 33, 64, 5)
    ws = torch.full((need // 4 + 64,), float("nan"), dtype=torch.float32, device="cuda")
    out = torch.full_like(qd, float("nan"))
    o = binding.sdpa_kv(qd, kd, vd, splits=5, workspace=ws, out=out)
    torch.cuda.synchronize()
    assert o.data_ptr() == out.data_ptr() and torch.isfinite(o.float()).all()
    ref = orc.sdpa(q.float().numpy(), k.float().numpy(), v.float().numpy())
    assert np.abs(o.cpu().double().numpy() - ref).max() <= TOL["f16"]
    assert torch.isnan(ws[need // 4:]).all(), "wrote past the stated workspace size"
    with pytest.raises(binding.TiledSdpaError):
        binding.sdpa_kv(qd, kd, vd, splits=5, workspace=ws[: need // 4 - 1])


def test_nothing_is_read_past_the_end_of_the_cache():
    """K and V sit inside larger NaN-filled buffers: a fetch past row Skv would poison the output."""
    B, H, Sq, Skv, D = 1, 3, 2, 333, 128
    q, k, v = make_q_kv(B, H, Sq, Skv, D, "bf16", seed=9700)
    pad = 4096
    kbuf = torch.full((B * H * Skv * D + 2 * pad,), float("nan"), dtype=torch.bfloat16, device="cuda")
    vbuf = torch.full_like(kbuf, float("nan"))
    kd = kbuf[pad:pad + B * H * Skv * D].view(B, H, Skv, D)
    vd = vbuf[pad:pad + B * H * Skv * D].view(B, H, Skv, D)
    kd.copy_(k)
    vd.copy_(v)
    # the last head is followed by NaN; earlier heads are followed by the next head's rows, which
    # must not leak in either: compared against the oracle below
    for splits in (1, 4):
        o = binding.sdpa_kv(q.cuda(), kd, vd, splits=splits, tile=(64, 64))
        torch.cuda.synchronize()
        assert torch.isfinite(o.float()).all()
        ref = orc.sdpa(q.float().numpy(), k.float().numpy(), v.float().numpy())
        assert np.abs(o.cpu().double().numpy() - ref).max() <= TOL["bf16"]


# ------------------------------------------------------------------ decoding at full size, sampled rows
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_long_cache_decode_full_size(dtype):
    # one new token per sequence against a 16384-entry cache (the length of the paper's longest
    # workload), and a 64-token chunk; heuristic splits
    for Sq in (1, 64):
        q, k, v = make_q_kv(2, 8, Sq, 16384, 128, dtype, seed=9800 + Sq)
        check_kv(q, k, v, dtype, causal=True, tag="long cache")
    q, k, v = make_q_kv(1, 2, 8192, 8192, 128, dtype, seed=9810, std=math.sqrt(2.0))
    rows = sample_rows(8192)
    check_kv(q, k, v, dtype, rows=rows, tag="few heads, long sequence")
    check_kv(q, k, v, dtype, rows=rows, causal=True, tag="few heads, long sequence, causal")


# ------------------------------------------------------------------ grouped heads (several query heads per key/value head)
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("B,H,Hkv,Sq,Skv,D,causal,splits", [
    (2, 8, 2, 1, 1000, 128, False, 0), (2, 8, 2, 1, 1000, 128, True, 0), (1, 32, 4, 1, 4096, 128, True, 8),
    (1, 12, 3, 5, 333, 64, False, 3), (1, 8, 8, 1, 257, 64, True, 0), (1, 16, 1, 7, 2048, 96, False, 0),
])
def test_grouped_heads_share_one_pass_over_their_keys(dtype, B, H, Hkv, Sq, Skv, D, causal, splits):
    """Query head h reads key/value head h // G.  The oracle gets K and V repeated G times along the
    head axis, i.e. the plain definition for every query head."""
    G = H // Hkv
    q = make_qkv(B, H, Sq, D, dtype, seed=71)[0]
    _, k, v = make_qkv(B, Hkv, Skv, D, dtype, seed=72)
    say(f"[case] grouped heads B={B} H={H} Hkv={Hkv} Sq={Sq} Skv={Skv} D={D} {dtype} causal={causal} splits={splits}")
    o, lse = binding.sdpa_kv(q.cuda(), k.cuda(), v.cuda(), causal=causal, splits=splits, return_lse=True)
    torch.cuda.synchronize()
    assert o.shape == q.shape and lse.shape == q.shape[:3]
    kx = np.repeat(k.float().numpy(), G, axis=1)
    vx = np.repeat(v.float().numpy(), G, axis=1)
    ref_o, ref_lse = orc.sdpa(q.float().numpy(), kx, vx, return_lse=True, causal=causal)
    err = float(np.abs(o.cpu().double().numpy() - ref_o).max())
    lerr = float(np.abs(lse.cpu().double().numpy() - ref_lse).max())
    say(f"        max|dO|={err:.3e} max|dLSE|={lerr:.3e}")
    assert err <= TOL[dtype] and lerr <= LSE_TOL * max(1.0, float(np.abs(ref_lse).max()) / 16)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("tile", [None, (64, 32), (128, 64)])
@pytest.mark.parametrize("B,H,Hkv,Sq,Skv,D,splits", [
    (1, 8, 2, 40, 200, 64, 0),        # four heads of 40 rows in one 160-row run: tiles cross head boundaries
    (2, 6, 3, 64, 64, 128, 0),        # square per head (prefill from an empty cache), two heads per group
    (1, 4, 1, 130, 1000, 128, 3),     # multi-query, a prefill chunk after 870 cached positions, split keys
    (1, 16, 2, 7, 7, 64, 0),          # groups of eight tiny heads inside one tile
    (1, 4, 2, 200, 333, 96, 2),
    (1, 3, 1, 33, 4096, 128, 0),      # split heuristic on a long cache
])
def test_grouped_heads_under_the_causal_mask(dtype, tile, B, H, Hkv, Sq, Skv, D, splits):
    """Every query head keeps its own causal limit (its rows are the last Sq positions) although the
    rows of a group run through the kernel as one block."""
    G = H // Hkv
    q = make_qkv(B, H, Sq, D, dtype, seed=75)[0]
    _, k, v = make_qkv(B, Hkv, Skv, D, dtype, seed=76)
    say(f"[case] grouped causal B={B} H={H} Hkv={Hkv} Sq={Sq} Skv={Skv} D={D} {dtype} tile={tile} splits={splits}")
    o, lse = binding.sdpa_kv(q.cuda(), k.cuda(), v.cuda(), causal=True, splits=splits, tile=tile, return_lse=True)
    torch.cuda.synchronize()
    kx = np.repeat(k.float().numpy(), G, axis=1)
    vx = np.repeat(v.float().numpy(), G, axis=1)
    ref_o, ref_lse = orc.sdpa(q.float().numpy(), kx, vx, return_lse=True, causal=True)
    err = float(np.abs(o.cpu().double().numpy() - ref_o).max())
    lerr = float(np.abs(lse.cpu().double().numpy() - ref_lse).max())
    say(f"        max|dO|={err:.3e} max|dLSE|={lerr:.3e}")
    assert torch.isfinite(o.float()).all()
    assert err <= TOL[dtype] and lerr <= LSE_TOL * max(1.0, float(np.abs(ref_lse).max()) / 16)


def test_grouped_heads_do_not_see_later_keys():
    """Changing keys and values after a head's last position changes nothing for it: with Sq = 3 rows per
    head at the end of 50 keys, row i of every head of the group must ignore keys > 47 + i."""
    q = make_qkv(1, 4, 3, 64, "f16", seed=77)[0].cuda()
    _, k, v = (t.cuda() for t in make_qkv(1, 1, 50, 64, "f16", seed=78))
    o1 = binding.sdpa_kv(q, k, v, causal=True)
    k2, v2 = k.clone(), v.clone()
    k2[:, :, 48:] = 9.0
    v2[:, :, 48:] = -7.0
    o2 = binding.sdpa_kv(q, k2, v2, causal=True)
    torch.cuda.synchronize()
    assert torch.equal(o1[:, :, 0], o2[:, :, 0])          # row 0 of every head sees keys 0..47 only
    assert not torch.equal(o1[:, :, 2], o2[:, :, 2])      # row 2 sees them all


def test_head_counts_that_do_not_divide_are_refused():
    q = make_qkv(1, 7, 4, 64, "f16", seed=73)[0].cuda()
    _, k, v = (t.cuda() for t in make_qkv(1, 2, 64, 64, "f16", seed=74))
    with pytest.raises(ValueError):
        binding.sdpa_kv(q, k, v)                          # 7 query heads over 2 key/value heads
    st = binding.tiled_sdpa_fwd_gqa(q.data_ptr(), k.data_ptr(), v.data_ptr(), q.data_ptr(), None,
                                    1, 7, 2, 4, 64, 64, 0.125, binding.F16, None)
    assert st == 2


# ------------------------------------------------------------------ KV cache with a length per batch entry
def check_kv_lens(B, H, Hkv, Sq, cap, D, dtype, lens, causal, splits, tile=None):
    """Entry b against the oracle on its first lens[b] key rows (the plain definition on the valid part of
    the cache).  Rows past the length are NaN in the device tensors: nothing of them may reach the output.
    A row that no key reaches must come back as exactly 0 with LSE = -inf."""
    G = H // Hkv
    q = make_qkv(B, H, Sq, D, dtype, seed=81)[0]
    _, k, v = make_qkv(B, Hkv, cap, D, dtype, seed=82)
    kd, vd = k.clone(), v.clone()
    for b, n in enumerate(lens):
        kd[b, :, n:] = float("nan")
        vd[b, :, n:] = float("nan")
    say(f"[case] kv_lens B={B} H={H} Hkv={Hkv} Sq={Sq} cap={cap} D={D} {dtype} lens={lens} causal={causal} splits={splits} tile={tile}")
    lens_d = torch.tensor(lens, dtype=torch.int32, device="cuda")
    o, lse = binding.sdpa_kv(q.cuda(), kd.cuda(), vd.cuda(), causal=causal, splits=splits, tile=tile,
                             return_lse=True, kv_lens=lens_d)
    torch.cuda.synchronize()
    o, lse = o.cpu(), lse.cpu()
    worst = 0.0
    for b, n in enumerate(lens):
        first = max(0, Sq - n) if causal else (Sq if n == 0 else 0)       # rows before `first` see no key
        assert torch.all(o[b, :, :first] == 0), f"entry {b}: rows without keys must be zero"
        assert torch.all(lse[b, :, :first] == float("-inf")), f"entry {b}: LSE of rows without keys must be -inf"
        if first == Sq:
            continue
        kx = np.repeat(k[b:b + 1, :, :n].float().numpy(), G, axis=1)
        vx = np.repeat(v[b:b + 1, :, :n].float().numpy(), G, axis=1)
        ref_o, ref_lse = orc.sdpa(q[b:b + 1, :, first:].float().numpy(), kx, vx, return_lse=True, causal=causal)
        got_o, got_lse = o[b:b + 1, :, first:].double().numpy(), lse[b:b + 1, :, first:].double().numpy()
        assert np.isfinite(got_o).all() and np.isfinite(got_lse).all(), f"entry {b}: non-finite output"
        err, lerr = float(np.abs(got_o - ref_o).max()), float(np.abs(got_lse - ref_lse).max())
        worst = max(worst, err)
        assert err <= TOL[dtype], f"entry {b} (len {n}): max|dO| {err}"
        assert lerr <= LSE_TOL * max(1.0, float(np.abs(ref_lse).max()) / 16), f"entry {b} (len {n}): max|dLSE| {lerr}"
    say(f"        worst max|dO|={worst:.3e}")


@pytest.mark.parametrize("D", [64, 96, 128, 160])
@pytest.mark.parametrize("splits", [5, 8, 9, 31, 64, 128])
def test_many_splits_take_the_one_row_per_workgroup_merge(D, splits):
    """Above eight splits (and up to 2048 output rows) the partial states of a row are combined by eight
    threads per column group through the LDS, otherwise by one thread that walks them: every head dim (its block is D/4 x 8 threads), split counts that do not divide by
    eight, entries whose later splits (or all of them) see no key, grouped heads and LSE."""
    dtype = "bf16" if D in (64, 160) else "f16"
    check_kv_lens(4, 4, 2, 1, 1100, D, dtype, [1100, 0, 65, 513], False, splits)
    check_kv_lens(2, 4, 1, 3, 900, D, dtype, [900, 2], True, splits)
    q, k, v = make_q_kv(1, 2, 70, 2100, D, dtype, seed=9300 + D + splits)     # two query tiles of 64 rows
    check_kv(q, k, v, dtype, splits=splits, causal=True, tile=(64, 64), tag="wide merge, chunk")


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("splits", [0, 1, 4])
def test_decoding_step_over_a_cache_with_a_length_per_entry(dtype, causal, splits):
    check_kv_lens(5, 8, 2, 1, 700, 128, dtype, [700, 1, 333, 0, 64], causal, splits)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("tile", [None, (64, 32), (128, 64)])
def test_prefill_chunks_over_a_cache_with_a_length_per_entry(dtype, tile):
    # entry 2 holds fewer positions than the chunk has rows: its first 28 rows precede every key
    check_kv_lens(3, 4, 4, 48, 300, 64, dtype, [300, 48, 20], True, 0, tile)
    check_kv_lens(3, 6, 2, 48, 300, 64, dtype, [257, 300, 5], True, 3, tile)
    check_kv_lens(2, 4, 1, 5, 1000, 96, dtype, [999, 31], False, 0, tile)


def test_lengths_beyond_the_capacity_are_clamped():
    check_kv_lens(2, 2, 2, 1, 100, 64, "f16", [100, 100], False, 0)
    q = make_qkv(2, 2, 1, 64, "f16", seed=83)[0].cuda()
    _, k, v = (t.cuda() for t in make_qkv(2, 2, 100, 64, "f16", seed=84))
    a = binding.sdpa_kv(q, k, v, kv_lens=torch.tensor([100, 100], dtype=torch.int32, device="cuda"))
    b = binding.sdpa_kv(q, k, v, kv_lens=torch.tensor([5000, -3], dtype=torch.int32, device="cuda"))
    torch.cuda.synchronize()
    assert torch.equal(a[0], b[0])                  # 5000 > capacity: the whole cache
    assert torch.all(b[1] == 0)                     # negative: an empty entry


# ------------------------------------------------------------------ paged cache
def check_paged(B, H, Hkv, Sq, D, dtype, lens, block_rows, causal, splits, tile=None, seed=91):
    """Dense per-entry caches are cut into pages that are scattered over a pool in a seeded random order
    (unused pool pages and the unused tail of every last page hold NaN); the oracle sees the dense rows."""
    G = H // Hkv
    cap = max(1, max(lens))
    max_blocks = (cap + block_rows - 1) // block_rows
    q = make_qkv(B, H, Sq, D, dtype, seed=seed)[0]
    _, k, v = make_qkv(B, Hkv, max_blocks * block_rows, D, dtype, seed=seed + 1)
    used = [(n + block_rows - 1) // block_rows for n in lens]
    pool = sum(used) + 3                                    # a few pages nobody owns
    rng = np.random.default_rng(seed)
    order = rng.permutation(pool)
    kp = torch.full((pool, Hkv, block_rows, D), float("nan"), dtype=k.dtype)
    vp = torch.full((pool, Hkv, block_rows, D), float("nan"), dtype=v.dtype)
    table = np.full((B, max(1, max_blocks)), -12345, dtype=np.int32)    # unused slots: garbage that must not be followed
    nxt = 0
    for b in range(B):
        for i in range(used[b]):
            page = int(order[nxt]); nxt += 1
            table[b, i] = page
            rows = min(block_rows, lens[b] - i * block_rows)
            kp[page, :, :rows] = k[b, :, i * block_rows:i * block_rows + rows]
            vp[page, :, :rows] = v[b, :, i * block_rows:i * block_rows + rows]
    say(f"[case] paged B={B} H={H} Hkv={Hkv} Sq={Sq} D={D} {dtype} lens={lens} block_rows={block_rows} causal={causal} splits={splits} tile={tile}")
    o, lse = binding.sdpa_paged(q.cuda(), kp.cuda(), vp.cuda(), torch.tensor(lens, dtype=torch.int32, device="cuda"),
                                torch.from_numpy(table).cuda(), causal=causal, splits=splits, tile=tile, return_lse=True)
    torch.cuda.synchronize()
    o, lse = o.cpu(), lse.cpu()
    for b, n in enumerate(lens):
        first = max(0, Sq - n) if causal else (Sq if n == 0 else 0)
        assert torch.all(o[b, :, :first] == 0) and torch.all(lse[b, :, :first] == float("-inf"))
        if first == Sq:
            continue
        kx = np.repeat(k[b:b + 1, :, :n].float().numpy(), G, axis=1)
        vx = np.repeat(v[b:b + 1, :, :n].float().numpy(), G, axis=1)
        ref_o, ref_lse = orc.sdpa(q[b:b + 1, :, first:].float().numpy(), kx, vx, return_lse=True, causal=causal)
        got_o, got_lse = o[b:b + 1, :, first:].double().numpy(), lse[b:b + 1, :, first:].double().numpy()
        assert np.isfinite(got_o).all() and np.isfinite(got_lse).all(), f"entry {b}: non-finite output"
        err, lerr = float(np.abs(got_o - ref_o).max()), float(np.abs(got_lse - ref_lse).max())
        assert err <= TOL[dtype], f"entry {b} (len {n}): max|dO| {err}"
        assert lerr <= LSE_TOL * max(1.0, float(np.abs(ref_lse).max()) / 16), f"entry {b} (len {n}): max|dLSE| {lerr}"


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("block_rows", [64, 256])
@pytest.mark.parametrize("splits", [0, 1, 5])
def test_decoding_step_over_a_paged_cache(dtype, block_rows, splits):
    check_paged(5, 8, 2, 1, 128, dtype, [700, 1, 333, 0, 64], block_rows, True, splits)
    check_paged(3, 4, 4, 1, 64, dtype, [block_rows, 2 * block_rows + 1, 3 * block_rows - 1], block_rows, False, splits)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("tile", [None, (64, 32), (64, 64), (128, 32), (128, 64)])
def test_prefill_chunks_over_a_paged_cache(dtype, tile):
    check_paged(3, 6, 2, 48, 64, dtype, [300, 48, 20], 64, True, 0, tile)
    check_paged(2, 4, 1, 130, 128, dtype, [1000, 131], 128, True, 3, tile)
    check_paged(2, 2, 2, 5, 96, dtype, [515, 31], 512, False, 0, tile)
    check_paged(1, 2, 1, 3, 160, dtype, [200], 64, True, 2, tile)


def test_paged_and_dense_caches_agree_bit_for_bit():
    """Same rows, same tiles, same order of operations: only the addresses differ.  (With more than one
    query tile per head; on a single one the dense path starts each workgroup's sweep at a tile of its
    own, so there the two agree to rounding only.)"""
    B, H, Hkv, D, block_rows, lens = 2, 4, 2, 128, 128, [1000, 513]
    _, k, v = (t.cuda() for t in make_qkv(B, Hkv, 1024, D, "bf16", seed=96))
    lens_d = torch.tensor(lens, dtype=torch.int32, device="cuda")
    # pages in reverse order of the dense blocks
    nb = 1024 // block_rows
    kp = k.view(B, Hkv, nb, block_rows, D).permute(0, 2, 1, 3, 4).reshape(B * nb, Hkv, block_rows, D).flip(0).contiguous()
    vp = v.view(B, Hkv, nb, block_rows, D).permute(0, 2, 1, 3, 4).reshape(B * nb, Hkv, block_rows, D).flip(0).contiguous()
    table = (B * nb - 1 - torch.arange(B * nb, dtype=torch.int32, device="cuda")).view(B, nb).contiguous()
    for Sq, causal, exact in ((200, True, True), (200, False, True), (1, False, False)):
        q = make_qkv(B, H, Sq, D, "bf16", seed=95)[0].cuda()
        dense = binding.sdpa_kv(q, k, v, kv_lens=lens_d, splits=4, causal=causal)
        paged = binding.sdpa_paged(q, kp, vp, lens_d, table, splits=4, causal=causal)
        torch.cuda.synchronize()
        if exact:
            assert torch.equal(dense, paged), f"Sq={Sq} causal={causal}"
        else:
            assert float((dense.float() - paged.float()).abs().max()) <= TOL["bf16"] / 4


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_long_query_blocks_without_mask_take_the_256_row_tile(dtype):
    """B*Hkv*ceil(G*Sq/256) >= 256 query tiles of 256 rows, no mask, one cache length, no split: the heuristic's
    choice on such shapes; checked in full on small ones (grouped heads fold G*Sq rows per key/value head, so a
    256-row tile crosses from one query head into the next), also pinned with splits, and refused on a paged cache."""
    for B, H, Hkv, Sq, Skv, D in ((16, 8, 4, 1100, 300, 128), (64, 2, 2, 2100, 130, 96)):
        G = H // Hkv
        q = make_qkv(B, H, Sq, D, dtype, seed=9700 + Sq)[0]
        _, k, v = make_qkv(B, Hkv, Skv, D, dtype, seed=9701 + Sq)
        ref_o, ref_lse = orc.sdpa(q.float().numpy(), np.repeat(k.float().numpy(), G, axis=1),
                                  np.repeat(v.float().numpy(), G, axis=1), return_lse=True)
        for tile, splits in ((None, 0), ((256, 64), 3), ((128, 64), 1)):
            say(f"[case] long query blocks B={B} H={H} Hkv={Hkv} Sq={Sq} Skv={Skv} D={D} {dtype} tile={tile} splits={splits}")
            o, lse = binding.sdpa_kv(q.cuda(), k.cuda(), v.cuda(), splits=splits, tile=tile, return_lse=True)
            torch.cuda.synchronize()
            err = float(np.abs(o.cpu().double().numpy() - ref_o).max())
            lerr = float(np.abs(lse.cpu().double().numpy() - ref_lse).max())
            say(f"        max|dO|={err:.3e}  max|dLSE|={lerr:.3e}")
            assert err <= TOL[dtype] and lerr <= LSE_TOL * max(1.0, float(np.abs(ref_lse).max()) / 16.0)
    with pytest.raises(binding.TiledSdpaError):
        check_paged(1, 2, 1, 3, 128, dtype, [200], 64, False, 1, (256, 64))
