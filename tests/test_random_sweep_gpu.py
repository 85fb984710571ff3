"""Seeded random sweep over every entry point: shapes, head dims, tiles, split counts, grouped heads,
cache lengths and page sizes drawn together, each case checked against the oracle with the tolerances of
the hand-picked tests.  The hand-picked cases aim at edges one at a time; this aims at their combinations.
The draws are fixed by the seeds below, so a failure names a reproducible case.
"""
import random

import pytest
import torch

import test_sdpa_bwd_gpu as bwd_cases
import test_sdpa_gpu as fwd_cases
import test_sdpa_kv_gpu as kv_cases
from paper_2603_01960_amd import binding
from paper_2603_01960_amd.workloads import make_qkv

pytestmark = pytest.mark.gpu

EDGE_LENGTHS = [1, 2, 31, 32, 33, 63, 64, 65, 127, 128, 129]


@pytest.fixture(scope="module", autouse=True)
def _device():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    binding.load_library()
    yield
    torch.cuda.synchronize()


def tiles_of(D, cache=False):
    tiles = [(64, 32), (64, 64), (128, 32), (128, 64), None]
    if D <= 128 and not cache:
        tiles += [(64, 128), (128, 128)]
    if not cache:
        tiles += [(256, 64)]          # the square problem only
    return tiles


def draw_common(rng):
    return rng.choice([64, 96, 128, 160]), rng.choice(["f16", "bf16"]), rng.random() < 0.5, rng.randrange(1 << 30)


@pytest.mark.parametrize("seed", [11, 12])
def test_forward_random_cases(seed):
    rng = random.Random(seed)
    for _ in range(40):
        D, dtype, causal, sd = draw_common(rng)
        B, H = rng.randint(1, 2), rng.randint(1, 3)
        S = rng.choice(EDGE_LENGTHS + [rng.randint(1, 900)])
        tile, scale = rng.choice(tiles_of(D)), rng.choice([None, None, 0.05, -0.1, 0.0])
        q, k, v = make_qkv(B, H, S, D, dtype, seed=sd)
        fwd_cases.check(q, k, v, dtype, scale=scale, tile=tile, causal=causal,
                        tag=f"random forward B={B} H={H} S={S} D={D} tile={tile} scale={scale} seed={sd}")


@pytest.mark.parametrize("seed", [21, 22])
def test_cache_random_cases(seed):
    rng = random.Random(seed)
    for _ in range(30):
        D, dtype, causal, sd = draw_common(rng)
        B, H = rng.randint(1, 3), rng.choice([2, 4, 6, 8])
        Hkv = rng.choice([h for h in (1, 2, 3, 4, 6, 8) if H % h == 0])
        Sq = rng.choice([1, 1, 1, 2, 5, 17, 64, 65, 130, rng.randint(1, 260)])
        splits, tile = rng.choice([0, 1, 2, 3, 4, 5, 7, 8, 16, 33, 64, 128]), rng.choice(tiles_of(D, cache=True))
        kind = rng.choice(["lengths", "pages"])
        if kind == "lengths":
            cap = rng.randint(Sq, 1500)
            lens = [rng.choice([0, 1, cap, rng.randint(0, cap)]) for _ in range(B)]
            kv_cases.check_kv_lens(B, H, Hkv, Sq, cap, D, dtype, lens, causal, splits, tile=tile)
        else:
            block_rows = rng.choice([64, 128, 256])
            lens = [rng.choice([0, 1, block_rows, block_rows + 1, rng.randint(0, 1400)]) for _ in range(B)]
            if causal and max(lens) < Sq:           # under the mask the cache holds at least the queries themselves
                lens[0] = Sq + rng.randint(0, 100)
            kv_cases.check_paged(B, H, Hkv, Sq, D, dtype, lens, block_rows, causal, splits, tile=tile, seed=sd % 100000)


@pytest.mark.parametrize("seed", [31, 32, 33, 34])
def test_backward_random_cases(seed):
    """Sequence lengths from one key upward.  Rows of one or two keys at D = 160 in BF16 used to exceed the bound
    (the rounding of the forward output inside Delta = rowsum(dO * O)); rows that see at most 64 keys now get
    Delta from its definition, sum_j P_ij dP_ij, in FP32."""
    rng = random.Random(seed)
    for _ in range(30):
        D, dtype, causal, sd = draw_common(rng)
        B, Hkv, G = rng.randint(1, 2), rng.randint(1, 2), rng.choice([1, 1, 2, 3, 4, 8])
        S = rng.choice([1, 2, 3, 8, 31, 33, 64, 65, 127, 129, rng.randint(1, 400)])
        H = Hkv * G
        q = make_qkv(B, H, S, D, dtype, seed=sd)[0]
        _, k, v = make_qkv(B, Hkv, S, D, dtype, seed=sd + 1)
        do = bwd_cases.make_dout(q.shape, dtype, sd + 2)
        tag = f"random backward B={B} H={H} Hkv={Hkv} S={S} D={D} {dtype} causal={causal} seed={sd}"
        bwd_cases.say(f"[case] {tag}")
        qd, kd, vd, dd = (t.cuda() for t in (q, k, v, do))
        o, lse = binding.sdpa_kv(qd, kd, vd, causal=causal, return_lse=True)
        grads = binding.sdpa_backward(qd, kd, vd, o, dd, lse, causal=causal)
        torch.cuda.synchronize()
        ref = bwd_cases.orc.sdpa_bwd_grouped(q.float().numpy(), k.float().numpy(), v.float().numpy(),
                                             do.float().numpy(), causal=causal)
        bwd_cases.compare(tuple(t.cpu() for t in grads), ref, dtype, tag)
