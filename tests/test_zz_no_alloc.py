"""The entry point that allocates nothing: tiled_sdpa_fwd_kvcache_static keeps its split states in a
device buffer that is part of the library, and must give, through the C-ABI, the very bits of
tiled_sdpa_fwd_kvcache with a caller's workspace (the same kernels run), also on a second, smaller call
that finds the first call's contents in the buffer.  Also checked against the float64 oracle."""
import math
import sys

import numpy as np
import pytest
import torch

from oracle import sdpa_oracle as orc
from paper_2603_01960_amd import binding
from paper_2603_01960_amd.workloads import make_qkv

pytestmark = pytest.mark.gpu

TOL = {"f16": 2e-3, "bf16": 1.6e-2}


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def both(B, H, Hkv, Sq, Skv, D, dtype, splits, causal, lens=None, seed=0):
    """(static entry point's o, lse), (workspace entry point's o, lse), oracle inputs -- raw C-ABI calls."""
    say(f"[case] static scratch B={B} H={H} Hkv={Hkv} Sq={Sq} Skv={Skv} D={D} {dtype} splits={splits} causal={causal} lens={lens}")
    q = make_qkv(B, H, Sq, D, dtype, seed=seed)[0]
    _, k, v = make_qkv(B, Hkv, Skv, D, dtype, seed=seed + 1)
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    code = binding.F16 if dtype == "f16" else binding.BF16
    flags = binding.FLAG_CAUSAL if causal else 0
    stream = torch.cuda.current_stream().cuda_stream
    lens_d = None if lens is None else torch.tensor(lens, dtype=torch.int32, device="cuda")
    lp = None if lens_d is None else lens_d.data_ptr()
    need = binding.kv_workspace_bytes(B, H, Sq, D, splits)
    assert 0 < need <= binding.STATIC_SCRATCH_BYTES
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    res = []
    for static in (True, False):
        o = torch.full_like(qd, float("nan"))
        lse = torch.full((B, H, Sq), float("nan"), dtype=torch.float32, device="cuda")
        if static:
            st = binding.tiled_sdpa_fwd_kvcache_static(qd.data_ptr(), kd.data_ptr(), vd.data_ptr(), o.data_ptr(),
                                                       lse.data_ptr(), lp, B, H, Hkv, Sq, Skv, D, math.nan, code, stream,
                                                       0, 0, flags, splits)
        else:
            st = binding.tiled_sdpa_fwd_kvcache(qd.data_ptr(), kd.data_ptr(), vd.data_ptr(), o.data_ptr(),
                                                lse.data_ptr(), lp, B, H, Hkv, Sq, Skv, D, math.nan, code, stream,
                                                0, 0, flags, splits, ws.data_ptr(), need)
        assert st == 0, binding.status_string(st)
        torch.cuda.synchronize()
        res.append((o.cpu(), lse.cpu()))
    return res[0], res[1], (q, k, v)


def against_oracle(o, q, k, v, G, dtype, causal):
    kk, vv = (t.repeat_interleave(G, dim=1) for t in (k, v))
    ref = orc.sdpa(q.float().numpy(), kk.float().numpy(), vv.float().numpy(), causal=causal)
    err = float(np.abs(o.double().numpy() - ref).max())
    say(f"        max|dO| vs oracle = {err:.3e} (tol {TOL[dtype]:.1e})")
    assert err <= TOL[dtype]


def test_two_calls_in_a_row_the_second_smaller_match_the_workspace_entry_point():
    binding.load_library()
    # a decoding step over a long cache with grouped heads, then a smaller problem (fewer heads, fewer
    # splits, shorter cache, other head dim) that finds the first call's states in the buffer
    for (B, H, Hkv, Sq, Skv, D, dtype, splits, causal) in ((2, 16, 4, 3, 5000, 128, "bf16", 16, True),
                                                           (1, 4, 4, 1, 700, 64, "f16", 3, False)):
        s, w, (q, k, v) = both(B, H, Hkv, Sq, Skv, D, dtype, splits, causal, seed=31000 + Skv)
        assert torch.isfinite(s[0].float()).all() and torch.isfinite(s[1]).all()
        assert torch.equal(s[0], w[0]) and torch.equal(s[1], w[1]), "static scratch and caller workspace disagree"
        against_oracle(s[0], q, k, v, H // Hkv, dtype, causal)


def test_lengths_per_entry_heuristic_splits_and_the_size_limit():
    binding.load_library()
    s, w, _ = both(3, 8, 2, 2, 2048, 96, "bf16", 8, True, lens=[2048, 5, 900], seed=31500)
    assert torch.equal(s[0], w[0]) and torch.equal(s[1], w[1])
    # splits = 0: the heuristic's count, the same in both entry points
    B, H, Sq, Skv, D = 1, 8, 1, 16384, 128
    q = make_qkv(B, H, Sq, D, "f16", seed=31600)[0].cuda()
    _, k, v = (t.cuda() for t in make_qkv(B, H, Skv, D, "f16", seed=31601))
    o = torch.empty_like(q)
    stream = torch.cuda.current_stream().cuda_stream
    st = binding.tiled_sdpa_fwd_kvcache_static(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), None, None,
                                               B, H, H, Sq, Skv, D, math.nan, binding.F16, stream, 0, 0, 0, 0)
    assert st == 0
    torch.cuda.synchronize()
    assert torch.equal(o, binding.sdpa_kv(q, k, v))
    # beyond the limit: refused with its own status, nothing enqueued, o untouched
    B, H, Sq, splits = 8, 32, 128, 64
    assert binding.kv_workspace_bytes(B, H, Sq, D, splits) > binding.STATIC_SCRATCH_BYTES
    q = torch.zeros(B, H, Sq, D, dtype=torch.float16, device="cuda")
    k = torch.zeros(B, H, 4096, D, dtype=torch.float16, device="cuda")
    o = torch.full_like(q, 5.0)
    st = binding.tiled_sdpa_fwd_kvcache_static(q.data_ptr(), k.data_ptr(), k.data_ptr(), o.data_ptr(), None, None,
                                               B, H, H, Sq, 4096, D, math.nan, binding.F16, stream, 0, 0, 0, splits)
    assert st == 11, binding.status_string(st)
    torch.cuda.synchronize()
    assert (o == 5.0).all()
