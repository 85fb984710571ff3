"""Parity of the backward pass (through the C-ABI) against the float64 CPU oracle.

Tolerance: the paper gives none for gradients.  Each gradient element is a sum of products of 16-bit
rounded factors, rounded once more on output, so the error scales with the magnitude of the
gradient tensor: max|g - ref| <= tol * max(1, max|ref|) with the forward tolerances tol = 2e-3
(FP16) and 1.6e-2 (BF16); all outputs finite.
"""
import sys

import numpy as np
import pytest
import torch

from oracle import sdpa_oracle as orc
from paper_2603_01960_amd import binding
from paper_2603_01960_amd.workloads import make_qkv, make_workload, sample_rows

pytestmark = pytest.mark.gpu

TOL = {"f16": 2e-3, "bf16": 1.6e-2}


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module", autouse=True)
def _device():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    binding.load_library()
    yield
    torch.cuda.synchronize()


def make_dout(shape, dtype, seed):
    g = torch.Generator(device="cpu").manual_seed(int(seed))
    return torch.randn(*shape, dtype=torch.float32, generator=g).to(torch.float16 if dtype == "f16" else torch.bfloat16)


def gpu_bwd(q, k, v, do, causal=False, scale=None):
    qd, kd, vd, dd = (t.cuda() for t in (q, k, v, do))
    o, lse = binding.sdpa(qd, kd, vd, causal=causal, scale=scale, return_lse=True)
    dq, dk, dv = binding.sdpa_backward(qd, kd, vd, o, dd, lse, causal=causal, scale=scale)
    torch.cuda.synchronize()
    return dq.cpu(), dk.cpu(), dv.cpu()


def compare(got, ref, dtype, tag):
    worst = 0.0
    for name, g, r in zip(("dq", "dk", "dv"), got, ref):
        assert torch.isfinite(g.float()).all(), f"{tag}: non-finite {name}"
        gn = g.double().numpy()
        if gn.size == 0:
            continue
        err = float(np.abs(gn - r).max())
        bound = TOL[dtype] * max(1.0, float(np.abs(r).max()))
        say(f"        {name}: max|err|={err:.3e}  bound={bound:.3e}  max|ref|={float(np.abs(r).max()):.3f}")
        assert err <= bound, f"{tag}: {name} error {err} > {bound}"
        worst = max(worst, err / bound)
    return worst


def check_bwd(q, k, v, do, dtype, causal=False, scale=None, tag=""):
    say(f"[case] bwd {tag} shape={tuple(q.shape)} dtype={dtype} causal={causal} scale={scale}")
    got = gpu_bwd(q, k, v, do, causal=causal, scale=scale)
    ref = orc.sdpa_bwd(q.float().numpy(), k.float().numpy(), v.float().numpy(), do.float().numpy(),
                       scale=scale, causal=causal)
    return compare(got, ref, dtype, tag)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("D", [64, 128])
def test_small_shapes(D, dtype, causal):
    # lengths around the 32/64-row tile and 128-row workgroup edges, a prime, one row
    for S in (1, 2, 31, 32, 33, 63, 64, 65, 127, 128, 129, 197, 257, 300, 517):
        q, k, v = make_qkv(2, 2, S, D, dtype, seed=12000 + S)
        do = make_dout(q.shape, dtype, 12500 + S)
        check_bwd(q, k, v, do, dtype, causal=causal, tag=f"small S={S}")


@pytest.mark.parametrize("scale", [0.0, -0.125, 0.5, 1e-3])
def test_scale_variants(scale):
    q, k, v = make_qkv(1, 2, 200, 64, "f16", seed=12100)
    check_bwd(q, k, v, make_dout(q.shape, "f16", 12101), "f16", scale=scale, tag=f"scale={scale}")
    q, k, v = make_qkv(1, 2, 150, 128, "bf16", seed=12102)
    check_bwd(q, k, v, make_dout(q.shape, "bf16", 12103), "bf16", scale=scale, causal=True, tag=f"scale={scale}")


def test_closed_forms_on_the_device():
    # one key: dV = dO, dQ = dK = 0 (up to the rounding of P = exp(s - lse) and of dP - Delta, both
    # differences of two FP32 evaluations of the same quantity)
    q, k, v = make_qkv(2, 2, 1, 64, "f16", seed=12200)
    do = make_dout(q.shape, "f16", 12201)
    dq, dk, dv = gpu_bwd(q, k, v, do)
    assert (dv.float() - do.float()).abs().max().item() <= 2e-3
    assert dq.float().abs().max().item() <= 1e-3 and dk.float().abs().max().item() <= 1e-3
    # dout = 0: every gradient is zero
    q, k, v = make_qkv(1, 2, 300, 128, "bf16", seed=12202)
    for g in gpu_bwd(q, k, v, torch.zeros_like(q), causal=True):
        assert not g.any()
    # identical value rows: the output does not depend on q or k
    v2 = v[:, :, :1].expand_as(v).contiguous()
    dq, dk, dv = gpu_bwd(q, k, v2, make_dout(q.shape, "bf16", 12203))
    assert dq.float().abs().max().item() <= 1.6e-2 and dk.float().abs().max().item() <= 1.6e-2


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("D", [64, 96, 128, 160])
def test_rows_that_see_one_or_two_keys(D, dtype):
    """dS = P (dP - Delta) cancels heavily on rows of one or two keys (P of order 1); there Delta comes
    from its definition in FP32, not from the 16-bit forward output.  Many seeds, at the usual bound."""
    for seed in range(12):
        for S, causal in ((1, False), (2, False), (3, True), (2, True), (40, True), (64, False), (65, True), (130, True)):
            q, k, v = make_qkv(1, 2, S, D, dtype, seed=12800 + 17 * seed + S)
            do = make_dout(q.shape, dtype, 12900 + seed)
            check_bwd(q, k, v, do, dtype, causal=causal, tag=f"few keys D={D} S={S} seed={seed}")


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_many_heads_of_a_few_hundred_rows_at_D128(dtype):
    """At D = 128 without the causal mask the passes take 256 resident rows per workgroup once that gives 256
    workgroups: 128 heads of 257 ... 700 rows do, with a ragged last tile, and are small enough to check in full."""
    for B, H, S in ((8, 16, 300), (2, 64, 257), (4, 32, 545)):
        q, k, v = make_qkv(B, H, S, 128, dtype, seed=13100 + S)
        do = make_dout(q.shape, dtype, 13150 + S)
        check_bwd(q, k, v, do, dtype, tag=f"wide workgroups B={B} H={H} S={S}")


def test_full_configurations_C2_and_C3():
    for name, dtype in (("C2", "f16"), ("C2", "bf16"), ("C3", "bf16")):
        w, q, k, v = make_workload(name, dtype)
        do = make_dout(q.shape, dtype, w.seed + 50)
        check_bwd(q, k, v, do, dtype, tag=name)
        check_bwd(q, k, v, do, dtype, causal=True, tag=name + " causal")


@pytest.mark.parametrize("name,dtype", [("C4", "bf16"), ("C5", "f16")])
def test_long_configurations_on_sampled_heads_and_rows(name, dtype):
    """The kernels run the whole configuration; the oracle checks two (batch, head) slices of it on
    sampled query rows (dQ) and key rows (dK, dV)."""
    w, q, k, v = make_workload(name, dtype)
    do = make_dout(q.shape, dtype, w.seed + 50)
    rows = sample_rows(w.S)
    for causal in (False, True):
        say(f"[case] bwd {name} {dtype} causal={causal} full size, sampled")
        got = gpu_bwd(q, k, v, do, causal=causal)
        for (b, h) in ((0, 0), (w.B - 1, w.H - 1)):
            sl = lambda t: t[b:b + 1, h:h + 1].float().numpy()
            ref = orc.sdpa_bwd(sl(q), sl(k), sl(v), sl(do), causal=causal, qrows=rows, krows=rows,
                               scale=None)
            compare([g[b:b + 1, h:h + 1][:, :, rows] for g in got], ref, dtype, f"{name} head ({b},{h})")


def test_results_are_deterministic_and_buffers_are_respected():
    q, k, v = make_qkv(2, 3, 333, 128, "bf16", seed=12300)
    do = make_dout(q.shape, "bf16", 12301)
    qd, kd, vd, dd = (t.cuda() for t in (q, k, v, do))
    o, lse = binding.sdpa(qd, kd, vd, causal=True, return_lse=True)
    a = binding.sdpa_backward(qd, kd, vd, o, dd, lse, causal=True)
    need = binding.bwd_workspace_bytes(2, 3, 333)
    ws = torch.full((need // 4 + 64,), float("nan"), dtype=torch.float32, device="cuda")
    grads = tuple(torch.full_like(qd, float("nan")) for _ in range(3))
    b = binding.sdpa_backward(qd, kd, vd, o, dd, lse, causal=True, workspace=ws, grads=grads)
    torch.cuda.synchronize()
    for x, y in zip(a, b):
        assert torch.equal(x, y) and torch.isfinite(y.float()).all()
    assert torch.isnan(ws[need // 4:]).all(), "wrote past the stated workspace size"
    with pytest.raises(binding.TiledSdpaError):
        binding.sdpa_backward(qd, kd, vd, o, dd, lse, workspace=ws[: need // 4 - 1])


def test_nothing_is_read_past_the_end_of_the_inputs():
    """q, k, v, dout sit inside NaN-filled buffers: a fetch past the last row would poison a gradient."""
    B, H, S, D = 1, 3, 197, 64
    q, k, v = make_qkv(B, H, S, D, "f16", seed=12400)
    do = make_dout(q.shape, "f16", 12401)
    pad, n = 8192, B * H * S * D

    def guarded(t):
        buf = torch.full((n + 2 * pad,), float("nan"), dtype=t.dtype, device="cuda")
        view = buf[pad:pad + n].view(B, H, S, D)
        view.copy_(t)
        return view
    qd, kd, vd, dd = (guarded(t) for t in (q, k, v, do))
    for causal in (False, True):
        o, lse = binding.sdpa(qd, kd, vd, causal=causal, return_lse=True)
        got = binding.sdpa_backward(qd, kd, vd, o, dd, lse, causal=causal)
        torch.cuda.synchronize()
        ref = orc.sdpa_bwd(q.float().numpy(), k.float().numpy(), v.float().numpy(), do.float().numpy(), causal=causal)
        compare([g.cpu() for g in got], ref, "f16", "guarded")


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("D", [96, 160])
def test_head_dims_96_and_160(D, dtype, causal):
    for S in (1, 33, 64, 130, 197, 300, 517, 1024):
        q, k, v = make_qkv(1, 3, S, D, dtype, seed=12600 + S + D)
        do = make_dout(q.shape, dtype, 12700 + S)
        check_bwd(q, k, v, do, dtype, causal=causal, tag=f"D={D} S={S}")


def test_unsupported_head_dims_are_refused():
    x = torch.zeros(1, 1, 16, 80, dtype=torch.float16, device="cuda")
    lse = torch.zeros(1, 1, 16, dtype=torch.float32, device="cuda")
    with pytest.raises(binding.TiledSdpaError) as e:
        binding.sdpa_backward(x, x, x, x, x, lse)
    assert e.value.status == 4


# ------------------------------------------------------------------ grouped heads
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("B,H,Hkv,S,D", [(2, 4, 2, 200, 64), (1, 8, 1, 333, 128), (1, 6, 2, 130, 96),
                                         (1, 4, 2, 100, 160), (1, 4, 4, 70, 128), (2, 8, 2, 1, 64)])
def test_grouped_heads(B, H, Hkv, S, D, dtype, causal):
    """dK and dV are sums over the query heads of a group, taken inside one workgroup per key tile."""
    q = make_qkv(B, H, S, D, dtype, seed=61)[0]
    _, k, v = make_qkv(B, Hkv, S, D, dtype, seed=62)
    do = make_dout(q.shape, dtype, 63)
    say(f"[case] bwd grouped B={B} H={H} Hkv={Hkv} S={S} D={D} {dtype} causal={causal}")
    qd, kd, vd, dd = (t.cuda() for t in (q, k, v, do))
    o, lse = binding.sdpa_kv(qd, kd, vd, causal=causal, return_lse=True)
    dq, dk, dv = binding.sdpa_backward(qd, kd, vd, o, dd, lse, causal=causal)
    torch.cuda.synchronize()
    assert dq.shape == q.shape and dk.shape == k.shape and dv.shape == v.shape
    ref = orc.sdpa_bwd_grouped(q.float().numpy(), k.float().numpy(), v.float().numpy(), do.float().numpy(),
                               causal=causal)
    compare((dq.cpu(), dk.cpu(), dv.cpu()), ref, dtype, "grouped")


def test_grouped_heads_at_a_long_sequence_on_sampled_rows():
    B, H, Hkv, S, D, dtype = 1, 8, 2, 4096, 128, "bf16"
    q = make_qkv(B, H, S, D, dtype, seed=64)[0]
    _, k, v = make_qkv(B, Hkv, S, D, dtype, seed=65)
    do = make_dout(q.shape, dtype, 66)
    rows = sample_rows(S)
    for causal in (False, True):
        say(f"[case] bwd grouped long S={S} causal={causal}")
        qd, kd, vd, dd = (t.cuda() for t in (q, k, v, do))
        o, lse = binding.sdpa_kv(qd, kd, vd, causal=causal, return_lse=True)
        got = binding.sdpa_backward(qd, kd, vd, o, dd, lse, causal=causal)
        torch.cuda.synchronize()
        ref = orc.sdpa_bwd_grouped(q.float().numpy(), k.float().numpy(), v.float().numpy(), do.float().numpy(),
                                   causal=causal, qrows=rows, krows=rows)
        compare([g.cpu()[:, :, rows] for g in got], ref, dtype, "grouped long")
