"""Pins for the backward-pass oracle (CPU only).

The paper prints no backward formula (Section 7 leaves it as future work), so the oracle's gradients
are pinned to things that do not share its derivation: (a) finite differences of a 50-digit Decimal
evaluation of Eq. 1 itself, (b) central differences of the float64 forward definition, (c) torch CPU
float64 autograd, (d) closed forms and invariants of the softmax Jacobian, (e) agreement of the
row-by-row C routine with the matrix-expression form and with row subsets, and (f) a mutation
check: planted mistakes in a copy of the formulas must each trip at least one pin.
"""
from decimal import Decimal, getcontext

import numpy as np
import pytest
import torch

from oracle import sdpa_oracle as orc


def _rand(shape, seed, dtype=np.float16, std=1.0):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal(shape) * std).astype(dtype)


def _inputs(S, D, seed, lead=(), std=1.2):
    return tuple(_rand((*lead, S, D), seed + i, std=std) for i in range(4))


# ------------------------------------------------- (a) finite differences in 50-digit arithmetic
def _forward_decimal(q, k, v, scale, causal):
    """Eq. 1 on lists of Decimals, no max subtraction, no float operations."""
    S, D = len(q), len(q[0])
    out = []
    for i in range(S):
        keys = range(i + 1) if causal else range(S)
        w = [(scale * sum(q[i][d] * k[j][d] for d in range(D))).exp() for j in keys]
        tot = sum(w)
        out.append([sum(wj * v[j][d] for wj, j in zip(w, keys)) / tot for d in range(D)])
    return out


@pytest.mark.parametrize("S,D", [(1, 2), (2, 2), (3, 2), (4, 3)])
@pytest.mark.parametrize("causal", [False, True])
def test_gradients_against_decimal_finite_differences(S, D, causal):
    getcontext().prec = 60
    q, k, v, do = _inputs(S, D, 700 + 10 * S + D, std=1.0)
    scale = float(np.float32(0.625))
    dec = lambda a: [[Decimal(float(x)) for x in row] for row in a]
    base = {"q": dec(q), "k": dec(k), "v": dec(v)}
    dO = dec(do)
    h = Decimal(10) ** -25

    def lam(args):
        o = _forward_decimal(args["q"], args["k"], args["v"], Decimal(scale), causal)
        return sum(dO[i][d] * o[i][d] for i in range(S) for d in range(D))

    grads = {}
    for name in ("q", "k", "v"):
        g = np.zeros((S, D))
        for i in range(S):
            for d in range(D):
                hi = {n: [row[:] for row in a] for n, a in base.items()}
                lo = {n: [row[:] for row in a] for n, a in base.items()}
                hi[name][i][d] += h
                lo[name][i][d] -= h
                g[i, d] = float((lam(hi) - lam(lo)) / (2 * h))
        grads[name] = g
    for fn in (orc.sdpa_bwd, orc.sdpa_bwd_numpy):
        dq, dk, dv = fn(q, k, v, do, scale=scale, causal=causal)
        np.testing.assert_allclose(dq, grads["q"], atol=1e-13, rtol=0)
        np.testing.assert_allclose(dk, grads["k"], atol=1e-13, rtol=0)
        np.testing.assert_allclose(dv, grads["v"], atol=1e-13, rtol=0)


# ------------------------------------------------- (b) central differences of the forward definition
@pytest.mark.parametrize("causal", [False, True])
def test_gradients_against_central_differences_of_the_forward_oracle(causal):
    S, D = 9, 5
    q, k, v, do = (x.astype(np.float64) for x in _inputs(S, D, 720))
    scale = float(np.float32(0.4375))
    lam = lambda qq, kk, vv: float((do * orc.sdpa_numpy(qq, kk, vv, scale=scale, causal=causal)).sum())
    dq, dk, dv = orc.sdpa_bwd(q, k, v, do, scale=scale, causal=causal)
    h = 1e-5
    for which, grad in enumerate((dq, dk, dv)):
        for (i, d) in [(0, 0), (3, 2), (8, 4), (5, 1)]:
            args_hi, args_lo = [q.copy(), k.copy(), v.copy()], [q.copy(), k.copy(), v.copy()]
            args_hi[which][i, d] += h
            args_lo[which][i, d] -= h
            fd = (lam(*args_hi) - lam(*args_lo)) / (2 * h)
            assert abs(fd - grad[i, d]) < 1e-8, (which, i, d, fd, grad[i, d])


# ------------------------------------------------- (c) library autograd
@pytest.mark.parametrize("shape", [(2, 2, 64, 64), (1, 2, 197, 64), (1, 1, 130, 128)])
@pytest.mark.parametrize("causal", [False, True])
def test_gradients_against_torch_float64_autograd(shape, causal):
    q, k, v, do = (_rand(shape, 730 + i, std=1.3) for i in range(4))
    scale = float(np.float32(shape[-1] ** -0.5))
    tq, tk, tv = (torch.tensor(x.astype(np.float64), requires_grad=True) for x in (q, k, v))
    o = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=causal, scale=scale)
    o.backward(torch.from_numpy(do.astype(np.float64)))
    dq, dk, dv = orc.sdpa_bwd(q, k, v, do, causal=causal)
    np.testing.assert_allclose(dq, tq.grad.numpy(), atol=1e-12, rtol=0)
    np.testing.assert_allclose(dk, tk.grad.numpy(), atol=1e-12, rtol=0)
    np.testing.assert_allclose(dv, tv.grad.numpy(), atol=1e-12, rtol=0)


def test_custom_and_negative_scale_against_torch_autograd():
    q, k, v, do = _inputs(50, 32, 740, lead=(2,))
    for scale in (0.375, -0.25, 0.0):
        tq, tk, tv = (torch.tensor(x.astype(np.float64), requires_grad=True) for x in (q, k, v))
        s = scale * (tq @ tk.transpose(-1, -2))
        (torch.softmax(s, -1) @ tv).backward(torch.from_numpy(do.astype(np.float64)))
        dq, dk, dv = orc.sdpa_bwd(q, k, v, do, scale=scale)
        for got, ref in ((dq, tq.grad), (dk, tk.grad), (dv, tv.grad)):
            np.testing.assert_allclose(got, ref.numpy(), atol=1e-12, rtol=0)


# ------------------------------------------------- (d) closed forms and invariants
def test_single_key_passes_dout_to_dv_and_nothing_else():
    q, k, v, do = _inputs(1, 8, 750)
    dq, dk, dv = orc.sdpa_bwd(q, k, v, do)
    assert np.array_equal(dv, do.astype(np.float64))
    assert np.all(dq == 0) and np.all(dk == 0)


def test_zero_queries_give_uniform_attention_gradients():
    S, D = 21, 6
    _, k, v, do = (x.astype(np.float64) for x in _inputs(S, D, 760))
    q = np.zeros((S, D))
    scale = 0.375
    dq, dk, dv = orc.sdpa_bwd(q, k, v, do, scale=scale)
    np.testing.assert_allclose(dv, np.broadcast_to(do.sum(0) / S, (S, D)), atol=1e-13)
    np.testing.assert_allclose(dk, 0.0, atol=1e-15)                       # dK = scale * dS^T Q with Q = 0
    dp = do @ v.T                                                         # uniform P = 1/S
    ds = (dp - dp.mean(1, keepdims=True)) / S
    np.testing.assert_allclose(dq, scale * ds @ k, atol=1e-13)
    # causal: row i attends keys 0..i uniformly
    dq, dk, dv = orc.sdpa_bwd(q, k, v, do, scale=scale, causal=True)
    ref_dv = np.stack([sum(do[i] / (i + 1) for i in range(j, S)) for j in range(S)])
    np.testing.assert_allclose(dv, ref_dv, atol=1e-13)


def test_invariants_of_the_softmax_jacobian():
    q, k, v, do = _inputs(33, 16, 770, lead=(2,))
    for causal in (False, True):
        dq, dk, dv = orc.sdpa_bwd(q, k, v, do, causal=causal)
        # adding one vector to every key shifts each score row by a constant and changes nothing:
        # the directional derivative sum_j dK_j vanishes (non-causal: every row sees every key)
        if not causal:
            np.testing.assert_allclose(dk.sum(-2), 0.0, atol=1e-12)
        # rows of P sum to one: sum_j dV_j = sum_i dO_i
        np.testing.assert_allclose(dv.sum(-2), do.astype(np.float64).sum(-2), atol=1e-12)
    # identical value rows: O does not depend on Q or K
    vconst = np.broadcast_to(v[:, :1], v.shape).copy()
    dq, dk, _ = orc.sdpa_bwd(q, k, vconst, do)
    np.testing.assert_allclose(dq, 0.0, atol=1e-13)
    np.testing.assert_allclose(dk, 0.0, atol=1e-13)
    # Lambda is linear in dout and in V
    a = orc.sdpa_bwd(q, k, v, do)
    b = orc.sdpa_bwd(q, k, v, (2 * do.astype(np.float32)).astype(np.float32))
    for x, y in zip(a, b):
        np.testing.assert_allclose(2 * x, y, atol=1e-12)


def test_causal_gradients_ignore_and_do_not_reach_later_positions():
    q, k, v, do = _inputs(40, 8, 780)
    dq, dk, dv = orc.sdpa_bwd(q, k, v, do, causal=True)
    # truncating the sequence at n leaves the first n rows of dQ alone only if later dout rows are
    # zero; zero them and compare with the truncated problem
    n = 17
    do0 = do.copy()
    do0[n:] = 0
    dq2, dk2, dv2 = orc.sdpa_bwd(q, k, v, do0, causal=True)
    dq3, dk3, dv3 = orc.sdpa_bwd(q[:n], k[:n], v[:n], do[:n], causal=True)
    np.testing.assert_allclose(dq2[:n], dq3, atol=1e-13)
    np.testing.assert_allclose(dk2[:n], dk3, atol=1e-13)
    np.testing.assert_allclose(dv2[:n], dv3, atol=1e-13)
    assert np.all(dq2[n:] == 0) and np.all(dk2[n:] == 0) and np.all(dv2[n:] == 0)
    # the last key is seen by the last query only: dV_last = P_last,last * dO_last
    p = orc.sdpa(q, k, v, causal=True, return_p=True)[1]
    np.testing.assert_allclose(dv[-1], p[-1, -1] * do[-1].astype(np.float64), atol=1e-13)


# ------------------------------------------------- (e) the C routine against the matrix form, subsets
def test_c_routine_matches_matrix_form_and_row_subsets():
    q, k, v, do = _inputs(130, 64, 790, lead=(2, 2))
    for causal in (False, True):
        full = orc.sdpa_bwd(q, k, v, do, causal=causal)
        ref = orc.sdpa_bwd_numpy(q, k, v, do, causal=causal)
        for x, y in zip(full, ref):
            np.testing.assert_allclose(x, y, atol=1e-12, rtol=0)
        qrows, krows = [0, 7, 129], [1, 64, 100, 128]
        dq, dk, dv = orc.sdpa_bwd(q, k, v, do, causal=causal, qrows=qrows, krows=krows)
        assert np.array_equal(dq, full[0][..., qrows, :])
        assert np.array_equal(dk, full[1][..., krows, :])
        assert np.array_equal(dv, full[2][..., krows, :])
    with pytest.raises(RuntimeError):
        orc.sdpa_bwd(q, k, v, do, qrows=[130])
    empty = np.zeros((0, 5, 8), np.float32)
    for g in orc.sdpa_bwd(empty, empty, empty, empty):
        assert g.shape == (0, 5, 8)


# ------------------------------------------------- (f) mutation check
def _formulas(q, k, v, do, scale, *, drop_inner=False, inner_over_dp_only=False, swap_dq_dk=False,
              drop_scale=False, dv_untransposed=False, ds_sign=1.0, inner_uses_p_squared=False):
    q, k, v, do = (np.asarray(x, np.float64) for x in (q, k, v, do))
    s = scale * (q @ k.T)
    e = np.exp(s - s.max(-1, keepdims=True))
    p = e / e.sum(-1, keepdims=True)
    dv = (p if dv_untransposed else p.T) @ do
    dp = do @ v.T
    inner = (p * dp).sum(-1, keepdims=True)
    if inner_over_dp_only:
        inner = dp.mean(-1, keepdims=True)
    if inner_uses_p_squared:
        inner = (p * p * dp).sum(-1, keepdims=True)
    if drop_inner:
        inner = 0.0
    ds = ds_sign * p * (dp - inner)
    sc = 1.0 if drop_scale else scale
    dq, dk = sc * (ds @ k), sc * (ds.T @ q)
    return (dk, dq, dv) if swap_dq_dk else (dq, dk, dv)


def _bwd_pin_suite(fn):
    failed = []
    q, k, v, do = (x.astype(np.float64) for x in _inputs(12, 12, 800))     # S = D so swapped operands still fit
    tq, tk, tv = (torch.tensor(x, requires_grad=True) for x in (q, k, v))
    (torch.softmax(0.375 * tq @ tk.T, -1) @ tv).backward(torch.from_numpy(do))
    got = fn(q, k, v, do, 0.375)
    for name, g, ref in zip("qkv", got, (tq.grad, tk.grad, tv.grad)):
        if not np.allclose(g, ref.numpy(), atol=1e-12):
            failed.append("torch-d" + name)
    lam = lambda qq, kk, vv: float((do * orc.sdpa_numpy(qq, kk, vv, scale=0.375)).sum())
    h = 1e-5
    for which in range(3):
        hi, lo = [q.copy(), k.copy(), v.copy()], [q.copy(), k.copy(), v.copy()]
        hi[which][2, 3] += h
        lo[which][2, 3] -= h
        if abs((lam(*hi) - lam(*lo)) / (2 * h) - got[which][2, 3]) > 1e-8:
            failed.append(f"fd-{which}")
    if not np.allclose(got[1].sum(0), 0.0, atol=1e-12):
        failed.append("dk-columns-sum-to-zero")
    if not np.allclose(got[2].sum(0), do.sum(0), atol=1e-12):
        failed.append("dv-columns-sum-to-dout")
    return failed


def test_backward_pins_pass_on_the_oracle_and_catch_planted_mistakes():
    real = lambda q, k, v, do, s: orc.sdpa_bwd(*(np.asarray(x, np.float32) for x in (q, k, v, do)), scale=s)
    # the finite-difference pin moves inputs off the float32 grid, which the C front end rejects: the
    # suite runs on the matrix form, and the C routine is tied to it on the same inputs below
    assert _bwd_pin_suite(lambda q, k, v, do, s: orc.sdpa_bwd_numpy(q, k, v, do, scale=s)) == []
    assert _bwd_pin_suite(lambda q, k, v, do, s: _formulas(q, k, v, do, s)) == []
    q, k, v, do = _inputs(12, 12, 800)
    for x, y in zip(real(q, k, v, do, 0.375), orc.sdpa_bwd_numpy(q, k, v, do, scale=0.375)):
        np.testing.assert_allclose(x, y, atol=1e-13)
    mutants = {
        "softmax Jacobian without the inner sum": dict(drop_inner=True),
        "inner sum as a plain mean of dP": dict(inner_over_dp_only=True),
        "inner sum weighted by P squared": dict(inner_uses_p_squared=True),
        "dQ and dK exchanged": dict(swap_dq_dk=True),
        "scale dropped from dQ and dK": dict(drop_scale=True),
        "dV = P dO instead of P^T dO": dict(dv_untransposed=True),
        "sign of dS": dict(ds_sign=-1.0),
    }
    for name, kw in mutants.items():
        bad = _bwd_pin_suite(lambda q, k, v, do, s, kw=kw: _formulas(q, k, v, do, s, **kw))
        assert bad, f"planted mistake not caught: {name}"


# ------------------------------------------------------------------ grouped heads
def _grouped_inputs(B, H, Hkv, S, D, seed):
    rng = np.random.default_rng(seed)
    f = lambda *shape: rng.standard_normal(shape).astype(np.float32)
    return f(B, H, S, D), f(B, Hkv, S, D), f(B, Hkv, S, D), f(B, H, S, D)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("B,H,Hkv,S,D", [(2, 4, 2, 7, 8), (1, 6, 1, 5, 4), (1, 3, 3, 9, 16)])
def test_grouped_backward_matches_torch_autograd_through_repeat_interleave(B, H, Hkv, S, D, causal):
    """Independent path: torch float64 autograd differentiates through the head repetition itself."""
    torch = pytest.importorskip("torch")
    q, k, v, do = _grouped_inputs(B, H, Hkv, S, D, seed=40 + S)
    tq, tk, tv = (torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in (q, k, v))
    G = H // Hkv
    o = torch.nn.functional.scaled_dot_product_attention(tq, tk.repeat_interleave(G, dim=1),
                                                         tv.repeat_interleave(G, dim=1), is_causal=causal,
                                                         scale=float(np.float32(1.0 / np.sqrt(D))))   # the oracle's default, as the float32 the device gets
    (o * torch.tensor(do, dtype=torch.float64)).sum().backward()
    dq, dk, dv = orc.sdpa_bwd_grouped(q, k, v, do, causal=causal)
    for got, want in ((dq, tq.grad), (dk, tk.grad), (dv, tv.grad)):
        np.testing.assert_allclose(got, want.numpy(), rtol=1e-10, atol=1e-12)


def test_grouped_backward_against_finite_differences_of_the_forward_definition():
    """Perturbing one key/value element moves the outputs of all G query heads of its group."""
    B, H, Hkv, S, D, G = 1, 4, 2, 5, 3, 2
    q, k, v, do = _grouped_inputs(B, H, Hkv, S, D, seed=77)
    scale = 0.4

    def loss(k_, v_):
        o = orc.sdpa(q, np.repeat(k_, G, axis=1), np.repeat(v_, G, axis=1), scale=scale, causal=True)
        return float((o * do.astype(np.float64)).sum())

    dq, dk, dv = orc.sdpa_bwd_grouped(q, k, v, do, scale=scale, causal=True)
    eps = 2.0 ** -9                    # exactly representable steps on float32 inputs
    for (h, j, d) in ((0, 0, 0), (1, 3, 2), (0, 4, 1)):
        for which, grad in (("k", dk), ("v", dv)):
            kp, km, vp, vm = k.copy(), k.copy(), v.copy(), v.copy()
            (kp if which == "k" else vp)[0, h, j, d] += eps
            (km if which == "k" else vm)[0, h, j, d] -= eps
            fd = (loss(kp, vp) - loss(km, vm)) / (2 * eps)
            assert abs(fd - grad[0, h, j, d]) <= 1e-5 * max(1.0, abs(fd)), (which, h, j, d, fd, grad[0, h, j, d])


def test_grouped_backward_special_cases_and_row_subsets():
    q, k, v, do = _grouped_inputs(2, 4, 2, 6, 8, seed=5)
    # one query head per key/value head: the plain backward pass
    a = orc.sdpa_bwd_grouped(q[:, :2], k, v, do[:, :2], causal=True)
    b = orc.sdpa_bwd(q[:, :2], k, v, do[:, :2], causal=True)
    for x, y in zip(a, b):
        np.testing.assert_array_equal(x, y)
    # identical query heads in a group (same q, same dout): dK, dV are G times one head's
    q2, do2 = np.repeat(q[:, :2], 2, axis=1), np.repeat(do[:, :2], 2, axis=1)      # heads (0,0,1,1) over 2 kv heads
    dq2, dk2, dv2 = orc.sdpa_bwd_grouped(q2, k, v, do2)
    _, dk1, dv1 = orc.sdpa_bwd(q[:, :2], k, v, do[:, :2])
    np.testing.assert_allclose(dk2, 2 * dk1, rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(dv2, 2 * dv1, rtol=1e-13, atol=1e-15)
    np.testing.assert_array_equal(dq2[:, 0], dq2[:, 1])
    # row subsets select rows of the full result
    full = orc.sdpa_bwd_grouped(q, k, v, do, causal=True)
    sub = orc.sdpa_bwd_grouped(q, k, v, do, causal=True, qrows=[0, 5], krows=[1, 2, 4])
    np.testing.assert_array_equal(sub[0], full[0][:, :, [0, 5]])
    np.testing.assert_array_equal(sub[1], full[1][:, :, [1, 2, 4]])
    np.testing.assert_array_equal(sub[2], full[2][:, :, [1, 2, 4]])
    with pytest.raises(ValueError):
        orc.sdpa_bwd_grouped(q[:, :3], k, v, do[:, :3])
