"""Pins for the CPU oracle: everything here runs without a GPU.

The paper prints no numeric attention example, so the oracle is pinned by
(a) hand-worked rational fixtures under tests/golden/ (Eq. 1, Section 3.1),
(b) closed forms and invariants of Eq. 1, (c) exact-rational brute force on tiny
inputs, (d) library routines (torch CPU float64 SDPA, scipy logsumexp), (e) the
merge identity between the materialised result and the blockwise recurrence of
Section 4.1.2 (Eqs. 2-4), and (f) a mutation check: planted mistakes in a copy
of the definition must each trip at least one pin.
"""
import math
from decimal import Decimal, getcontext
from fractions import Fraction
from pathlib import Path

import numpy as np
import pytest
import torch

from oracle import sdpa_oracle as orc

GOLDEN = Path(__file__).resolve().parent / "golden"
LN2_F32 = float(np.float32(math.log(2.0)))


# ----------------------------------------------------------------------------- fixtures
def _parse_matrix(text, conv=float):
    return [[conv(tok) for tok in row.split()] for row in text.split(";")]


def load_golden(name):
    fields = {}
    for line in (GOLDEN / name).read_text().splitlines():
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        key, _, rest = line.partition(" ")
        fields[key] = rest.strip()
    S, D = int(fields["S"]), int(fields["D"])
    assert fields["scale_is"] == "ln2"
    g = {
        "S": S, "D": D, "scale": LN2_F32, "tol": float(fields["tol"]),
        "causal": fields.get("mask", "none") == "causal",
        "Q": np.array(_parse_matrix(fields["Q"])), "K": np.array(_parse_matrix(fields["K"])),
        "V": np.array(_parse_matrix(fields["V"])),
        "O": np.array(_parse_matrix(fields["O"], lambda t: float(Fraction(t)))),
        "P": np.array(_parse_matrix(fields["P"], lambda t: float(Fraction(t)))),
        "LSE": np.array([math.log(float(Fraction(t))) for t in fields["LSE_exp"].split()]),
    }
    assert g["Q"].shape == (S, D) and g["K"].shape == (S, D) and g["V"].shape == (S, D)
    return g


GOLDEN_FILES = ["pow2_softmax.txt", "two_key_sigmoid.txt", "pow2_softmax_causal.txt"]


def _rand(shape, seed, dtype=np.float16, std=1.0):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal(shape) * std).astype(dtype)


def _bf16_round(x):
    t = torch.from_numpy(np.asarray(x, dtype=np.float32)).to(torch.bfloat16).to(torch.float32)
    return t.numpy()


# ------------------------------------------------------------------- (a) golden fixtures
@pytest.mark.parametrize("name", GOLDEN_FILES)
@pytest.mark.parametrize("impl", ["c", "numpy", "online"])
def test_golden_rational_examples(name, impl):
    g = load_golden(name)
    q, k, v = (g[x].astype(np.float32) for x in "QKV")
    cz = g["causal"]
    if impl == "c":
        o, lse, p = orc.sdpa(q, k, v, scale=g["scale"], return_lse=True, return_p=True, causal=cz)
        np.testing.assert_allclose(p, g["P"], atol=g["tol"], rtol=0)
    elif impl == "numpy":
        o, lse = orc.sdpa_numpy(q, k, v, scale=g["scale"], return_lse=True, causal=cz)
    else:
        o, lse = orc.sdpa_online(q, k, v, scale=g["scale"],
                                 tile_bounds=list(range(g["S"] + 1)), return_lse=True, causal=cz)
    np.testing.assert_allclose(o, g["O"], atol=g["tol"], rtol=0)
    np.testing.assert_allclose(lse, g["LSE"], atol=g["tol"], rtol=0)


# ------------------------------------------------------------- (b) closed forms, invariants
def test_zero_queries_give_column_mean_and_log_S():
    k, v = _rand((3, 37, 8), 1), _rand((3, 37, 8), 2)
    q = np.zeros_like(k)
    o, lse = orc.sdpa(q, k, v, return_lse=True)
    mean = v.astype(np.float64).mean(axis=1, keepdims=True)
    np.testing.assert_allclose(o, np.broadcast_to(mean, o.shape), atol=1e-13)
    np.testing.assert_allclose(lse, math.log(37), atol=1e-13)
    # scale = 0 is the same statement for arbitrary Q
    o0, lse0 = orc.sdpa(_rand((3, 37, 8), 3), k, v, scale=0.0, return_lse=True)
    np.testing.assert_allclose(o0, np.broadcast_to(mean, o.shape), atol=1e-13)
    np.testing.assert_allclose(lse0, math.log(37), atol=1e-13)


def test_identical_keys_give_column_mean():
    q, v = _rand((2, 19, 4), 4), _rand((2, 19, 4), 5)
    k = np.broadcast_to(_rand((2, 1, 4), 6), (2, 19, 4)).copy()
    o = orc.sdpa(q, k, v)
    mean = v.astype(np.float64).mean(axis=1, keepdims=True)
    np.testing.assert_allclose(o, np.broadcast_to(mean, o.shape), atol=1e-13)


def test_single_key_returns_value_row_exactly():
    q, k, v = _rand((4, 1, 64), 7), _rand((4, 1, 64), 8), _rand((4, 1, 64), 9)
    o, lse = orc.sdpa(q, k, v, return_lse=True)
    assert np.array_equal(o, v.astype(np.float64))
    s = (q.astype(np.float64) * k.astype(np.float64)).sum(-1) * float(np.float32(1 / 8.0))
    np.testing.assert_allclose(lse, s, atol=1e-13)


def test_constant_value_rows_give_that_row():
    q, k = _rand((2, 33, 16), 10), _rand((2, 33, 16), 11)
    row = _rand((2, 1, 16), 12)
    v = np.broadcast_to(row, (2, 33, 16)).copy()
    o = orc.sdpa(q, k, v)
    np.testing.assert_allclose(o, np.broadcast_to(row.astype(np.float64), o.shape), atol=1e-13)


def test_dominant_logit_selects_value_row():
    S, D = 24, 16
    q = np.zeros((S, D), np.float32)
    q[:, 0] = 1.0
    k = np.zeros((S, D), np.float32)
    v = _rand((S, D), 13).astype(np.float32)
    star, gap = 17, 40.0
    k[star, 0] = gap                       # logit gap = scale*gap with scale=1
    o, p = orc.sdpa(q, k, v, scale=1.0, return_p=True)
    bound = (S - 1) * math.exp(-gap) * 2 * np.abs(v).max()
    np.testing.assert_allclose(o, np.broadcast_to(v[star].astype(np.float64), o.shape), atol=bound)
    assert np.all(p[:, star] > 1 - (S - 1) * math.exp(-gap))


def test_softmax_rows_sum_to_one_and_are_positive():
    q, k, v = _rand((2, 3, 50, 8), 14, std=2.0), _rand((2, 3, 50, 8), 15, std=2.0), _rand((2, 3, 50, 8), 16)
    _, p = orc.sdpa(q, k, v, return_p=True)
    assert p.shape == (2, 3, 50, 50)
    assert np.all(p >= 0)
    np.testing.assert_allclose(p.sum(-1), 1.0, atol=1e-13)


def test_output_is_convex_combination_of_value_rows():
    q, k, v = _rand((5, 40, 8), 17, std=3.0), _rand((5, 40, 8), 18, std=3.0), _rand((5, 40, 8), 19)
    o = orc.sdpa(q, k, v)
    v64 = v.astype(np.float64)
    assert np.all(o <= v64.max(axis=1, keepdims=True) + 1e-13)
    assert np.all(o >= v64.min(axis=1, keepdims=True) - 1e-13)


def test_joint_permutation_of_keys_and_values_leaves_output_unchanged():
    q, k, v = _rand((2, 31, 8), 20), _rand((2, 31, 8), 21), _rand((2, 31, 8), 22)
    perm = np.random.default_rng(23).permutation(31)
    o1, l1 = orc.sdpa(q, k, v, return_lse=True)
    o2, l2 = orc.sdpa(q, k[:, perm], v[:, perm], return_lse=True)
    np.testing.assert_allclose(o1, o2, atol=1e-13)
    np.testing.assert_allclose(l1, l2, atol=1e-13)
    # permuting only K (not V) must change the result: guards against an index that ignores j
    o3 = orc.sdpa(q, k[:, perm], v)
    assert np.abs(o3 - o1).max() > 1e-3


def test_key_shift_changes_lse_by_scaled_dot_only():
    q, k, v = _rand((29, 8), 24), _rand((29, 8), 25), _rand((29, 8), 26)
    c = np.array([1, -2, 0.5, 0, 3, -1, 0.25, 2], np.float16)
    k2 = (k.astype(np.float32) + c.astype(np.float32))
    scale = float(np.float32(1 / math.sqrt(8)))
    o1, l1 = orc.sdpa(q, k, v, return_lse=True)
    o2, l2 = orc.sdpa(q, k2, v, return_lse=True)
    np.testing.assert_allclose(o1, o2, atol=1e-12)
    shift = scale * (q.astype(np.float64) @ c.astype(np.float64))
    np.testing.assert_allclose(l2 - l1, shift, atol=1e-12)


def test_heads_are_independent():
    q, k, v = _rand((2, 3, 20, 8), 27), _rand((2, 3, 20, 8), 28), _rand((2, 3, 20, 8), 29)
    o1 = orc.sdpa(q, k, v)
    k2, v2 = k.copy(), v.copy()
    k2[1, 2] += 1
    v2[1, 2] -= 1
    o2 = orc.sdpa(q, k2, v2)
    mask = np.ones((2, 3), bool)
    mask[1, 2] = False
    assert np.array_equal(o1[mask], o2[mask])
    assert np.abs(o1[1, 2] - o2[1, 2]).max() > 1e-3


# ---------------------------------------------------------- (c) exact-rational brute force
def _brute_force(q, k, v, scale):
    """Rational dot products, 50-digit exponentials; no max subtraction, no float ops."""
    getcontext().prec = 50
    S, D = q.shape
    out, lses = [], []
    sc = Fraction(float(scale))
    for i in range(S):
        logits = []
        for j in range(S):
            dot = sum(Fraction(float(q[i, d])) * Fraction(float(k[j, d])) for d in range(D))
            x = sc * dot
            logits.append(Decimal(x.numerator) / Decimal(x.denominator))
        w = [x.exp() for x in logits]
        tot = sum(w)
        row = []
        for d in range(D):
            num = sum(w[j] * Decimal(float(v[j, d])) for j in range(S))
            row.append(float(num / tot))
        out.append(row)
        lses.append(float(tot.ln()))
    return np.array(out), np.array(lses)


@pytest.mark.parametrize("S,D", [(1, 1), (2, 4), (3, 1), (5, 4), (8, 64), (7, 3)])
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_brute_force_tiny(S, D, dtype):
    q, k, v = (_rand((S, D), 100 + 7 * S + D + i, np.float32, std=1.5) for i in range(3))
    if dtype == "f16":
        q, k, v = (x.astype(np.float16).astype(np.float32) for x in (q, k, v))
    else:
        q, k, v = (_bf16_round(x) for x in (q, k, v))
    scale = float(np.float32(1 / math.sqrt(D)))
    ref_o, ref_lse = _brute_force(q, k, v, scale)
    for fn in (orc.sdpa, orc.sdpa_numpy):
        o, lse = fn(q, k, v, return_lse=True)
        np.testing.assert_allclose(o, ref_o, atol=1e-12, rtol=0)
        np.testing.assert_allclose(lse, ref_lse, atol=1e-12, rtol=0)


# ------------------------------------------------------------------- (d) library routines
@pytest.mark.parametrize("shape", [(2, 3, 64, 64), (1, 2, 197, 64), (1, 1, 300, 128), (1, 2, 1024, 64)])
def test_against_torch_float64_sdpa(shape):
    q, k, v = (_rand(shape, 200 + i, std=1.3) for i in range(3))
    o, lse = orc.sdpa(q, k, v, return_lse=True)
    tq, tk, tv = (torch.from_numpy(x.astype(np.float64)) for x in (q, k, v))
    # the oracle takes the float32 value of 1/sqrt(D) (what the device receives), so torch gets the same
    scale = float(np.float32(1 / math.sqrt(shape[-1])))
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, scale=scale).numpy()
    np.testing.assert_allclose(o, ref, atol=1e-12, rtol=0)
    from scipy.special import logsumexp
    logits = scale * (tq @ tk.transpose(-1, -2)).numpy()
    np.testing.assert_allclose(lse, logsumexp(logits, axis=-1), atol=1e-12, rtol=0)


def test_custom_scale_against_torch():
    q, k, v = (_rand((2, 45, 16), 210 + i) for i in range(3))
    for scale in (0.3, -0.7, 2.0):
        o = orc.sdpa(q, k, v, scale=scale)
        tq, tk, tv = (torch.from_numpy(x.astype(np.float64)) for x in (q, k, v))
        ref = torch.nn.functional.scaled_dot_product_attention(
            tq, tk, tv, scale=float(np.float32(scale))).numpy()
        np.testing.assert_allclose(o, ref, atol=1e-12, rtol=0)


# ---------------------------------------------------------------- (e) merge identity
@pytest.mark.parametrize("S", [1, 5, 64, 197])
def test_online_recurrence_reaches_materialised_result(S):
    D = 16
    q, k, v = (_rand((S, D), 300 + S + i, std=2.0) for i in range(3))
    ref_o, ref_lse = orc.sdpa(q, k, v, return_lse=True)
    rng = np.random.default_rng(S)
    splits = [[0, S], list(range(S + 1))]
    if S > 2:
        cuts = sorted(set(rng.integers(1, S, size=min(6, S - 1)).tolist()))
        splits.append([0] + cuts + [S])
        splits.append(list(range(0, S, 32)) + [S])
    for tb in splits:
        o, lse = orc.sdpa_online(q, k, v, tile_bounds=tb, return_lse=True)
        np.testing.assert_allclose(o, ref_o, atol=1e-12, rtol=0)
        np.testing.assert_allclose(lse, ref_lse, atol=1e-12, rtol=0)


def test_online_recurrence_with_increasing_maxima():
    """Keys ordered so that the running max rises in every tile: the rescale of Eqs. 3-4 is exercised."""
    S, D = 48, 4
    q = np.ones((S, D), np.float32)
    k = np.tile(np.arange(S, dtype=np.float32)[:, None] * 0.5, (1, D))
    v = _rand((S, D), 310).astype(np.float32)
    ref = orc.sdpa(q, k, v, scale=1.0)
    o = orc.sdpa_online(q, k, v, scale=1.0, tile_bounds=list(range(0, S + 1, 4)))
    np.testing.assert_allclose(o, ref, atol=1e-12, rtol=0)


# ------------------------------------------------------------------- C-oracle mechanics
def test_c_oracle_matches_numpy_definition_and_row_subsets():
    q, k, v = (_rand((2, 2, 130, 64), 400 + i) for i in range(3))
    o, lse = orc.sdpa(q, k, v, return_lse=True)
    o_np, lse_np = orc.sdpa_numpy(q, k, v, return_lse=True)
    np.testing.assert_allclose(o, o_np, atol=1e-13, rtol=0)
    np.testing.assert_allclose(lse, lse_np, atol=1e-13, rtol=0)
    rows = [0, 1, 63, 64, 129]
    o_r, lse_r = orc.sdpa(q, k, v, rows=rows, return_lse=True)
    assert np.array_equal(o_r, o[:, :, rows])
    assert np.array_equal(lse_r, lse[:, :, rows])


def test_c_oracle_rejects_bad_arguments():
    q = np.zeros((4, 8), np.float32)
    with pytest.raises(ValueError):
        orc.sdpa(q, np.zeros((5, 8), np.float32), q)
    with pytest.raises(RuntimeError):
        orc.sdpa(q, q, q, rows=[4])
    with pytest.raises(TypeError):
        orc.sdpa(q.astype(np.int32), q, q)
    assert orc.num_threads() >= 1


def test_empty_problem():
    q = np.zeros((0, 5, 8), np.float32)
    assert orc.sdpa(q, q, q).shape == (0, 5, 8)


# ------------------------------------------------------------------ (f) mutation check
def _pin_suite(fn):
    """Run a compact set of the pins above on fn(q,k,v,scale)->(o,lse); return names that fail."""
    failed = []

    def check(name, cond):
        if not cond:
            failed.append(name)

    for gname in GOLDEN_FILES:
        g = load_golden(gname)
        if g["causal"]:
            continue            # the causal fixtures have their own suite below
        o, lse = fn(g["Q"], g["K"], g["V"], g["scale"])
        check("golden-o:" + gname, np.allclose(o, g["O"], atol=g["tol"], rtol=0))
        check("golden-lse:" + gname, np.allclose(lse, g["LSE"], atol=g["tol"], rtol=0))
    k, v = _rand((37, 8), 1).astype(np.float64), _rand((37, 8), 2).astype(np.float64)
    o, lse = fn(np.zeros_like(k), k, v, 0.375)
    check("q0-mean", np.allclose(o, v.mean(0, keepdims=True), atol=1e-12))
    check("q0-lse", np.allclose(lse, math.log(37), atol=1e-12))
    q = _rand((37, 8), 3).astype(np.float64)
    row = _rand((1, 8), 4).astype(np.float64)
    o, _ = fn(q, k, np.broadcast_to(row, (37, 8)).copy(), 0.375)
    check("const-v", np.allclose(o, row, atol=1e-12))
    tq, tk, tv = (torch.from_numpy(x) for x in (q, k, v))
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, scale=0.375).numpy()
    o, _ = fn(q, k, v, 0.375)
    check("torch", np.allclose(o, ref, atol=1e-12))
    return failed


def _definition(q, k, v, scale, *, sign=1.0, transpose_qk=False, drop_scale=False,
                skip_normalise=False, no_max_in_lse=False, v_index_shift=0, normalise_by_count=False):
    q, k, v = (np.asarray(x, np.float64) for x in (q, k, v))
    s = (k @ q.T) if transpose_qk else (q @ k.T)
    if not drop_scale:
        s = s * scale
    s = sign * s
    m = s.max(-1, keepdims=True)
    e = np.exp(s - m)
    L = e.sum(-1, keepdims=True)
    vv = np.roll(v, v_index_shift, axis=0)
    o = e @ vv
    if normalise_by_count:
        o = o / s.shape[-1]
    elif not skip_normalise:
        o = o / L
    lse = (np.log(L) if no_max_in_lse else m + np.log(L))[:, 0]
    return o, lse


def test_pins_pass_on_the_oracle_and_catch_planted_mistakes():
    real = lambda q, k, v, s: orc.sdpa(np.asarray(q, np.float32), np.asarray(k, np.float32),
                                       np.asarray(v, np.float32), scale=s, return_lse=True)
    assert _pin_suite(real) == []
    assert _pin_suite(lambda q, k, v, s: _definition(q, k, v, float(np.float32(s)))) == []
    mutants = {
        "negated logits": dict(sign=-1.0),
        "K Q^T instead of Q K^T": dict(transpose_qk=True),
        "scale dropped": dict(drop_scale=True),
        "no division by the normaliser": dict(skip_normalise=True),
        "divide by S instead of the normaliser": dict(normalise_by_count=True),
        "row max left out of LSE": dict(no_max_in_lse=True),
        "value rows off by one": dict(v_index_shift=1),
    }
    for name, kw in mutants.items():
        bad = _pin_suite(lambda q, k, v, s, kw=kw: _definition(q, k, v, float(np.float32(s)), **kw))
        assert bad, f"planted mistake not caught: {name}"


# ------------------------------------------------------------------ causal mask (Section 4.1.3)
def test_causal_row_i_equals_plain_attention_over_the_first_i_plus_one_keys():
    """Eq. 1 with the causal mask: row i attends keys 0..i, i.e. the unmasked problem truncated at i."""
    q, k, v = (_rand((2, 41, 16), 500 + i, std=1.5) for i in range(3))
    o, lse, p = orc.sdpa(q, k, v, causal=True, return_lse=True, return_p=True)
    assert np.array_equal(o[:, 0], v[:, 0].astype(np.float64))          # first row: its own value row
    np.testing.assert_allclose(p.sum(-1), 1.0, atol=1e-13)
    assert np.all(np.triu(p, k=1) == 0)                                  # nothing after the query
    for i in (0, 1, 7, 20, 40):
        # plain attention of query i over keys 0..i, written out with numpy
        for b in range(2):
            s = float(np.float32(1 / math.sqrt(16))) * (k[b, :i + 1].astype(np.float64) @ q[b, i].astype(np.float64))
            w = np.exp(s - s.max())
            ref = (w[:, None] * v[b, :i + 1].astype(np.float64)).sum(0) / w.sum()
            np.testing.assert_allclose(o[b, i], ref, atol=1e-13)
            np.testing.assert_allclose(lse[b, i], s.max() + math.log(w.sum()), atol=1e-13)


def test_causal_against_torch_float64_and_numpy_and_online():
    q, k, v = (_rand((2, 3, 150, 64), 510 + i, std=1.3) for i in range(3))
    o, lse = orc.sdpa(q, k, v, causal=True, return_lse=True)
    tq, tk, tv = (torch.from_numpy(x.astype(np.float64)) for x in (q, k, v))
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True, scale=0.125).numpy()
    np.testing.assert_allclose(o, ref, atol=1e-12, rtol=0)
    o_np, lse_np = orc.sdpa_numpy(q, k, v, causal=True, return_lse=True)
    np.testing.assert_allclose(o, o_np, atol=1e-13, rtol=0)
    np.testing.assert_allclose(lse, lse_np, atol=1e-13, rtol=0)
    o_on, lse_on = orc.sdpa_online(q[0, 0], k[0, 0], v[0, 0], causal=True, return_lse=True,
                                   tile_bounds=[0, 7, 64, 65, 128, 150])
    np.testing.assert_allclose(o_on, o[0, 0], atol=1e-12, rtol=0)
    np.testing.assert_allclose(lse_on, lse[0, 0], atol=1e-12, rtol=0)


def test_causal_output_ignores_later_keys_and_values():
    q, k, v = (_rand((33, 8), 520 + i) for i in range(3))
    o1 = orc.sdpa(q, k, v, causal=True)
    k2, v2 = k.copy(), v.copy()
    k2[20:] += 3
    v2[20:] -= 5
    o2 = orc.sdpa(q, k2, v2, causal=True)
    assert np.array_equal(o1[:20], o2[:20])
    assert np.abs(o1[20:] - o2[20:]).max() > 1e-2
    rows = [0, 5, 32]
    assert np.array_equal(orc.sdpa(q, k, v, causal=True, rows=rows), o1[rows])


def test_causal_pins_catch_planted_mask_mistakes():
    g = load_golden("pow2_softmax_causal.txt")
    q, k, v = (_rand((19, 8), 530 + i) for i in range(3))
    tq, tk, tv = (torch.from_numpy(x.astype(np.float64)) for x in (q, k, v))
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True).numpy()

    def masked(qq, kk, vv, scale, keep):
        qq, kk, vv = (np.asarray(x, np.float64) for x in (qq, kk, vv))
        s = scale * (qq @ kk.T)
        n = s.shape[0]
        s = np.where(keep(np.arange(n)[:, None], np.arange(n)[None, :]), s, -np.inf)
        w = np.exp(s - s.max(-1, keepdims=True))
        return (w @ vv) / w.sum(-1, keepdims=True)

    def fails(keep):
        bad = not np.allclose(masked(g["Q"], g["K"], g["V"], g["scale"], keep), g["O"], atol=g["tol"])
        bad |= not np.allclose(masked(q, k, v, float(np.float32(8 ** -0.5)), keep), ref, atol=1e-12)
        return bad

    assert not fails(lambda i, j: j <= i)                       # the right mask passes
    assert fails(lambda i, j: j <= i + 1)                       # diagonal off by one (too wide)
    assert fails(lambda i, j: (j < i) | (i == 0))               # diagonal off by one (too narrow)
    assert fails(lambda i, j: j >= i)                           # mask transposed
    assert fails(lambda i, j: j == j)                           # no mask


# ------------------------------------------- Sq query rows against Skv keys (decoding shapes, Section 7)
def _brute_force_kv(q, k, v, scale, causal):
    """Rational dot products and 50-digit exponentials for q [Sq, D] against k, v [Skv, D]; under the
    causal mask the queries are the last Sq positions of the sequence."""
    getcontext().prec = 50
    (Sq, D), Skv = q.shape, k.shape[0]
    sc = Fraction(float(scale))
    out, lses = [], []
    for i in range(Sq):
        pos = i + (Skv - Sq)                          # position of query i in the Skv-long sequence
        keys = [j for j in range(Skv) if not causal or j <= pos]
        w = []
        for j in keys:
            x = sc * sum(Fraction(float(q[i, d])) * Fraction(float(k[j, d])) for d in range(D))
            w.append((Decimal(x.numerator) / Decimal(x.denominator)).exp())
        tot = sum(w)
        out.append([float(sum(wj * Decimal(float(v[j, d])) for wj, j in zip(w, keys)) / tot) for d in range(D)])
        lses.append(float(tot.ln()))
    return np.array(out), np.array(lses)


@pytest.mark.parametrize("Sq,Skv,D", [(1, 1, 2), (1, 9, 4), (3, 7, 4), (4, 5, 3), (6, 6, 2), (7, 3, 2)])
@pytest.mark.parametrize("causal", [False, True])
def test_kv_shapes_brute_force_tiny(Sq, Skv, D, causal):
    if causal and Skv < Sq:
        pytest.skip("causal needs Skv >= Sq")
    q = _rand((Sq, D), 600 + Sq, std=1.5)
    k, v = _rand((Skv, D), 601 + Skv, std=1.5), _rand((Skv, D), 602 + Skv, std=1.5)
    scale = float(np.float32(1 / math.sqrt(D)))
    ref_o, ref_lse = _brute_force_kv(q, k, v, scale, causal)
    for fn in (orc.sdpa, orc.sdpa_numpy):
        o, lse = fn(q, k, v, return_lse=True, causal=causal)
        assert o.shape == (Sq, D) and lse.shape == (Sq,)
        np.testing.assert_allclose(o, ref_o, atol=1e-12, rtol=0)
        np.testing.assert_allclose(lse, ref_lse, atol=1e-12, rtol=0)
    o, lse = orc.sdpa_online(q, k, v, return_lse=True, causal=causal, tile_bounds=sorted({0, (Skv + 1) // 2, Skv}))
    np.testing.assert_allclose(o, ref_o, atol=1e-12, rtol=0)
    np.testing.assert_allclose(lse, ref_lse, atol=1e-12, rtol=0)


@pytest.mark.parametrize("Sq,Skv", [(1, 300), (17, 130), (64, 64), (100, 257)])
def test_kv_shapes_against_torch_float64(Sq, Skv):
    q = _rand((2, 2, Sq, 64), 610, std=1.3)
    k, v = _rand((2, 2, Skv, 64), 611, std=1.3), _rand((2, 2, Skv, 64), 612, std=1.3)
    tq, tk, tv = (torch.from_numpy(x.astype(np.float64)) for x in (q, k, v))
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, scale=0.125).numpy()
    np.testing.assert_allclose(orc.sdpa(q, k, v), ref, atol=1e-12, rtol=0)
    # causal: an explicit boolean mask with the queries as the last Sq positions
    keep = torch.ones(Sq, Skv, dtype=torch.bool).tril(diagonal=Skv - Sq)
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=keep, scale=0.125).numpy()
    o, lse = orc.sdpa(q, k, v, causal=True, return_lse=True)
    np.testing.assert_allclose(o, ref, atol=1e-12, rtol=0)
    s = 0.125 * (tq @ tk.transpose(-1, -2)).masked_fill(~keep, -math.inf)
    np.testing.assert_allclose(lse, torch.logsumexp(s, -1).numpy(), atol=1e-12, rtol=0)
    rows = sorted({0, Sq // 2, Sq - 1})
    assert np.array_equal(orc.sdpa(q, k, v, causal=True, rows=rows), o[..., rows, :])


def test_decode_step_is_the_last_row_of_the_square_causal_problem():
    """One new query against a cache of Skv keys = the last row of causal self-attention over Skv
    positions; a chunk of queries a..b-1 against keys 0..b-1 = rows a..b-1 of the square problem."""
    q, k, v = (_rand((3, 90, 32), 620 + i, std=1.4) for i in range(3))
    tq, tk, tv = (torch.from_numpy(x.astype(np.float64)) for x in (q, k, v))
    scale = float(np.float32(32 ** -0.5))
    sq = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True, scale=scale).numpy()
    np.testing.assert_allclose(orc.sdpa(q[:, -1:], k, v, causal=True), sq[:, -1:], atol=1e-12, rtol=0)
    np.testing.assert_allclose(orc.sdpa(q[:, -1:], k, v, causal=False), sq[:, -1:], atol=1e-12, rtol=0)
    a, b = 40, 77
    np.testing.assert_allclose(orc.sdpa(q[:, a:b], k[:, :b], v[:, :b], causal=True), sq[:, a:b], atol=1e-12, rtol=0)


def test_kv_shapes_closed_forms_and_planted_offset_mistakes():
    # zero queries: row i is the mean of the value rows it may see (all Skv, or the first i+Skv-Sq+1)
    k, v = _rand((23, 8), 630), _rand((23, 8), 631).astype(np.float64)
    q0 = np.zeros((5, 8), np.float16)
    o, lse = orc.sdpa(q0, k, v.astype(np.float32), return_lse=True)
    np.testing.assert_allclose(o, np.broadcast_to(v.mean(0), (5, 8)), atol=1e-13)
    np.testing.assert_allclose(lse, math.log(23), atol=1e-13)
    o, lse = orc.sdpa(q0, k, v.astype(np.float32), return_lse=True, causal=True)
    for i in range(5):
        n = i + 23 - 5 + 1
        np.testing.assert_allclose(o[i], v[:n].mean(0), atol=1e-13)
        np.testing.assert_allclose(lse[i], math.log(n), atol=1e-13)

    # the same closed form rejects plausible wrong alignments of the mask
    def mean_rows(offset):
        return np.stack([v[:max(1, min(23, i + offset + 1))].mean(0) for i in range(5)])
    assert np.allclose(o, mean_rows(23 - 5), atol=1e-13)
    assert not np.allclose(o, mean_rows(0), atol=1e-6)              # top-left alignment
    assert not np.allclose(o, mean_rows(23 - 5 - 1), atol=1e-6)     # one position short
    assert not np.allclose(o, mean_rows(23 - 5 + 1), atol=1e-6)     # one position long
    with pytest.raises(RuntimeError):
        orc.sdpa(np.zeros((6, 8), np.float16), k[:5], v[:5].astype(np.float32), causal=True)   # Skv < Sq
