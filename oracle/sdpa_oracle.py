"""CPU oracle for the SDPA forward pass.  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's ``cpu_baseline`` leg may import
this module; the product path never does, and the two share no code.

Three independent float64 routines for the forward pass live here (and two for the backward
pass, :func:`sdpa_bwd` in C and :func:`sdpa_bwd_numpy`, described at the end):

* :func:`sdpa` -- ctypes front end of ``sdpa_oracle.c`` (plain C + OpenMP), the
  materialised row-by-row definition of the paper's Eq. 1 (Section 3.1) with
  M = 0 and the final division of Section 4.1.2.  This is *the* oracle used for
  parity at every size (it can evaluate a subset of query rows).
* :func:`sdpa_numpy` -- the same definition as three numpy matrix expressions,
  for small shapes; kept because it can be checked against Eq. 1 by eye.
* :func:`sdpa_online` -- the blockwise recurrence of Section 4.1.2 (Eqs. 2-4)
  taken step by step in float64 with arbitrary tile boundaries.  It exists to
  show that the recurrence reaches the materialised result (merge identity).

Inputs are numpy arrays holding FP16/BF16-rounded values (Section 4.1.3); they
are converted to float32 (exact for 16-bit floats) for the C routine, which
promotes every operand to double.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "sdpa_oracle.c"
_LIB = _HERE / "libsdpa_oracle.so"
_lib = None


def build(force: bool = False) -> Path:
    """Compile ``sdpa_oracle.c`` with gcc (no fast-math: IEEE double throughout)."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        tmp = _LIB.with_suffix(f".tmp{os.getpid()}.so")
        cmd = ["gcc", "-O2", "-fopenmp", "-fno-fast-math", "-shared", "-fPIC",
               str(_SRC), "-o", str(tmp), "-lm"]
        subprocess.run(cmd, check=True)
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(str(_LIB))
        lib.sdpa_oracle_rows_kv.restype = ctypes.c_int
        lib.sdpa_oracle_rows_kv.argtypes = [
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_long, ctypes.c_long, ctypes.c_long, ctypes.c_long, ctypes.c_double,
            ctypes.c_void_p, ctypes.c_long, ctypes.c_int,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        lib.sdpa_oracle_bwd.restype = ctypes.c_int
        lib.sdpa_oracle_bwd.argtypes = [
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_long, ctypes.c_long, ctypes.c_long, ctypes.c_double, ctypes.c_int,
            ctypes.c_void_p, ctypes.c_long, ctypes.c_void_p, ctypes.c_long,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        lib.sdpa_oracle_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def num_threads() -> int:
    """OpenMP threads the C oracle will use."""
    return int(_load().sdpa_oracle_num_threads())


def _as_f32(x) -> np.ndarray:
    a = np.asarray(x)
    if a.dtype not in (np.float16, np.float32, np.float64):
        raise TypeError(f"unsupported dtype {a.dtype}")
    a32 = np.ascontiguousarray(a, dtype=np.float32)
    if a.dtype == np.float64 and not np.array_equal(a32.astype(np.float64), a):
        raise ValueError("float64 input is not exactly representable in float32")
    return a32


def sdpa(q, k, v, scale=None, rows=None, return_lse=False, return_p=False, causal=False):
    """Materialised float64 attention, Eq. 1 (Section 3.1) with M = 0, or with the causal mask of
    Section 4.1.3 (keys after the query are left out) when ``causal`` is set.

    q: [..., Sq, D]; k, v: [..., Skv, D] (leading dims are batch/head and must
    agree; Sq = Skv = S is the paper's case, Sq != Skv the KV-cache / decoding
    shapes of its roadmap, Section 7, where under ``causal`` the queries are the
    last Sq positions of the Skv-long sequence: row i sees keys j <= i + Skv - Sq).
    scale: defaults to 1/sqrt(D) (Section 4.2.1); if given it is used
    as the float32 value the device receives, promoted to double.
    rows: optional 1-D sequence of query-row indices evaluated for every
    batch/head.  Returns o [..., nrows, D] float64 (and lse [..., nrows],
    p [..., nrows, Skv] on request).
    """
    q32, k32, v32 = _as_f32(q), _as_f32(k), _as_f32(v)
    if (k32.shape != v32.shape or q32.ndim < 2 or q32.ndim != k32.ndim
            or q32.shape[:-2] != k32.shape[:-2] or q32.shape[-1] != k32.shape[-1]):
        raise ValueError("q must be [..., Sq, D] and k, v [..., Skv, D] with equal leading dims and D")
    lead, (Sq, D) = q32.shape[:-2], q32.shape[-2:]
    S = k32.shape[-2]
    BH = int(np.prod(lead, dtype=np.int64)) if lead else 1
    if scale is None:
        scale = 1.0 / np.sqrt(np.float64(D))
    scale = float(np.float32(scale))
    if rows is None:
        rows_arr, nrows, rows_ptr = None, Sq, None
    else:
        rows_arr = np.ascontiguousarray(rows, dtype=np.int64)
        if rows_arr.ndim != 1:
            raise ValueError("rows must be one-dimensional")
        nrows, rows_ptr = rows_arr.size, rows_arr.ctypes.data
    o = np.empty((BH, nrows, D), dtype=np.float64)
    lse = np.empty((BH, nrows), dtype=np.float64) if return_lse else None
    p = np.empty((BH, nrows, S), dtype=np.float64) if return_p else None
    rc = _load().sdpa_oracle_rows_kv(
        q32.ctypes.data, k32.ctypes.data, v32.ctypes.data, BH, Sq, S, D, scale,
        rows_ptr, nrows, 1 if causal else 0, o.ctypes.data,
        lse.ctypes.data if lse is not None else None,
        p.ctypes.data if p is not None else None)
    if rc != 0:
        raise RuntimeError(f"sdpa_oracle_rows_kv failed with status {rc}")
    out = [o.reshape(*lead, nrows, D)]
    if return_lse:
        out.append(lse.reshape(*lead, nrows))
    if return_p:
        out.append(p.reshape(*lead, nrows, S))
    return out[0] if len(out) == 1 else tuple(out)


def sdpa_numpy(q, k, v, scale=None, return_lse=False, causal=False):
    """Eq. 1 (Section 3.1) as numpy float64 matrix expressions; M = 0, or the causal mask
    (M_ij = -inf for j > i, Section 4.1.3) added to the scaled scores exactly as Eq. 1 writes it.
    With Sq query rows against Skv >= Sq keys the mask is M_ij = -inf for j > i + Skv - Sq."""
    q64 = np.asarray(q, dtype=np.float64)
    k64 = np.asarray(k, dtype=np.float64)
    v64 = np.asarray(v, dtype=np.float64)
    D = q64.shape[-1]
    if scale is None:
        scale = 1.0 / np.sqrt(np.float64(D))
    scale = float(np.float32(scale))
    s = scale * (q64 @ np.swapaxes(k64, -1, -2))
    if causal:
        Sq, S = s.shape[-2:]
        if S < Sq:
            raise ValueError("causal needs Skv >= Sq")
        s = s + np.where(np.arange(S)[None, :] > np.arange(Sq)[:, None] + (S - Sq), -np.inf, 0.0)
    m = s.max(axis=-1, keepdims=True)
    e = np.exp(s - m)
    L = e.sum(axis=-1, keepdims=True)
    o = (e @ v64) / L
    if return_lse:
        return o, (m + np.log(L))[..., 0]
    return o


def sdpa_online(q, k, v, scale=None, tile_bounds=None, return_lse=False, causal=False):
    """Blockwise online-softmax attention, Section 4.1.2 (Eqs. 2-4), in float64.

    One problem: q [Sq, D] against k, v [S, D] (Sq = S in the paper).  ``tile_bounds`` is an
    increasing list of key indices 0 = b_0 < b_1 < ... < b_T = S; tile t holds keys b_t .. b_{t+1}-1.  For each
    tile, in the paper's order: scores, running max (Eq. 2), normaliser (Eq. 3),
    output accumulator (Eq. 4); after the last tile O_i = o_i / l_i.  The state
    starts at m = -inf, l = 0, o = 0 (the paper does not state the start; any
    start with l = 0, o = 0 and m below every score gives the same result).
    With ``causal`` the scores of keys after the query (j > i + S - Sq) are set to -inf before
    the update (a row whose keys in a tile are all masked keeps its state).
    """
    q64 = np.asarray(q, dtype=np.float64)
    k64 = np.asarray(k, dtype=np.float64)
    v64 = np.asarray(v, dtype=np.float64)
    Sq, D = q64.shape
    S = k64.shape[0]
    if scale is None:
        scale = 1.0 / np.sqrt(np.float64(D))
    scale = float(np.float32(scale))
    if tile_bounds is None:
        tile_bounds = [0, S]
    m = np.full(Sq, -np.inf)
    l = np.zeros(Sq)
    o = np.zeros((Sq, D))
    for lo, hi in zip(tile_bounds[:-1], tile_bounds[1:]):
        s_tile = scale * (q64 @ k64[lo:hi].T)                    # S_ij for this tile
        if causal:                                               # mask, then update (Section 4.1.2)
            s_tile = np.where(np.arange(lo, hi)[None, :] > np.arange(Sq)[:, None] + (S - Sq), -np.inf, s_tile)
        m_old = m
        m = np.maximum(m_old, s_tile.max(axis=1))                # Eq. 2
        with np.errstate(invalid="ignore"):
            alpha = np.where(np.isneginf(m), 0.0, np.exp(m_old - m))   # e^{m_old - m}; rows with no key yet
            e = np.where(np.isneginf(s_tile), 0.0, np.exp(s_tile - m[:, None]))
        l = l * alpha + e.sum(axis=1)                            # Eq. 3
        o = o * alpha[:, None] + e @ v64[lo:hi]                  # Eq. 4
    out = o / l[:, None]
    if return_lse:
        return out, m + np.log(l)
    return out


def sdpa_bwd(q, k, v, dout, scale=None, causal=False, qrows=None, krows=None):
    """Gradients of sum(dout * O) with respect to q, k, v for O of Eq. 1 (Section 3.1), float64, through
    the row-by-row C routine ``sdpa_oracle_bwd`` (the paper leaves the backward pass as future work,
    Section 7, so the formulas are the derivative of Eq. 1 written out; see the C source).

    q, k, v, dout: [..., S, D] with equal shapes.  ``qrows`` / ``krows`` optionally select the rows
    for which dq / (dk, dv) are returned.  Returns (dq [..., nq, D], dk [..., nk, D], dv [..., nk, D]).
    """
    q32, k32, v32, d32 = _as_f32(q), _as_f32(k), _as_f32(v), _as_f32(dout)
    if not (q32.shape == k32.shape == v32.shape == d32.shape) or q32.ndim < 2:
        raise ValueError("q, k, v, dout must have identical shape [..., S, D]")
    lead, (S, D) = q32.shape[:-2], q32.shape[-2:]
    BH = int(np.prod(lead, dtype=np.int64)) if lead else 1
    if scale is None:
        scale = 1.0 / np.sqrt(np.float64(D))
    scale = float(np.float32(scale))

    def subset(rows):
        if rows is None:
            return None, S, None
        arr = np.ascontiguousarray(rows, dtype=np.int64)
        if arr.ndim != 1:
            raise ValueError("row subsets must be one-dimensional")
        return arr, arr.size, arr.ctypes.data

    qarr, nq, qptr = subset(qrows)
    karr, nk, kptr = subset(krows)
    dq = np.zeros((BH, nq, D), dtype=np.float64)
    dk = np.zeros((BH, nk, D), dtype=np.float64)
    dv = np.zeros((BH, nk, D), dtype=np.float64)
    rc = _load().sdpa_oracle_bwd(q32.ctypes.data, k32.ctypes.data, v32.ctypes.data, d32.ctypes.data,
                                 BH, S, D, scale, 1 if causal else 0, qptr, nq, kptr, nk,
                                 dq.ctypes.data, dk.ctypes.data, dv.ctypes.data)
    if rc != 0:
        raise RuntimeError(f"sdpa_oracle_bwd failed with status {rc}")
    return dq.reshape(*lead, nq, D), dk.reshape(*lead, nk, D), dv.reshape(*lead, nk, D)


def sdpa_bwd_grouped(q, k, v, dout, scale=None, causal=False, qrows=None, krows=None):
    """Backward pass with grouped heads: q, dout [B, H, S, D], k, v [B, Hkv, S, D], H = G * Hkv, query head h
    reading key/value head h // G (the paper has G = 1, Section 3.1).  The forward pass is Eq. 1 per query
    head on the key/value rows of its group, i.e. on K and V repeated G times along the head axis, so by the
    chain rule of that repetition dQ is the gradient of the repeated problem and dK, dV are its gradients
    summed over the G query heads of each group.  That is what is computed here, literally, with
    :func:`sdpa_bwd` (the pinned row-by-row routine) on the repeated tensors.

    Returns (dq [B, H, nq, D], dk [B, Hkv, nk, D], dv [B, Hkv, nk, D])."""
    q32, k32, v32 = _as_f32(q), _as_f32(k), _as_f32(v)
    if q32.ndim != 4 or k32.ndim != 4 or k32.shape != v32.shape or q32.shape[0] != k32.shape[0] or \
            q32.shape[2:] != k32.shape[2:] or k32.shape[1] == 0 or q32.shape[1] % k32.shape[1] != 0:
        raise ValueError("q must be [B, H, S, D] and k, v [B, Hkv, S, D] with H a multiple of Hkv")
    B, H, S, D = q32.shape
    Hkv = k32.shape[1]
    G = H // Hkv
    dq, dkx, dvx = sdpa_bwd(q32, np.repeat(k32, G, axis=1), np.repeat(v32, G, axis=1), dout,
                            scale=scale, causal=causal, qrows=qrows, krows=krows)
    nk = dkx.shape[2]
    return dq, dkx.reshape(B, Hkv, G, nk, D).sum(axis=2), dvx.reshape(B, Hkv, G, nk, D).sum(axis=2)


def sdpa_bwd_numpy(q, k, v, dout, scale=None, causal=False):
    """The same gradients as numpy float64 matrix expressions (small shapes): with P the row softmax
    of the scaled, masked scores, dV = P^T dO, dP = dO V^T, dS = P * (dP - rowsum(P * dP)),
    dQ = scale * dS K, dK = scale * dS^T Q."""
    q64, k64, v64, d64 = (np.asarray(x, dtype=np.float64) for x in (q, k, v, dout))
    D = q64.shape[-1]
    if scale is None:
        scale = 1.0 / np.sqrt(np.float64(D))
    scale = float(np.float32(scale))
    s = scale * (q64 @ np.swapaxes(k64, -1, -2))
    if causal:
        S = s.shape[-1]
        s = s + np.where(np.arange(S)[None, :] > np.arange(S)[:, None], -np.inf, 0.0)
    e = np.exp(s - s.max(axis=-1, keepdims=True))
    p = e / e.sum(axis=-1, keepdims=True)
    dv = np.swapaxes(p, -1, -2) @ d64
    dp = d64 @ np.swapaxes(v64, -1, -2)
    ds = p * (dp - (p * dp).sum(axis=-1, keepdims=True))
    dq = scale * (ds @ k64)
    dk = scale * (np.swapaxes(ds, -1, -2) @ q64)
    return dq, dk, dv
