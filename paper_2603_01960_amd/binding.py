"""ctypes binding of libtiled_sdpa.so: argument marshalling only.

Every step of the forward pass runs in the HIP kernels behind the C-ABI declared
in include/tiled_sdpa.h.  PyTorch supplies device memory and the current stream.
There is no CPU fallback: if the library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import math
from pathlib import Path

F16, BF16 = 0, 1
FLAG_LINEAR_GRID = 1
FLAG_EXACT_MAX = 2
FLAG_CAUSAL = 8

_PKG = Path(__file__).resolve().parent
_LIB_PATH = _PKG / "libtiled_sdpa.so"
_lib = None

EXPORTS = (
    "tiled_sdpa_fwd",
    "tiled_sdpa_fwd_ex",
    "tiled_sdpa_bwd",
    "tiled_sdpa_bwd_gqa",
    "tiled_sdpa_bwd_workspace_bytes",
    "tiled_sdpa_default_tile",
    "tiled_sdpa_tune_tile",
    "tiled_sdpa_fwd_kv",
    "tiled_sdpa_fwd_gqa",
    "tiled_sdpa_fwd_kvcache",
    "tiled_sdpa_fwd_kvcache_static",
    "tiled_sdpa_fwd_paged",
    "tiled_sdpa_kv_default_splits",
    "tiled_sdpa_kv_workspace_bytes",
    "tiled_sdpa_probe_mfma",
    "tiled_sdpa_probe_hbm_read",
    "tiled_sdpa_status_string",
    "tiled_sdpa_version",
)


class TiledSdpaError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"tiled_sdpa status {status}: {text}")
        self.status = status


def library_path() -> Path:
    return _LIB_PATH


def load_library():
    """Load the HIP library; raises if it has not been built (python -m paper_2603_01960_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not _LIB_PATH.exists():
        raise FileNotFoundError(
            f"{_LIB_PATH} not found: build it with `python -m paper_2603_01960_amd.build` "
            "(there is no fallback path)")
    lib = ctypes.CDLL(str(_LIB_PATH))
    vp, ci, cf = ctypes.c_void_p, ctypes.c_int, ctypes.c_float
    lib.tiled_sdpa_fwd.restype = ci
    lib.tiled_sdpa_fwd.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, cf, ci, vp]
    lib.tiled_sdpa_fwd_ex.restype = ci
    lib.tiled_sdpa_fwd_ex.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, cf, ci, vp, ci, ci, ctypes.c_uint]
    lib.tiled_sdpa_default_tile.restype = ci
    lib.tiled_sdpa_default_tile.argtypes = [ci, ci, ci, ci, ci, ctypes.c_uint, ctypes.POINTER(ci), ctypes.POINTER(ci)]
    lib.tiled_sdpa_fwd_kv.restype = ci
    lib.tiled_sdpa_fwd_kv.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, cf, ci, vp, ci, ci, ctypes.c_uint,
                                      ci, vp, ctypes.c_ulonglong]
    lib.tiled_sdpa_kv_default_splits.restype = ci
    lib.tiled_sdpa_kv_default_splits.argtypes = [ci, ci, ci, ci, ci, ci, ctypes.c_uint, ctypes.POINTER(ci)]
    lib.tiled_sdpa_kv_workspace_bytes.restype = ctypes.c_ulonglong
    lib.tiled_sdpa_kv_workspace_bytes.argtypes = [ci, ci, ci, ci, ci]
    lib.tiled_sdpa_bwd.restype = ci
    lib.tiled_sdpa_fwd_gqa.restype = ci
    lib.tiled_sdpa_fwd_gqa.argtypes = [vp] * 5 + [ci] * 6 + [cf, ci, vp, ci, ci, ctypes.c_uint, ci, vp, ctypes.c_ulonglong]
    lib.tiled_sdpa_fwd_kvcache.restype = ci
    lib.tiled_sdpa_fwd_kvcache.argtypes = [vp] * 6 + [ci] * 6 + [cf, ci, vp, ci, ci, ctypes.c_uint, ci, vp, ctypes.c_ulonglong]
    lib.tiled_sdpa_fwd_kvcache_static.restype = ci
    lib.tiled_sdpa_fwd_kvcache_static.argtypes = [vp] * 6 + [ci] * 6 + [cf, ci, vp, ci, ci, ctypes.c_uint, ci]
    lib.tiled_sdpa_fwd_paged.restype = ci
    lib.tiled_sdpa_fwd_paged.argtypes = [vp] * 7 + [ci] * 7 + [cf, ci, vp, ci, ci, ctypes.c_uint, ci, vp, ctypes.c_ulonglong]
    lib.tiled_sdpa_tune_tile.restype = ci
    lib.tiled_sdpa_tune_tile.argtypes = [vp] * 4 + [ci] * 4 + [cf, ci, vp, ctypes.c_uint, ci,
                                         ctypes.POINTER(ci), ctypes.POINTER(ci), ctypes.POINTER(cf)]
    lib.tiled_sdpa_bwd.argtypes = [vp] * 9 + [ci, ci, ci, ci, cf, ci, ctypes.c_uint, vp, ctypes.c_ulonglong, vp]
    lib.tiled_sdpa_bwd_gqa.restype = ci
    lib.tiled_sdpa_bwd_gqa.argtypes = [vp] * 9 + [ci, ci, ci, ci, ci, cf, ci, ctypes.c_uint, vp, ctypes.c_ulonglong, vp]
    lib.tiled_sdpa_bwd_workspace_bytes.restype = ctypes.c_ulonglong
    lib.tiled_sdpa_bwd_workspace_bytes.argtypes = [ci, ci, ci]
    lib.tiled_sdpa_probe_hbm_read.restype = ci
    lib.tiled_sdpa_probe_hbm_read.argtypes = [vp, ctypes.c_ulonglong, vp, ctypes.POINTER(ctypes.c_double), vp]
    lib.tiled_sdpa_probe_mfma.restype = ci
    lib.tiled_sdpa_probe_mfma.argtypes = [ci, ci, ci, vp, ctypes.POINTER(ctypes.c_double), vp]
    lib.tiled_sdpa_status_string.restype = ctypes.c_char_p
    lib.tiled_sdpa_status_string.argtypes = [ci]
    lib.tiled_sdpa_version.restype = ci
    lib.tiled_sdpa_version.argtypes = []
    _lib = lib
    return lib


def version() -> int:
    return int(load_library().tiled_sdpa_version())


def status_string(status: int) -> str:
    return load_library().tiled_sdpa_status_string(int(status)).decode()


TILE_ORDER = ((64, 32), (64, 64), (64, 128), (128, 32), (128, 64), (128, 128), (256, 64))


def tune_tile(q, k, v, causal: bool = False, scale=None, *, launches: int = 10, flags: int = 0):
    """Time every legal (T_M, T_N) on these tensors (tiled_sdpa_tune_tile; waits for the stream) and
    return ``((tile_m, tile_n), {tile: ms per launch})``.  Pass the tile to :func:`sdpa`."""
    import torch

    if causal:
        flags |= FLAG_CAUSAL
    for t in (q, k, v):
        if not isinstance(t, torch.Tensor) or not t.is_cuda or t.dim() != 4 or not t.is_contiguous():
            raise ValueError("q, k, v must be contiguous [B, H, S, D] device tensors")
    if q.dtype not in (torch.float16, torch.bfloat16) or k.dtype != q.dtype or v.dtype != q.dtype or \
            k.shape != q.shape or v.shape != q.shape:
        raise ValueError("q, k, v must share shape and dtype float16 or bfloat16")
    B, H, S, D = q.shape
    out = torch.empty_like(q)
    tm, tn = ctypes.c_int(0), ctypes.c_int(0)
    ms = (ctypes.c_float * len(TILE_ORDER))()
    guard, stream = _guard_and_stream(torch, q.device)
    with guard:
        st = load_library().tiled_sdpa_tune_tile(q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(), B, H, S, D,
                                                 math.nan if scale is None else float(scale),
                                                 F16 if q.dtype == torch.float16 else BF16, stream, flags, launches,
                                                 ctypes.byref(tm), ctypes.byref(tn), ms)
    if st != 0:
        raise TiledSdpaError(st, status_string(st))
    return (tm.value, tn.value), {t: float(x) for t, x in zip(TILE_ORDER, ms) if x >= 0}


def default_tile(B: int, H: int, S: int, D: int, dtype: int, flags: int = 0):
    tm, tn = ctypes.c_int(0), ctypes.c_int(0)
    st = load_library().tiled_sdpa_default_tile(B, H, S, D, dtype, flags, ctypes.byref(tm), ctypes.byref(tn))
    if st != 0:
        raise TiledSdpaError(st, status_string(st))
    return tm.value, tn.value


def kv_default_splits(B: int, H: int, Sq: int, Skv: int, D: int, dtype: int, flags: int = 0) -> int:
    n = ctypes.c_int(0)
    st = load_library().tiled_sdpa_kv_default_splits(B, H, Sq, Skv, D, dtype, flags, ctypes.byref(n))
    if st != 0:
        raise TiledSdpaError(st, status_string(st))
    return n.value


def kv_workspace_bytes(B: int, H: int, Sq: int, D: int, splits: int) -> int:
    return int(load_library().tiled_sdpa_kv_workspace_bytes(B, H, Sq, D, splits))


def probe_mfma(dtype: int, random_operands, iters: int, sink=None, stream=None) -> float:
    """Enqueue the MFMA stream (see tiled_sdpa_probe_mfma); returns its flop count.

    ``random_operands``: False/0 constant operands, True/1 random ones, 2 random ones plus the
    attention loop's LDS-read and vector-ALU mix.

    With ``iters=0`` nothing is launched (flop count only) and ``sink`` may be None; a launch
    (``iters > 0``) needs a real device buffer of 512*256 floats."""
    if sink is None and iters != 0:
        raise ValueError("probe_mfma: iters > 0 launches a kernel that writes 512*256 floats to `sink`")
    flops = ctypes.c_double(0.0)
    st = load_library().tiled_sdpa_probe_mfma(dtype, int(random_operands), iters, sink, ctypes.byref(flops), stream)
    if st != 0:
        raise TiledSdpaError(st, status_string(st))
    return flops.value


def probe_hbm_read(src_ptr: int, nbytes: int, sink_ptr: int, stream=None) -> float:
    """Enqueue the read-only stream over ``nbytes`` at ``src_ptr`` (see tiled_sdpa_probe_hbm_read); returns
    the bytes it reads."""
    done = ctypes.c_double(0.0)
    st = load_library().tiled_sdpa_probe_hbm_read(src_ptr, nbytes, sink_ptr, ctypes.byref(done), stream)
    if st != 0:
        raise TiledSdpaError(st, status_string(st))
    return done.value


def tiled_sdpa_fwd(q_ptr, k_ptr, v_ptr, o_ptr, lse_ptr, B, H, S, D, scale, dtype, stream) -> int:
    """Raw call: integer device addresses in, status code out (same argument order as the C-ABI)."""
    return int(load_library().tiled_sdpa_fwd(q_ptr, k_ptr, v_ptr, o_ptr, lse_ptr, B, H, S, D,
                                             float(scale), dtype, stream))



class _NoGuard:
    def __enter__(self):
        return self

    def __exit__(self, *exc):
        return False


_NO_GUARD = _NoGuard()


def _guard_and_stream(torch, device):
    """(context manager that makes ``device`` current for the launch, raw handle of the stream that is
    current on it).  A short call is dominated by host time, so the usual case -- the tensors live on
    the current device -- takes no device switch and reads the raw stream handle directly."""
    current = torch.cuda.current_device()
    index = current if device.index is None else device.index
    guard = _NO_GUARD if index == current else torch.cuda.device(index)
    raw = getattr(torch._C, "_cuda_getCurrentRawStream", None)
    stream = raw(index) if raw is not None else torch.cuda.current_stream(index).cuda_stream
    return guard, stream


def tiled_sdpa_fwd_ex(q_ptr, k_ptr, v_ptr, o_ptr, lse_ptr, B, H, S, D, scale, dtype, stream,
                      tile_m=0, tile_n=0, flags=0) -> int:
    return int(load_library().tiled_sdpa_fwd_ex(q_ptr, k_ptr, v_ptr, o_ptr, lse_ptr, B, H, S, D,
                                                float(scale), dtype, stream, tile_m, tile_n, flags))


def tiled_sdpa_fwd_kv(q_ptr, k_ptr, v_ptr, o_ptr, lse_ptr, B, H, Sq, Skv, D, scale, dtype, stream,
                      tile_m=0, tile_n=0, flags=0, splits=0, workspace_ptr=None, workspace_bytes=0) -> int:
    return int(load_library().tiled_sdpa_fwd_kv(q_ptr, k_ptr, v_ptr, o_ptr, lse_ptr, B, H, Sq, Skv, D,
                                                float(scale), dtype, stream, tile_m, tile_n, flags,
                                                splits, workspace_ptr, workspace_bytes))


def tiled_sdpa_fwd_gqa(q_ptr, k_ptr, v_ptr, o_ptr, lse_ptr, B, H, Hkv, Sq, Skv, D, scale, dtype, stream,
                       tile_m=0, tile_n=0, flags=0, splits=0, workspace_ptr=None, workspace_bytes=0) -> int:
    return int(load_library().tiled_sdpa_fwd_gqa(q_ptr, k_ptr, v_ptr, o_ptr, lse_ptr, B, H, Hkv, Sq, Skv, D,
                                                 float(scale), dtype, stream, tile_m, tile_n, flags,
                                                 splits, workspace_ptr, workspace_bytes))


def tiled_sdpa_fwd_kvcache(q_ptr, k_ptr, v_ptr, o_ptr, lse_ptr, kv_lens_ptr, B, H, Hkv, Sq, Skv, D, scale, dtype,
                           stream, tile_m=0, tile_n=0, flags=0, splits=0, workspace_ptr=None, workspace_bytes=0) -> int:
    return int(load_library().tiled_sdpa_fwd_kvcache(q_ptr, k_ptr, v_ptr, o_ptr, lse_ptr, kv_lens_ptr, B, H, Hkv, Sq,
                                                     Skv, D, float(scale), dtype, stream, tile_m, tile_n, flags,
                                                     splits, workspace_ptr, workspace_bytes))


STATIC_SCRATCH_BYTES = 32 * 1024 * 1024


def tiled_sdpa_fwd_kvcache_static(q_ptr, k_ptr, v_ptr, o_ptr, lse_ptr, kv_lens_ptr, B, H, Hkv, Sq, Skv, D, scale, dtype,
                                  stream, tile_m=0, tile_n=0, flags=0, splits=0) -> int:
    """tiled_sdpa_fwd_kvcache with the split states in the library's own static device buffer."""
    return int(load_library().tiled_sdpa_fwd_kvcache_static(q_ptr, k_ptr, v_ptr, o_ptr, lse_ptr, kv_lens_ptr, B, H, Hkv,
                                                            Sq, Skv, D, float(scale), dtype, stream, tile_m, tile_n,
                                                            flags, splits))


def sdpa_kv(q, k, v, causal: bool = False, scale=None, *, splits: int = 0, return_lse: bool = False,
            out=None, workspace=None, tile=None, flags: int = 0, kv_lens=None):
    """Attention of q [B, H, Sq, D] over k, v [B, H, Skv, D] (KV-cache / decoding shapes), the key range
    split over ``splits`` workgroups per query tile (0 = heuristic).  Under ``causal`` the queries are
    the last Sq positions of the sequence.  ``workspace`` (any contiguous device tensor of enough bytes)
    is allocated through torch when not given and needed.

    Grouped heads: k, v may be [B, Hkv, Skv, D] with H = G * Hkv, query head h reading key/value head
    h // G (tiled_sdpa_fwd_gqa): the rows of a group share one pass over its keys.

    ``kv_lens`` (int32 device tensor [B]): k, v are a cache of capacity Skv of which batch entry b holds
    kv_lens[b] valid rows (tiled_sdpa_fwd_kvcache); rows no key reaches come back as zeros.
    """
    import torch

    if causal:
        flags |= FLAG_CAUSAL
    for name, t in (("q", q), ("k", k), ("v", v)):
        if not isinstance(t, torch.Tensor) or not t.is_cuda:
            raise ValueError(f"{name} must be a device tensor")
        if t.dim() != 4 or not t.is_contiguous():
            raise ValueError(f"{name} must be contiguous [B, H, S, D]")
    if q.dtype not in (torch.float16, torch.bfloat16) or k.dtype != q.dtype or v.dtype != q.dtype:
        raise ValueError("q, k, v must share dtype float16 or bfloat16")
    if k.shape != v.shape or q.shape[0] != k.shape[0] or q.shape[3] != k.shape[3]:
        raise ValueError("q must be [B, H, Sq, D] and k, v [B, Hkv, Skv, D]")
    if k.shape[1] == 0 or q.shape[1] % k.shape[1] != 0:
        raise ValueError("the number of query heads must be a multiple of the number of key/value heads")
    if k.device != q.device or v.device != q.device:
        raise ValueError("q, k, v must be on one device")
    if kv_lens is not None:
        if (not isinstance(kv_lens, torch.Tensor) or kv_lens.dtype != torch.int32 or kv_lens.device != q.device
                or kv_lens.shape != (q.shape[0],) or not kv_lens.is_contiguous()):
            raise ValueError("kv_lens must be a contiguous int32 tensor [B] on the device of q")
    B, H, Sq, D = q.shape
    Hkv, Skv = k.shape[1], k.shape[2]
    group = H // Hkv
    out_shape = q.shape
    dtype = F16 if q.dtype == torch.float16 else BF16
    if out is None:
        out = torch.empty(out_shape, dtype=q.dtype, device=q.device)
    elif out.shape != out_shape or out.dtype != q.dtype or not out.is_contiguous() or out.device != q.device:
        raise ValueError("out must match q in shape, dtype, device and be contiguous")
    lse = torch.empty(out_shape[:3], dtype=torch.float32, device=q.device) if return_lse else None
    tm, tn = tile if tile is not None else (0, 0)
    # the library's heuristics see B * Hkv heads of group * Sq rows each
    n = splits if splits else kv_default_splits(B, Hkv, group * Sq, Skv, D, dtype,
                                                flags if group == 1 else flags & ~FLAG_CAUSAL)
    need = kv_workspace_bytes(B, H, Sq, D, n)
    if workspace is None and need:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    guard, stream = _guard_and_stream(torch, q.device)
    with guard:
        st = tiled_sdpa_fwd_kvcache(q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(),
                                    lse.data_ptr() if lse is not None else None,
                                    kv_lens.data_ptr() if kv_lens is not None else None,
                                    B, H, Hkv, Sq, Skv, D, math.nan if scale is None else scale, dtype, stream,
                                    tm, tn, flags, n, ws_ptr, ws_bytes)
    if st != 0:
        raise TiledSdpaError(st, status_string(st))
    return (out, lse) if return_lse else out


def tiled_sdpa_fwd_paged(q_ptr, k_ptr, v_ptr, o_ptr, lse_ptr, kv_lens_ptr, block_table_ptr, B, H, Hkv, Sq, max_blocks,
                         block_rows, D, scale, dtype, stream, tile_m=0, tile_n=0, flags=0, splits=0,
                         workspace_ptr=None, workspace_bytes=0) -> int:
    return int(load_library().tiled_sdpa_fwd_paged(q_ptr, k_ptr, v_ptr, o_ptr, lse_ptr, kv_lens_ptr, block_table_ptr,
                                                   B, H, Hkv, Sq, max_blocks, block_rows, D, float(scale), dtype,
                                                   stream, tile_m, tile_n, flags, splits, workspace_ptr, workspace_bytes))


def sdpa_paged(q, k_pages, v_pages, kv_lens, block_table, causal: bool = False, scale=None, *, splits: int = 0,
               return_lse: bool = False, out=None, workspace=None, tile=None, flags: int = 0):
    """Attention of q [B, H, Sq, D] over a paged cache: k_pages, v_pages [P, Hkv, block_rows, D],
    block_table int32 [B, max_blocks] (page of every block of every batch entry), kv_lens int32 [B]
    (valid key rows per entry).  See tiled_sdpa_fwd_paged; otherwise as :func:`sdpa_kv`."""
    import torch

    if causal:
        flags |= FLAG_CAUSAL
    for name, t in (("q", q), ("k_pages", k_pages), ("v_pages", v_pages)):
        if not isinstance(t, torch.Tensor) or not t.is_cuda or t.dim() != 4 or not t.is_contiguous():
            raise ValueError(f"{name} must be a contiguous 4-d device tensor")
    if q.dtype not in (torch.float16, torch.bfloat16) or k_pages.dtype != q.dtype or v_pages.dtype != q.dtype:
        raise ValueError("q, k_pages, v_pages must share dtype float16 or bfloat16")
    if k_pages.shape != v_pages.shape or k_pages.shape[3] != q.shape[3] or k_pages.device != q.device or v_pages.device != q.device:
        raise ValueError("k_pages, v_pages must be [P, Hkv, block_rows, D] on the device of q")
    B, H, Sq, D = q.shape
    P, Hkv, block_rows = k_pages.shape[:3]
    if Hkv == 0 or H % Hkv != 0:
        raise ValueError("the number of query heads must be a multiple of the number of key/value heads")
    for name, t, shape in (("kv_lens", kv_lens, (B,)), ("block_table", block_table, None)):
        if (not isinstance(t, torch.Tensor) or t.dtype != torch.int32 or t.device != q.device or not t.is_contiguous()
                or (shape is not None and tuple(t.shape) != shape)):
            raise ValueError(f"{name} must be a contiguous int32 device tensor" + (f" {list(shape)}" if shape else ""))
    if block_table.dim() != 2 or block_table.shape[0] != B:
        raise ValueError("block_table must be [B, max_blocks]")
    max_blocks = block_table.shape[1]
    dtype = F16 if q.dtype == torch.float16 else BF16
    if out is None:
        out = torch.empty_like(q)
    elif out.shape != q.shape or out.dtype != q.dtype or not out.is_contiguous() or out.device != q.device:
        raise ValueError("out must match q in shape, dtype, device and be contiguous")
    lse = torch.empty((B, H, Sq), dtype=torch.float32, device=q.device) if return_lse else None
    tm, tn = tile if tile is not None else (0, 0)
    group = H // Hkv
    n = splits if splits else kv_default_splits(B, Hkv, group * Sq, max(1, max_blocks * block_rows), D, dtype,
                                                flags & ~FLAG_CAUSAL)
    need = kv_workspace_bytes(B, H, Sq, D, n)
    if workspace is None and need:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    guard, stream = _guard_and_stream(torch, q.device)
    with guard:
        st = tiled_sdpa_fwd_paged(q.data_ptr(), k_pages.data_ptr(), v_pages.data_ptr(), out.data_ptr(),
                                  lse.data_ptr() if lse is not None else None, kv_lens.data_ptr(),
                                  block_table.data_ptr(), B, H, Hkv, Sq, max_blocks, block_rows, D,
                                  math.nan if scale is None else scale, dtype, stream, tm, tn, flags, n, ws_ptr, ws_bytes)
    if st != 0:
        raise TiledSdpaError(st, status_string(st))
    return (out, lse) if return_lse else out


def bwd_workspace_bytes(B: int, H: int, S: int) -> int:
    return int(load_library().tiled_sdpa_bwd_workspace_bytes(B, H, S))


def tiled_sdpa_bwd(q_ptr, k_ptr, v_ptr, o_ptr, dout_ptr, lse_ptr, dq_ptr, dk_ptr, dv_ptr, B, H, S, D, scale,
                   dtype, flags, workspace_ptr, workspace_bytes, stream) -> int:
    return int(load_library().tiled_sdpa_bwd(q_ptr, k_ptr, v_ptr, o_ptr, dout_ptr, lse_ptr, dq_ptr, dk_ptr,
                                             dv_ptr, B, H, S, D, float(scale), dtype, flags,
                                             workspace_ptr, workspace_bytes, stream))


def sdpa_backward(q, k, v, o, dout, lse, causal: bool = False, scale=None, *, workspace=None, grads=None):
    """(dq, dk, dv) for the attention of :func:`sdpa`; ``o`` and ``lse`` are that call's outputs
    (``return_lse=True``) for the same q, k, v, causal and scale.  ``grads=(dq, dk, dv)`` and
    ``workspace`` let the caller own the buffers; otherwise torch allocates them.

    Grouped heads: k, v [B, Hkv, S, D] with H a multiple of Hkv (the forward of ``sdpa_kv`` at Sq = Skv);
    dk, dv then have the shape of k and hold the sum over the query heads of each group."""
    import torch

    for name, t, like in (("q", q, q), ("k", k, k), ("v", v, k), ("o", o, q), ("dout", dout, q)):
        if not isinstance(t, torch.Tensor) or not t.is_cuda:
            raise ValueError(f"{name} must be a device tensor")
        if t.dim() != 4 or not t.is_contiguous():
            raise ValueError(f"{name} must be contiguous [B, H, S, D]")
        if t.shape != like.shape or t.dtype != q.dtype or t.device != q.device:
            raise ValueError("q, o, dout and k, v must agree in shape, dtype and device")
    if q.dtype not in (torch.float16, torch.bfloat16):
        raise ValueError("dtype must be float16 or bfloat16")
    B, H, S, D = q.shape
    Hkv = k.shape[1]
    if k.shape[0] != B or k.shape[2:] != q.shape[2:] or Hkv == 0 or H % Hkv != 0:
        raise ValueError("k, v must be [B, Hkv, S, D] with H a multiple of Hkv")
    if lse.shape != (B, H, S) or lse.dtype != torch.float32 or not lse.is_contiguous() or lse.device != q.device:
        raise ValueError("lse must be contiguous float32 [B, H, S] on the same device")
    dtype = F16 if q.dtype == torch.float16 else BF16
    if grads is None:
        grads = (torch.empty_like(q), torch.empty_like(k), torch.empty_like(k))
    for gname, t, like in zip(("dq", "dk", "dv"), grads, (q, k, k)):
        if t.shape != like.shape or t.dtype != q.dtype or not t.is_contiguous() or t.device != q.device:
            raise ValueError(f"{gname} must match {'q' if like is q else 'k'} in shape, dtype, device and be contiguous")
    need = bwd_workspace_bytes(B, H, S)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    ws_bytes = workspace.numel() * workspace.element_size()
    guard, stream = _guard_and_stream(torch, q.device)
    with guard:
        st = int(load_library().tiled_sdpa_bwd_gqa(
            q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), dout.data_ptr(),
            lse.data_ptr(), grads[0].data_ptr(), grads[1].data_ptr(), grads[2].data_ptr(),
            B, H, Hkv, S, D, math.nan if scale is None else float(scale), dtype,
            FLAG_CAUSAL if causal else 0, workspace.data_ptr(), ws_bytes, stream))
    if st != 0:
        raise TiledSdpaError(st, status_string(st))
    return grads


def sdpa(q, k, v, causal: bool = False, scale=None, *, return_lse: bool = False, out=None,
         lse_out=None, tile=None, flags: int = 0):
    """o = softmax(q k^T * scale [+ causal mask]) v for contiguous [B, H, S, D] FP16/BF16 device tensors.

    Mirrors the functional API of Section 4.2.1 of the paper (scale defaults to 1/sqrt(D)).
    ``tile=(T_M, T_N)`` pins the schedule; ``out`` / ``lse_out`` let the caller own the outputs.
    """
    import torch

    if causal:
        flags |= FLAG_CAUSAL
    for name, t in (("q", q), ("k", k), ("v", v)):
        if not isinstance(t, torch.Tensor) or not t.is_cuda:
            raise ValueError(f"{name} must be a device tensor")
        if t.dim() != 4:
            raise ValueError(f"{name} must be [B, H, S, D]")
        if not t.is_contiguous():
            raise ValueError(f"{name} must be contiguous")
    if q.dtype not in (torch.float16, torch.bfloat16) or k.dtype != q.dtype or v.dtype != q.dtype:
        raise ValueError("q, k, v must share dtype float16 or bfloat16")
    if q.shape != k.shape or q.shape != v.shape or k.device != q.device or v.device != q.device:
        raise ValueError("q, k, v must have identical shape and device")
    B, H, S, D = q.shape
    dtype = F16 if q.dtype == torch.float16 else BF16
    if out is None:
        out = torch.empty_like(q)
    elif out.shape != q.shape or out.dtype != q.dtype or not out.is_contiguous() or out.device != q.device:
        raise ValueError("out must match q in shape, dtype, device and be contiguous")
    lse = None
    if return_lse:
        lse = lse_out if lse_out is not None else torch.empty((B, H, S), dtype=torch.float32, device=q.device)
        if lse.shape != (B, H, S) or lse.dtype != torch.float32 or not lse.is_contiguous():
            raise ValueError("lse_out must be contiguous float32 [B, H, S]")
    tm, tn = tile if tile is not None else (0, 0)
    guard, stream = _guard_and_stream(torch, q.device)
    with guard:
        st = tiled_sdpa_fwd_ex(q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(),
                               lse.data_ptr() if lse is not None else None,
                               B, H, S, D, math.nan if scale is None else scale, dtype, stream,
                               tm, tn, flags)
    if st != 0:
        raise TiledSdpaError(st, status_string(st))
    return (out, lse) if return_lse else out
