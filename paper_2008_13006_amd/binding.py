"""ctypes binding of the C-ABI library ``libtw.so`` (see ``include/tw.h``).

Argument marshalling only: every step of the path (tiling analysis, compaction, schedule,
the GEMMs) runs inside the library.  PyTorch appears here solely as the owner of device
memory and streams.  Importing this module without a built library raises; there is no
fallback of any kind.
"""
from __future__ import annotations

import ctypes
import os
from typing import Dict, Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtw.so")

TW_F16, TW_BF16 = 0, 1
_DT = {"f16": TW_F16, "bf16": TW_BF16}

SYMBOLS = ["tw_pack_size", "tw_pack", "tw_pack_tew_size", "tw_pack_tew", "tw_restore_ew", "tw_unpack", "tw_info", "tw_prune", "tw_gemm_workspace", "tw_gemm_plan", "tw_gemm", "tw_gemm_static",
           "tw_gemm_bias_act", "tw_gemm_t", "tw_gemm_t_bias_act", "tw_transpose", "tw_dense_gemm", "tw_dense_gemm_bias_act", "tw_strerror",
           "tw_version"]
TW_ACT_NONE, TW_ACT_RELU, TW_ACT_GELU = 0, 1, 2
TW_STATIC_SCRATCH_BYTES = 8 << 20   # include/tw.h
_ACT = {None: TW_ACT_NONE, "none": TW_ACT_NONE, "relu": TW_ACT_RELU, "gelu": TW_ACT_GELU}


class TwError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {_strerror(status)} ({status})")


class TwInfo(ctypes.Structure):
    _fields_ = [("version", ctypes.c_int32), ("dtype", ctypes.c_int32), ("K", ctypes.c_int32),
                ("N", ctypes.c_int32), ("G", ctypes.c_int32), ("T", ctypes.c_int32),
                ("n_kept_cols", ctypes.c_int32), ("k_chunk", ctypes.c_int32),
                ("nnz", ctypes.c_int64), ("ew_nnz", ctypes.c_int64), ("padded_macs_per_row", ctypes.c_int64),
                ("blob_bytes", ctypes.c_uint64),
                ("off_col_idx", ctypes.c_uint64), ("off_tile_col_ptr", ctypes.c_uint64),
                ("off_tile_row_ptr", ctypes.c_uint64), ("off_row_idx", ctypes.c_uint64),
                ("off_tile_span", ctypes.c_uint64), ("off_sched_order", ctypes.c_uint64)]


class TwPlan(ctypes.Structure):
    _fields_ = [("mode", ctypes.c_int32), ("rows_per_block", ctypes.c_int32), ("tiles_per_set", ctypes.c_int32),
                ("n_row_blocks", ctypes.c_int32), ("n_sets", ctypes.c_int32), ("n_items", ctypes.c_int32),
                ("grid", ctypes.c_int32), ("lds_bytes", ctypes.c_uint32), ("row_lists", ctypes.c_int32),
                ("k_parts", ctypes.c_int32), ("reserved", ctypes.c_int32 * 6)]


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "(hipcc, gfx950) first; there is no fallback path")
    lib = ctypes.CDLL(LIB_PATH)
    vp, sz, i = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
    lib.tw_pack_size.argtypes = [vp, i, i, i, i, ctypes.POINTER(sz)]
    lib.tw_pack.argtypes = [vp, i, vp, i, i, i, i, vp, sz]
    lib.tw_unpack.argtypes = [vp, vp, i, vp]
    lib.tw_pack_tew_size.argtypes = [vp, vp, i, i, i, i, ctypes.POINTER(sz)]
    lib.tw_pack_tew.argtypes = [vp, i, vp, vp, i, i, i, i, vp, sz]
    lib.tw_restore_ew.argtypes = [vp, i, i, i, i, vp, ctypes.c_double, vp]
    lib.tw_info.argtypes = [vp, ctypes.POINTER(TwInfo)]
    lib.tw_gemm_workspace.argtypes = [vp, i, ctypes.POINTER(sz)]
    lib.tw_gemm_plan.argtypes = [vp, i, i, i, ctypes.POINTER(TwPlan)]
    lib.tw_gemm.argtypes = [vp, vp, vp, i, i, vp, i, vp, sz, vp]
    lib.tw_gemm_static.argtypes = [vp, vp, vp, i, i, vp, i, vp]
    lib.tw_dense_gemm.argtypes = [vp, i, vp, i, vp, i, i, i, i, i, vp]
    lib.tw_gemm_bias_act.argtypes = [vp, vp, vp, i, i, vp, i, vp, i, vp, sz, vp]
    lib.tw_gemm_t.argtypes = [vp, vp, vp, i, i, vp, i, vp, sz, vp]
    lib.tw_gemm_t_bias_act.argtypes = [vp, vp, vp, i, i, vp, i, vp, i, vp, sz, vp]
    lib.tw_transpose.argtypes = [vp, i, i, i, vp, i, vp]
    lib.tw_dense_gemm_bias_act.argtypes = [vp, i, vp, i, vp, i, vp, i, i, i, i, i, vp]
    lib.tw_strerror.argtypes = [i]
    lib.tw_strerror.restype = ctypes.c_char_p
    for name in SYMBOLS:
        if name != "tw_strerror":
            getattr(lib, name).restype = ctypes.c_int
    return lib


_lib = _load()


def _strerror(status: int) -> str:
    return _lib.tw_strerror(int(status)).decode()


def _check(status: int, where: str) -> None:
    if status != 0:
        raise TwError(status, where)


def _np_ptr(a: np.ndarray) -> ctypes.c_void_p:
    return ctypes.c_void_p(a.ctypes.data)


def tw_version() -> int:
    return int(_lib.tw_version())


# --------------------------------------------------------------------------- host side
def tw_pack_size(mask: np.ndarray, G: int, dtype: str) -> int:
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    K, N = mask.shape
    n = ctypes.c_size_t(0)
    _check(_lib.tw_pack_size(_np_ptr(mask), K, N, int(G), _DT[dtype], ctypes.byref(n)), "tw_pack_size")
    return int(n.value)


def tw_pack(B_bits: np.ndarray, mask: np.ndarray, G: int, dtype: str) -> np.ndarray:
    """B_bits: uint16 [K, N] (row stride may exceed N), mask: uint8 [K, N].  Returns the blob (uint8)."""
    assert B_bits.dtype == np.uint16 and B_bits.ndim == 2 and B_bits.strides[1] == 2
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    K, N = mask.shape
    assert B_bits.shape == (K, N)
    ldb = B_bits.strides[0] // 2 if K > 1 else N
    nbytes = tw_pack_size(mask, G, dtype)
    blob = _aligned_bytes(nbytes, 256)
    _check(_lib.tw_pack(_np_ptr(B_bits), ldb, _np_ptr(mask), K, N, int(G), _DT[dtype], _np_ptr(blob), nbytes),
           "tw_pack")
    return blob


def tw_pack_tew(B_bits: np.ndarray, mask: np.ndarray, ew_mask: np.ndarray, G: int, dtype: str) -> np.ndarray:
    """TW pattern `mask` plus the element-wise residual `ew_mask` (both uint8 [K, N]).  Returns the blob."""
    assert B_bits.dtype == np.uint16 and B_bits.ndim == 2 and B_bits.strides[1] == 2
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    ew_mask = np.ascontiguousarray(ew_mask, dtype=np.uint8)
    K, N = mask.shape
    assert B_bits.shape == (K, N) and ew_mask.shape == (K, N)
    ldb = B_bits.strides[0] // 2 if K > 1 else N
    n = ctypes.c_size_t(0)
    _check(_lib.tw_pack_tew_size(_np_ptr(mask), _np_ptr(ew_mask), K, N, int(G), _DT[dtype], ctypes.byref(n)),
           "tw_pack_tew_size")
    blob = _aligned_bytes(int(n.value), 256)
    _check(_lib.tw_pack_tew(_np_ptr(B_bits), ldb, _np_ptr(mask), _np_ptr(ew_mask), K, N, int(G), _DT[dtype],
                            _np_ptr(blob), int(n.value)), "tw_pack_tew")
    return blob


def tw_restore_ew(B_bits: np.ndarray, mask: np.ndarray, delta: float, dtype: str) -> np.ndarray:
    """The delta*K*N pruned weights of largest magnitude in surviving columns, as a uint8 [K, N] mask."""
    assert B_bits.dtype == np.uint16 and B_bits.ndim == 2 and B_bits.strides[1] == 2
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    K, N = mask.shape
    ldb = B_bits.strides[0] // 2 if K > 1 else N
    out = np.empty((K, N), dtype=np.uint8)
    _check(_lib.tw_restore_ew(_np_ptr(B_bits), ldb, K, N, _DT[dtype], _np_ptr(mask), ctypes.c_double(delta),
                              _np_ptr(out)), "tw_restore_ew")
    return out


def _aligned_bytes(n: int, align: int) -> np.ndarray:
    raw = np.zeros(n + align, dtype=np.uint8)
    off = (-raw.ctypes.data) % align
    return raw[off:off + n]


def tw_prune(B_bits: np.ndarray, G: int, dtype: str, col_prune: float, sparsity: float) -> np.ndarray:
    """One-shot magnitude pruning into the TW pattern; returns the uint8 [K, N] mask."""
    assert B_bits.dtype == np.uint16 and B_bits.ndim == 2 and B_bits.strides[1] == 2
    K, N = B_bits.shape
    ldb = B_bits.strides[0] // 2 if K > 1 else N
    mask = np.empty((K, N), dtype=np.uint8)
    _check(_lib.tw_prune(_np_ptr(B_bits), ldb, K, N, G, _DT[dtype], ctypes.c_double(col_prune),
                         ctypes.c_double(sparsity), _np_ptr(mask)), "tw_prune")
    return mask


def tw_unpack(blob: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    inf = tw_info(blob)
    K, N = inf["K"], inf["N"]
    B = np.empty((K, N), dtype=np.uint16)
    mask = np.empty((K, N), dtype=np.uint8)
    _check(_lib.tw_unpack(_np_ptr(blob), _np_ptr(B), N, _np_ptr(mask)), "tw_unpack")
    return B, mask


def tw_info(blob: np.ndarray) -> Dict:
    """Header fields plus views of the canonical int32 index arrays inside the blob."""
    assert blob.dtype == np.uint8 and blob.flags["C_CONTIGUOUS"]
    ti = TwInfo()
    _check(_lib.tw_info(_np_ptr(blob), ctypes.byref(ti)), "tw_info")
    out = {f: getattr(ti, f) for f, _ in TwInfo._fields_}
    T, nk = ti.T, ti.n_kept_cols

    def arr(off, n):
        return blob[off:off + 4 * n].view(np.int32)

    out["tile_row_ptr"] = arr(ti.off_tile_row_ptr, T + 1)
    out["tile_col_ptr"] = arr(ti.off_tile_col_ptr, T + 1)
    out["col_idx"] = arr(ti.off_col_idx, nk)
    out["row_idx"] = arr(ti.off_row_idx, int(out["tile_row_ptr"][T]) if T > 0 else 0)
    out["tile_span"] = arr(ti.off_tile_span, T + 1)
    out["sched_order"] = arr(ti.off_sched_order, T)
    return out


def tw_gemm_plan(blob: np.ndarray, M: int, n_cu: int = 256, transposed: bool = False) -> Dict:
    """How tw_gemm / tw_gemm_t would run this weight on M rows on a GPU of n_cu compute units (host only)."""
    assert blob.dtype == np.uint8 and blob.flags["C_CONTIGUOUS"]
    pl = TwPlan()
    _check(_lib.tw_gemm_plan(_np_ptr(blob), int(M), int(n_cu), int(bool(transposed)), ctypes.byref(pl)), "tw_gemm_plan")
    return {f: getattr(pl, f) for f, _ in TwPlan._fields_ if f != "reserved"}


# --------------------------------------------------------------------------- device side
def _torch():
    import torch
    return torch


def _tdtype(dtype: str):
    torch = _torch()
    return torch.float16 if dtype == "f16" else torch.bfloat16


def _stream_ptr(stream=None) -> ctypes.c_void_p:
    torch = _torch()
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def tw_gemm_workspace(blob: np.ndarray, M: int) -> int:
    n = ctypes.c_size_t(0)
    _check(_lib.tw_gemm_workspace(_np_ptr(blob), int(M), ctypes.byref(n)), "tw_gemm_workspace")
    return int(n.value)


class TwWeight:
    """A packed weight resident on one GPU: host blob, device copy and a workspace (zeroed scheduler counters and,
    for few rows and a long K, room for the partial results of a split-K plan).  The library's rule applies:
    calls on ONE workspace must not overlap in time, so launches of one weight that may run concurrently (two
    streams) need a TwWeight each: `sibling()` gives another one on the same device copy of the blob."""

    def __init__(self, blob: np.ndarray, device="cuda:0"):
        torch = _torch()
        self.blob = blob
        self.info = tw_info(blob)
        self.dtype = "f16" if self.info["dtype"] == TW_F16 else "bf16"
        self.blob_dev = torch.from_numpy(blob).to(device)
        assert self.blob_dev.data_ptr() % 256 == 0
        self.workspace = torch.zeros(256, dtype=torch.uint8, device=device)
        self.ws_limit = None        # bytes of workspace handed to the library at most (None: what it asks for)
        self._retired = []          # outgrown workspaces: kept, kernels already enqueued may still use them
        self._ws_need = {}          # M -> bytes the library wants (asked once per M)

    def sibling(self):
        """Another TwWeight on the same host and device copy of the blob, with a workspace of its own."""
        torch = _torch()
        other = object.__new__(TwWeight)
        other.blob, other.info, other.dtype, other.blob_dev = self.blob, self.info, self.dtype, self.blob_dev
        other.workspace = torch.zeros(256, dtype=torch.uint8, device=self.workspace.device)
        other.ws_limit, other._retired, other._ws_need = self.ws_limit, [], {}
        return other

    def workspace_for(self, M: int):
        """(pointer, bytes) of a zero-initialised workspace of the size the library wants for M rows."""
        need = self._ws_need.get(M)
        if need is None:
            need = self._ws_need[M] = max(256, tw_gemm_workspace(self.blob, M))
        if self.ws_limit is not None:
            need = max(256, min(need, int(self.ws_limit)))
        if need > self.workspace.numel():
            torch = _torch()
            self._retired.append(self.workspace)
            self.workspace = torch.zeros(need, dtype=torch.uint8, device=self.workspace.device)
        return ctypes.c_void_p(self.workspace.data_ptr()), need

    @classmethod
    def from_dense(cls, B_bits: np.ndarray, mask: np.ndarray, G: int, dtype: str, device="cuda:0"):
        return cls(tw_pack(B_bits, mask, G, dtype), device)


def tw_gemm(w: TwWeight, A, C=None, stream=None):
    """C = A . (B * mask).  A: torch tensor [M, K] (f16/bf16, cuda, unit column stride)."""
    torch = _torch()
    assert A.is_cuda and A.dtype == _tdtype(w.dtype) and A.dim() == 2 and A.stride(1) == 1
    M, K = A.shape
    assert K == w.info["K"]
    N = w.info["N"]
    if C is None:
        C = torch.empty((M, N), dtype=A.dtype, device=A.device)
    assert C.is_cuda and C.dtype == A.dtype and C.shape == (M, N) and C.stride(1) == 1
    lda = A.stride(0) if M > 1 else max(K, A.stride(0))
    ldc = C.stride(0) if M > 1 else max(N, C.stride(0))
    ws, ws_bytes = w.workspace_for(M)
    _check(_lib.tw_gemm(_np_ptr(w.blob), ctypes.c_void_p(w.blob_dev.data_ptr()), ctypes.c_void_p(A.data_ptr()),
                        M, lda, ctypes.c_void_p(C.data_ptr()), ldc, ws, ws_bytes, _stream_ptr(stream)), "tw_gemm")
    return C


def tw_gemm_static(w: TwWeight, A, C, stream=None):
    """tw_gemm without a workspace and without any allocation: the library's own per-GPU scratch array holds the
    scheduler's counters and the partial results of a split-K plan.  C must be given (the caller owns every buffer).  Calls must not overlap on one GPU."""
    assert A.is_cuda and A.dtype == _tdtype(w.dtype) and A.dim() == 2 and A.stride(1) == 1
    M, K = A.shape
    N = w.info["N"]
    assert K == w.info["K"]
    assert C.is_cuda and C.dtype == A.dtype and C.shape == (M, N) and C.stride(1) == 1
    lda = A.stride(0) if M > 1 else max(K, A.stride(0))
    ldc = C.stride(0) if M > 1 else max(N, C.stride(0))
    _check(_lib.tw_gemm_static(_np_ptr(w.blob), ctypes.c_void_p(w.blob_dev.data_ptr()), ctypes.c_void_p(A.data_ptr()),
                               M, lda, ctypes.c_void_p(C.data_ptr()), ldc, _stream_ptr(stream)), "tw_gemm_static")
    return C


def tw_gemm_t(w: TwWeight, At, Ct=None, stream=None):
    """Ct = (A . (B * mask))^T from At = A^T.  At: torch tensor [K, M], Ct: [N, M] (unit column stride)."""
    return tw_gemm_t_bias_act(w, At, None, "none", Ct, stream)


def tw_gemm_t_bias_act(w: TwWeight, At, bias=None, act="none", Ct=None, stream=None):
    """Ct = act(A . (B * mask) + bias)^T from At = A^T; bias: torch tensor [N] or None."""
    torch = _torch()
    assert At.is_cuda and At.dtype == _tdtype(w.dtype) and At.dim() == 2 and At.stride(1) == 1
    K, M = At.shape
    assert K == w.info["K"]
    N = w.info["N"]
    if Ct is None:
        ld = (M + 63) // 64 * 64
        Ct = torch.empty((N, ld), dtype=At.dtype, device=At.device)[:, :M]
    assert Ct.is_cuda and Ct.dtype == At.dtype and Ct.shape == (N, M) and Ct.stride(1) == 1
    ldat = At.stride(0) if K > 1 else max(M, At.stride(0))
    ldct = Ct.stride(0) if N > 1 else max(M, Ct.stride(0))
    bptr = ctypes.c_void_p(0)
    if bias is not None:
        assert bias.is_cuda and bias.dtype == At.dtype and bias.shape == (N,) and bias.stride(0) == 1
        bptr = ctypes.c_void_p(bias.data_ptr())
    ws, ws_bytes = w.workspace_for(M)
    if bias is None and _act_code(act) == TW_ACT_NONE:
        _check(_lib.tw_gemm_t(_np_ptr(w.blob), ctypes.c_void_p(w.blob_dev.data_ptr()), ctypes.c_void_p(At.data_ptr()),
                              M, ldat, ctypes.c_void_p(Ct.data_ptr()), ldct, ws, ws_bytes, _stream_ptr(stream)), "tw_gemm_t")
    else:
        _check(_lib.tw_gemm_t_bias_act(_np_ptr(w.blob), ctypes.c_void_p(w.blob_dev.data_ptr()),
                                       ctypes.c_void_p(At.data_ptr()), M, ldat, bptr, _act_code(act),
                                       ctypes.c_void_p(Ct.data_ptr()), ldct, ws, ws_bytes, _stream_ptr(stream)),
               "tw_gemm_t_bias_act")
    return Ct


def tw_transpose(src, dst=None, stream=None):
    """dst = src^T for a 2-D torch tensor of a 16-bit type (unit column stride)."""
    torch = _torch()
    assert src.is_cuda and src.dim() == 2 and src.stride(1) == 1 and src.element_size() == 2
    rows, cols = src.shape
    if dst is None:
        ld = (rows + 63) // 64 * 64
        dst = torch.empty((cols, ld), dtype=src.dtype, device=src.device)[:, :rows]
    assert dst.shape == (cols, rows) and dst.dtype == src.dtype and dst.stride(1) == 1
    lds = src.stride(0) if rows > 1 else max(cols, src.stride(0))
    ldd = dst.stride(0) if cols > 1 else max(rows, dst.stride(0))
    _check(_lib.tw_transpose(ctypes.c_void_p(src.data_ptr()), lds, rows, cols, ctypes.c_void_p(dst.data_ptr()), ldd,
                             _stream_ptr(stream)), "tw_transpose")
    return dst


def _act_code(act) -> int:
    if isinstance(act, int):
        return act
    if act not in _ACT:
        raise ValueError(f"unknown activation {act!r}")
    return _ACT[act]


def tw_gemm_bias_act(w: TwWeight, A, bias=None, act="none", C=None, stream=None):
    """C = act(A . (B * mask) + bias).  bias: torch tensor [N] of A's dtype on the GPU, or None."""
    torch = _torch()
    assert A.is_cuda and A.dtype == _tdtype(w.dtype) and A.dim() == 2 and A.stride(1) == 1
    M, K = A.shape
    assert K == w.info["K"]
    N = w.info["N"]
    if C is None:
        C = torch.empty((M, N), dtype=A.dtype, device=A.device)
    assert C.is_cuda and C.dtype == A.dtype and C.shape == (M, N) and C.stride(1) == 1
    bptr = ctypes.c_void_p(0)
    if bias is not None:
        assert bias.is_cuda and bias.dtype == A.dtype and bias.shape == (N,) and bias.stride(0) == 1
        bptr = ctypes.c_void_p(bias.data_ptr())
    lda = A.stride(0) if M > 1 else max(K, A.stride(0))
    ldc = C.stride(0) if M > 1 else max(N, C.stride(0))
    ws, ws_bytes = w.workspace_for(M)
    _check(_lib.tw_gemm_bias_act(_np_ptr(w.blob), ctypes.c_void_p(w.blob_dev.data_ptr()),
                                 ctypes.c_void_p(A.data_ptr()), M, lda, bptr, _act_code(act),
                                 ctypes.c_void_p(C.data_ptr()), ldc, ws, ws_bytes, _stream_ptr(stream)), "tw_gemm_bias_act")
    return C


def tw_dense_gemm_bias_act(A, B, bias=None, act="none", C=None, stream=None):
    """C = act(A . B + bias), both matrices row-major torch tensors on the GPU."""
    torch = _torch()
    assert A.is_cuda and B.is_cuda and A.dtype == B.dtype and A.dtype in (torch.float16, torch.bfloat16)
    assert A.dim() == 2 and B.dim() == 2 and A.stride(1) == 1 and B.stride(1) == 1
    M, K = A.shape
    K2, N = B.shape
    assert K == K2
    if C is None:
        C = torch.empty((M, N), dtype=A.dtype, device=A.device)
    assert C.shape == (M, N) and C.dtype == A.dtype and C.stride(1) == 1
    bptr = ctypes.c_void_p(0)
    if bias is not None:
        assert bias.is_cuda and bias.dtype == A.dtype and bias.shape == (N,) and bias.stride(0) == 1
        bptr = ctypes.c_void_p(bias.data_ptr())
    dt = TW_F16 if A.dtype == torch.float16 else TW_BF16
    lda = A.stride(0) if M > 1 else max(K, A.stride(0))
    ldb = B.stride(0) if K > 1 else max(N, B.stride(0))
    ldc = C.stride(0) if M > 1 else max(N, C.stride(0))
    _check(_lib.tw_dense_gemm_bias_act(ctypes.c_void_p(A.data_ptr()), lda, ctypes.c_void_p(B.data_ptr()), ldb, bptr,
                                       _act_code(act), ctypes.c_void_p(C.data_ptr()), ldc, M, N, K, dt,
                                       _stream_ptr(stream)), "tw_dense_gemm_bias_act")
    return C


def tw_dense_gemm(A, B, C=None, stream=None):
    """C = A . B, both row-major torch tensors on the GPU."""
    torch = _torch()
    assert A.is_cuda and B.is_cuda and A.dtype == B.dtype and A.dtype in (torch.float16, torch.bfloat16)
    assert A.dim() == 2 and B.dim() == 2 and A.stride(1) == 1 and B.stride(1) == 1
    M, K = A.shape
    K2, N = B.shape
    assert K == K2
    if C is None:
        C = torch.empty((M, N), dtype=A.dtype, device=A.device)
    assert C.shape == (M, N) and C.dtype == A.dtype and C.stride(1) == 1
    dt = TW_F16 if A.dtype == torch.float16 else TW_BF16
    lda = A.stride(0) if M > 1 else max(K, A.stride(0))
    ldb = B.stride(0) if K > 1 else max(N, B.stride(0))
    ldc = C.stride(0) if M > 1 else max(N, C.stride(0))
    _check(_lib.tw_dense_gemm(ctypes.c_void_p(A.data_ptr()), lda, ctypes.c_void_p(B.data_ptr()), ldb,
                              ctypes.c_void_p(C.data_ptr()), ldc, M, N, K, dt, _stream_ptr(stream)), "tw_dense_gemm")
    return C


def bits_to_tensor(bits: np.ndarray, dtype: str, device="cuda:0"):
    """uint16 bit patterns -> torch tensor of the 16-bit float type on `device` (a pure reinterpretation)."""
    torch = _torch()
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(device)
    return t.view(_tdtype(dtype))


def tensor_to_bits(t) -> np.ndarray:
    torch = _torch()
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
