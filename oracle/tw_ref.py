"""Python side of the CPU oracle (TEST INFRASTRUCTURE ONLY, never on the product path).

* ``masked_gemm``      - ctypes call into ``tw_oracle.c`` (fp64 masked product, the definition).
* ``tile_structure``   - the TW format's integer side written out from the paper's description
                         (Sec. IV-A): column pruning first, surviving columns re-grouped G at a
                         time, each group keeping its own ascending list of K rows; a tile owns
                         the stretch of original columns up to the next tile's first column
                         (the "G+4, G+3, G+2, G-9" stretches of the worked example).
* ``masked_weight_bits`` - what pack -> unpack must give back: B where kept, +0 elsewhere.
* ``prune_one_shot``   - one stage of Alg. 1 (Sec. V) with the weight magnitude as importance score: columns
                         first, then row segments of the regrouped tiles ranked across all tiles.
* ``restore_ew``       - which pruned weights the TEW hybrid puts back (Sec. IV-A "Hybrid Pattern": prune
                         alpha + delta tile-wise, then restore the delta most important elements): ANY
                         pruned weight may come back, also one in a column the tile-wise pattern removed;
                         the weight magnitude is the importance; the hybrid's product is the masked product
                         over mask | ew_mask, which ``masked_gemm`` already defines.
* ``bias_act``         - the fused epilogue's definition: act(C + bias) in fp64 (bias addition and
                         activation are the operators the paper fuses around its GEMMs, Sec. VI
                         "Kernel Fusion"; GELU in its exact erf form, as in BERT), evaluated by
                         ``two_bias_act`` in tw_oracle.c with the C library's erf.

Nothing here imports the HIP package, and the HIP package imports nothing from here.
Parity status: every function is pinned by tests/test_oracle_pins.py and tests/test_tile_structure_pins.py
(``prune_one_shot`` and ``restore_ew`` by hand-worked cases written out in the tests).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Dict

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tw_oracle.c")
_LIB = os.path.join(_HERE, "libtw_oracle.so")
_DT = {"f16": 0, "bf16": 1}
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (no fast-math, no FMA contraction: the sum is the plain one)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        u16p = ctypes.POINTER(ctypes.c_uint16)
        lib.two_masked_gemm.restype = ctypes.c_int
        lib.two_masked_gemm.argtypes = [u16p, ctypes.c_long, u16p, ctypes.c_long,
                                        ctypes.POINTER(ctypes.c_uint8), ctypes.c_long, ctypes.c_long,
                                        ctypes.c_long, ctypes.c_int,
                                        ctypes.POINTER(ctypes.c_double), ctypes.c_long]
        lib.two_decode.restype = ctypes.c_int
        lib.two_decode.argtypes = [u16p, ctypes.c_long, ctypes.c_int, ctypes.POINTER(ctypes.c_double)]
        lib.two_num_threads.restype = ctypes.c_int
        lib.two_bias_act.restype = ctypes.c_int
        lib.two_bias_act.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.c_long, ctypes.c_long, ctypes.c_long,
                                     ctypes.POINTER(ctypes.c_double), ctypes.c_int]
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().two_num_threads())


def decode(bits: np.ndarray, dtype: str) -> np.ndarray:
    """16-bit patterns -> float64 through the oracle's own decoder."""
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    out = np.empty(b.shape, dtype=np.float64)
    rc = _load().two_decode(b.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16)), b.size, _DT[dtype],
                            out.ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
    if rc != 0:
        raise RuntimeError("two_decode failed")
    return out


def masked_gemm(A_bits: np.ndarray, B_bits: np.ndarray, mask: np.ndarray, dtype: str) -> np.ndarray:
    """C = A . (B * mask) in fp64 from 16-bit inputs.  A [M,K] (row stride may exceed K), B [K,N], mask [K,N]."""
    assert A_bits.dtype == np.uint16 and B_bits.dtype == np.uint16
    assert A_bits.ndim == 2 and B_bits.ndim == 2 and mask.shape == B_bits.shape
    assert A_bits.strides[1] == 2 and B_bits.strides[1] == 2
    M, K = A_bits.shape
    K2, N = B_bits.shape
    assert K == K2
    lda = A_bits.strides[0] // 2 if M > 1 else K
    ldb = B_bits.strides[0] // 2 if K > 1 else N
    mk = np.ascontiguousarray(mask, dtype=np.uint8)
    C = np.empty((M, N), dtype=np.float64)
    rc = _load().two_masked_gemm(
        A_bits.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16)), lda,
        B_bits.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16)), ldb,
        mk.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)), M, K, N, _DT[dtype],
        C.ctypes.data_as(ctypes.POINTER(ctypes.c_double)), N)
    if rc != 0:
        raise RuntimeError(f"two_masked_gemm failed: {rc}")
    return C


class NotTileWise(ValueError):
    pass


def tile_structure(mask: np.ndarray, G: int) -> Dict[str, np.ndarray]:
    """Integer description of a TW mask.

    1. A column survives iff it keeps at least one weight (column pruning comes first).
    2. Surviving columns, ascending, are swept left to right; a tile is closed when it holds G
       columns or when the next column keeps a different set of rows.
    3. Tile t keeps the ascending rows of that shared set; it owns original columns
       [span[t], span[t+1]) with span[0] = 0, span[t] = its first column, span[T] = N.
    4. More than 2*ceil(N/G) tiles means the mask is not tile-wise for this G.
    """
    mask = np.asarray(mask)
    K, N = mask.shape
    m = mask != 0
    col_idx = np.flatnonzero(m.any(axis=0)).astype(np.int32)
    tile_col_ptr = [0]
    rows = []
    i = 0
    while i < len(col_idx):
        pat = m[:, col_idx[i]]
        j = i + 1
        while j < len(col_idx) and j - i < G and np.array_equal(m[:, col_idx[j]], pat):
            j += 1
        rows.append(np.flatnonzero(pat).astype(np.int32))
        tile_col_ptr.append(j)
        i = j
    T = len(rows)
    if T > 2 * ((N + G - 1) // G):
        raise NotTileWise(f"{T} tiles for N={N}, G={G}")
    tile_row_ptr = np.zeros(T + 1, dtype=np.int32)
    for t, r in enumerate(rows):
        tile_row_ptr[t + 1] = tile_row_ptr[t] + len(r)
    span = np.zeros(T + 1, dtype=np.int32)
    for t in range(1, T):
        span[t] = col_idx[tile_col_ptr[t]]
    span[T] = N if T > 0 else 0
    return dict(
        K=K, N=N, G=G, T=T,
        col_idx=col_idx,
        tile_col_ptr=np.asarray(tile_col_ptr, dtype=np.int32),
        tile_row_ptr=tile_row_ptr,
        row_idx=(np.concatenate(rows).astype(np.int32) if rows else np.zeros(0, np.int32)),
        tile_span=span,
        nnz=int(m.sum()),
    )


def masked_weight_bits(B_bits: np.ndarray, mask: np.ndarray) -> np.ndarray:
    """B where the mask keeps it, the +0 pattern elsewhere."""
    return np.where(np.asarray(mask) != 0, B_bits, np.uint16(0)).astype(np.uint16)


def prune_one_shot(B_bits: np.ndarray, G: int, dtype: str, col_prune: float, sparsity: float) -> np.ndarray:
    """One stage of the paper's pruning algorithm (Sec. V, Alg. 1) with |w| as importance score, no apriori
    tuning, no fine-tuning: columns first (a column is a K x 1 tile, scored by the sum of its magnitudes; the
    floor(p*N + 0.5) lowest go, lower index first among equals), then the surviving columns are regrouped
    G at a time and row segments (1 x G tiles, scored by their mean magnitude) are pruned across all tiles
    in ascending score until zeros / (K*N) >= sparsity; a tile keeps at least one row.
    Written out with plain loops over rows and columns; scores accumulate in float64 in index order."""
    K, N = B_bits.shape
    absB = np.abs(decode(B_bits, dtype))
    cscore = np.zeros(N, dtype=np.float64)
    for k in range(K):
        cscore += absB[k]
    n_prune = int(np.floor(col_prune * N + 0.5))
    order = sorted(range(N), key=lambda n: (cscore[n], n))
    pruned = set(order[:n_prune])
    cols = [n for n in range(N) if n not in pruned]
    mask = np.zeros((K, N), dtype=np.uint8)
    if not cols:
        return mask
    tiles = [cols[i:i + G] for i in range(0, len(cols), G)]
    segs = []                                   # (score, tile, row, width)
    for t, tc in enumerate(tiles):
        acc = np.zeros(K, dtype=np.float64)
        for n in tc:
            acc += absB[:, n]
        sc = acc / len(tc)
        for k in range(K):
            segs.append((float(sc[k]), t, k, len(tc)))
    segs.sort(key=lambda x: (x[0], x[1], x[2]))
    want = int(np.ceil(sparsity * float(K * N)))
    zeros = K * (N - len(cols))
    left = [K] * len(tiles)
    drop = set()
    for sc, t, k, w in segs:
        if zeros >= want:
            break
        if left[t] <= 1:
            continue
        drop.add((t, k))
        left[t] -= 1
        zeros += w
    for t, tc in enumerate(tiles):
        for k in range(K):
            if (t, k) not in drop:
                mask[k, tc] = 1
    return mask


def bias_act(C: np.ndarray, bias64, act: str = "none") -> np.ndarray:
    """act(C + bias), fp64.  C: [M, N] fp64 (the masked product), bias64: [N] fp64 or None.
    relu(x) = max(x, 0); gelu(x) = x/2 * (1 + erf(x / sqrt 2)) = x * Phi(x) (the exact form)."""
    codes = {None: 0, "none": 0, "relu": 1, "gelu": 2}
    if act not in codes:
        raise ValueError(f"unknown activation {act!r}")
    x = np.array(C, dtype=np.float64, order="C", copy=True)
    assert x.ndim == 2
    M, N = x.shape
    b = None
    if bias64 is not None:
        b = np.ascontiguousarray(bias64, dtype=np.float64)
        assert b.shape == (N,)
    if M == 0:
        return x
    dp = ctypes.POINTER(ctypes.c_double)
    rc = _load().two_bias_act(x.ctypes.data_as(dp), M, N, N, b.ctypes.data_as(dp) if b is not None else None,
                              codes[act])
    if rc != 0:
        raise RuntimeError(f"two_bias_act failed: {rc}")
    return x


def restore_ew(B_bits: np.ndarray, mask: np.ndarray, delta: float, dtype: str) -> np.ndarray:
    """uint8 [K, N]: the floor(delta*K*N + 0.5) weights of largest magnitude among ALL weights that `mask`
    prunes (Sec. IV-A "Hybrid Pattern" restores the most important pruned elements, wherever they lie: also in
    columns that the tile-wise pattern removed altogether); ties go to the lower (k, n) (row-major position)."""
    K, N = mask.shape
    mag = np.abs(decode(B_bits, dtype))
    cand = [(-mag[k, n], k * N + n) for k in range(K) for n in range(N) if not mask[k, n]]
    cand.sort()
    want = min(len(cand), int(np.floor(delta * K * N + 0.5)))
    out = np.zeros((K, N), dtype=np.uint8)
    for _, pos in cand[:want]:
        out[pos // N, pos % N] = 1
    return out
