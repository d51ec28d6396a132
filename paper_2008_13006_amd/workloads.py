"""Seeded synthetic inputs for the tile-wise (TW) sparse GEMM: activations A, weights B
and TW-structured masks with the GEMM shapes of BERT-base, BERT-large and an im2col
3x3 convolution.

This module only *draws inputs*.  It holds none of the GEMM's arithmetic and is the one
piece of code that both the CPU oracle's tests and the HIP path's tests/bench consume.
It imports neither of them.

The masks stand in for what the paper's pruning algorithm (Alg. 1) produces on trained
models: whole columns are pruned first, the surviving columns are re-grouped G at a
time (Sec. IV-A, "Pruning Order"), and each group then keeps its own subset of the K
rows.  The importance score is the magnitude score the paper calls the most intuitive
one (Sec. V, "Importance Score"): the L1 norm of a column, resp. of a 1xG row segment.
Uneven per-tile keep counts imitate the uneven sparsity that global ranking produces
(Sec. IV-B, "Against VW").

All values are rounded once to the 16-bit storage type and handed out as raw uint16 bit
patterns, so every consumer sees the same bits.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Tuple

import numpy as np

F16 = "f16"
BF16 = "bf16"
BASE_SEED = 20200813


# --------------------------------------------------------------------------- bits
def f32_to_bits(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round float32 values to fp16/bf16 (round-to-nearest-even), return uint16 bits."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == F16:
        return x.astype(np.float16).view(np.uint16)
    if dtype == BF16:
        u = x.view(np.uint32)
        r = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
        return (r >> np.uint32(16)).astype(np.uint16)
    raise ValueError(dtype)


def bits_to_f32(b: np.ndarray, dtype: str) -> np.ndarray:
    """Exact widening of fp16/bf16 bit patterns to float32 (for scoring and for tests)."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    if dtype == F16:
        return b.view(np.float16).astype(np.float32)
    if dtype == BF16:
        return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)
    raise ValueError(dtype)


# --------------------------------------------------------------------------- specs
@dataclass(frozen=True)
class GemmSpec:
    """One weight GEMM C[M,N] = A[M,K] . (B[K,N] * mask)."""
    name: str
    M: int
    K: int
    N: int
    dtype: str = F16
    G: int = 128
    a_dist: str = "normal"          # "normal" | "relu_normal" | "smallint"
    b_sigma: float = 0.02
    col_prune: float = 0.0          # fraction of whole columns pruned first
    keep: Tuple = ("const", 0.5)    # ("const", f) | ("upow", lo, hi) | ("zipf", lo, hi, s)
    sparsity: Optional[float] = None  # overall target (zeros / (K*N)); None = whatever keep gives
    seed_offset: int = 0
    grid: str = "regrouped"         # "regrouped": tiles of G SURVIVING columns | "fixed": the survivors of every
                                    # block of G original columns form a tile (the other description in Sec. IV-A)


def _bert_base(M: int) -> List[GemmSpec]:
    kw = dict(M=M, dtype=F16, G=128, col_prune=0.05, keep=("upow", 0.10, 0.50), sparsity=0.75)
    return [
        GemmSpec(name="qkv_768x2304", K=768, N=2304, seed_offset=0, **kw),
        GemmSpec(name="attn_out_768x768", K=768, N=768, seed_offset=100, **kw),
        GemmSpec(name="ffn_up_768x3072", K=768, N=3072, seed_offset=200, **kw),
        GemmSpec(name="ffn_down_3072x768", K=3072, N=768, seed_offset=300, **kw),
    ]


CONFIGS: Dict[str, List[GemmSpec]] = {
    # single small GEMM, every tile keeps the top half of its rows, no column pruning
    "c1_single": [GemmSpec(name="single_256x768x768", M=256, K=768, N=768, dtype=F16, G=128,
                           col_prune=0.0, keep=("const", 0.5), sparsity=None, seed_offset=1000)],
    # BERT-base FFN-up, 75 % overall, tiles between 10 % and 50 % kept, 5 % of columns gone
    "c2_bert_base_ffn_up": [GemmSpec(name="ffn_up_768x3072", M=16384, K=768, N=3072, dtype=F16,
                                     G=128, col_prune=0.05, keep=("upow", 0.10, 0.50),
                                     sparsity=0.75, seed_offset=2000)],
    # the four weight GEMMs of one BERT-base encoder layer (QKV fused)
    "c3_bert_base_layer": [GemmSpec(**{**s.__dict__, "seed_offset": 3000 + s.seed_offset})
                           for s in _bert_base(16384)],
    # BERT-large FFN pair, bf16, Zipf(1.2)-skewed tiles from 2 % to 60 % kept, 10 % columns gone
    "c4_bert_large_skewed": [
        GemmSpec(name="ffn_up_1024x4096", M=8192, K=1024, N=4096, dtype=BF16, G=128,
                 col_prune=0.10, keep=("zipf", 0.02, 0.60, 1.2), sparsity=0.875, seed_offset=4000),
        GemmSpec(name="ffn_down_4096x1024", M=8192, K=4096, N=1024, dtype=BF16, G=128,
                 col_prune=0.10, keep=("zipf", 0.02, 0.60, 1.2), sparsity=0.875, seed_offset=4100),
    ],
    # 3x3 conv 256->256 on a 56x56 map, batch 32, lowered with im2col; activations post-ReLU
    "c5_conv_im2col": [GemmSpec(name="conv3x3_256_56x56_b32", M=32 * 56 * 56, K=3 * 3 * 256, N=256,
                                dtype=F16, G=64, a_dist="relu_normal", b_sigma=0.05, col_prune=0.0,
                                keep=("upow", 0.10, 0.50), sparsity=0.75, seed_offset=5000)],
}


@dataclass
class Workload:
    spec: GemmSpec
    A: Optional[np.ndarray]     # uint16 [M, K] bit patterns (None when not requested)
    B: np.ndarray               # uint16 [K, N]
    mask: np.ndarray            # uint8  [K, N], 1 = kept
    info: dict = field(default_factory=dict)


# --------------------------------------------------------------------------- masks
def _keep_fractions(kind: Tuple, widths: np.ndarray, K: int, N: int, target_sparsity, rng) -> np.ndarray:
    """Per-tile kept-row fractions.  With a target, the exponent gamma of f = lo + (hi-lo)*u**gamma
    is found by bisection so that sum_t w_t*round(f_t*K) / (K*N) hits 1 - target."""
    T = len(widths)
    if kind[0] == "const":
        return np.full(T, float(kind[1]))
    lo, hi = float(kind[1]), float(kind[2])
    if kind[0] == "upow":
        u = rng.random(T)
        if T > 1:
            u = (u - u.min()) / (u.max() - u.min())      # force the end points 0 and 1
        else:
            u = np.array([0.5])
    elif kind[0] == "zipf":
        s = float(kind[3])
        ranks = rng.permutation(T) + 1                    # random rank 1..T for every tile
        z = ranks.astype(np.float64) ** (-s)
        zT, z1 = float(T) ** (-s), 1.0
        u = (z - zT) / (z1 - zT) if T > 1 else np.array([0.5])
    else:
        raise ValueError(kind)
    if target_sparsity is None:
        return lo + (hi - lo) * u

    want = 1.0 - float(target_sparsity)

    def density(gamma: float) -> float:
        with np.errstate(divide="ignore"):
            f = lo + (hi - lo) * np.where(u > 0, u ** gamma, 0.0)
        kt = np.maximum(1, np.floor(f * K + 0.5))
        return float((widths * kt).sum()) / (K * N)

    g_lo, g_hi = 1e-3, 1e3                                # density falls as gamma grows
    if density(g_lo) < want or density(g_hi) > want:
        raise ValueError("target sparsity not reachable with these keep bounds")
    for _ in range(200):
        g = (g_lo * g_hi) ** 0.5
        if density(g) > want:
            g_lo = g
        else:
            g_hi = g
    g = (g_lo * g_hi) ** 0.5
    return lo + (hi - lo) * np.where(u > 0, u ** g, 0.0)


def tw_mask_from_scores(absB: np.ndarray, G: int, col_prune: float, keep: Tuple,
                        target_sparsity, rng, grid: str = "regrouped") -> Tuple[np.ndarray, dict]:
    """Column pruning, re-grouping, then per-group row pruning (Sec. IV-A), with L1 scores.

    absB: float64 |B| of the already rounded weights.  Ties: the smaller index is the more
    important one when keeping, and the first one to go when pruning columns."""
    K, N = absB.shape
    n_prune = int(np.floor(col_prune * N + 0.5))
    col_score = absB.sum(axis=0)
    order = np.argsort(col_score, kind="stable")          # ascending, ties -> smaller n first
    pruned_cols = np.sort(order[:n_prune])
    kept_cols = np.setdiff1d(np.arange(N), pruned_cols)
    if grid == "fixed":
        groups = [kept_cols[(kept_cols >= t * G) & (kept_cols < (t + 1) * G)] for t in range((N + G - 1) // G)]
        groups = [g for g in groups if len(g)]
    else:
        groups = [kept_cols[t * G:(t + 1) * G] for t in range((len(kept_cols) + G - 1) // G)]
    T = len(groups)
    widths = np.array([len(g) for g in groups], dtype=np.float64)
    f = _keep_fractions(keep, widths, K, N, target_sparsity, rng)
    mask = np.zeros((K, N), dtype=np.uint8)
    k_t = []
    for t, cols in enumerate(groups):
        kt = int(max(1, np.floor(f[t] * K + 0.5)))
        kt = min(kt, K)
        seg = absB[:, cols].sum(axis=1)
        top = np.argsort(-seg, kind="stable")[:kt]        # descending, ties -> smaller k
        rows = np.sort(top)
        mask[np.ix_(rows, cols)] = 1
        k_t.append(kt)
    info = dict(T=T, k_t=k_t, widths=[int(w) for w in widths], n_pruned_cols=n_prune,
                sparsity=1.0 - float(mask.sum()) / (K * N))
    return mask, info


# --------------------------------------------------------------------------- draw
def generate(spec: GemmSpec, with_A: bool = True, M: Optional[int] = None) -> Workload:
    """Draw A, then B, then the mask's random numbers, from PCG64(BASE_SEED + seed_offset).

    M overrides the row count (the first M rows of the full A are what is returned, the
    stream of draws for B and the mask does not depend on it)."""
    rng = np.random.Generator(np.random.PCG64(BASE_SEED + spec.seed_offset))
    rows = spec.M if M is None else int(M)
    A_bits = None
    # A is drawn in row blocks so the float32 temporary stays small; the full-size stream
    # is always consumed so that B and the mask do not change with `M` or `with_A`.
    blk = 8192
    if with_A:
        A_bits = np.empty((rows, spec.K), dtype=np.uint16)
    for r0 in range(0, spec.M, blk):
        r1 = min(spec.M, r0 + blk)
        if spec.a_dist == "smallint":
            a = rng.integers(-3, 4, size=(r1 - r0, spec.K)).astype(np.float32)
        else:
            a = rng.standard_normal((r1 - r0, spec.K), dtype=np.float32)
            if spec.a_dist == "relu_normal":
                np.maximum(a, 0.0, out=a)
        if with_A and r0 < rows:
            e = min(r1, rows)
            A_bits[r0:e] = f32_to_bits(a[: e - r0], spec.dtype)
    if spec.a_dist == "smallint":
        b = rng.integers(-2, 3, size=(spec.K, spec.N)).astype(np.float32)
    else:
        b = rng.standard_normal((spec.K, spec.N), dtype=np.float32) * np.float32(spec.b_sigma)
    B_bits = f32_to_bits(b, spec.dtype)
    absB = np.abs(bits_to_f32(B_bits, spec.dtype).astype(np.float64))
    if spec.a_dist == "smallint":
        # break the many ties of integer weights deterministically without touching B itself
        absB = absB + 1e-3 * rng.random(absB.shape)
    mask, info = tw_mask_from_scores(absB, spec.G, spec.col_prune, spec.keep, spec.sparsity, rng, spec.grid)
    info.update(seed=BASE_SEED + spec.seed_offset, M=rows, K=spec.K, N=spec.N, G=spec.G,
                dtype=spec.dtype, name=spec.name)
    return Workload(spec=spec, A=A_bits, B=B_bits, mask=mask, info=info)


def small_spec(name: str, M: int, K: int, N: int, G: int, dtype: str = F16, col_prune: float = 0.0,
               keep: Tuple = ("upow", 0.10, 0.60), sparsity=None, seed_offset: int = 9000,
               a_dist: str = "normal", b_sigma: float = 0.02) -> GemmSpec:
    """Convenience for tests: an arbitrary small TW GEMM drawn with the same recipe."""
    return GemmSpec(name=name, M=M, K=K, N=N, dtype=dtype, G=G, a_dist=a_dist, b_sigma=b_sigma,
                    col_prune=col_prune, keep=keep, sparsity=sparsity, seed_offset=seed_offset)


def sweep_spec(G: int, sparsity: float, M: int = 16384, K: int = 768, N: int = 3072, dtype: str = F16) -> GemmSpec:
    """Sparsity x granularity sweep on the BERT-base FFN-up shape (the experiment of Sec. VII-B, Fig. 8b and
    Fig. 10, on synthetic masks): 5 % of the columns pruned (none at 0 % sparsity), per-tile keep
    fractions spread between 0.4x and 1.9x of the mean, bisected onto the target."""
    if sparsity <= 0.0:
        return GemmSpec(name=f"sweep_G{G}_s0", M=M, K=K, N=N, dtype=dtype, G=G, col_prune=0.0,
                        keep=("const", 1.0), seed_offset=7000 + G)
    cp = min(0.05, sparsity / 2)
    f = (1.0 - sparsity) / (1.0 - cp)
    lo, hi = max(0.4 * f, 1.0 / K), min(1.9 * f, 1.0)
    return GemmSpec(name=f"sweep_G{G}_s{int(round(sparsity * 1000))}", M=M, K=K, N=N, dtype=dtype, G=G,
                    col_prune=cp, keep=("upow", lo, hi), sparsity=sparsity,
                    seed_offset=7000 + G + int(round(sparsity * 1000)))


# The headline workload under the other description of the pattern in Sec. IV-A: B is cut into tiles of G original
# columns first and every tile prunes columns and rows of its own, so a tile's span is a whole number of 128-byte
# lines of C.  Reported next to the five workloads, not one of them.
C2_FIXED_GRID = GemmSpec(name="ffn_up_768x3072_fixed_grid", M=16384, K=768, N=3072, dtype=F16, G=128, col_prune=0.05,
                         keep=("upow", 0.10, 0.50), sparsity=0.75, seed_offset=2000, grid="fixed")


def nonzero_flops(mask: np.ndarray, M: int) -> int:
    """2*M*(number of kept weights): the work the TW method itself has to do."""
    return 2 * int(M) * int(mask.sum(dtype=np.int64))
