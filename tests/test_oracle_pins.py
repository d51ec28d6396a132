"""Pins for the CPU oracle's masked GEMM (oracle/tw_oracle.c): none of them re-types the
oracle's loop.  They fix it against library routines on special cases, closed forms with exact
integer answers, selector inputs that expose a wrong index or a transposed operand, and the
paper's own statements (TW product = union of small dense GEMMs; linearity used for TEW)."""
import numpy as np
import pytest
import torch

from oracle import tw_ref
from paper_2008_13006_amd import workloads as W


def _f64(bits, dtype):
    """Independent widening: numpy's float16 / torch's bfloat16, not the oracle's decoder."""
    if dtype == "f16":
        return bits.view(np.float16).astype(np.float64)
    t = torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16)
    return t.to(torch.float64).numpy()


def test_decode_every_f16_pattern_matches_numpy():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    got = tw_ref.decode(bits, "f16")
    want = bits.view(np.float16).astype(np.float64)
    assert np.array_equal(np.isnan(got), np.isnan(want))
    ok = ~np.isnan(want)
    assert np.array_equal(got[ok], want[ok])
    assert np.array_equal(np.signbit(got[ok]), np.signbit(want[ok]))


def test_decode_every_bf16_pattern_matches_torch():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    got = tw_ref.decode(bits, "bf16")
    want = _f64(bits, "bf16")
    assert np.array_equal(np.isnan(got), np.isnan(want))
    ok = ~np.isnan(want)
    assert np.array_equal(got[ok], want[ok])
    assert np.array_equal(np.signbit(got[ok]), np.signbit(want[ok]))


def test_decode_known_values():
    # textbook constants: 1.0, -2.0, smallest f16 subnormal 2^-24, max f16 65504, bf16 1.0 and pi-ish 3.140625
    assert tw_ref.decode(np.array([0x3C00, 0xC000, 0x0001, 0x7BFF], np.uint16), "f16").tolist() == \
        [1.0, -2.0, 2.0 ** -24, 65504.0]
    assert tw_ref.decode(np.array([0x3F80, 0x4049, 0x0001], np.uint16), "bf16").tolist() == \
        [1.0, 3.140625, 2.0 ** -133]


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_dense_special_case_equals_blas_dgemm(dtype):
    """0 % sparsity: the masked product is the ordinary product (library routine special case)."""
    rng = np.random.default_rng(1)
    M, K, N = 37, 53, 29                               # all different: a transposed operand cannot pass
    A = W.f32_to_bits(rng.standard_normal((M, K), dtype=np.float32), dtype)
    B = W.f32_to_bits(rng.standard_normal((K, N), dtype=np.float32), dtype)
    C = tw_ref.masked_gemm(A, B, np.ones((K, N), np.uint8), dtype)
    ref = _f64(A, dtype) @ _f64(B, dtype)
    assert np.max(np.abs(C - ref)) <= 1e-13 * np.max(np.abs(ref))


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_masked_equals_dgemm_on_zeroed_weights(dtype):
    """Skipping a weight and multiplying by an explicit zero give the same sum for finite inputs."""
    rng = np.random.default_rng(2)
    M, K, N = 19, 64, 48
    A = W.f32_to_bits(rng.standard_normal((M, K), dtype=np.float32), dtype)
    B = W.f32_to_bits(rng.standard_normal((K, N), dtype=np.float32), dtype)
    mask = (rng.random((K, N)) < 0.3).astype(np.uint8)   # even an unstructured mask: the oracle knows no tiles
    C = tw_ref.masked_gemm(A, B, mask, dtype)
    ref = _f64(A, dtype) @ (_f64(B, dtype) * mask)
    assert np.max(np.abs(C - ref)) <= 1e-13 * np.max(np.abs(ref))


def test_all_ones_counts_kept_weights_exactly():
    """A = 1, B = 1: C[m,n] is the number of kept weights in column n (closed form, exact)."""
    rng = np.random.default_rng(3)
    M, K, N = 5, 40, 33
    one = np.uint16(0x3C00)
    mask = (rng.random((K, N)) < 0.5).astype(np.uint8)
    mask[:, 7] = 0
    C = tw_ref.masked_gemm(np.full((M, K), one), np.full((K, N), one), mask, "f16")
    assert np.array_equal(C, np.tile(mask.sum(axis=0).astype(np.float64), (M, 1)))
    assert np.all(C[:, 7] == 0.0) and not np.any(np.signbit(C[:, 7]))


def test_selector_rows_pick_single_weights():
    """A = rows of the identity (M = K): C must be B where kept and 0 elsewhere - any index
    mix-up (k vs n, m vs k) or a transposed B shows up as a wrong element."""
    rng = np.random.default_rng(4)
    K, N = 24, 17
    A = W.f32_to_bits(np.eye(K, dtype=np.float32), "f16")
    Bf = rng.integers(-8, 9, size=(K, N)).astype(np.float32)
    B = W.f32_to_bits(Bf, "f16")
    mask = (rng.random((K, N)) < 0.6).astype(np.uint8)
    C = tw_ref.masked_gemm(A, B, mask, "f16")
    assert np.array_equal(C, Bf.astype(np.float64) * mask)


def test_weighted_row_sum_closed_form():
    """A[m,k] = (m+1), B[k,n] = (k+1) on a mask keeping rows k < n+1 of column n:
    C[m,n] = (m+1) * (n+1)(n+2)/2, exact in double."""
    M, K, N = 6, 12, 12
    A = W.f32_to_bits(np.tile(np.arange(1, M + 1, dtype=np.float32)[:, None], (1, K)), "f16")
    B = W.f32_to_bits(np.tile(np.arange(1, K + 1, dtype=np.float32)[:, None], (1, N)), "f16")
    mask = (np.arange(K)[:, None] <= np.arange(N)[None, :]).astype(np.uint8)
    C = tw_ref.masked_gemm(A, B, mask, "f16")
    n = np.arange(N, dtype=np.float64)
    want = np.arange(1, M + 1, dtype=np.float64)[:, None] * ((n + 1) * (n + 2) / 2)[None, :]
    assert np.array_equal(C, want)


def test_row_strides_are_honoured():
    rng = np.random.default_rng(5)
    M, K, N = 9, 16, 11
    Abig = W.f32_to_bits(rng.standard_normal((M, K + 5), dtype=np.float32), "f16")
    Bbig = W.f32_to_bits(rng.standard_normal((K, N + 3), dtype=np.float32), "f16")
    mask = (rng.random((K, N)) < 0.5).astype(np.uint8)
    C = tw_ref.masked_gemm(Abig[:, :K], Bbig[:, :N], mask, "f16")
    ref = _f64(np.ascontiguousarray(Abig[:, :K]), "f16") @ (_f64(np.ascontiguousarray(Bbig[:, :N]), "f16") * mask)
    assert np.max(np.abs(C - ref)) <= 1e-13 * np.max(np.abs(ref))


def test_tile_wise_product_is_union_of_small_dense_gemms():
    """Sec. IV-A / Fig. 4 step 4 and Sec. VI: on a TW mask every tile is a dense GEMM over the
    tile's kept rows and columns; pruned columns are exactly zero."""
    spec = W.small_spec("pin_tiles", M=23, K=96, N=200, G=32, col_prune=0.1, keep=("upow", 0.1, 0.7))
    w = W.generate(spec)
    C = tw_ref.masked_gemm(w.A, w.B, w.mask, "f16")
    A64, B64 = _f64(w.A, "f16"), _f64(w.B, "f16")
    kept_cols = np.flatnonzero(w.mask.any(axis=0))
    assert len(kept_cols) == 200 - 20
    for t in range(0, len(kept_cols), 32):
        cols = kept_cols[t:t + 32]
        rows = np.flatnonzero(w.mask[:, cols[0]])
        assert all(np.array_equal(np.flatnonzero(w.mask[:, c]), rows) for c in cols)
        small = A64[:, rows] @ B64[np.ix_(rows, cols)]
        assert np.max(np.abs(C[:, cols] - small)) <= 1e-13 * np.max(np.abs(small))
    pruned = np.setdiff1d(np.arange(200), kept_cols)
    assert np.all(C[:, pruned] == 0.0)


def test_linearity_over_disjoint_masks():
    """Sec. IV-A, last paragraph: the product is linear in the weight, so two disjoint masks add up."""
    rng = np.random.default_rng(6)
    M, K, N = 8, 32, 24
    A = W.f32_to_bits(rng.integers(-4, 5, size=(M, K)).astype(np.float32), "f16")
    B = W.f32_to_bits(rng.integers(-4, 5, size=(K, N)).astype(np.float32), "f16")
    m1 = (rng.random((K, N)) < 0.4).astype(np.uint8)
    m2 = ((rng.random((K, N)) < 0.5) & (m1 == 0)).astype(np.uint8)
    C1 = tw_ref.masked_gemm(A, B, m1, "f16")
    C2 = tw_ref.masked_gemm(A, B, m2, "f16")
    C12 = tw_ref.masked_gemm(A, B, m1 | m2, "f16")
    assert np.array_equal(C1 + C2, C12)                 # integers: exact


def test_brute_force_tiny_with_python_integers():
    """2 x 3 x 2 by hand: A = [[1,2,3],[4,5,6]], B = [[1,-1],[2,0],[3,5]], mask = [[1,0],[0,1],[1,1]].
    C = [[1*1+3*3, 2*0+3*5], [4*1+6*3, 5*0+6*5]] = [[10,15],[22,30]]."""
    A = W.f32_to_bits(np.array([[1, 2, 3], [4, 5, 6]], np.float32), "bf16")
    B = W.f32_to_bits(np.array([[1, -1], [2, 0], [3, 5]], np.float32), "bf16")
    mask = np.array([[1, 0], [0, 1], [1, 1]], np.uint8)
    assert tw_ref.masked_gemm(A, B, mask, "bf16").tolist() == [[10.0, 15.0], [22.0, 30.0]]


def test_bad_arguments_are_rejected():
    A = np.zeros((2, 4), np.uint16)
    B = np.zeros((4, 3), np.uint16)
    with pytest.raises(AssertionError):
        tw_ref.masked_gemm(A, B, np.zeros((3, 4), np.uint8), "f16")


# ------------------------------------------------------------------ fused epilogue definition
def test_bias_act_pins():
    """bias_act against closed forms: gelu(x) = x * Phi(x) with Phi the standard normal CDF
    (Phi(1) = 0.8413447460685429..., a table value), gelu(x) - gelu(-x) = x, relu, bias broadcast
    along rows, and a pruned column (C = 0) holding act(bias)."""
    import math
    x = np.array([[-3.0, -1.0, -0.5, 0.0, 0.5, 1.0, 3.0]])
    g = tw_ref.bias_act(x, None, "gelu")
    assert abs(g[0, 5] - 0.8413447460685429) < 1e-15
    assert g[0, 3] == 0.0
    assert np.allclose(g - tw_ref.bias_act(-x, None, "gelu"), x, rtol=0, atol=1e-15)
    phi = np.array([0.5 * (1.0 + math.erf(v / math.sqrt(2.0))) for v in x[0]])
    assert np.allclose(g[0], x[0] * phi, rtol=0, atol=1e-15)
    assert np.array_equal(tw_ref.bias_act(x, None, "relu"), np.maximum(x, 0.0))
    assert np.array_equal(tw_ref.bias_act(x, None, "none"), x)
    C = np.zeros((3, 4)); C[:, 1] = [1.0, -2.0, 0.25]
    b = np.array([0.5, -0.5, 2.0, -1.0])
    out = tw_ref.bias_act(C, b, "relu")
    assert np.array_equal(out[:, 0], [0.5, 0.5, 0.5]) and np.array_equal(out[:, 3], [0.0, 0.0, 0.0])
    assert np.array_equal(out[:, 1], [0.5, 0.0, 0.0])
    # a dropped bias or a bias added along the wrong axis fails the line above; a tanh-form GELU fails Phi(1)
    with pytest.raises(ValueError):
        tw_ref.bias_act(x, None, "swish")


# ------------------------------------------------------------------ one-shot pruning (Alg. 1, one stage, magnitude score)
# Hand-worked case.  K = 3, N = 6, G = 2.  Magnitudes |B| (B[2,1] is negative: the score is the magnitude):
#         n=0  1  2  3  4  5
#   k=0    1   4  1  2  8  3
#   k=1    2   5  1  6  1  3
#   k=2    3   6  4  1  3  4
# Column stage, one column to prune (floor(6/6 + 0.5) = 1): column sums 6, 15, 6, 9, 12, 10; columns 0 and 2 tie
# for the lowest score and the lower index goes: column 0.  Survivors 1..5 regroup as t0 = {1,2}, t1 = {3,4},
# t2 = {5} (the narrower last tile).  Row-segment scores = MEAN magnitude over the tile's columns:
#   t0: 2.5, 3, 5     t1: 5, 3.5, 2     t2: 3, 3, 4
# ascending, ties by (tile, row): (t1,k2) 2, (t0,k0) 2.5, (t0,k1) 3, (t2,k0) 3, (t2,k1) 3, (t1,k1) 3.5, (t2,k2) 4,
# (t0,k2) 5, (t1,k0) 5.  Zeros start at 3 (the pruned column) of K*N = 18.
_PRUNE_B = np.array([[1, 4, 1, 2, 8, 3], [2, 5, 1, 6, 1, 3], [3, -6, 4, 1, 3, 4]], np.float32)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_prune_one_shot_hand_worked_half(dtype):
    """Target 0.5: 9 zeros wanted.  (t1,k2) -> 5 zeros, (t0,k0) -> 7, (t0,k1) -> 9: stop.  t2 is untouched, which a
    SUM score would not give (t2's sums 3, 3, 4 are the lowest of all), and (t0,k1) goes before the equally scored
    (t2,k0), (t2,k1), which a tie order by row first or by descending tile would not give."""
    B = W.f32_to_bits(_PRUNE_B, dtype)
    want = np.array([[0, 0, 0, 1, 1, 1],
                     [0, 0, 0, 1, 1, 1],
                     [0, 1, 1, 0, 0, 1]], np.uint8)
    assert np.array_equal(tw_ref.prune_one_shot(B, 2, dtype, 1.0 / 6.0, 0.5), want)


def test_prune_one_shot_hand_worked_keep_one_row():
    """Target 0.75: 14 zeros wanted, which cannot be reached.  After the three segments above: (t2,k0) -> 10,
    (t2,k1) -> 11 and t2 is down to one row; (t1,k1) -> 13 and t1 is down to one row; (t2,k2), (t0,k2), (t1,k0) are
    the last rows of their tiles and stay.  Every tile keeps exactly its most important row."""
    B = W.f32_to_bits(_PRUNE_B, "f16")
    want = np.array([[0, 0, 0, 1, 1, 0],
                     [0, 0, 0, 0, 0, 0],
                     [0, 1, 1, 0, 0, 1]], np.uint8)
    assert np.array_equal(tw_ref.prune_one_shot(B, 2, "f16", 1.0 / 6.0, 0.75), want)


def test_prune_one_shot_degenerate_targets():
    B = W.f32_to_bits(_PRUNE_B, "f16")
    assert np.array_equal(tw_ref.prune_one_shot(B, 2, "f16", 0.0, 0.0), np.ones((3, 6), np.uint8))
    # whole-matrix granularity: one tile, rows ranked by their mean magnitude: 19/6, 18/6, 21/6 -> k1 goes first
    m = tw_ref.prune_one_shot(B, 6, "f16", 0.0, 1.0 / 3.0)
    assert np.array_equal(m, np.array([[1] * 6, [0] * 6, [1] * 6], np.uint8))


def test_prune_one_shot_properties():
    """What Alg. 1 states, checked on the oracle's own output: whole columns go first (the least important ones),
    then whole row segments of the regrouped tiles; the target is met with less than one segment to spare;
    every tile keeps a row."""
    rng = np.random.default_rng(777)
    K, N, G = 96, 260, 64
    B = W.f32_to_bits((rng.standard_normal((K, N)) * 0.05).astype(np.float32), "f16")
    mask = tw_ref.prune_one_shot(B, G, "f16", 0.1, 0.75)
    kept_cols = np.flatnonzero(mask.any(axis=0))
    assert N - len(kept_cols) == int(np.floor(0.1 * N + 0.5))
    cs = np.abs(B.view(np.float16).astype(np.float64)).sum(axis=0)
    assert cs[kept_cols].min() >= np.delete(cs, kept_cols).max()
    zeros = mask.size - int(mask.sum())
    assert zeros >= 0.75 * mask.size and zeros - G < 0.75 * mask.size
    kts = []
    for i in range(0, len(kept_cols), G):
        seg = mask[:, kept_cols[i:i + G]]
        assert np.all((seg.sum(axis=1) == 0) | (seg.sum(axis=1) == seg.shape[1]))
        assert seg.any()
        kts.append(int(seg.any(axis=1).sum()))
    assert len(set(kts)) > 1                      # ranking across tiles: tiles end up with different heights
    s = tw_ref.tile_structure(mask, G)
    assert s["T"] <= -(-len(kept_cols) // G) + 1


# ------------------------------------------------------------------ TEW: which pruned weights come back
# Hand-worked case.  K = 4, N = 6; the tile-wise pattern (G = 3) keeps rows {0,1} of columns 0..2, prunes column 3
# altogether and keeps rows {2,3} of columns 4..5:
#         n=0  1  2  3  4  5                 mask
#   k=0    1  -9  2  7  3  1              1 1 1 0 0 0
#   k=1    5   2 -8  7  1  2              1 1 1 0 0 0
#   k=2   -3   4  6 -7  2  3              0 0 0 0 1 1
#   k=3    2   1  5  1  8  4              0 0 0 0 1 1
# Pruned weights by magnitude: 7 at (0,3), (1,3), (2,3) (a three-way tie, all in the pruned column), 6 at (2,2),
# 5 at (3,2), 4 at (2,1), 3 at (2,0) and (0,4), ...
_TEW_B = np.array([[1, -9, 2, 7, 3, 1], [5, 2, -8, 7, 1, 2], [-3, 4, 6, -7, 2, 3], [2, 1, 5, 1, 8, 4]], np.float32)
_TEW_MASK = np.array([[1, 1, 1, 0, 0, 0], [1, 1, 1, 0, 0, 0], [0, 0, 0, 0, 1, 1], [0, 0, 0, 0, 1, 1]], np.uint8)


@pytest.mark.parametrize("n_restore,want_pos", [
    (2, [(0, 3), (1, 3)]),                                   # the tie goes to the lower (k, n)
    (4, [(0, 3), (1, 3), (2, 3), (2, 2)]),
    (5, [(0, 3), (1, 3), (2, 3), (2, 2), (3, 2)]),
    (8, [(0, 3), (1, 3), (2, 3), (2, 2), (3, 2), (2, 1), (2, 0), (0, 4)]),   # both weights of magnitude 3
])
def test_restore_ew_hand_worked(n_restore, want_pos):
    """The most important pruned elements come back wherever they lie: here the first three are in the column
    that the tile-wise pattern pruned altogether."""
    B = W.f32_to_bits(_TEW_B, "f16")
    got = tw_ref.restore_ew(B, _TEW_MASK, n_restore / 24.0, "f16")
    want = np.zeros((4, 6), np.uint8)
    for k, n in want_pos:
        want[k, n] = 1
    assert np.array_equal(got, want)
    assert not np.any(got & _TEW_MASK)


def test_restore_ew_tie_order_is_row_major():
    """Seven restored weights: 7,7,7,6,5,4 and ONE of the two 3s - the one at the lower row-major position, (0,4)."""
    B = W.f32_to_bits(_TEW_B, "bf16")
    got = tw_ref.restore_ew(B, _TEW_MASK, 7 / 24.0, "bf16")
    assert got[0, 4] == 1 and got[2, 0] == 0 and int(got.sum()) == 7


def test_restore_ew_limits():
    B = W.f32_to_bits(_TEW_B, "f16")
    assert not tw_ref.restore_ew(B, _TEW_MASK, 0.0, "f16").any()
    everything = tw_ref.restore_ew(B, _TEW_MASK, 0.99, "f16")          # more than there are pruned weights
    assert np.array_equal(everything, 1 - _TEW_MASK)
