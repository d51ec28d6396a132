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
