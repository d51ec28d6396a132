"""GPU parity: tw_gemm and tw_dense_gemm, called through the C-ABI, against the fp64 CPU oracle on
the same seeded inputs, EVERY element of C at every size (the full-size workloads included).
Tolerance (max|err| / max|ref|): 2e-3 for fp16, 1e-2 for bf16 - the output rounding (2^-11, 2^-8)
dominates, fp32 accumulation adds ~1e-6.  On top of that norm-wise bound every element is held to
its own bound (one rounding of the element plus a small share of the largest one), so that a single
wrong small element cannot hide behind a large one.  Integer-valued inputs make every product and
sum exact, so those cases are compared bit for bit, once per kernel mode and boundary."""
import sys

import numpy as np
import pytest
import torch

from oracle import tw_ref
from paper_2008_13006_amd import workloads as W

pytestmark = pytest.mark.gpu
TOL = {"f16": 2e-3, "bf16": 1e-2}


@pytest.fixture(scope="module")
def tw():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2008_13006_amd import binding
    return binding


def _say(msg):
    print(f"[case] {msg}", flush=True)
    sys.stdout.flush()


def _to_f64(t):
    return t.to(torch.float64).cpu().numpy()


def _rel_err(got64, ref):
    scale = np.max(np.abs(ref))
    return float(np.max(np.abs(got64 - ref)) / scale) if scale > 0 else float(np.max(np.abs(got64)))


# one rounding to the storage type, relative to the element
ULP = {"f16": 2.0 ** -11, "bf16": 2.0 ** -8}


def _assert_close(got64, ref, dtype, what=""):
    """The benchmark spec's bound on max|err| / max|ref| AND an element-wise bound: the output rounding of that element
    (with 2 % slack) plus 1e-4 of the largest reference value for the fp32 accumulation."""
    assert got64.shape == ref.shape
    assert np.isfinite(got64).all(), f"{what}: some element was not written"
    scale = float(np.max(np.abs(ref))) if ref.size else 0.0
    err = np.abs(got64 - ref)
    rel = float(err.max() / scale) if scale > 0 else float(err.max()) if err.size else 0.0
    assert rel <= TOL[dtype], f"{what}: max|err|/max|ref| = {rel:.3e}"
    bound = 1.02 * ULP[dtype] * np.abs(ref) + 1e-4 * max(scale, 1e-30)
    bad = err > bound
    assert not bad.any(), f"{what}: {int(bad.sum())} elements beyond their own bound, first at {np.argwhere(bad)[0]}"
    return rel


def _compare_whole(C, A_bits, B_bits, mask, dtype, transposed=False, chunk=8192, what="", post=None):
    """Every element of C (or of Ct = C^T with transposed=True) against the oracle, in blocks of rows of A so that
    the fp64 copies stay small.  post(ref_block) maps the oracle's product to the expected values (fused epilogue)."""
    M = A_bits.shape[0]
    worst = 0.0
    for r0 in range(0, M, chunk):
        r1 = min(M, r0 + chunk)
        ref = tw_ref.masked_gemm(np.ascontiguousarray(A_bits[r0:r1]), B_bits, mask, dtype)
        if post is not None:
            ref = post(ref)
        got = _to_f64(C[:, r0:r1]).T if transposed else _to_f64(C[r0:r1])
        worst = max(worst, _assert_close(got, ref, dtype, f"{what} rows {r0}..{r1}"))
    return worst


def _device_A(tw, A_bits, dtype, pad_to=8):
    """A on the GPU with a row stride that is a multiple of 8 elements."""
    M, K = A_bits.shape
    lda = (K + pad_to - 1) // pad_to * pad_to
    buf = torch.zeros((M, lda), dtype=torch.float16 if dtype == "f16" else torch.bfloat16, device="cuda:0")
    buf[:, :K] = tw.bits_to_tensor(A_bits, dtype)
    return buf[:, :K]


def _run_tw(tw, w, poison=True):
    spec = w.spec
    wt = tw.TwWeight.from_dense(w.B, w.mask, spec.G, spec.dtype)
    A = _device_A(tw, w.A, spec.dtype)
    M = A.shape[0]
    C = torch.full((M, spec.N), float("nan"), dtype=A.dtype, device="cuda:0") if poison else None
    C = tw.tw_gemm(wt, A, C)
    torch.cuda.synchronize()
    ws = wt.workspace.view(torch.int32)[:4].cpu().tolist()
    assert ws[0] == 0 and ws[1] == 0, "scheduler counters not reset"
    assert ws[3] == 0, "a bounded wait inside the kernel ran out"
    return wt, A, C


def _check_tw(tw, w):
    """tw_gemm on the workload, every element of C against the oracle."""
    spec = w.spec
    wt, A, C = _run_tw(tw, w)
    err = _compare_whole(C, w.A, w.B, w.mask, spec.dtype, what=spec.name)
    _say(f"{spec.name}: rel err {err:.3e} (all {spec.M} x {spec.N} elements)")
    # pruned columns are exact zeros
    pruned = np.flatnonzero(~w.mask.any(axis=0))
    if len(pruned):
        assert float(C[:, torch.as_tensor(pruned, device="cuda:0")].float().abs().max().item()) == 0.0
    return wt, A, C


# ------------------------------------------------------------------ small, element by element
SMALL = [
    # name, M, K, N, G, dtype, col_prune, keep
    ("tiny_one_tile", 5, 24, 32, 32, "f16", 0.0, ("const", 0.5)),
    ("ragged_rows_gaps", 77, 200, 300, 128, "f16", 0.07, ("upow", 0.05, 0.7)),
    ("k_not_mult_of_8", 33, 203, 190, 64, "f16", 0.1, ("upow", 0.1, 0.9)),
    ("bf16_g64", 130, 320, 256, 64, "bf16", 0.05, ("upow", 0.1, 0.6)),
    ("g32_many_tiles", 65, 96, 320, 32, "f16", 0.2, ("upow", 0.02, 1.0)),
    ("one_row", 1, 128, 256, 128, "bf16", 0.0, ("upow", 0.1, 0.5)),
    ("several_row_blocks", 300, 512, 640, 128, "f16", 0.05, ("upow", 0.1, 0.5)),
    ("kept_one_row_each", 40, 64, 256, 128, "f16", 0.0, ("const", 0.0)),
    ("streamed_k", 100, 2304, 200, 64, "f16", 0.1, ("upow", 0.05, 0.5)),
    ("streamed_k_bf16_ragged", 67, 2100, 300, 128, "bf16", 0.05, ("upow", 0.02, 0.6)),
    # 70 % of the columns pruned: a tile of 128 kept columns spans ~430 original columns, more than one
    # staging window of the epilogue
    ("wide_spans", 90, 256, 1400, 128, "f16", 0.7, ("upow", 0.1, 0.6)),
    ("wide_spans_bf16_g64", 45, 160, 900, 64, "bf16", 0.8, ("upow", 0.1, 0.9)),
    # few kept columns: spans narrower than a 16-byte group
    ("thin_tiles", 37, 64, 24, 32, "f16", 0.75, ("const", 0.5)),
    ("odd_everything", 71, 333, 1001, 128, "f16", 0.33, ("upow", 0.05, 0.8)),
]


@pytest.mark.parametrize("case", SMALL, ids=[c[0] for c in SMALL])
def test_tw_gemm_small_cases(tw, case):
    name, M, K, N, G, dtype, cp, keep = case
    _say(f"tw_gemm small {name} M={M} K={K} N={N} G={G} {dtype}")
    spec = W.small_spec(name, M=M, K=K, N=N, G=G, dtype=dtype, col_prune=cp, keep=keep,
                        seed_offset=9500 + len(name))
    _check_tw(tw, W.generate(spec))


def test_tw_gemm_integer_inputs_bit_exact(tw):
    """Small integers: every product and partial sum is exact in fp32 and the result is exact in fp16."""
    _say("tw_gemm integer inputs, bit exact")
    spec = W.small_spec("ints", M=150, K=256, N=384, G=128, dtype="f16", col_prune=0.05,
                        keep=("upow", 0.1, 0.6), a_dist="smallint", seed_offset=9600)
    w = W.generate(spec)
    _, _, C = _run_tw(tw, w)
    ref = tw_ref.masked_gemm(w.A, w.B, w.mask, "f16")
    assert np.max(np.abs(ref)) < 2048                    # integers below 2^11 are exact in fp16
    assert np.array_equal(_to_f64(C), ref)


def test_tw_gemm_zero_sparsity_equals_dense(tw):
    """0 % sparsity: TW result, dense kernel result and the oracle agree (spec invariant)."""
    _say("tw_gemm at 0 % sparsity vs tw_dense_gemm")
    spec = W.small_spec("dense0", M=200, K=256, N=384, G=128, dtype="f16", keep=("const", 1.0), seed_offset=9700)
    w = W.generate(spec)
    assert w.mask.all()
    wt, A, C = _check_tw(tw, w)
    B = tw.bits_to_tensor(w.B, "f16")
    Cd = tw.tw_dense_gemm(A.contiguous(), B)
    torch.cuda.synchronize()
    ref = tw_ref.masked_gemm(w.A, w.B, w.mask, "f16")
    assert _rel_err(_to_f64(Cd), ref) <= TOL["f16"]
    assert _rel_err(_to_f64(C), _to_f64(Cd)) <= TOL["f16"]


def test_tw_gemm_all_pruned_tile_and_empty_weight(tw):
    _say("tw_gemm all-pruned tile / empty weight")
    spec = W.small_spec("holes", M=70, K=64, N=384, G=128, dtype="f16", keep=("const", 0.5), seed_offset=9800)
    w = W.generate(spec)
    w.mask[:, 128:256] = 0                               # the middle tile disappears entirely
    _, _, C = _check_tw(tw, w)
    assert float(C[:, 128:256].float().abs().max().item()) == 0.0
    w.mask[:] = 0
    _, _, C = _run_tw(tw, w)
    assert float(C.float().abs().max().item()) == 0.0


def test_tw_gemm_is_deterministic_and_workspace_reusable(tw):
    _say("tw_gemm twice on one workspace, bit-identical")
    w = W.generate(W.CONFIGS["c1_single"][0])
    wt, A, C1 = _run_tw(tw, w)
    C2 = tw.tw_gemm(wt, A)
    C3 = tw.tw_gemm(wt, A)
    torch.cuda.synchronize()
    assert torch.equal(C1, C2) and torch.equal(C1, C3)


def test_two_streams_with_a_workspace_each(tw):
    """Launches of one weight on two streams that may overlap: a TwWeight (a workspace) per stream on one device copy
    of the blob; a resident-K weight with more items than compute units (the counters are in use) and a split-K plan
    (the workspace holds partial results)."""
    for name, M, K, N, G in (("two_streams_resident", 20000, 256, 512, 128), ("two_streams_split", 512, 2304, 512, 128)):
        spec = W.small_spec(name, M=M, K=K, N=N, G=G, dtype="f16", col_prune=0.05, keep=("upow", 0.1, 0.5), seed_offset=9900 + K)
        w = W.generate(spec)
        w0 = tw.TwWeight.from_dense(w.B, w.mask, G, "f16")
        w1 = w0.sibling()
        assert w1.blob_dev.data_ptr() == w0.blob_dev.data_ptr() and w1.workspace.data_ptr() != w0.workspace.data_ptr()
        A = _device_A(tw, w.A, "f16")
        ref = tw.tw_gemm(w0, A)
        torch.cuda.synchronize()
        s0, s1 = torch.cuda.Stream(), torch.cuda.Stream()
        outs = [[], []]
        for rep in range(6):
            for wt, st, o in ((w0, s0, outs[0]), (w1, s1, outs[1])):
                with torch.cuda.stream(st):
                    o.append(tw.tw_gemm(wt, A, stream=st))
        torch.cuda.synchronize()
        for o in outs[0] + outs[1]:
            assert torch.equal(o, ref)
        for wt in (w0, w1):
            assert wt.workspace.view(torch.int32)[:4].cpu().tolist() == [0, 0, 0, 0]
        _say(f"{name}: 2 x 6 launches on two streams, all equal to the single-stream result")
    torch.cuda.empty_cache()


def test_tw_gemm_strided_output(tw):
    _say("tw_gemm into a strided C")
    spec = W.small_spec("ldc", M=50, K=128, N=200, G=64, dtype="f16", col_prune=0.1, seed_offset=9900)
    w = W.generate(spec)
    wt = tw.TwWeight.from_dense(w.B, w.mask, 64, "f16")
    A = _device_A(tw, w.A, "f16")
    big = torch.full((50, 333), 7.0, dtype=torch.float16, device="cuda:0")
    tw.tw_gemm(wt, A, big[:, 11:211])
    torch.cuda.synchronize()
    ref = tw_ref.masked_gemm(w.A, w.B, w.mask, "f16")
    assert _rel_err(_to_f64(big[:, 11:211]), ref) <= TOL["f16"]
    assert bool((big[:, :11] == 7.0).all()) and bool((big[:, 211:] == 7.0).all())


def test_bad_device_arguments_are_refused(tw):
    spec = W.small_spec("args", M=8, K=64, N=128, G=64, seed_offset=9950)
    w = W.generate(spec)
    wt = tw.TwWeight.from_dense(w.B, w.mask, 64, "f16")
    A = torch.zeros((8, 65), dtype=torch.float16, device="cuda:0")[:, :64]   # row stride 65: not a multiple of 8
    with pytest.raises(tw.TwError) as e:
        tw.tw_gemm(wt, A)
    assert e.value.status == -4


# ------------------------------------------------------------------ dense kernel
DENSE = [("d_small", 70, 96, 130, "f16"), ("d_ragged", 300, 200, 520, "bf16"), ("d_blocks", 512, 256, 512, "f16"),
         ("d_k_tail", 257, 1000, 264, "f16")]


@pytest.mark.parametrize("case", DENSE, ids=[c[0] for c in DENSE])
def test_dense_gemm_small_cases(tw, case):
    name, M, K, N, dtype = case
    _say(f"tw_dense_gemm {name} M={M} K={K} N={N} {dtype}")
    rng = np.random.default_rng(sum(map(ord, name)))
    A_bits = W.f32_to_bits(rng.standard_normal((M, K), dtype=np.float32), dtype)
    B_bits = W.f32_to_bits(rng.standard_normal((K, N), dtype=np.float32) * np.float32(0.05), dtype)
    lda, ldb, ldc = (K + 7) // 8 * 8, (N + 7) // 8 * 8, (N + 7) // 8 * 8 + 8
    td = torch.float16 if dtype == "f16" else torch.bfloat16
    A = torch.zeros((M, lda), dtype=td, device="cuda:0"); A[:, :K] = tw.bits_to_tensor(A_bits, dtype)
    B = torch.zeros((K, ldb), dtype=td, device="cuda:0"); B[:, :N] = tw.bits_to_tensor(B_bits, dtype)
    Cbuf = torch.full((M, ldc), float("nan"), dtype=td, device="cuda:0")
    tw.tw_dense_gemm(A[:, :K], B[:, :N], Cbuf[:, :N])
    torch.cuda.synchronize()
    ref = tw_ref.masked_gemm(A_bits, B_bits, np.ones((K, N), np.uint8), dtype)
    got = _to_f64(Cbuf[:, :N])
    assert np.isfinite(got).all()
    assert _rel_err(got, ref) <= TOL[dtype]
    assert bool(torch.isnan(Cbuf[:, N:].float()).all().item()), "wrote outside C"


# ------------------------------------------------------------------ the five workloads, full size
def test_config1_full(tw):
    _say("config 1, every element")
    _check_tw(tw, W.generate(W.CONFIGS["c1_single"][0]))


@pytest.mark.parametrize("cfg", ["c2_bert_base_ffn_up", "c3_bert_base_layer", "c4_bert_large_skewed", "c5_conv_im2col"])
def test_full_size_workloads_every_element(tw, cfg):
    """Full-size launch (the configuration bench.py times): every element of C against the oracle."""
    for spec in W.CONFIGS[cfg]:
        _say(f"{cfg} / {spec.name} M={spec.M} K={spec.K} N={spec.N}")
        w = W.generate(spec)
        wt, A, C = _check_tw(tw, w)
        if cfg == "c2_bert_base_ffn_up":
            # the dense yardstick at the same shape
            B = tw.bits_to_tensor(w.B, spec.dtype)
            Cd = tw.tw_dense_gemm(A.contiguous(), B)
            torch.cuda.synchronize()
            _compare_whole(Cd, w.A, w.B, np.ones_like(w.mask), spec.dtype, what="tw_dense_gemm " + spec.name)
            del Cd
        del wt, A, C
        torch.cuda.empty_cache()


def test_full_size_fixed_grid_mask_every_element(tw):
    """The headline shape with tiles cut on a fixed grid of G original columns (spans are whole lines of C)."""
    spec = W.C2_FIXED_GRID
    _say(f"fixed grid / {spec.name} M={spec.M} K={spec.K} N={spec.N}")
    _check_tw(tw, W.generate(spec))
    torch.cuda.empty_cache()


# ------------------------------------------------------------------ fused epilogue: act(A.(B*mask) + bias)
def _bias_bits(N, dtype, seed):
    rng = np.random.default_rng(seed)
    return W.f32_to_bits(rng.standard_normal(N, dtype=np.float32) * np.float32(0.5), dtype)


FUSED = [
    # SMALL case name, bias?, activation
    ("ragged_rows_gaps", True, "gelu"), ("ragged_rows_gaps", True, "none"), ("ragged_rows_gaps", False, "relu"),
    ("bf16_g64", True, "gelu"), ("g32_many_tiles", True, "relu"), ("several_row_blocks", True, "gelu"),
    ("streamed_k", True, "gelu"), ("streamed_k_bf16_ragged", True, "relu"), ("wide_spans", True, "gelu"),
    ("thin_tiles", True, "gelu"), ("odd_everything", True, "relu"), ("one_row", False, "gelu"),
]


@pytest.mark.parametrize("case", FUSED, ids=[f"{c[0]}-{'bias' if c[1] else 'nobias'}-{c[2]}" for c in FUSED])
def test_tw_gemm_bias_act(tw, case):
    """tw_gemm_bias_act against the oracle's act(C_ref + bias); pruned columns must hold act(bias)."""
    cname, with_bias, act = case
    name, M, K, N, G, dtype, cp, keep = next(c for c in SMALL if c[0] == cname)
    _say(f"tw_gemm_bias_act {name} bias={with_bias} act={act}")
    spec = W.small_spec(name, M=M, K=K, N=N, G=G, dtype=dtype, col_prune=cp, keep=keep, seed_offset=9500 + len(name))
    w = W.generate(spec)
    wt = tw.TwWeight.from_dense(w.B, w.mask, G, dtype)
    A = _device_A(tw, w.A, dtype)
    bbits = _bias_bits(N, dtype, 77 + N) if with_bias else None
    bias = tw.bits_to_tensor(bbits, dtype) if with_bias else None
    C = torch.full((M, N), float("nan"), dtype=A.dtype, device="cuda:0")
    tw.tw_gemm_bias_act(wt, A, bias, act, C)
    torch.cuda.synchronize()
    ref = tw_ref.bias_act(tw_ref.masked_gemm(w.A, w.B, w.mask, dtype),
                          tw_ref.decode(bbits, dtype) if with_bias else None, act)
    got = _to_f64(C)
    assert np.isfinite(got).all(), "some element of C was not written"
    err = _rel_err(got, ref)
    _say(f"  rel err {err:.3e}")
    assert err <= TOL[dtype]
    pruned = np.flatnonzero(~w.mask.any(axis=0))
    if len(pruned):      # act(bias) there, the same value in every row
        col = got[:, pruned]
        assert np.all(col == col[0:1, :])
        assert np.max(np.abs(col[0] - ref[0, pruned])) <= TOL[dtype] * max(1.0, np.max(np.abs(ref)))


def test_tw_gemm_bias_act_empty_weight_and_bad_act(tw):
    M, K, N, G = 9, 32, 64, 32
    B_bits = W.f32_to_bits(np.ones((K, N), np.float32), "f16")
    wt = tw.TwWeight.from_dense(B_bits, np.zeros((K, N), np.uint8), G, "f16")
    A = torch.ones((M, K), dtype=torch.float16, device="cuda:0")
    bbits = _bias_bits(N, "f16", 5)
    C = tw.tw_gemm_bias_act(wt, A, tw.bits_to_tensor(bbits, "f16"), "relu")
    torch.cuda.synchronize()
    ref = tw_ref.bias_act(np.zeros((M, N)), tw_ref.decode(bbits, "f16"), "relu")
    assert np.array_equal(_to_f64(C), ref)          # relu of a 16-bit value is exact
    with pytest.raises(tw.TwError):
        tw.tw_gemm_bias_act(wt, A, None, 7)


@pytest.mark.parametrize("case", [("d_ragged", "gelu"), ("d_blocks", "relu"), ("d_small", "none")],
                         ids=["d_ragged-gelu", "d_blocks-relu", "d_small-none"])
def test_dense_gemm_bias_act(tw, case):
    dname, act = case
    name, M, K, N, dtype = next(c for c in DENSE if c[0] == dname)
    _say(f"tw_dense_gemm_bias_act {name} act={act}")
    rng = np.random.default_rng(sum(map(ord, name)) + 1)
    A_bits = W.f32_to_bits(rng.standard_normal((M, K), dtype=np.float32), dtype)
    B_bits = W.f32_to_bits(rng.standard_normal((K, N), dtype=np.float32) * np.float32(0.05), dtype)
    bbits = _bias_bits(N, dtype, 11)
    lda, ldb, ldc = (K + 7) // 8 * 8, (N + 7) // 8 * 8, (N + 7) // 8 * 8 + 8
    td = torch.float16 if dtype == "f16" else torch.bfloat16
    A = torch.zeros((M, lda), dtype=td, device="cuda:0"); A[:, :K] = tw.bits_to_tensor(A_bits, dtype)
    B = torch.zeros((K, ldb), dtype=td, device="cuda:0"); B[:, :N] = tw.bits_to_tensor(B_bits, dtype)
    Cbuf = torch.full((M, ldc), float("nan"), dtype=td, device="cuda:0")
    tw.tw_dense_gemm_bias_act(A[:, :K], B[:, :N], tw.bits_to_tensor(bbits, dtype), act, Cbuf[:, :N])
    torch.cuda.synchronize()
    ref = tw_ref.bias_act(tw_ref.masked_gemm(A_bits, B_bits, np.ones((K, N), np.uint8), dtype),
                          tw_ref.decode(bbits, dtype), act)
    got = _to_f64(Cbuf[:, :N])
    assert np.isfinite(got).all()
    assert _rel_err(got, ref) <= TOL[dtype]
    assert bool(torch.isnan(Cbuf[:, N:].float()).all().item()), "wrote outside C"


def test_full_size_ffn_up_with_gelu(tw):
    """BERT-base FFN-up at full size with its bias and GELU fused, every element."""
    spec = W.CONFIGS["c2_bert_base_ffn_up"][0]
    w = W.generate(spec)
    wt = tw.TwWeight.from_dense(w.B, w.mask, spec.G, spec.dtype)
    A = _device_A(tw, w.A, spec.dtype)
    bbits = _bias_bits(spec.N, spec.dtype, 3)
    C = tw.tw_gemm_bias_act(wt, A, tw.bits_to_tensor(bbits, spec.dtype), "gelu")
    torch.cuda.synchronize()
    b64 = tw_ref.decode(bbits, spec.dtype)
    _compare_whole(C, w.A, w.B, w.mask, spec.dtype, what="ffn_up + bias + gelu",
                   post=lambda r: tw_ref.bias_act(r, b64, "gelu"))


# ------------------------------------------------------------------ transposed boundary: Ct = (A.(B*mask))^T from At
def _device_At(tw, A_bits, dtype):
    """A^T on the GPU (K x M) with a row stride that is a multiple of 8 elements."""
    M, K = A_bits.shape
    ld = (M + 7) // 8 * 8
    buf = torch.zeros((K, ld), dtype=torch.float16 if dtype == "f16" else torch.bfloat16, device="cuda:0")
    buf[:, :M] = tw.bits_to_tensor(np.ascontiguousarray(A_bits.T), dtype)
    return buf[:, :M]


TRANSPOSED = [c[0] for c in SMALL] + ["t_k1024", "t_k1400_bf16", "t_stream_8tiles", "t_stream_3tiles"]
SMALL_T = SMALL + [
    ("t_k1024", 150, 1024, 384, 128, "f16", 0.05, ("upow", 0.05, 0.5)),          # resident, blocks of 32 tokens
    ("t_k1400_bf16", 90, 1400, 200, 64, "bf16", 0.0, ("upow", 0.1, 0.4)),
    ("t_stream_8tiles", 200, 1700, 1100, 128, "f16", 0.08, ("upow", 0.05, 0.5)),  # streamed, a wave per tile
    ("t_stream_3tiles", 333, 2304, 180, 64, "f16", 0.0, ("upow", 0.1, 0.5)),      # streamed, loading waves
]


@pytest.mark.parametrize("cname", TRANSPOSED)
def test_tw_gemm_t_small_cases(tw, cname):
    name, M, K, N, G, dtype, cp, keep = next(c for c in SMALL_T if c[0] == cname)
    _say(f"tw_gemm_t small {name} M={M} K={K} N={N} G={G} {dtype}")
    spec = W.small_spec(name, M=M, K=K, N=N, G=G, dtype=dtype, col_prune=cp, keep=keep, seed_offset=9500 + len(name))
    w = W.generate(spec)
    wt = tw.TwWeight.from_dense(w.B, w.mask, G, dtype)
    At = _device_At(tw, w.A, dtype)
    ldct = (M + 7) // 8 * 8 + 8
    Cbuf = torch.full((N, ldct), float("nan"), dtype=At.dtype, device="cuda:0")
    tw.tw_gemm_t(wt, At, Cbuf[:, :M])
    torch.cuda.synchronize()
    ref = tw_ref.masked_gemm(w.A, w.B, w.mask, dtype)
    got = _to_f64(Cbuf[:, :M]).T
    assert np.isfinite(got).all(), "some element of Ct was not written"
    err = _rel_err(got, ref)
    _say(f"  rel err {err:.3e}")
    assert err <= TOL[dtype]
    pruned = np.flatnonzero(~w.mask.any(axis=0))
    if len(pruned):
        assert float(np.abs(got[:, pruned]).max()) == 0.0
    assert bool(torch.isnan(Cbuf[:, M:].float()).all().item()), "wrote outside Ct"
    ws = wt.workspace.view(torch.int32)[:2].cpu().tolist()
    assert ws == [0, 0], "scheduler counters not reset"


def test_tw_gemm_t_matches_tw_gemm_bit_for_bit(tw):
    """Same products in the same order: the transposed path must give exactly the bits of tw_gemm."""
    spec = W.small_spec("t_vs_plain", M=192, K=384, N=520, G=128, dtype="f16", col_prune=0.1, keep=("upow", 0.1, 0.7),
                        seed_offset=9911)
    w = W.generate(spec)
    wt = tw.TwWeight.from_dense(w.B, w.mask, spec.G, spec.dtype)
    C = tw.tw_gemm(wt, _device_A(tw, w.A, spec.dtype))
    Ct = tw.tw_gemm_t(wt, _device_At(tw, w.A, spec.dtype))
    torch.cuda.synchronize()
    assert torch.equal(C, Ct.T.contiguous())


def test_tw_transpose(tw):
    rng = np.random.default_rng(5)
    # (whole 64 x 64 tiles on aligned rows take 16-byte loads and stores, everything else goes element by element)
    for rows, cols in ((1, 1), (70, 130), (64, 64), (257, 33), (192, 320), (200, 136), (128, 72)):
        x = torch.from_numpy(rng.integers(0, 65536, size=(rows, cols), dtype=np.int64).astype(np.int16)).to("cuda:0").view(torch.float16)
        y = tw.tw_transpose(x)
        torch.cuda.synchronize()
        assert torch.equal(y.view(torch.int16), x.view(torch.int16).T)
    # a view with an odd offset: rows that are not 16-byte aligned
    big = torch.from_numpy(rng.integers(0, 65536, size=(130, 200), dtype=np.int64).astype(np.int16)).to("cuda:0").view(torch.float16)
    x = big[1:129, 3:131]
    out = torch.full((128, 136), float("nan"), dtype=torch.float16, device="cuda:0")
    tw.tw_transpose(x, out[:, :128])
    torch.cuda.synchronize()
    assert torch.equal(out[:, :128].view(torch.int16), x.view(torch.int16).T)
    assert bool(torch.isnan(out[:, 128:]).all().item())


def test_full_size_ffn_up_transposed(tw):
    spec = W.CONFIGS["c2_bert_base_ffn_up"][0]
    w = W.generate(spec)
    wt = tw.TwWeight.from_dense(w.B, w.mask, spec.G, spec.dtype)
    At = tw.tw_transpose(_device_A(tw, w.A, spec.dtype))
    Ct = tw.tw_gemm_t(wt, At)
    torch.cuda.synchronize()
    _compare_whole(Ct, w.A, w.B, w.mask, spec.dtype, transposed=True, what="tw_gemm_t ffn_up")
    pruned = np.flatnonzero(~w.mask.any(axis=0))
    assert float(Ct[torch.as_tensor(pruned, device="cuda:0")].float().abs().max().item()) == 0.0


FUSED_T = [("ragged_rows_gaps", True, "gelu"), ("bf16_g64", True, "relu"), ("wide_spans", True, "gelu"),
           ("t_k1024", True, "gelu"), ("t_stream_8tiles", True, "relu"), ("t_stream_3tiles", False, "gelu"),
           ("thin_tiles", True, "none")]


@pytest.mark.parametrize("case", FUSED_T, ids=[f"{c[0]}-{'bias' if c[1] else 'nobias'}-{c[2]}" for c in FUSED_T])
def test_tw_gemm_t_bias_act(tw, case):
    cname, with_bias, act = case
    name, M, K, N, G, dtype, cp, keep = next(c for c in SMALL_T if c[0] == cname)
    _say(f"tw_gemm_t_bias_act {name} bias={with_bias} act={act}")
    spec = W.small_spec(name, M=M, K=K, N=N, G=G, dtype=dtype, col_prune=cp, keep=keep, seed_offset=9500 + len(name))
    w = W.generate(spec)
    wt = tw.TwWeight.from_dense(w.B, w.mask, G, dtype)
    At = _device_At(tw, w.A, dtype)
    bbits = _bias_bits(N, dtype, 78 + N) if with_bias else None
    bias = tw.bits_to_tensor(bbits, dtype) if with_bias else None
    ldct = (M + 7) // 8 * 8
    Cbuf = torch.full((N, ldct + 8), float("nan"), dtype=At.dtype, device="cuda:0")
    tw.tw_gemm_t_bias_act(wt, At, bias, act, Cbuf[:, :M])
    torch.cuda.synchronize()
    ref = tw_ref.bias_act(tw_ref.masked_gemm(w.A, w.B, w.mask, dtype),
                          tw_ref.decode(bbits, dtype) if with_bias else None, act)
    got = _to_f64(Cbuf[:, :M]).T
    assert np.isfinite(got).all(), "some element of Ct was not written"
    err = _rel_err(got, ref)
    _say(f"  rel err {err:.3e}")
    assert err <= TOL[dtype]
    assert bool(torch.isnan(Cbuf[:, M:].float()).all().item()), "wrote outside Ct"


# ------------------------------------------------------------------ TEW hybrid: tile-wise pattern + element-wise residual
TEW = [("ragged_rows_gaps", 0.02), ("bf16_g64", 0.01), ("g32_many_tiles", 0.05), ("several_row_blocks", 0.01),
       ("wide_spans", 0.03), ("t_k1024", 0.01), ("kept_one_row_each", 0.1),
       # streamed K: a wave per tile with 32- and 64-row blocks, loading waves; the residual is added chunk by chunk
       ("streamed_k", 0.01), ("streamed_k_bf16_ragged", 0.02), ("t_stream_8tiles", 0.01), ("t_stream_3tiles", 0.02)]


@pytest.mark.parametrize("case", TEW, ids=[f"{c[0]}-delta{c[1]}" for c in TEW])
def test_tew_gemm_all_boundaries(tw, case):
    """A.(B*(mask | ew)) through tw_gemm, tw_gemm_t and the fused epilogue on a TEW blob, against the oracle's
    masked product over the union mask."""
    cname, delta = case
    name, M, K, N, G, dtype, cp, keep = next(c for c in SMALL_T if c[0] == cname)
    _say(f"TEW {name} delta={delta}")
    spec = W.small_spec(name, M=M, K=K, N=N, G=G, dtype=dtype, col_prune=cp, keep=keep, seed_offset=9500 + len(name))
    w = W.generate(spec)
    ew = tw_ref.restore_ew(w.B, w.mask, delta, dtype)
    assert ew.any()
    wt = tw.TwWeight(tw.tw_pack_tew(w.B, w.mask, ew, G, dtype))
    union = (w.mask | ew).astype(np.uint8)
    ref = tw_ref.masked_gemm(w.A, w.B, union, dtype)
    ref_tw_only = tw_ref.masked_gemm(w.A, w.B, w.mask, dtype)
    assert _rel_err(ref_tw_only, ref) > 10 * TOL[dtype] or delta < 0.02     # the residual matters in this case
    C = tw.tw_gemm(wt, _device_A(tw, w.A, dtype))
    Ct = tw.tw_gemm_t(wt, _device_At(tw, w.A, dtype))
    bbits = _bias_bits(N, dtype, 5)
    Cg = tw.tw_gemm_bias_act(wt, _device_A(tw, w.A, dtype), tw.bits_to_tensor(bbits, dtype), "relu")
    torch.cuda.synchronize()
    assert _rel_err(_to_f64(C), ref) <= TOL[dtype]
    assert _rel_err(_to_f64(Ct).T, ref) <= TOL[dtype]
    assert _rel_err(_to_f64(Cg), tw_ref.bias_act(ref, tw_ref.decode(bbits, dtype), "relu")) <= TOL[dtype]
    pruned = np.flatnonzero(~union.any(axis=0))
    if len(pruned):
        assert float(C[:, torch.as_tensor(pruned, device="cuda:0")].float().abs().max().item()) == 0.0


def test_tew_full_size_ffn_up(tw):
    """The hybrid on the headline workload, every element.  One per cent of the weights come back; about one in
    twenty of them lies in a column that the tile-wise pattern pruned altogether (they run in the pass of their own)."""
    spec = W.CONFIGS["c2_bert_base_ffn_up"][0]
    w = W.generate(spec)
    ew = tw.tw_restore_ew(w.B, w.mask, 0.01, spec.dtype)
    assert ew[:, ~w.mask.any(axis=0)].any()
    wt = tw.TwWeight(tw.tw_pack_tew(w.B, w.mask, ew, spec.G, spec.dtype))
    assert wt.info["ew_nnz"] == int(np.floor(0.01 * spec.K * spec.N + 0.5))
    union = (w.mask | ew).astype(np.uint8)
    C = tw.tw_gemm(wt, _device_A(tw, w.A, spec.dtype))
    torch.cuda.synchronize()
    _compare_whole(C, w.A, w.B, union, spec.dtype, what="TEW ffn_up")
    del C
    Ct = tw.tw_gemm_t(wt, tw.tw_transpose(_device_A(tw, w.A, spec.dtype)))
    torch.cuda.synchronize()
    _compare_whole(Ct, w.A, w.B, union, spec.dtype, transposed=True, what="TEW ffn_up transposed")


@pytest.mark.parametrize("cfg,idx", [("c3_bert_base_layer", 3), ("c4_bert_large_skewed", 1), ("c5_conv_im2col", 0)],
                         ids=["ffn_down_wave_per_tile", "ffn_down_skewed_sets_of_four", "conv_loading_waves"])
def test_tew_full_size_streamed_k(tw, cfg, idx):
    """The hybrid on the workloads whose K is streamed (64-row blocks: a wave per tile, sets of four tiles, loading
    waves), both boundaries, every element.  The residual comes from the library's tw_restore_ew, which the CPU
    tests hold bit for bit against the oracle's."""
    spec = W.CONFIGS[cfg][idx]
    _say(f"TEW streamed {cfg} / {spec.name}")
    w = W.generate(spec)
    ew = tw.tw_restore_ew(w.B, w.mask, 0.005, spec.dtype)
    wt = tw.TwWeight(tw.tw_pack_tew(w.B, w.mask, ew, spec.G, spec.dtype))
    assert wt.info["ew_nnz"] == int(np.floor(0.005 * spec.K * spec.N + 0.5)) and wt.info["k_chunk"] < spec.K
    union = (w.mask | ew).astype(np.uint8)
    rows = np.arange(0, spec.M, max(1, spec.M // 64))
    ref = tw_ref.masked_gemm(np.ascontiguousarray(w.A[rows]), w.B, union, spec.dtype)
    ref_tw_only = tw_ref.masked_gemm(np.ascontiguousarray(w.A[rows]), w.B, w.mask, spec.dtype)
    assert _rel_err(ref_tw_only, ref) > TOL[spec.dtype], "the residual should matter in this case"
    C = tw.tw_gemm(wt, _device_A(tw, w.A, spec.dtype))
    torch.cuda.synchronize()
    ws = wt.workspace.view(torch.int32)[:4].cpu().tolist()
    assert ws[0] == 0 and ws[1] == 0 and ws[3] == 0, f"workspace after the call: {ws}"
    _compare_whole(C, w.A, w.B, union, spec.dtype, what="TEW " + spec.name)
    del C
    torch.cuda.empty_cache()
    Ct = tw.tw_gemm_t(wt, _device_At(tw, w.A, spec.dtype))
    torch.cuda.synchronize()
    ws = wt.workspace.view(torch.int32)[:4].cpu().tolist()
    assert ws[0] == 0 and ws[1] == 0 and ws[3] == 0, f"workspace after the call: {ws}"
    _compare_whole(Ct, w.A, w.B, union, spec.dtype, transposed=True, what="TEW transposed " + spec.name)
    del Ct, wt
    torch.cuda.empty_cache()


def test_bad_arguments_of_the_newer_entry_points_are_refused(tw):
    """Documented error codes of tw_gemm_t, tw_gemm_*_bias_act and tw_transpose; nothing is enqueued on error."""
    import ctypes
    spec = W.small_spec("args2", M=16, K=64, N=128, G=64, seed_offset=9951)
    w = W.generate(spec)
    wt = tw.TwWeight.from_dense(w.B, w.mask, 64, "f16")
    lib = tw._lib
    vp = ctypes.c_void_p
    At = torch.zeros((64, 24), dtype=torch.float16, device="cuda:0")
    Ct = torch.full((128, 24), 7.0, dtype=torch.float16, device="cuda:0")
    blob_h, blob_d, ws = tw._np_ptr(wt.blob), vp(wt.blob_dev.data_ptr()), vp(wt.workspace.data_ptr())
    def call_t(at_ptr, M, ldat, ct_ptr, ldct, bias=None, act=0):
        return lib.tw_gemm_t_bias_act(blob_h, blob_d, vp(at_ptr), M, ldat, vp(bias or 0), act, vp(ct_ptr), ldct, ws, 256, None)
    assert call_t(At.data_ptr(), 16, 24, Ct.data_ptr(), 24) == 0                       # baseline: fine
    assert call_t(At.data_ptr(), 16, 20, Ct.data_ptr(), 24) == -4                      # ldat % 8 != 0
    assert call_t(At.data_ptr(), 16, 24, Ct.data_ptr(), 12) == -1                      # ldct < M
    assert call_t(At.data_ptr() + 2, 16, 24, Ct.data_ptr(), 24) == -4                  # At not 16-byte aligned
    assert call_t(At.data_ptr(), 16, 24, Ct.data_ptr(), 24, act=9) == -1               # unknown activation
    assert call_t(At.data_ptr(), 16, 24, Ct.data_ptr(), 24, bias=Ct.data_ptr() + 1) == -4   # odd bias address
    assert call_t(0, 16, 24, Ct.data_ptr(), 24) == -1                                  # null pointer
    assert call_t(At.data_ptr(), 0, 24, Ct.data_ptr(), 24) == 0                        # M = 0: nothing to do
    assert lib.tw_gemm_t(blob_h, blob_d, vp(At.data_ptr()), 16, 24, vp(Ct.data_ptr()), 24, ws, 8, None) == -3   # workspace too small
    torch.cuda.synchronize()
    x = torch.zeros((4, 8), dtype=torch.float16, device="cuda:0")
    y = torch.zeros((8, 4), dtype=torch.float16, device="cuda:0")
    assert lib.tw_transpose(vp(x.data_ptr()), 4, 4, 8, vp(y.data_ptr()), 4, None) == -1    # ld_src < cols
    assert lib.tw_transpose(vp(x.data_ptr()), 8, 4, 8, vp(y.data_ptr()), 2, None) == -1    # ld_dst < rows
    assert lib.tw_transpose(vp(x.data_ptr()), 8, 0, 8, vp(y.data_ptr()), 4, None) == 0
    with pytest.raises(ValueError):
        tw.tw_gemm_bias_act(wt, torch.zeros((16, 64), dtype=torch.float16, device="cuda:0"), None, "swish")


@pytest.mark.parametrize("cfg", ["c3_bert_base_layer", "c4_bert_large_skewed", "c5_conv_im2col"])
def test_full_size_workloads_transposed_every_element(tw, cfg):
    """tw_gemm_t at the sizes bench.py times (resident K with 64- and 32-token blocks, streamed K with a wave
    per tile and with loading waves that read only the kept rows), every element of Ct."""
    for spec in W.CONFIGS[cfg]:
        _say(f"transposed {cfg} / {spec.name} M={spec.M} K={spec.K} N={spec.N}")
        w = W.generate(spec)
        wt = tw.TwWeight.from_dense(w.B, w.mask, spec.G, spec.dtype)
        At = tw.tw_transpose(_device_A(tw, w.A, spec.dtype))
        Ct = tw.tw_gemm_t(wt, At)
        torch.cuda.synchronize()
        err = _compare_whole(Ct, w.A, w.B, w.mask, spec.dtype, transposed=True, what="tw_gemm_t " + spec.name)
        _say(f"  rel err {err:.3e}")
        pruned = np.flatnonzero(~w.mask.any(axis=0))
        if len(pruned):
            assert float(Ct[torch.as_tensor(pruned, device="cuda:0")].float().abs().max().item()) == 0.0
        del At, Ct
        torch.cuda.empty_cache()


# ------------------------------------------------------------------ seeded random shapes, every boundary per shape
def _random_case(seed):
    """Shape, G, dtype and mask recipe drawn from a seeded generator: M spans one to several row blocks with a
    ragged tail, K spans the resident and both streamed regimes, N spans one to a dozen tiles."""
    rng = np.random.default_rng(77000 + seed)
    M = int(rng.choice([1, 7, 31, 64, 65, 130, 257, 333]))
    K = int(rng.choice([16, 40, 129, 384, 770, 1100, 1536, 1544, 2050, 3000]))
    G = int(rng.choice([32, 64, 128]))
    N = int(rng.integers(8, 12 * G))
    dtype = "f16" if rng.random() < 0.6 else "bf16"
    cp = float(rng.choice([0.0, 0.05, 0.3, 0.8]))
    lo = float(rng.choice([0.0, 0.02, 0.1]))
    hi = float(rng.choice([0.3, 0.6, 1.0]))
    return M, K, N, G, dtype, cp, ("upow", lo, hi)


@pytest.mark.parametrize("seed", range(20))
def test_random_shapes_all_boundaries(tw, seed):
    M, K, N, G, dtype, cp, keep = _random_case(seed)
    _say(f"random seed {seed}: M={M} K={K} N={N} G={G} {dtype} col_prune={cp} keep={keep}")
    spec = W.small_spec(f"rand{seed}", M=M, K=K, N=N, G=G, dtype=dtype, col_prune=cp, keep=keep,
                        seed_offset=88000 + seed)
    w = W.generate(spec)
    ref = tw_ref.masked_gemm(w.A, w.B, w.mask, dtype)
    wt = tw.TwWeight.from_dense(w.B, w.mask, G, dtype)
    A = _device_A(tw, w.A, dtype)
    At = _device_At(tw, w.A, dtype)
    td = A.dtype
    # row-major boundary
    C = torch.full((M, N), float("nan"), dtype=td, device="cuda:0")
    tw.tw_gemm(wt, A, C)
    # transposed boundary, output with a padded row stride
    ldct = (M + 7) // 8 * 8 + 8
    Ctb = torch.full((N, ldct), float("nan"), dtype=td, device="cuda:0")
    tw.tw_gemm_t(wt, At, Ctb[:, :M])
    # fused epilogue on both
    rng = np.random.default_rng(99000 + seed)
    bbits = W.f32_to_bits(rng.standard_normal(N).astype(np.float32), dtype)
    bias = tw.bits_to_tensor(bbits, dtype)
    Cf = torch.full((M, N), float("nan"), dtype=td, device="cuda:0")
    tw.tw_gemm_bias_act(wt, A, bias, "gelu", Cf)
    Cft = torch.full((N, ldct), float("nan"), dtype=td, device="cuda:0")
    tw.tw_gemm_t_bias_act(wt, At, bias, "relu", Cft[:, :M])
    torch.cuda.synchronize()
    ws = wt.workspace.view(torch.int32)[:4].cpu().tolist()
    assert ws[0] == 0 and ws[1] == 0 and ws[3] == 0, f"workspace after the calls: {ws}"

    got = _to_f64(C)
    assert np.isfinite(got).all()
    assert _rel_err(got, ref) <= TOL[dtype]
    assert torch.equal(Ctb[:, :M].T.contiguous(), C), "the two boundaries differ in some bit"
    assert bool(torch.isnan(Ctb[:, M:].float()).all().item()), "wrote outside Ct"
    b64 = tw_ref.decode(bbits, dtype)
    ref_g = tw_ref.bias_act(ref, b64, "gelu")
    ref_r = tw_ref.bias_act(ref, b64, "relu")
    assert _rel_err(_to_f64(Cf), ref_g) <= TOL[dtype]
    assert _rel_err(_to_f64(Cft[:, :M]).T, ref_r) <= TOL[dtype]
    assert bool(torch.isnan(Cft[:, M:].float()).all().item()), "wrote outside Ct (fused)"


def test_streamed_k_sets_of_four_tiles(tw):
    """More than four tiles, K streamed, and too few 64-row blocks to give every compute unit one with eight tiles
    per workgroup: the plan then carves sets of four tiles (half of the waves only load A).  20 tiles, 52 row
    blocks: 3 sets of eight would make 156 items, 5 sets of four make 260."""
    M, K, N, G, dtype = 3300, 1600, 660, 32, "f16"
    _say(f"sets of four: M={M} K={K} N={N} G={G} {dtype}")
    spec = W.small_spec("sets_of_four", M=M, K=K, N=N, G=G, dtype=dtype, col_prune=0.04, keep=("upow", 0.05, 0.6),
                        seed_offset=9977)
    w = W.generate(spec)
    wt = tw.TwWeight.from_dense(w.B, w.mask, G, dtype)
    assert wt.info["T"] > 4
    n_cu = torch.cuda.get_device_properties(0).multi_processor_count
    for tr in (False, True):
        pl = tw.tw_gemm_plan(tw.tw_pack(w.B, w.mask, G, dtype), M, n_cu=n_cu, transposed=tr)
        _say(f"  plan on {n_cu} compute units, transposed={tr}: {pl}")
        if n_cu == 256:
            assert pl["mode"] == 2 and pl["tiles_per_set"] == 4
            # (260 items of 64 rows would be two rounds with an almost empty second one: the row-major boundary
            # takes lower row blocks instead, the transposed one keeps whole lines of 64 tokens)
            assert pl["rows_per_block"] == (64 if tr else 40)
    rng = np.random.default_rng(5)
    A = _device_A(tw, w.A, dtype)
    C = torch.full((M, N), float("nan"), dtype=A.dtype, device="cuda:0")
    tw.tw_gemm(wt, A, C)
    At = _device_At(tw, w.A, dtype)
    ldct = (M + 7) // 8 * 8 + 8
    Ctb = torch.full((N, ldct), float("nan"), dtype=A.dtype, device="cuda:0")
    tw.tw_gemm_t(wt, At, Ctb[:, :M])
    bbits = W.f32_to_bits(rng.standard_normal(N).astype(np.float32), dtype)
    Cf = torch.full((M, N), float("nan"), dtype=A.dtype, device="cuda:0")
    tw.tw_gemm_bias_act(wt, A, tw.bits_to_tensor(bbits, dtype), "relu", Cf)
    torch.cuda.synchronize()
    ws = wt.workspace.view(torch.int32)[:4].cpu().tolist()
    assert ws[0] == 0 and ws[1] == 0 and ws[3] == 0, f"workspace after the calls: {ws}"
    _compare_whole(C, w.A, w.B, w.mask, dtype, what="sets of four")
    assert torch.equal(Ctb[:, :M].T.contiguous(), C), "the two boundaries differ in some bit"
    assert bool(torch.isnan(Ctb[:, M:].float()).all().item()), "wrote outside Ct"
    b64 = tw_ref.decode(bbits, dtype)
    _compare_whole(Cf, w.A, w.B, w.mask, dtype, what="sets of four, relu", post=lambda r: tw_ref.bias_act(r, b64, "relu"))
    pruned = np.flatnonzero(~w.mask.any(axis=0))
    if len(pruned):
        assert float(C[:, torch.as_tensor(pruned, device="cuda:0")].float().abs().max().item()) == 0.0


# ------------------------------------------------------------------ a chain of launches inside a HIP graph
def test_hip_graph_replays_match_eager(tw):
    """The four weight GEMMs of a BERT-base layer (QKV, attention output on a strided view, FFN-up with bias and
    GELU, FFN-down) chained on one stream, captured in a HIP graph and replayed with new inputs; eager work of the
    same library runs between the replays.  Every replay must give the bits of the eager chain, and the eager
    chain's last output is held against the oracle.  (The library enqueues kernels only: the scheduler counters
    in the workspace are put back by the kernel itself, so a capture records no memset.)"""
    M = 512
    specs = W.CONFIGS["c3_bert_base_layer"]
    ws = [W.generate(s, M=M) for s in specs]
    wts = [tw.TwWeight.from_dense(w.B, w.mask, s.G, s.dtype) for w, s in zip(ws, specs)]
    dtype = specs[0].dtype
    bbits = _bias_bits(specs[2].N, dtype, 11)
    bias = tw.bits_to_tensor(bbits, dtype)
    td = torch.float16
    X = torch.empty((M, 768), dtype=td, device="cuda:0")
    QKV = torch.empty((M, 2304), dtype=td, device="cuda:0")
    AO = torch.empty((M, 768), dtype=td, device="cuda:0")
    H = torch.empty((M, 3072), dtype=td, device="cuda:0")
    Y = torch.empty((M, 768), dtype=td, device="cuda:0")

    def chain():
        tw.tw_gemm(wts[0], X, QKV)
        tw.tw_gemm(wts[1], QKV[:, :768], AO)          # row stride 2304
        tw.tw_gemm_bias_act(wts[2], AO, bias, "gelu", H)
        tw.tw_gemm(wts[3], H, Y)

    rng = np.random.default_rng(21)
    inputs = [W.f32_to_bits(rng.standard_normal((M, 768)).astype(np.float32), dtype) for _ in range(3)]
    X.copy_(tw.bits_to_tensor(inputs[0], dtype))
    chain()                                            # warm-up outside the capture (first-use attribute calls)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        chain()
    torch.cuda.synchronize()
    for i, xb in enumerate(inputs):
        _say(f"  replay {i}")
        X.copy_(tw.bits_to_tensor(xb, dtype))
        chain()
        torch.cuda.synchronize()
        eager = [t.clone() for t in (QKV, AO, H, Y)]
        for t in (QKV, AO, H, Y):
            t.fill_(float("nan"))
        g.replay()
        torch.cuda.synchronize()
        for name, a, b in zip(("QKV", "AO", "H", "Y"), eager, (QKV, AO, H, Y)):
            assert torch.equal(a, b), f"replay {i}: {name} differs from the eager chain"
        for wt in wts:
            assert wt.workspace.view(torch.int32)[:4].cpu().tolist() == [0, 0, 0, 0]
        # unrelated eager work of the library between replays
        tw.tw_gemm(wts[1], X)
        torch.cuda.synchronize()
    # the last eager chain against the oracle, stage by stage on the device's own intermediate results
    def bits(t):
        return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    ref_y = tw_ref.masked_gemm(bits(H), ws[3].B, ws[3].mask, dtype)
    assert _rel_err(_to_f64(Y), ref_y) <= TOL[dtype]
    ref_h = tw_ref.bias_act(tw_ref.masked_gemm(bits(AO), ws[2].B, ws[2].mask, dtype), tw_ref.decode(bbits, dtype), "gelu")
    assert _rel_err(_to_f64(H), ref_h) <= TOL[dtype]
    ref_ao = tw_ref.masked_gemm(bits(QKV[:, :768]), ws[1].B, ws[1].mask, dtype)
    assert _rel_err(_to_f64(AO), ref_ao) <= TOL[dtype]


# ------------------------------------------------------------------ seeded random shapes at full occupancy
def _random_big_case(seed):
    """Enough rows to give every compute unit a 64-row block (so the 64-row kernels of all three modes run), a
    ragged last block, K in the resident and the streamed regime, few and many tiles."""
    rng = np.random.default_rng(55000 + seed)
    M = int(rng.choice([16384, 16411, 20001, 33000]))
    K = int(rng.choice([200, 768, 1536, 1600, 2304, 3100]))
    G = int(rng.choice([32, 64, 128]))
    N = int(rng.choice([G * 2 + 5, G * 4, G * 6 - 3, G * 9 + 1]))
    dtype = "f16" if rng.random() < 0.5 else "bf16"
    cp = float(rng.choice([0.0, 0.05, 0.25]))
    return M, K, N, G, dtype, cp, ("upow", 0.05, float(rng.choice([0.3, 0.7])))


@pytest.mark.parametrize("seed", range(8))
def test_random_big_shapes_on_sampled_rows(tw, seed):
    M, K, N, G, dtype, cp, keep = _random_big_case(seed)
    spec = W.small_spec(f"randbig{seed}", M=M, K=K, N=N, G=G, dtype=dtype, col_prune=cp, keep=keep,
                        seed_offset=66000 + seed)
    w = W.generate(spec)
    blob = tw.tw_pack(w.B, w.mask, G, dtype)
    n_cu = torch.cuda.get_device_properties(0).multi_processor_count
    pl, plt = tw.tw_gemm_plan(blob, M, n_cu=n_cu), tw.tw_gemm_plan(blob, M, n_cu=n_cu, transposed=True)
    _say(f"random big seed {seed}: M={M} K={K} N={N} G={G} {dtype} col_prune={cp} keep={keep} "
         f"plan mode {pl['mode']}/{plt['mode']} rows {pl['rows_per_block']} tiles per set {pl['tiles_per_set']}")
    wt = tw.TwWeight(blob)
    A = _device_A(tw, w.A, dtype)
    C = torch.full((M, N), float("nan"), dtype=A.dtype, device="cuda:0")
    tw.tw_gemm(wt, A, C)
    At = _device_At(tw, w.A, dtype)
    del A
    ldct = (M + 7) // 8 * 8 + 8
    Ctb = torch.full((N, ldct), float("nan"), dtype=C.dtype, device="cuda:0")
    tw.tw_gemm_t(wt, At, Ctb[:, :M])
    torch.cuda.synchronize()
    ws = wt.workspace.view(torch.int32)[:4].cpu().tolist()
    assert ws[0] == 0 and ws[1] == 0 and ws[3] == 0, f"workspace after the calls: {ws}"
    _compare_whole(C, w.A, w.B, w.mask, dtype, what=f"random big {seed}")
    assert torch.equal(Ctb[:, :M].T.contiguous(), C), "the two boundaries differ in some bit"
    assert bool(torch.isnan(Ctb[:, M:].float()).all().item()), "wrote outside Ct"
    pruned = np.flatnonzero(~w.mask.any(axis=0))
    if len(pruned):
        assert float(C[:, torch.as_tensor(pruned, device="cuda:0")].float().abs().max().item()) == 0.0
    del Ctb, At
    # the fused epilogue and, where K is resident or streamed alike, the hybrid's residual on the same plan
    bbits = _bias_bits(N, dtype, 100 + seed)
    b64 = tw_ref.decode(bbits, dtype)
    C.fill_(float("nan"))
    tw.tw_gemm_bias_act(wt, _device_A(tw, w.A, dtype), tw.bits_to_tensor(bbits, dtype), "relu", C)
    torch.cuda.synchronize()
    _compare_whole(C, w.A, w.B, w.mask, dtype, what=f"random big {seed} relu", post=lambda r: tw_ref.bias_act(r, b64, "relu"))
    ew = tw.tw_restore_ew(w.B, w.mask, 0.004, dtype)
    wte = tw.TwWeight(tw.tw_pack_tew(w.B, w.mask, ew, G, dtype))
    C.fill_(float("nan"))
    tw.tw_gemm(wte, _device_A(tw, w.A, dtype), C)
    torch.cuda.synchronize()
    _compare_whole(C, w.A, w.B, (w.mask | ew).astype(np.uint8), dtype, what=f"random big {seed} TEW")
    del C, wt, wte
    torch.cuda.empty_cache()


def test_a_million_rows_byte_offsets_beyond_2_31(tw):
    """The largest launch of the suite: 1 048 583 rows (a ragged last block, 16 385 row blocks: 65 rounds of
    workgroups through the item counter), C of 2.3 GB so that byte offsets into C and into Ct pass 2^31.  Every
    element against the oracle, both boundaries."""
    M, K, N, G = 1048583, 64, 1100, 128
    spec = W.small_spec("million_rows", M=M, K=K, N=N, G=G, dtype="f16", col_prune=0.4, keep=("upow", 0.2, 0.5),
                        seed_offset=31000)
    w = W.generate(spec)
    wt = tw.TwWeight.from_dense(w.B, w.mask, G, "f16")
    A = _device_A(tw, w.A, "f16")
    C = torch.full((M, N), float("nan"), dtype=A.dtype, device="cuda:0")
    assert C.numel() * 2 > 2 ** 31
    tw.tw_gemm(wt, A, C)
    At = _device_At(tw, w.A, "f16")
    Ct = tw.tw_gemm_t(wt, At)
    torch.cuda.synchronize()
    assert wt.workspace.view(torch.int32)[:4].cpu().tolist() == [0, 0, 0, 0]
    worst = worst_t = 0.0
    chunk = 65536
    for r0 in range(0, M, chunk):                      # the oracle once per block of rows, both outputs against it
        r1 = min(M, r0 + chunk)
        ref = tw_ref.masked_gemm(np.ascontiguousarray(w.A[r0:r1]), w.B, w.mask, "f16")
        worst = max(worst, _assert_close(_to_f64(C[r0:r1]), ref, "f16", f"million rows {r0}..{r1}"))
        worst_t = max(worst_t, _assert_close(_to_f64(Ct[:, r0:r1]).T, ref, "f16", f"million rows transposed {r0}..{r1}"))
    _say(f"million rows: rel err {worst:.3e} / transposed {worst_t:.3e}")
    del C, Ct, At, A
    torch.cuda.empty_cache()


# ------------------------------------------------------------------ integer inputs: bit for bit, per kernel mode
# A in {-3..3}, B in {-2..2}: every product and every partial sum is an integer that fp32 holds exactly, and the
# result is exact in the storage type while |C| stays below 2^11 (fp16) or 2^8 (bf16); the cases assert that.
# The shapes are chosen for the plan they give on 256 compute units; the plan is asserted.
EXACT = [
    # name, M, K, N, G, dtype, col_prune, keep, expected (mode, rows_per_block, tiles_per_set, k_parts) row-major / transposed
    ("resident_32rows", 150, 256, 384, 128, "f16", 0.05, ("upow", 0.1, 0.6), (0, 32, 0, 1), (0, 32, 0, 1)),
    ("resident_64rows", 8192, 256, 390, 128, "f16", 0.05, ("upow", 0.1, 0.6), (0, 64, 0, 1), (0, 64, 0, 1)),
    ("resident_64rows_bf16", 8192, 96, 200, 64, "bf16", 0.1, ("upow", 0.1, 0.5), (0, 64, 0, 1), (0, 64, 0, 1)),
    ("resident_lowered_blocks", 17000, 256, 250, 128, "f16", 0.0, ("upow", 0.1, 0.6), (0, 40, 0, 1), (0, 64, 0, 1)),
    ("streamed_wave_per_tile", 16384, 1600, 380, 64, "f16", 0.05, ("upow", 0.02, 0.15), (1, 64, 8, 1), (1, 64, 8, 1)),
    ("streamed_sets_of_4", 16400, 1600, 250, 64, "f16", 0.0, ("upow", 0.02, 0.15), (2, 40, 4, 1), (2, 64, 4, 1)),
    ("streamed_sets_of_2", 8192, 1700, 256, 64, "f16", 0.0, ("upow", 0.02, 0.15), (2, 64, 2, 1), (2, 64, 2, 1)),
    ("streamed_sets_of_1", 4096, 1600, 128, 32, "f16", 0.0, ("upow", 0.02, 0.15), (2, 64, 1, 1), (2, 64, 1, 1)),
    ("streamed_bf16", 16384, 1600, 256, 64, "bf16", 0.0, ("upow", 0.01, 0.04), (2, 64, 4, 1), (2, 64, 4, 1)),
    # split K: few row blocks and a streamed K; the parts' partial results go through the workspace
    ("split_one_row_block", 64, 3072, 768, 128, "f16", 0.0, ("upow", 0.02, 0.15), (1, 64, 1, 8), (1, 64, 1, 8)),
    ("split_sets_apart", 512, 3072, 768, 128, "f16", 0.05, ("upow", 0.02, 0.15), (1, 64, 2, 8), (1, 64, 2, 8)),
    ("split_bf16_ragged_chunk", 700, 2000, 300, 64, "bf16", 0.0, ("upow", 0.01, 0.04), (1, 64, 2, 6), (1, 64, 2, 6)),
    ("split_g32_parts_of_two", 1100, 1600, 250, 32, "f16", 0.1, ("upow", 0.02, 0.15), (1, 64, 4, 5), (1, 64, 4, 5)),
]


@pytest.mark.parametrize("case", EXACT, ids=[c[0] for c in EXACT])
def test_integer_inputs_bit_exact_per_mode(tw, case):
    name, M, K, N, G, dtype, cp, keep, plan_n, plan_t = case
    spec = W.small_spec("exact_" + name, M=M, K=K, N=N, G=G, dtype=dtype, col_prune=cp, keep=keep, a_dist="smallint",
                        seed_offset=12000 + len(name) + K)
    w = W.generate(spec)
    blob = tw.tw_pack(w.B, w.mask, G, dtype)
    n_cu = torch.cuda.get_device_properties(0).multi_processor_count
    pl, plt = tw.tw_gemm_plan(blob, M, n_cu=n_cu), tw.tw_gemm_plan(blob, M, n_cu=n_cu, transposed=True)
    _say(f"exact {name}: M={M} K={K} N={N} G={G} {dtype} T={tw.tw_info(blob)['T']} plan {pl} / transposed {plt}")
    if n_cu == 256:
        assert (pl["mode"], pl["rows_per_block"], pl["tiles_per_set"], pl["k_parts"]) == plan_n
        assert (plt["mode"], plt["rows_per_block"], plt["tiles_per_set"], plt["k_parts"]) == plan_t
    ref = tw_ref.masked_gemm(w.A, w.B, w.mask, dtype)
    limit = 2048 if dtype == "f16" else 256
    assert np.max(np.abs(ref)) <= limit, "the case must stay exactly representable"
    wt = tw.TwWeight(blob)
    A = _device_A(tw, w.A, dtype)
    C = torch.full((M, N), float("nan"), dtype=A.dtype, device="cuda:0")
    tw.tw_gemm(wt, A, C)
    torch.cuda.synchronize()
    assert np.array_equal(_to_f64(C), ref), "tw_gemm differs from the oracle in some bit"
    if pl["k_parts"] > 1:
        # the same product with the counters' 256 bytes of workspace only: no split, a different kernel plan
        assert tw.tw_gemm_workspace(blob, M) > 256
        wu = tw.TwWeight(blob)
        wu.ws_limit = 256
        Cu = torch.full((M, N), float("nan"), dtype=A.dtype, device="cuda:0")
        tw.tw_gemm(wu, A, Cu)
        torch.cuda.synchronize()
        assert wu.workspace.numel() == 256 and torch.equal(C, Cu), "split and unsplit plans differ on exact inputs"
        del Cu
    del C
    At = _device_At(tw, w.A, dtype)
    ldct = (M + 7) // 8 * 8 + 8
    Ctb = torch.full((N, ldct), float("nan"), dtype=A.dtype, device="cuda:0")
    tw.tw_gemm_t(wt, At, Ctb[:, :M])
    torch.cuda.synchronize()
    assert np.array_equal(_to_f64(Ctb[:, :M]).T, ref), "tw_gemm_t differs from the oracle in some bit"
    del Ctb, At
    # fused bias + ReLU: integer bias, exact as well
    rng = np.random.default_rng(31 + M)
    bias_i = rng.integers(-5, 6, size=N).astype(np.float32)
    bbits = W.f32_to_bits(bias_i, dtype)
    ref_r = tw_ref.bias_act(ref, bias_i.astype(np.float64), "relu")
    assert np.max(np.abs(ref_r)) <= limit
    Cf = tw.tw_gemm_bias_act(wt, A, tw.bits_to_tensor(bbits, dtype), "relu")
    torch.cuda.synchronize()
    assert np.array_equal(_to_f64(Cf), ref_r), "tw_gemm_bias_act differs from the oracle in some bit"
    del Cf
    # the hybrid's residual, weights in pruned columns included
    ew = tw_ref.restore_ew(w.B, w.mask, 0.004, dtype) if K * N <= 200000 else tw.tw_restore_ew(w.B, w.mask, 0.004, dtype)
    union = (w.mask | ew).astype(np.uint8)
    ref_e = tw_ref.masked_gemm(w.A, w.B, union, dtype)
    if np.max(np.abs(ref_e)) <= limit:
        wte = tw.TwWeight(tw.tw_pack_tew(w.B, w.mask, ew, G, dtype))
        Ce = tw.tw_gemm(wte, A)
        torch.cuda.synchronize()
        assert np.array_equal(_to_f64(Ce), ref_e), "tw_gemm on the TEW blob differs from the oracle in some bit"
        del Ce
        Cet = tw.tw_gemm_t(wte, _device_At(tw, w.A, dtype))
        torch.cuda.synchronize()
        assert np.array_equal(_to_f64(Cet).T, ref_e), "tw_gemm_t on the TEW blob differs from the oracle in some bit"
    torch.cuda.empty_cache()


# ------------------------------------------------------------------ split K: few rows, streamed K
@pytest.mark.parametrize("M", [64, 512, 2048, 1000])
def test_split_k_small_batches_of_the_ffn_down(tw, M):
    """FFN-down of BERT-base (K = 3072 in eight chunks, the c3 workload's weight and value distributions) at batch
    sizes that leave most compute units without a row block: the K chunks are split over workgroups, the parts'
    fp32 results go through the workspace and a second kernel adds them in a fixed order.  Every element of C
    against the oracle on both boundaries, with the fused epilogue and with a TEW residual; repeated calls are
    bit-identical (no atomics on floating point); a workspace that is too small for the parts falls back to
    the unsplit plan instead of failing."""
    import dataclasses
    base = W.CONFIGS["c3_bert_base_layer"][3]
    spec = dataclasses.replace(base, name=f"{base.name}_M{M}", M=M)
    w = W.generate(spec)
    dtype = spec.dtype
    wt = tw.TwWeight.from_dense(w.B, w.mask, spec.G, dtype)
    n_cu = torch.cuda.get_device_properties(0).multi_processor_count
    pl, plt = tw.tw_gemm_plan(wt.blob, M, n_cu=n_cu), tw.tw_gemm_plan(wt.blob, M, n_cu=n_cu, transposed=True)
    need = tw.tw_gemm_workspace(wt.blob, M)
    _say(f"split K {spec.name}: K={spec.K} N={spec.N} T={wt.info['T']} plan {pl} / transposed {plt}, workspace {need} bytes")
    if n_cu == 256:
        assert pl["k_parts"] > 1 and plt["k_parts"] > 1 and pl["mode"] == 1 and pl["n_items"] <= n_cu
        tile_bytes = 64 * spec.G * 4
        assert need == 256 + max(pl["k_parts"], plt["k_parts"]) * pl["n_row_blocks"] * wt.info["T"] * tile_bytes
    A = _device_A(tw, w.A, dtype)
    C = torch.full((M, spec.N), float("nan"), dtype=A.dtype, device="cuda:0")
    tw.tw_gemm(wt, A, C)
    torch.cuda.synchronize()
    assert wt.workspace.numel() == need
    err = _compare_whole(C, w.A, w.B, w.mask, dtype, what=spec.name)
    assert wt.workspace.view(torch.int32)[:4].cpu().tolist() == [0, 0, 0, 0]
    for _ in range(3):
        assert torch.equal(C, tw.tw_gemm(wt, A)), "two calls of a split-K plan differ in some bit"
    # transposed boundary
    At = _device_At(tw, w.A, dtype)
    Ct = tw.tw_gemm_t(wt, At)
    torch.cuda.synchronize()
    errt = _compare_whole(Ct, w.A, w.B, w.mask, dtype, transposed=True, what=spec.name + " transposed")
    assert torch.equal(Ct, tw.tw_gemm_t(wt, At))
    # fused bias + GELU in the second kernel's epilogue, both boundaries
    bbits = _bias_bits(spec.N, dtype, 77 + M)
    bias = tw.bits_to_tensor(bbits, dtype)
    bias64 = tw_ref.decode(bbits, dtype)
    post = lambda ref: tw_ref.bias_act(ref, bias64, "gelu")
    Cf = tw.tw_gemm_bias_act(wt, A, bias, "gelu")
    Cft = tw.tw_gemm_t_bias_act(wt, At, bias, "gelu")
    torch.cuda.synchronize()
    _compare_whole(Cf, w.A, w.B, w.mask, dtype, what=spec.name + " gelu", post=post)
    _compare_whole(Cft, w.A, w.B, w.mask, dtype, transposed=True, what=spec.name + " gelu transposed", post=post)
    # too little workspace for the parts: the unsplit plan, same tolerance
    wu = tw.TwWeight(wt.blob)
    wu.ws_limit = 4096
    Cu = tw.tw_gemm(wu, A)
    torch.cuda.synchronize()
    assert wu.workspace.numel() <= 4096
    _compare_whole(Cu, w.A, w.B, w.mask, dtype, what=spec.name + " small workspace")
    # the hybrid: residual weights inside the tiles' columns (added per chunk by the part that holds the chunk)
    # and in pruned columns (transposed: the pass of their own runs behind the second kernel; row-major: the
    # tiles add them themselves, which takes an unsplit plan)
    ew = tw.tw_restore_ew(w.B, w.mask, 0.01, dtype)
    union = (w.mask | ew).astype(np.uint8)
    wte = tw.TwWeight(tw.tw_pack_tew(w.B, w.mask, ew, spec.G, dtype))
    Ce = tw.tw_gemm(wte, A)
    Cet = tw.tw_gemm_t(wte, At)
    torch.cuda.synchronize()
    assert wte.info["ew_nnz"] > 0 and tw.tw_gemm_plan(wte.blob, M, n_cu=n_cu, transposed=True)["k_parts"] == plt["k_parts"]
    assert tw.tw_gemm_plan(wte.blob, M, n_cu=n_cu)["k_parts"] == 1
    _compare_whole(Ce, w.A, w.B, union, dtype, what=spec.name + " TEW")
    _compare_whole(Cet, w.A, w.B, union, dtype, transposed=True, what=spec.name + " TEW transposed")
    _say(f"split K {spec.name}: rel err {err:.3e} / transposed {errt:.3e}")
    torch.cuda.empty_cache()


@pytest.mark.parametrize("K", [300, 1536, 1700], ids=["k_resident", "k_resident_no_lds_left", "k_streamed_ragged_chunk"])
def test_tew_many_residual_only_columns_per_tile_bit_exact(tw, K):
    """Tiles whose spans hold more residual-only columns than a tile adds itself (16): the first 16 leave with the
    tile's stores (row-major: through the staging window; transposed: in place of the lines of zeros), the others
    in the pass of their own; with a residual inside the kept columns as well, K resident and streamed (five
    chunks, the last one ragged; the columns' sums then wait in LDS between chunks); several row blocks with a
    ragged last one; integers, bit for bit, both boundaries and the fused epilogue.  K = 1536 is the largest resident K:
    its LDS copy of A leaves no room for the waves' areas for these columns, so all of them take the pass of their own."""
    spec = W.small_spec(f"xcols_many_{K}", M=205, K=K, N=300, G=64, dtype="f16", col_prune=0.45, keep=("upow", 0.1, 0.5),
                        a_dist="smallint", seed_offset=4242)
    w = W.generate(spec)
    rng = np.random.default_rng(17)
    alive = w.mask.any(axis=0)
    pruned = np.flatnonzero(~alive)
    ew = np.zeros_like(w.mask)
    for n in pruned:
        ew[rng.choice(spec.K, size=int(rng.integers(1, 12)), replace=False), n] = 1
    kept_res = (rng.random(w.mask.shape) < 0.02) & (w.mask == 0) & alive[None, :]
    ew |= kept_res.astype(np.uint8)
    wt = tw.TwWeight(tw.tw_pack_tew(w.B, w.mask, ew, spec.G, "f16"))
    span = wt.info["tile_span"]
    per_tile = np.histogram(pruned, bins=span)[0]
    assert per_tile.max() > 16 and wt.info["ew_nnz"] == int(ew.sum())
    pl, plt = tw.tw_gemm_plan(wt.blob, spec.M), tw.tw_gemm_plan(wt.blob, spec.M, transposed=True)
    _say(f"{spec.name}: residual-only columns per tile {per_tile.tolist()}, plan {pl} / {plt}")
    assert (pl["mode"] == 0) == (K <= 1536) and pl["k_parts"] == 1
    if K == 1536:
        assert pl["lds_bytes"] + 8 * 16 * 64 * 2 > 160 * 1024      # no room for eight waves x 16 columns x 64 rows
    bias_i = rng.integers(-5, 6, size=spec.N).astype(np.float32)
    bias = tw.bits_to_tensor(W.f32_to_bits(bias_i, "f16"), "f16")
    A, At = _device_A(tw, w.A, "f16"), _device_At(tw, w.A, "f16")
    ref = tw_ref.masked_gemm(w.A, w.B, (w.mask | ew).astype(np.uint8), "f16")
    ref_r = tw_ref.bias_act(ref, bias_i.astype(np.float64), "relu")
    C, Ct = tw.tw_gemm(wt, A), tw.tw_gemm_t(wt, At)
    Cf, Cft = tw.tw_gemm_bias_act(wt, A, bias, "relu"), tw.tw_gemm_t_bias_act(wt, At, bias, "relu")
    torch.cuda.synchronize()
    assert np.abs(ref).max() < 2048                      # fp16 holds every result exactly
    assert np.array_equal(_to_f64(C), ref) and np.array_equal(_to_f64(Ct).T, ref)
    assert np.array_equal(_to_f64(Cf), ref_r) and np.array_equal(_to_f64(Cft).T, ref_r)
    assert np.any(ref[:, pruned] != 0)


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_tew_random_shapes_bit_exact(tw, seed):
    """Seeded random hybrids (shape, granularity, dtype, share of pruned columns, share of restored weights; every
    third one with residual weights in ALL pruned columns), integer data: tw_unpack gives the union back, and both
    boundaries with and without the fused epilogue equal the oracle bit for bit.  Cases whose results an output
    element cannot hold exactly are skipped."""
    rng = np.random.default_rng(1000 + seed)
    checked = 0
    for case in range(16):
        G = int(rng.choice([32, 64, 128]))
        K = int(rng.choice([40, 200, 520, 1000, 1536, 1544, 1704, 2400]))
        N = int(rng.integers(G, 5 * G + 40))
        M = int(rng.choice([1, 31, 64, 100, 200, 333, 700, 1500]))
        dtype = str(rng.choice(["f16", "bf16"]))
        cp = float(rng.choice([0.0, 0.1, 0.3, 0.5]))
        delta = float(rng.choice([0.005, 0.02, 0.05]))
        spec = W.small_spec(f"tew_random_{seed}_{case}", M=M, K=K, N=N, G=G, dtype=dtype, col_prune=cp,
                            keep=("upow", 0.05, 0.5), a_dist="smallint", seed_offset=60000 + 100 * seed + case)
        w = W.generate(spec)
        ew = tw.tw_restore_ew(w.B, w.mask, delta, dtype)
        if case % 3 == 0:
            for n in np.flatnonzero(~w.mask.any(axis=0)):
                ew[rng.choice(K, size=int(rng.integers(1, 9)), replace=False), n] = 1
        _say(f"TEW random {seed}/{case}: M={M} K={K} N={N} G={G} {dtype} col_prune={cp} delta={delta} residual {int(ew.sum())}")
        wt = tw.TwWeight(tw.tw_pack_tew(w.B, w.mask, ew, G, dtype))
        union = (w.mask | ew).astype(np.uint8)
        Bu, mu = tw.tw_unpack(wt.blob)
        assert np.array_equal(mu, union) and np.array_equal(Bu, tw_ref.masked_weight_bits(w.B, union))
        bias_i = rng.integers(-3, 4, size=N).astype(np.float32)
        ref = tw_ref.masked_gemm(w.A, w.B, union, dtype)
        ref_r = tw_ref.bias_act(ref, bias_i.astype(np.float64), "relu")
        if max(np.abs(ref).max(), np.abs(ref_r).max()) >= (2048 if dtype == "f16" else 256):
            continue
        A, At = _device_A(tw, w.A, dtype), _device_At(tw, w.A, dtype)
        bias = tw.bits_to_tensor(W.f32_to_bits(bias_i, dtype), dtype)
        C, Ct = tw.tw_gemm(wt, A), tw.tw_gemm_t(wt, At)
        Cf, Cft = tw.tw_gemm_bias_act(wt, A, bias, "relu"), tw.tw_gemm_t_bias_act(wt, At, bias, "relu")
        torch.cuda.synchronize()
        assert np.array_equal(_to_f64(C), ref) and np.array_equal(_to_f64(Ct).T, ref), (seed, case)
        assert np.array_equal(_to_f64(Cf), ref_r) and np.array_equal(_to_f64(Cft).T, ref_r), (seed, case)
        checked += 1
    assert checked >= 6


def test_tew_residual_only_in_pruned_columns_bit_exact(tw):
    """A weight whose tile-wise pattern is EMPTY plus a residual (every column is of the kind that runs in the
    pass of its own), and one whose residual lies only in the pruned columns; integers, bit for bit, both boundaries
    and the fused epilogue (a pruned column then holds act(bias + its residual's product))."""
    spec = W.small_spec("xcols", M=333, K=300, N=200, G=64, dtype="f16", col_prune=0.2, keep=("upow", 0.1, 0.5),
                        a_dist="smallint", seed_offset=12345)
    w = W.generate(spec)
    rng = np.random.default_rng(9)
    pruned = np.flatnonzero(~w.mask.any(axis=0))
    ew = np.zeros_like(w.mask)
    for n in pruned[::2]:
        ew[rng.choice(spec.K, size=int(rng.integers(1, 12)), replace=False), n] = 1
    bias_i = rng.integers(-5, 6, size=spec.N).astype(np.float32)
    bbits = W.f32_to_bits(bias_i, "f16")
    A, At = _device_A(tw, w.A, "f16"), _device_At(tw, w.A, "f16")
    for mask in (w.mask, np.zeros_like(w.mask)):
        wt = tw.TwWeight(tw.tw_pack_tew(w.B, mask, ew, spec.G, "f16"))
        assert wt.info["ew_nnz"] == int(ew.sum())
        ref = tw_ref.masked_gemm(w.A, w.B, (mask | ew).astype(np.uint8), "f16")
        C = tw.tw_gemm(wt, A)
        Ct = tw.tw_gemm_t(wt, At)
        Cf = tw.tw_gemm_bias_act(wt, A, tw.bits_to_tensor(bbits, "f16"), "relu")
        Cft = tw.tw_gemm_t_bias_act(wt, At, tw.bits_to_tensor(bbits, "f16"), "relu")
        torch.cuda.synchronize()
        assert np.array_equal(_to_f64(C), ref)
        assert np.array_equal(_to_f64(Ct).T, ref)
        ref_r = tw_ref.bias_act(ref, bias_i.astype(np.float64), "relu")
        assert np.array_equal(_to_f64(Cf), ref_r)
        assert np.array_equal(_to_f64(Cft).T, ref_r)
        assert np.any(ref[:, pruned[::2]] != 0)
