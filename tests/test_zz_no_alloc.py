"""tw_gemm_static: the entry point that allocates nothing and takes no workspace (the scheduler's counters and the
partial results of split-K plans live in a device array of the library).  Called through the C ABI on two inputs in
a row, the second smaller than the first, and held to the oracle at the parity tolerance and to tw_gemm's output
bit for bit (tw_gemm on a workspace of the array's size plans the same kernels)."""
import numpy as np
import pytest
import torch

from oracle import tw_ref
from paper_2008_13006_amd import workloads as W

pytestmark = pytest.mark.gpu
TOL = {"f16": 2e-3, "bf16": 1e-2}


def _case(tw, name, M, K, N, G, dtype, seed):
    spec = W.small_spec(name, M=M, K=K, N=N, G=G, dtype=dtype, col_prune=0.06, keep=("upow", 0.1, 0.6), seed_offset=seed)
    w = W.generate(spec)
    wt = tw.TwWeight.from_dense(w.B, w.mask, G, dtype)
    wt.ws_limit = tw.TW_STATIC_SCRATCH_BYTES        # tw_gemm then plans what tw_gemm_static plans
    A = tw.bits_to_tensor(w.A, dtype)
    return w, wt, A


def test_tw_gemm_static_two_calls_in_a_row():
    assert torch.cuda.is_available(), "this test needs the MI355X"
    from paper_2008_13006_amd import binding as tw
    # first call: more work items than compute units with 64-row blocks (the counters are used: 300 row blocks);
    # second call: a smaller input on the same GPU's array, which still holds what the first call left
    big = _case(tw, "static_big", 19200, 512, 640, 128, "f16", 13001)
    small = _case(tw, "static_small", 700, 320, 200, 64, "f16", 13002)
    outs = []
    for w, wt, A in (big, small):
        C = torch.full((A.shape[0], w.spec.N), float("nan"), dtype=A.dtype, device="cuda:0")
        before = torch.cuda.memory_allocated()
        tw.tw_gemm_static(wt, A, C)
        assert torch.cuda.memory_allocated() == before
        outs.append(C)
    torch.cuda.synchronize()
    for (w, wt, A), C in zip((big, small), outs):
        spec = w.spec
        ref = tw_ref.masked_gemm(w.A, w.B, w.mask, spec.dtype)
        got = C.to(torch.float64).cpu().numpy()
        assert np.isfinite(got).all(), "some element of C was not written"
        err = float(np.max(np.abs(got - ref)) / np.max(np.abs(ref)))
        print(f"[case] tw_gemm_static {spec.name}: rel err {err:.3e}", flush=True)
        assert err <= TOL[spec.dtype]
        Cw = tw.tw_gemm(wt, A)                       # the existing entry point on the caller's workspace
        torch.cuda.synchronize()
        assert torch.equal(C, Cw), "tw_gemm_static and tw_gemm differ in some bit"
        ws = wt.workspace.view(torch.int32)[:4].cpu().tolist()
        assert ws[0] == 0 and ws[1] == 0
    # streamed-K weights and bf16 right behind, still the same array: few rows (a split-K plan: the array holds the
    # parts' partial results), then more rows than a split's partial results fit the array for (fewer parts)
    n_cu = torch.cuda.get_device_properties(0).multi_processor_count
    for name, M, K, N, G, seed in (("static_stream", 300, 2000, 260, 64, 13003), ("static_stream_big", 1000, 3096, 500, 128, 13005)):
        w, wt, A = _case(tw, name, M, K, N, G, "bf16", seed)
        full = tw.tw_gemm_plan(wt.blob, M, n_cu=n_cu)
        print(f"[case] tw_gemm_static {name}: plan with a full workspace {full}, wants {tw.tw_gemm_workspace(wt.blob, M)} bytes", flush=True)
        if n_cu == 256:
            assert full["k_parts"] > 1
            assert (tw.tw_gemm_workspace(wt.blob, M) > tw.TW_STATIC_SCRATCH_BYTES) == (name == "static_stream_big")
        C = torch.full((M, N), float("nan"), dtype=A.dtype, device="cuda:0")
        before = torch.cuda.memory_allocated()
        tw.tw_gemm_static(wt, A, C)
        assert torch.cuda.memory_allocated() == before
        torch.cuda.synchronize()
        ref = tw_ref.masked_gemm(w.A, w.B, w.mask, "bf16")
        got = C.to(torch.float64).cpu().numpy()
        assert np.isfinite(got).all(), "some element of C was not written"
        assert float(np.max(np.abs(got - ref)) / np.max(np.abs(ref))) <= TOL["bf16"]
        assert torch.equal(C, tw.tw_gemm(wt, A))


def test_tw_gemm_static_refuses_what_tw_gemm_refuses():
    from paper_2008_13006_amd import binding as tw
    import ctypes
    w, wt, A = _case(tw, "static_err", 64, 64, 64, 32, "f16", 13004)
    C = torch.empty((64, 64), dtype=A.dtype, device="cuda:0")
    lib = tw._lib
    vp = ctypes.c_void_p
    blob, bd = vp(wt.blob.ctypes.data), vp(wt.blob_dev.data_ptr())
    assert lib.tw_gemm_static(blob, bd, vp(A.data_ptr()), 64, 60, vp(C.data_ptr()), 64, None) == -1      # lda < K
    assert lib.tw_gemm_static(blob, bd, None, 64, 64, vp(C.data_ptr()), 64, None) == -1                   # null A
    assert lib.tw_gemm_static(blob, bd, vp(A.data_ptr() + 2), 64, 64, vp(C.data_ptr()), 64, None) == -4   # alignment
    assert lib.tw_gemm_static(vp(C.data_ptr() * 0), bd, vp(A.data_ptr()), 64, 64, vp(C.data_ptr()), 64, None) == -1
    assert lib.tw_gemm_static(blob, bd, vp(A.data_ptr()), 0, 64, vp(C.data_ptr()), 64, None) == 0         # M = 0: nothing
    torch.cuda.synchronize()
