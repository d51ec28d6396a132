#!/usr/bin/env python3
"""Benchmark of the TW-sparse GEMM hot path on one MI355X.

A "step" is one tw_gemm launch on the BERT-base FFN-up workload (M=16384 tokens, K=768, N=3072,
fp16, G=128, 75 % tile-wise sparsity, 5 % of columns pruned), inputs resident in HBM.  The packer
runs once before the timed region (the paper packs offline, Sec. VI "Tiling"); its time is reported
separately.  The timed launches rotate over several (A, C) buffer sets that together exceed the
256 MB last-level cache, so `value` is the cold-cache time (`--report` also gives the warm time).
Every tw_gemm launch of the default run is such a cold launch, so a kernel trace of the same command
averages the same population that `value` does.

Prints ONE JSON line on stdout.  `--report FILE` additionally writes a per-GEMM table for all five
workloads (time, nonzero TFLOP/s, bytes/s, dense time, speedup) to FILE.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X published HBM3E bandwidth
MFMA_PEAK_TFLOPS = 2500.0    # dense fp16/bf16 MFMA
# HBM bytes per launch on this workload come from the two rocprofv3 --pmc runs (FETCH_SIZE, then WRITE_SIZE)
# summarised in these files, each counter scaled by what it reads for the copy kernel of known size that
# `--pmc-calibration` launches.  A summary names the kernel sources it was measured on (`source_sha256:`); if the
# sources in this tree are different ones, the figure is stale and `traffic` is reported as null.
TRAFFIC_FILES = {False: os.path.join(ROOT, "profiles", "tw_gemm_c2_hbm_traffic.txt"),
                 True: os.path.join(ROOT, "profiles", "tw_gemm_t_c2_hbm_traffic.txt")}
KERNEL_SOURCES = ["paper_2008_13006_amd/csrc/tw_gemm.hip", "paper_2008_13006_amd/csrc/tw_device.hpp",
                  "paper_2008_13006_amd/csrc/tw_format.h", "paper_2008_13006_amd/csrc/tw_pack.cpp"]
PAPER_CONTEXT = {"tw128_speedup_vs_dense_75pct": 2.26, "hardware": "NVIDIA V100 tensor cores, FP16",
                 "where": "Sec. VII-B, Fig. 8b"}


def kernel_source_hash() -> str:
    """sha256 over the sources of the TW kernel and the packer (what decides the kernel's memory traffic)."""
    import hashlib
    h = hashlib.sha256()
    for rel in KERNEL_SOURCES:
        with open(os.path.join(ROOT, rel), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def measured_traffic(transposed: bool):
    """(bytes per launch, note) from the counter summary under profiles/, or (None, why) if it was measured on
    other sources than the ones in this tree."""
    path = TRAFFIC_FILES[transposed]
    try:
        text = open(path).read()
    except OSError:
        return None, f"{os.path.relpath(path, ROOT)} missing"
    fields = {}
    for line in text.splitlines():
        if ":" in line:
            k, v = line.split(":", 1)
            fields[k.strip()] = v.strip()
    if fields.get("source_sha256") != kernel_source_hash():
        return None, f"{os.path.relpath(path, ROOT)} was measured on other kernel sources (stale)"
    try:
        return int(fields["traffic_bytes_per_launch"]), os.path.relpath(path, ROOT)
    except (KeyError, ValueError):
        return None, f"{os.path.relpath(path, ROOT)} has no traffic_bytes_per_launch line"


def algorithmic_bytes(info: dict, M: int) -> int:
    """Bytes the method itself must move per launch: A once, the compacted tiles and their kept-row
    lists once, C once (16-bit elements, 4-byte indices)."""
    sum_kt = int(info["tile_row_ptr"][-1]) if info["T"] > 0 else 0
    return 2 * M * info["K"] + 2 * int(info["nnz"]) + 4 * sum_kt + 2 * M * info["N"]


def time_launches(torch, fn, n_sets: int, steps: int, warmup: int):
    """Average duration of `steps` back-to-back launches, by HIP events on the launch stream."""
    for i in range(warmup):
        fn(i % n_sets)
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for i in range(steps):
        fn(i % n_sets)
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    return e0.elapsed_time(e1) / steps, wall_ms / steps


def per_launch_stats(torch, fn, n_sets: int, steps: int):
    """Individually bracketed launches: median / min in ms."""
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    for i, (a, b) in enumerate(evs):
        a.record()
        fn(i % n_sets)
        b.record()
    torch.cuda.synchronize()
    ts = sorted(a.elapsed_time(b) for a, b in evs)
    return ts[len(ts) // 2], ts[0]


def bench_gemm(torch, tw, W, spec, steps: int, warmup: int, with_dense: bool = True, n_sets=None,
               with_warm: bool = False, with_steady: bool = False, settle: int = 0, with_unsplit: bool = False):
    w = W.generate(spec)
    t0 = time.perf_counter()
    blob = tw.tw_pack(w.B, w.mask, spec.G, spec.dtype)
    pack_ms = (time.perf_counter() - t0) * 1e3
    wt = tw.TwWeight(blob)
    info = wt.info
    M = spec.M
    td = torch.float16 if spec.dtype == "f16" else torch.bfloat16
    set_bytes = 2 * M * (spec.K + spec.N)
    if n_sets is None:
        n_sets = max(3, -(-320 * 2 ** 20 // set_bytes))       # > 256 MB in rotation
    A0 = tw.bits_to_tensor(w.A, spec.dtype)
    As = [A0] + [A0.clone() for _ in range(n_sets - 1)]
    Cs = [torch.empty((M, spec.N), dtype=td, device="cuda:0") for _ in range(n_sets)]
    Bd = tw.bits_to_tensor(w.B, spec.dtype)

    # Clocks and queues settle during the first few hundred launches of a process (the same launch is 10 % slower
    # before): they are spent here, untimed, before the warm-up steps and the timed steps that the caller asked for.
    for i in range(settle):
        tw.tw_gemm(wt, As[i % n_sets], Cs[i % n_sets])
    torch.cuda.synchronize()
    cold_ms, cold_wall = time_launches(torch, lambda i: tw.tw_gemm(wt, As[i], Cs[i]), n_sets, steps, warmup)
    warm_ms = None
    if with_warm:     # same buffers every launch: A and part of C stay in the last-level cache
        warm_ms, _ = time_launches(torch, lambda i: tw.tw_gemm(wt, As[0], Cs[0]), 1, steps, warmup)
    med_ms, min_ms = per_launch_stats(torch, lambda i: tw.tw_gemm(wt, As[i], Cs[i]), n_sets, min(steps, 50))
    steady_ms = None
    if with_steady:   # whatever --steps says: 200 launches after 50 warm-ups, clocks and queues settled
        steady_ms, _ = time_launches(torch, lambda i: tw.tw_gemm(wt, As[i], Cs[i]), n_sets, 200, 50)
    # the same product on the transposed boundary (At in, Ct out): same algorithmic bytes
    Ats = [tw.tw_transpose(a).contiguous() for a in As]
    Cts = [torch.empty((spec.N, M), dtype=td, device="cuda:0") for _ in range(n_sets)]
    t_ms, _ = time_launches(torch, lambda i: tw.tw_gemm_t(wt, Ats[i], Cts[i]), n_sets, steps, warmup)
    del Ats, Cts
    out = dict(name=spec.name, M=M, K=spec.K, N=spec.N, G=spec.G, dtype=spec.dtype, T=int(info["T"]),
               sparsity=w.info["sparsity"], tw_ms=cold_ms, tw_ms_warm=warm_ms, tw_ms_median=med_ms,
               tw_ms_min=min_ms, tw_wall_ms=cold_wall, pack_ms=pack_ms, n_buffer_sets=n_sets, tw_t_ms=t_ms,
               tw_ms_steady=steady_ms)
    if with_unsplit:  # the same launches with the counters' 256 bytes of workspace only: no split-K plan
        wu = tw.TwWeight(blob)
        wu.ws_limit = 256
        u_ms, _ = time_launches(torch, lambda i: tw.tw_gemm(wu, As[i], Cs[i]), n_sets, steps, warmup)
        n_cu = torch.cuda.get_device_properties(0).multi_processor_count
        out.update(tw_ms_unsplit=u_ms, plan=tw.tw_gemm_plan(blob, M, n_cu=n_cu),
                   plan_t=tw.tw_gemm_plan(blob, M, n_cu=n_cu, transposed=True), workspace_bytes=tw.tw_gemm_workspace(blob, M))
    nz_flops = W.nonzero_flops(w.mask, M)
    dense_flops = 2.0 * M * spec.K * spec.N
    abytes = algorithmic_bytes(info, M)
    out.update(nonzero_gflop=nz_flops / 1e9, tw_tflops_nonzero=nz_flops / (cold_ms * 1e-3) / 1e12,
               tw_mfma_frac_nonzero=nz_flops / (cold_ms * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS,
               padded_mfma_frac=2.0 * M * int(info["padded_macs_per_row"]) / (cold_ms * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS,
               algorithmic_bytes=abytes, tw_gbs=abytes / (cold_ms * 1e-3) / 1e9,
               tw_hbm_frac=abytes / (cold_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
               tw_t_gbs=abytes / (t_ms * 1e-3) / 1e9, tw_t_hbm_frac=abytes / (t_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
               tw_t_tflops_nonzero=nz_flops / (t_ms * 1e-3) / 1e12)
    if with_dense:
        d_ms, _ = time_launches(torch, lambda i: tw.tw_dense_gemm(As[i], Bd, Cs[i]), n_sets, steps, warmup)
        out.update(dense_ms=d_ms, dense_tflops=dense_flops / (d_ms * 1e-3) / 1e12,
                   dense_mfma_frac=dense_flops / (d_ms * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS,
                   speedup_vs_dense=d_ms / cold_ms)
        # context only: the vendor library's dense GEMM through torch
        t_ms, _ = time_launches(torch, lambda i: torch.matmul(As[i], Bd, out=Cs[i]), n_sets, steps, warmup)
        out.update(torch_matmul_ms=t_ms, speedup_vs_vendor_dense=t_ms / cold_ms)
    return out, w, info


def cpu_baseline(W, w, spec, budget_s: float = 15.0):
    """The oracle as it stands, timed on the host cores on a bounded sample of the same workload."""
    import numpy as np
    from oracle import tw_ref
    cal_rows = min(128, spec.M)
    t0 = time.perf_counter()
    tw_ref.masked_gemm(np.ascontiguousarray(w.A[:cal_rows]), w.B, w.mask, spec.dtype)
    cal = time.perf_counter() - t0
    rows = int(min(spec.M, max(cal_rows, budget_s / max(cal, 1e-6) * cal_rows)))
    rows = max(8, rows // 8 * 8)
    t0 = time.perf_counter()
    tw_ref.masked_gemm(np.ascontiguousarray(w.A[:rows]), w.B, w.mask, spec.dtype)
    dt = time.perf_counter() - t0
    full_ms = dt / rows * spec.M * 1e3
    return {"value": full_ms, "unit": "ms", "cores": tw_ref.num_threads(), "kind": "oracle",
            "sample": f"first {rows} of {spec.M} rows of A in {dt:.2f} s (fp64 masked triple loop, OpenMP), "
                      f"scaled to all rows"}


def pmc_calibration(torch, tw, W, spec, steps: int, transposed: bool = False) -> int:
    """What a hardware-counter run profiles: a plain copy kernel that reads and writes COPY_BYTES each
    (an elementwise pass over int32, larger than the last-level cache), then `steps` tw_gemm launches
    over rotating buffers.  The copy's known size turns counter units into bytes."""
    COPY_BYTES = 512 * 2 ** 20
    src = torch.arange(COPY_BYTES // 4, dtype=torch.int32, device="cuda:0")
    dst = torch.empty_like(src)
    for _ in range(5):
        torch.add(src, 0, out=dst)
    torch.cuda.synchronize()
    w = W.generate(spec)
    wt = tw.TwWeight(tw.tw_pack(w.B, w.mask, spec.G, spec.dtype))
    td = torch.float16 if spec.dtype == "f16" else torch.bfloat16
    n_sets = 4
    A0 = tw.bits_to_tensor(w.A, spec.dtype)
    As = [A0] + [A0.clone() for _ in range(n_sets - 1)]
    Cs = [torch.empty((spec.M, spec.N), dtype=td, device="cuda:0") for _ in range(n_sets)]
    if transposed:
        Ats = [tw.tw_transpose(a).contiguous() for a in As]
        Cts = [torch.empty((spec.N, spec.M), dtype=td, device="cuda:0") for _ in range(n_sets)]
        torch.cuda.synchronize()
        for i in range(steps):
            tw.tw_gemm_t(wt, Ats[i % n_sets], Cts[i % n_sets])
    else:
        for i in range(steps):
            tw.tw_gemm(wt, As[i % n_sets], Cs[i % n_sets])
    torch.cuda.synchronize()
    print(json.dumps({"pmc_calibration": {"copy_kernel_reads_bytes": COPY_BYTES, "copy_kernel_writes_bytes": COPY_BYTES,
                                          "copy_launches": 5, "tw_gemm_launches": steps,
                                          "algorithmic_bytes_per_launch": algorithmic_bytes(wt.info, spec.M)}}))
    return 0


def pmc_sweep(torch, tw, W, reps: int = 3) -> int:
    """What the counter runs of the sparsity sweep profile (the paper's Fig. 10 on this chip: memory requests
    and matrix-unit work against sparsity, normalised to dense): on the FFN-up shape with G = 128, `reps` launches
    each of tw_dense_gemm (first), then per sparsity of tw_gemm and of tw_gemm_t, in this order.  Prints the order."""
    order = []
    spec0 = W.sweep_spec(128, 0.0)
    w0 = W.generate(spec0)
    td = torch.float16
    A = tw.bits_to_tensor(w0.A, spec0.dtype)
    At = tw.tw_transpose(A).contiguous()
    Bd = tw.bits_to_tensor(w0.B, spec0.dtype)
    C = torch.empty((spec0.M, spec0.N), dtype=td, device="cuda:0")
    Ct = torch.empty((spec0.N, spec0.M), dtype=td, device="cuda:0")
    torch.cuda.synchronize()
    for _ in range(reps):
        tw.tw_dense_gemm(A, Bd, C)
    order.append({"kernel": "tw_dense_gemm", "sparsity": 0.0, "launches": reps})
    for sp in (0.0, 0.25, 0.5, 0.75, 0.875, 0.95, 0.99):
        spec = W.sweep_spec(128, sp)
        w = W.generate(spec)
        wt = tw.TwWeight(tw.tw_pack(w.B, w.mask, spec.G, spec.dtype))
        for _ in range(reps):
            tw.tw_gemm(wt, A, C)
        for _ in range(reps):
            tw.tw_gemm_t(wt, At, Ct)
        torch.cuda.synchronize()
        order.append({"kernel": "tw_gemm then tw_gemm_t", "sparsity": float(w.info["sparsity"]), "launches": reps,
                      "nnz": int(wt.info["nnz"]), "T": int(wt.info["T"])})
    print(json.dumps({"pmc_sweep": order}))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--report", type=str, default=None, help="also time all five workloads, write a table here")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--sweep", type=str, default=None,
                    help="also run the sparsity x G sweep on the FFN-up shape, write a table (JSON) here")
    ap.add_argument("--transposed", action="store_true", help="with --pmc-calibration: launch tw_gemm_t instead of tw_gemm")
    ap.add_argument("--pmc-sweep", action="store_true", help="counter runs of the sparsity sweep (G = 128)")
    ap.add_argument("--source-hash", action="store_true", help="print the hash that the counter summaries record")
    ap.add_argument("--small-batch", type=int, default=0, metavar="M",
                    help="time only the FFN-down of BERT-base (K = 3072, streamed) on M rows: the split-K plan, the "
                         "unsplit plan and the dense GEMMs; prints its own JSON line")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="counter runs: launch only a copy kernel of known size, then the tw_gemm steps")
    args = ap.parse_args()
    if args.source_hash:
        print(kernel_source_hash())
        return 0
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (rows of A and C are independent, so the path would "
              "shard over M with no collective); re-run with --gpus 1", file=sys.stderr)
        return 2

    import torch
    from paper_2008_13006_amd import binding as tw
    from paper_2008_13006_amd import workloads as W
    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    torch.cuda.set_device(0)

    spec = W.CONFIGS["c2_bert_base_ffn_up"][0]
    if args.small_batch > 0:
        import dataclasses
        s_ = dataclasses.replace(W.CONFIGS["c3_bert_base_layer"][3], M=args.small_batch)
        r, _, _ = bench_gemm(torch, tw, W, s_, args.steps, args.warmup, n_sets=16, with_unsplit=True, settle=100)
        print(json.dumps({"workload": f"c3 {s_.name} at M={s_.M}", "tw_ms": r["tw_ms"], "tw_ms_unsplit": r["tw_ms_unsplit"],
                          "tw_t_ms": r["tw_t_ms"], "dense_ms": r["dense_ms"], "vendor_dense_ms": r["torch_matmul_ms"],
                          "plan": r["plan"], "plan_t": r["plan_t"], "workspace_bytes": r["workspace_bytes"]}), flush=True)
        return 0
    if args.pmc_sweep:
        return pmc_sweep(torch, tw, W)
    if args.pmc_calibration:
        return pmc_calibration(torch, tw, W, spec, args.steps, args.transposed)
    res, w, info = bench_gemm(torch, tw, W, spec, args.steps, args.warmup, with_steady=True, settle=400)
    traffic, traffic_note = measured_traffic(False)
    traffic_t, traffic_t_note = measured_traffic(True)
    line = {
        "metric": "tw_gemm_ms (TW-sparse GEMM time, BERT-base FFN-up, 75% tile-wise sparsity)",
        "value": res["tw_ms"], "unit": "ms", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": res["tw_ms"], "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "data": "synthetic",
        "config": {"workload": "c2_bert_base_ffn_up: M=16384 K=768 N=3072 fp16 G=128, 75% TW sparsity, "
                               "5% columns pruned, tiles 10-50% kept", "T": res["T"],
                   "sparsity": round(res["sparsity"], 4), "cache": f"cold: {res['n_buffer_sets']} rotating (A,C) sets"},
        "speedup_vs_dense": res["speedup_vs_dense"], "speedup_vs_vendor_dense": res["speedup_vs_vendor_dense"],
        "dense_ms": res["dense_ms"],
        "dense_tflops": res["dense_tflops"], "dense_mfma_frac": res["dense_mfma_frac"],
        "tw_tflops_nonzero": res["tw_tflops_nonzero"], "mfma_util_nonzero": res["tw_mfma_frac_nonzero"],
        "mfma_util_issued": res["padded_mfma_frac"],
        "tw_ms_median": res["tw_ms_median"], "tw_ms_min": res["tw_ms_min"], "tw_ms_steady": res["tw_ms_steady"],
        "torch_matmul_dense_ms_context": res["torch_matmul_ms"], "pack_ms_offline": res["pack_ms"],
        "roofline": {"bound": "hbm", "achieved": res["tw_gbs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": res["tw_hbm_frac"], "traffic": traffic, "traffic_source": traffic_note,
                     "frac_steady": res["algorithmic_bytes"] / (res["tw_ms_steady"] * 1e-3) / 1e9 / HBM_PEAK_GBS,
                     "kernel": "tw_gemm_kernel<f16, MS=2 (64 rows), NCB=4 (G=128), MODE 0 (K resident)>",
                     "algorithmic_bytes_per_launch": res["algorithmic_bytes"]},
        # the same GEMM through tw_gemm_t (activations and result transposed, the paper's layout): not `value`
        "transposed_boundary": {"tw_gemm_t_ms": res["tw_t_ms"], "speedup_vs_dense": res["dense_ms"] / res["tw_t_ms"],
                                "tflops_nonzero": res["tw_t_tflops_nonzero"],
                                "roofline": {"bound": "hbm", "achieved": res["tw_t_gbs"], "peak": HBM_PEAK_GBS,
                                             "unit": "GB/s", "frac": res["tw_t_hbm_frac"],
                                             "traffic": traffic_t, "traffic_source": traffic_t_note,
                                             "kernel": "tw_gemm_kernel<f16, MS=2 (64 tokens), NCB=4, MODE 0, transposed>"}},
        "paper_context": PAPER_CONTEXT,
    }
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(W, w, spec)
    if args.report:
        rows = []
        for cfg, specs in list(W.CONFIGS.items()) + [("c2_fixed_grid_mask", [W.C2_FIXED_GRID])]:
            for s in specs:
                r, _, _ = bench_gemm(torch, tw, W, s, max(20, args.steps // 4), 5, with_warm=True)
                r["config"] = cfg
                rows.append(r)
                print(f"[report] {cfg}/{s.name}: tw {r['tw_ms']*1e3:.1f} us  tw_t {r['tw_t_ms']*1e3:.1f} us  "
                      f"dense {r['dense_ms']*1e3:.1f} us  "
                      f"x{r['speedup_vs_dense']:.2f}  nz {r['tw_tflops_nonzero']:.0f} TF  {r['tw_gbs']:.0f} GB/s",
                      file=sys.stderr, flush=True)
                torch.cuda.empty_cache()
        # the fused epilogue on the headline workload: FFN-up with its bias and GELU inside the GEMM, against
        # the GEMM followed by a separate bias + GELU pass over C (torch's elementwise kernels)
        M, N = spec.M, spec.N
        td = torch.float16
        wt = tw.TwWeight(tw.tw_pack(w.B, w.mask, spec.G, spec.dtype))
        n_sets = 4
        A0 = tw.bits_to_tensor(w.A, spec.dtype)
        As = [A0] + [A0.clone() for _ in range(n_sets - 1)]
        Cs = [torch.empty((M, N), dtype=td, device="cuda:0") for _ in range(n_sets)]
        Bd = tw.bits_to_tensor(w.B, spec.dtype)
        bias = (torch.randn(N, device="cuda:0") * 0.5).to(td)
        gelu = torch.nn.functional.gelu
        st = max(20, args.steps // 4)
        fused_ms, _ = time_launches(torch, lambda i: tw.tw_gemm_bias_act(wt, As[i], bias, "gelu", Cs[i]), n_sets, st, 5)
        plain_ms, _ = time_launches(torch, lambda i: tw.tw_gemm(wt, As[i], Cs[i]), n_sets, st, 5)
        sep_ms, _ = time_launches(torch, lambda i: Cs[i].copy_(gelu(tw.tw_gemm(wt, As[i], Cs[i]) + bias)), n_sets, st, 5)
        dfused_ms, _ = time_launches(torch, lambda i: tw.tw_dense_gemm_bias_act(As[i], Bd, bias, "gelu", Cs[i]), n_sets, st, 5)
        rows.append({"config": "fused_epilogue_c2", "name": "ffn_up_768x3072 + bias + GELU", "tw_fused_ms": fused_ms,
                     "tw_plain_ms": plain_ms, "tw_then_separate_bias_gelu_ms": sep_ms, "dense_fused_ms": dfused_ms})
        print(f"[report] fused epilogue on c2: tw_gemm_bias_act(gelu) {fused_ms*1e3:.1f} us, tw_gemm {plain_ms*1e3:.1f} us, "
              f"tw_gemm + separate bias/GELU pass {sep_ms*1e3:.1f} us, tw_dense_gemm_bias_act {dfused_ms*1e3:.1f} us",
              file=sys.stderr, flush=True)
        # the TEW hybrid on the headline workload (the experiment of Sec. VII-B, Fig. 9, latency side): the
        # delta*K*N pruned weights of largest magnitude put back as an element-wise residual
        Ats = [tw.tw_transpose(a).contiguous() for a in As]
        Cts = [torch.empty((N, M), dtype=td, device="cuda:0") for _ in range(n_sets)]
        for delta in (0.0, 0.005, 0.01, 0.02, 0.05):
            ew = tw.tw_restore_ew(w.B, w.mask, delta, spec.dtype)
            wte = tw.TwWeight(tw.tw_pack_tew(w.B, w.mask, ew, spec.G, spec.dtype))
            a_ms, _ = time_launches(torch, lambda i: tw.tw_gemm(wte, As[i], Cs[i]), n_sets, st, 5)
            b_ms, _ = time_launches(torch, lambda i: tw.tw_gemm_t(wte, Ats[i], Cts[i]), n_sets, st, 5)
            rows.append({"config": "tew_c2", "name": f"ffn_up_768x3072 delta={delta}", "delta": delta,
                         "ew_nnz": int(wte.info["ew_nnz"]), "tw_ms": a_ms, "tw_t_ms": b_ms})
            print(f"[report] TEW on c2, delta {delta:.3f} ({int(wte.info['ew_nnz'])} residual weights): tw_gemm {a_ms*1e3:.1f} us, "
                  f"tw_gemm_t {b_ms*1e3:.1f} us", file=sys.stderr, flush=True)
        del Ats, Cts, As, Cs
        # the same with a streamed K: the FFN-down of BERT-base (K = 3072 in eight chunks)
        spec_d = W.CONFIGS["c3_bert_base_layer"][3]
        wd = W.generate(spec_d)
        Ad = [tw.bits_to_tensor(wd.A, spec_d.dtype)]
        Ad += [Ad[0].clone() for _ in range(n_sets - 1)]
        Adt = [tw.tw_transpose(a).contiguous() for a in Ad]
        Cd = [torch.empty((spec_d.M, spec_d.N), dtype=td, device="cuda:0") for _ in range(n_sets)]
        Cdt = [torch.empty((spec_d.N, spec_d.M), dtype=td, device="cuda:0") for _ in range(n_sets)]
        for delta in (0.0, 0.01):
            ew = tw.tw_restore_ew(wd.B, wd.mask, delta, spec_d.dtype)
            wte = tw.TwWeight(tw.tw_pack_tew(wd.B, wd.mask, ew, spec_d.G, spec_d.dtype))
            a_ms, _ = time_launches(torch, lambda i: tw.tw_gemm(wte, Ad[i], Cd[i]), n_sets, st, 5)
            b_ms, _ = time_launches(torch, lambda i: tw.tw_gemm_t(wte, Adt[i], Cdt[i]), n_sets, st, 5)
            rows.append({"config": "tew_ffn_down", "name": f"ffn_down_3072x768 delta={delta}", "delta": delta,
                         "ew_nnz": int(wte.info["ew_nnz"]), "tw_ms": a_ms, "tw_t_ms": b_ms})
            print(f"[report] TEW on the FFN-down of c3 (streamed K), delta {delta:.3f} ({int(wte.info['ew_nnz'])} residual weights): "
                  f"tw_gemm {a_ms*1e3:.1f} us, tw_gemm_t {b_ms*1e3:.1f} us", file=sys.stderr, flush=True)
        del Ad, Adt, Cd, Cdt
        # Few rows and a streamed K (the GEMMs with K > 1536 at serving batch sizes): split-K plans against the
        # unsplit plan and the dense GEMMs
        import dataclasses
        for cfg, idx in (("c3_bert_base_layer", 3), ("c4_bert_large_skewed", 1), ("c5_conv_im2col", 0)):
            for Ms in (64, 512, 2048):
                s_ = dataclasses.replace(W.CONFIGS[cfg][idx], M=Ms)
                r, _, _ = bench_gemm(torch, tw, W, s_, max(50, args.steps // 2), 10, n_sets=16, with_unsplit=True)
                r["config"] = "small_batch"
                r["of"] = cfg
                rows.append(r)
                print(f"[report] small batch {cfg}/{s_.name} M={Ms}: tw {r['tw_ms']*1e3:.1f} us (k_parts {r['plan']['k_parts']}, "
                      f"unsplit {r['tw_ms_unsplit']*1e3:.1f} us)  tw_t {r['tw_t_ms']*1e3:.1f} us  dense {r['dense_ms']*1e3:.1f} us  "
                      f"vendor dense {r['torch_matmul_ms']*1e3:.1f} us", file=sys.stderr, flush=True)
                torch.cuda.empty_cache()
        # The four weight GEMMs of a BERT-base layer chained on one stream (QKV, attention output on a strided view,
        # FFN-up with bias + GELU, FFN-down), launch by launch and as one HIP graph: at small M the launches bound it.
        for Ml in (512, 16384):
            lspecs = W.CONFIGS["c3_bert_base_layer"]
            lws = [W.generate(s_, M=Ml) for s_ in lspecs]
            lwt = [tw.TwWeight(tw.tw_pack(w_.B, w_.mask, s_.G, s_.dtype)) for w_, s_ in zip(lws, lspecs)]
            X = tw.bits_to_tensor(lws[0].A, lspecs[0].dtype)
            QKV = torch.empty((Ml, 2304), dtype=td, device="cuda:0")
            AO = torch.empty((Ml, 768), dtype=td, device="cuda:0")
            Hh = torch.empty((Ml, 3072), dtype=td, device="cuda:0")
            Y = torch.empty((Ml, 768), dtype=td, device="cuda:0")

            def chain():
                tw.tw_gemm(lwt[0], X, QKV)
                tw.tw_gemm(lwt[1], QKV[:, :768], AO)
                tw.tw_gemm_bias_act(lwt[2], AO, bias, "gelu", Hh)
                tw.tw_gemm(lwt[3], Hh, Y)

            chain()
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                chain()
            torch.cuda.synchronize()
            eager_ms, _ = time_launches(torch, lambda i: chain(), 1, st, 5)
            graph_ms, _ = time_launches(torch, lambda i: graph.replay(), 1, st, 5)
            rows.append({"config": "layer_chain", "name": f"bert_base_layer_M{Ml}", "M": Ml, "eager_ms": eager_ms,
                         "graph_ms": graph_ms})
            print(f"[report] BERT-base layer chain, M={Ml}: four launches {eager_ms*1e3:.1f} us, one HIP graph replay "
                  f"{graph_ms*1e3:.1f} us", file=sys.stderr, flush=True)
            del lwt, X, QKV, AO, Hh, Y, graph
            torch.cuda.empty_cache()
        with open(args.report, "w") as f:
            json.dump(rows, f, indent=1)
    if args.sweep:
        rows = []
        dense_ms = None
        for G in (32, 64, 128):
            for sp in (0.0, 0.25, 0.5, 0.625, 0.75, 0.875, 0.95, 0.99):
                spec_s = W.sweep_spec(G, sp)
                r, _, _ = bench_gemm(torch, tw, W, spec_s, max(20, args.steps // 4), 5, with_dense=dense_ms is None)
                if dense_ms is None:
                    dense_ms = r["dense_ms"]
                r["dense_ms"] = dense_ms
                r["speedup_vs_dense"] = dense_ms / r["tw_ms"]
                rows.append(r)
                print(f"[sweep] G={G:3d} sparsity {r['sparsity']:.3f} T={r['T']:3d}: tw {r['tw_ms']*1e3:6.1f} us  "
                      f"tw_t {r['tw_t_ms']*1e3:6.1f} us  "
                      f"x{r['speedup_vs_dense']:.2f} vs dense {dense_ms*1e3:.1f} us  nz {r['tw_tflops_nonzero']:.0f} TF "
                      f"({100*r['tw_mfma_frac_nonzero']:.1f} % of MFMA peak)  {r['tw_gbs']:.0f} GB/s", file=sys.stderr, flush=True)
                torch.cuda.empty_cache()
        with open(args.sweep, "w") as f:
            json.dump(rows, f, indent=1)
    print(json.dumps(line), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
