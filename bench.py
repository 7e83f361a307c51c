#!/usr/bin/env python3
"""Benchmark: bf16 GEMM 4096^3 (A row-major, B column-major, fp32 accumulate and output) on one
MI355X through the C ABI, with the int8 GEMM, batched-GEMM and convolution workloads timed
beside it, the MFMA roofline fraction of the dominant kernel, and the CPU oracle timed on the
host cores as a reported baseline.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--only-main] [--no-cpu]

A step is one xp_gemm call on inputs already resident in HBM.  One JSON line is printed.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

PEAK_BF16_TFLOPS = 2516.6     # 256 CU x 4096 FLOP/clk/CU x 2.4 GHz, dense
PEAK_INT8_TOPS = 5033.2
PEAK_HBM_GBS = 8000.0

# Bytes per launch between the L2s and the memory fabric, from rocprofv3 --pmc FETCH_SIZE and
# WRITE_SIZE runs scaled by a plain 256 MiB copy (factors 2.00 and 1.00), see
# profiles/dl_kernel_bf16_256x256_ring3a2b_asm_reads_gemm_4096.md (for the variants with compiler-issued reads
# profiles/dl_kernel_bf16_256x256_ring3a2b_mfma16_gemm_4096.md and, for the two-buffer variant,
# profiles/dl_kernel_bf16_256x256_mfma16_gemm_4096.md).  Keyed by kernel variant: a different
# kernel than the profiled ones reports null.
TRAFFIC_BYTES = {"bf16 256x256x128B waves 2x4 ring 3(A)+2(B) direct-to-lds, reads as assembly, mfma16": 268.7e6,
                 "bf16 256x256x128B waves 2x4 ring 3(A)+2(B) direct-to-lds mfma16": 268.7e6,
                 "bf16 256x256x128B waves 2x4 ring 2 direct-to-lds mfma16": 268.6e6}


def _time_calls(torch, fn, steps, warmup):
    """Average duration of one call in ms: HIP events on the stream the kernels are launched on."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    start = torch.cuda.Event(enable_timing=True)
    stop = torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    start.record()
    for _ in range(steps):
        fn()
    stop.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    return start.elapsed_time(stop) / steps, wall_ms / steps


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=500)
    ap.add_argument("--only-main", action="store_true", help="skip the int8 / batched / conv side measurements")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--force-variant", type=int, default=-1,
                    help="force this kernel variant index for the main workload (profiling a sweep candidate)")
    ap.add_argument("--force-batched-variant", type=int, default=-1,
                    help="force this kernel variant index for the two batched side workloads")
    ap.add_argument("--force-attention-variant", type=int, default=-1,
                    help="time this attention variant instead of the library's choice")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 256 MiB device-to-device copy (a known-size reference for "
                         "scaling the profiler's FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        return 2

    import torch
    from paper_2505_02146_amd import inputs, xp          # fails loudly if libxp.so is missing
    from tests.helpers import dev

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)

    # ---- main workload: bf16 GEMM 4096^3, NT
    w = inputs.workload("gemm_bf16_4096")
    M, N, K = w["M"], w["N"], w["K"]
    dA, dB = dev(w["A"].reshape(-1)), dev(w["B"].reshape(-1))
    dC = torch.empty((M, N), dtype=torch.float32, device="cuda")

    if args.force_variant >= 0:
        xp.xp_force_config(xp.XP_OP_GEMM, "bf16", args.force_variant)

    def step():
        xp.xp_gemm(M, N, K, 1.0, dA, "row", K, dB, "col", K, 0.0, dC, "row", N, a_type="bf16", b_type="bf16")

    ev_ms, wall_ms = _time_calls(torch, step, args.steps, args.warmup)
    flops = 2.0 * M * N * K
    tflops = flops / (ev_ms * 1e-3) / 1e12
    variant = xp.xp_describe_config(0, "bf16", xp.xp_last_config(0, "bf16"))

    out = {
        "metric": "bf16 GEMM TFLOP/s + % MFMA peak at 4096^3; int8 TOPS; conv TFLOP/s",
        "value": round(flops / (wall_ms * 1e-3) / 1e12, 2),
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(wall_ms, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "gemm_bf16_4096: M=N=K=4096, A row-major, B column-major, N(0,1) entries, "
                               "fp32 accumulate and output, alpha=1, beta=0", "kernel": variant},
        "pct_mfma_peak": round(100.0 * tflops / PEAK_BF16_TFLOPS, 2),
        "roofline": {"bound": "mfma", "achieved": round(tflops, 2), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(tflops / PEAK_BF16_TFLOPS, 4), "traffic": TRAFFIC_BYTES.get(variant),
                     "kernel_ms": round(ev_ms, 5)},
    }

    xp.xp_force_config(xp.XP_OP_GEMM, "bf16", -1)

    if args.calibrate_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- side measurements named by the metric
    if not args.only_main:
        side = {}
        steps2, warm2 = max(20, args.steps // 4), max(5, args.warmup // 4)
        del dA, dB, dC
        w8 = inputs.workload("gemm_i8_4096x4096x8192")
        a8, b8 = dev(w8["A"].reshape(-1)), dev(w8["B"].reshape(-1))
        c8 = torch.empty((4096, 4096), dtype=torch.int32, device="cuda")
        ms, _ = _time_calls(torch, lambda: xp.xp_gemm(4096, 4096, 8192, 1.0, a8, "row", 8192, b8, "col", 8192, 0.0,
                                                      c8, "row", 4096), steps2, warm2)
        tops = 2.0 * 4096 * 4096 * 8192 / (ms * 1e-3) / 1e12
        side["gemm_i8_4096x4096x8192"] = {"ms": round(ms, 5), "TOPS": round(tops, 1),
                                          "pct_int8_mfma_peak": round(100 * tops / PEAK_INT8_TOPS, 2),
                                          "kernel": xp.xp_describe_config(0, "i8", xp.xp_last_config(0, "i8"))}
        del a8, b8, c8
        wc = inputs.workload("conv_bf16_56")
        xin, fil = dev(wc["input"].reshape(-1)), dev(wc["filter"].reshape(-1))
        oc = torch.empty((32, 56, 56, 256), dtype=torch.float32, device="cuda")
        ms, _ = _time_calls(torch, lambda: xp.xp_conv2d_nhwc(32, 56, 56, 256, 256, 3, 3, 1, 1, 1, 1, xin, fil, "krsc",
                                                             oc, in_type="bf16", w_type="bf16"), steps2, warm2)
        tf = 2.0 * 32 * 56 * 56 * 256 * 9 * 256 / (ms * 1e-3) / 1e12
        side["conv_bf16_56"] = {"ms": round(ms, 5), "TFLOP/s": round(tf, 1),
                                "pct_bf16_mfma_peak": round(100 * tf / PEAK_BF16_TFLOPS, 2),
                                "kernel": xp.xp_describe_config(2, "bf16", xp.xp_last_config(2, "bf16"))}
        del xin, fil, oc
        for name, alg_bytes in (("bgemm_bf16_qk", 113.2e6), ("bgemm_bf16_pv", 69.2e6)):
            wb = inputs.workload(name)
            b, m, n, k = wb["batch"], wb["M"], wb["N"], wb["K"]
            lb = wb["b_layout"]
            ldb = n if lb == "row" else k
            # rotate through buffer sets larger than the 256 MB last-level cache: HBM-cold timing
            sets = max(2, int(600e6 // alg_bytes) + 1)
            As = [dev(wb["A"].reshape(-1)) for _ in range(sets)]
            Bs = [dev(wb["B"].reshape(-1)) for _ in range(sets)]
            Cs = [torch.empty((b, m, n), dtype=torch.float32, device="cuda") for _ in range(sets)]
            it = {"i": 0}

            def call():
                i = it["i"] % sets
                it["i"] += 1
                xp.xp_gemm_batched(b, m, n, k, 1.0, As[i], "row", k, m * k, Bs[i], lb, ldb, k * n, 0.0, Cs[i], "row", n,
                                   m * n, a_type="bf16", b_type="bf16")
            if args.force_batched_variant >= 0:
                xp.xp_force_config(xp.XP_OP_GEMM_BATCHED, "bf16", args.force_batched_variant)
            try:
                ms, _ = _time_calls(torch, call, steps2 * 2, warm2)
            except xp.XpError:                       # the forced variant does not serve this layout
                xp.xp_force_config(xp.XP_OP_GEMM_BATCHED, "bf16", -1)
                ms, _ = _time_calls(torch, call, steps2 * 2, warm2)
            finally:
                xp.xp_force_config(xp.XP_OP_GEMM_BATCHED, "bf16", -1)
            side[name] = {"ms": round(ms, 5), "TFLOP/s": round(2.0 * b * m * n * k / (ms * 1e-3) / 1e12, 1),
                          "GB/s": round(alg_bytes / (ms * 1e-3) / 1e9, 1),
                          "pct_hbm_peak": round(100 * alg_bytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 2),
                          "buffers": f"{sets} rotating sets (HBM-cold)",
                          "kernel": xp.xp_describe_config(1, "bf16", xp.xp_last_config(1, "bf16"))}
            del As, Bs, Cs
        # fused attention: the two batched stages with the row softmax between them, as one launch
        wa = inputs.workload("attention_bf16_512")
        b, L, d = wa["batch"], wa["Lq"], wa["d"]
        alg_bytes = 3 * b * L * d * 2 + b * L * d * 4        # Q, K, V read once, O written once
        sets = max(2, int(600e6 // alg_bytes) + 1)
        Qs, Ks, Vs = ([dev(wa[t].reshape(-1)) for _ in range(sets)] for t in ("Q", "K", "V"))
        Os = [torch.empty((b, L, d), dtype=torch.float32, device="cuda") for _ in range(sets)]
        it = {"i": 0}

        def call_attention():
            i = it["i"] % sets
            it["i"] += 1
            xp.xp_attention(b, L, L, d, d, wa["scale"], Qs[i], d, L * d, Ks[i], d, L * d, Vs[i], d, L * d, Os[i], d, L * d,
                            q_type="bf16", k_type="bf16", v_type="bf16")
        if args.force_attention_variant >= 0:
            xp.xp_force_config(xp.XP_OP_ATTENTION, "bf16", args.force_attention_variant)
        try:
            ms, _ = _time_calls(torch, call_attention, steps2 * 2, warm2)
        finally:
            xp.xp_force_config(xp.XP_OP_ATTENTION, "bf16", -1)
        unfused = side["bgemm_bf16_qk"]["ms"] + side["bgemm_bf16_pv"]["ms"]
        side["attention_bf16_512"] = {"ms": round(ms, 5), "TFLOP/s": round(4.0 * b * L * L * d / (ms * 1e-3) / 1e12, 1),
                                      "GB/s": round(alg_bytes / (ms * 1e-3) / 1e9, 1),
                                      "buffers": f"{sets} rotating sets (HBM-cold)",
                                      "vs_two_batched_gemm_stages_without_softmax": round(unfused / ms, 2),
                                      "kernel": xp.xp_describe_config(3, "bf16", xp.xp_last_config(3, "bf16"))}
        del Qs, Ks, Vs, Os
        # the same operator at a decoder block's shape: 32 heads of 128 over 2048 positions (compute-bound)
        w2 = inputs.workload("attention_bf16_2048_d128")
        b2, L2, d2 = w2["batch"], w2["Lq"], w2["d"]
        Q2, K2, V2 = dev(w2["Q"].reshape(-1)), dev(w2["K"].reshape(-1)), dev(w2["V"].reshape(-1))
        O2 = torch.empty((b2 * L2 * d2,), dtype=torch.float32, device="cuda")
        ms2, _ = _time_calls(torch, lambda: xp.xp_attention(b2, L2, L2, d2, d2, w2["scale"], Q2, d2, L2 * d2, K2, d2, L2 * d2, V2, d2,
                                                            L2 * d2, O2, d2, L2 * d2, q_type="bf16", k_type="bf16", v_type="bf16"),
                             steps2, warm2)
        side["attention_bf16_2048_d128"] = {"ms": round(ms2, 5), "TFLOP/s": round(4.0 * b2 * L2 * L2 * d2 / (ms2 * 1e-3) / 1e12, 1),
                                            "pct_bf16_mfma_peak": round(100 * 4.0 * b2 * L2 * L2 * d2 / (ms2 * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 2),
                                            "kernel": xp.xp_describe_config(3, "bf16", xp.xp_last_config(3, "bf16"))}
        del Q2, K2, V2, O2
        # matrix-vector product: one pass over a 134 MB matrix, HBM-cold by rotation
        wv = inputs.workload("gemv_bf16_8192")
        mv, kv = wv["M"], wv["K"]
        alg_bytes = mv * kv * 2 + kv * 2 + mv * 4
        sets = 5
        Av = [dev(wv["A"].reshape(-1)) for _ in range(sets)]
        xv = dev(wv["B"].reshape(-1))
        yv = torch.empty((mv,), dtype=torch.float32, device="cuda")
        it = {"i": 0}

        def call_gemv():
            i = it["i"] % sets
            it["i"] += 1
            xp.xp_gemm(mv, 1, kv, 1.0, Av[i], "row", kv, xv, "col", kv, 0.0, yv, "row", 1, a_type="bf16", b_type="bf16")
        ms, _ = _time_calls(torch, call_gemv, steps2 * 2, warm2)
        side["gemv_bf16_8192"] = {"ms": round(ms, 5), "GB/s": round(alg_bytes / (ms * 1e-3) / 1e9, 1),
                                  "pct_hbm_peak": round(100 * alg_bytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 2),
                                  "buffers": f"{sets} rotating matrices (HBM-cold)",
                                  "kernel": xp.xp_describe_config(0, "bf16", xp.xp_last_config(0, "bf16"))}
        del Av, xv, yv
        # the convolution workload with NCHW tensors: two layout-change passes in front of the same kernels
        torch.manual_seed(0)
        xn = torch.randn(32, 256, 56, 56, device="cuda").bfloat16()
        wn = (torch.randn(256, 256, 3, 3, device="cuda") / 48.0).bfloat16()
        on = torch.empty(32, 256, 56, 56, device="cuda")
        wsn = torch.empty(xp.xp_conv2d_nchw_workspace_bytes(32, 56, 56, 256, 256, 3, 3, 1, 1, 1, 1, "bf16"), dtype=torch.uint8, device="cuda")
        ms, _ = _time_calls(torch, lambda: xp.xp_conv2d_nchw(32, 56, 56, 256, 256, 3, 3, 1, 1, 1, 1, xn, wn, on, wsn), steps2, warm2)
        side["conv_bf16_56_nchw"] = {"ms": round(ms, 5), "TFLOP/s": round(2.0 * 32 * 56 * 56 * 256 * 9 * 256 / (ms * 1e-3) / 1e12, 1),
                                     "note": "input NCHW -> NHWC and filter KCRS -> KRSC passes included; the kernel writes NCHW directly"}
        del xn, wn, on, wsn
        # operators that are not contractions: achieved algorithmic bytes/s against the HBM peak, HBM-cold
        # (rotating buffer sets larger than the 256 MB last-level cache; workloads in opbench.py)
        from paper_2505_02146_amd import opbench
        mem = {}
        for op in opbench.BENCH_OPS:
            name, ms, nbytes, note = opbench.time_op(op, steps2 * 2, warm2)
            mem[name] = {"ms": round(ms, 5), "GB/s": round(nbytes / (ms * 1e-3) / 1e9, 1),
                         "pct_hbm_peak": round(100 * nbytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 2), "buffers": note}
        side["memory_bound"] = mem
        out["other_workloads"] = side

    # ---- CPU oracle on a bounded sample of the main workload (reported baseline, not the target)
    if not args.no_cpu:
        import oracle
        rows = M          # the whole job: about 4-10 s on 16 host cores
        a_sample = np.ascontiguousarray(w["A"][:rows]).reshape(-1)
        t0 = time.perf_counter()
        oracle.gemm_float(rows, N, K, a_sample, "row", w["B"].reshape(-1), "col")
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": round(2.0 * rows * N * K / dt / 1e12, 5), "unit": "TFLOP/s",
                               "cores": oracle.num_threads(), "kind": "oracle",
                               "sample": f"all {rows} rows of C (the whole 4096^3 workload), {dt:.1f} s",
                               "host_cpus": os.cpu_count()}

    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
