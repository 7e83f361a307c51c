#!/usr/bin/env python3
"""Benchmark: bf16 GEMM 4096^3 (A row-major, B column-major, fp32 accumulate and output) on one
MI355X through the C ABI, with the other workloads (fp32 256^3, int8 GEMM, the two batched-GEMM stages,
the convolution stage) timed beside it.  For every workload: time (mean, median and minimum), rate,
fraction of its roofline, the accuracy gates of the timed output against the CPU oracle, and the oracle's
own time on the host cores.  For the dominant kernel: its fraction of the nominal MFMA peak and of the
rate a register-resident MFMA loop sustains on this device.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--only-main] [--no-cpu]

A step is one xp_gemm call on inputs already resident in HBM.  Every timed region is preceded by a fixed
load of the same kernel (`preload_ms`, not counted) that lets the clock settle: after idle the chip runs the
first tens of milliseconds up to 25 % slower.  One JSON line is printed; a failed gate makes the exit code 1.
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

import numpy as np

PEAK_BF16_TFLOPS = 2516.6     # 256 CU x 4096 FLOP/clk/CU x 2.4 GHz, dense
PEAK_INT8_TOPS = 5033.2
PEAK_F32_TFLOPS = 157.3
PEAK_HBM_GBS = 8000.0
GATE_ELEM, GATE_FRO = 1e-2, 5e-3

PRELOAD_MS = 100.0            # load in front of every timed region
BATCHES = 60                  # event pairs for median / minimum
# Bytes per launch between the L2s and the memory fabric for the kernel variants that have been profiled
# (rocprofv3 --pmc FETCH_SIZE, then WRITE_SIZE, scaled by a plain 256 MiB copy; the profile is named beside the
# figure).  Not measured by this run; a variant without a profile reports null.
TRAFFIC = {
    "bf16 256x256x128B waves 2x2 ring 3(A)+2(B) direct-to-lds, reads as assembly, sub-steps paired, mfma16":
        (269.9e6, "profiles/dl_kernel_bf16_256x256_waves2x2_paired_gemm_4096.md"),
    "bf16 256x256x128B waves 2x4 ring 3(A)+2(B) direct-to-lds, reads as assembly, mfma16":
        (268.6e6, "profiles/dl_kernel_bf16_256x256_ring3a2b_asm_reads_gemm_4096.md"),
}


def _settle(torch, fn, ms):
    """Runs fn back to back for about `ms` milliseconds of GPU time."""
    t0 = time.perf_counter()
    n = 0
    while (time.perf_counter() - t0) * 1e3 < ms:
        for _ in range(25):
            fn()
        n += 25
        torch.cuda.synchronize()
    return n


def _region(torch, fn, steps, warmup):
    """`warmup` untimed calls, then exactly `steps` calls between two synchronisations: (event ms, wall ms) per call."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    start.record()
    for _ in range(steps):
        fn()
    stop.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    return start.elapsed_time(stop) / steps, wall_ms / steps


def _spread(torch, fn, per_batch, batches=BATCHES):
    """Median and minimum over `batches` event pairs around `per_batch` calls each (per call, ms), and
    over `batches` event pairs around single calls (those include the events' own overhead)."""
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(batches)]
    for a, b in pairs:
        a.record()
        for _ in range(per_batch):
            fn()
        b.record()
    torch.cuda.synchronize()
    per = [a.elapsed_time(b) / per_batch for a, b in pairs]
    for a, b in pairs:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    single = [a.elapsed_time(b) for a, b in pairs]
    return {"median_ms": round(statistics.median(per), 5), "min_ms": round(min(per), 5),
            "launches": batches * per_batch, "single_launch_median_ms": round(statistics.median(single), 5),
            "single_launch_min_ms": round(min(single), 5)}


def _measure(torch, fn, per_batch, preload_ms=PRELOAD_MS):
    _settle(torch, fn, preload_ms)
    return _spread(torch, fn, per_batch)


def _gates(gpu, ref):
    """The two accuracy gates against the fp64 oracle: margins and verdict."""
    from paper_2505_02146_amd.gates import margins
    worst, fro = margins(gpu, ref)
    return {"max_elem_err_over_absref_plus_1": float(f"{worst:.3e}"), "elem_gate": GATE_ELEM,
            "rel_frobenius": float(f"{fro:.3e}"), "frobenius_gate": GATE_FRO,
            "elements": int(np.asarray(ref).size), "pass": bool(worst <= GATE_ELEM and fro <= GATE_FRO)}


def _exact(gpu, ref):
    same = bool(np.array_equal(np.asarray(gpu), np.asarray(ref)))
    return {"bit_exact": same, "elements": int(np.asarray(ref).size), "pass": same}


def _timed_oracle(fn, repeats=1):
    """Best of `repeats` runs: (result of the last run, seconds)."""
    best, res = None, None
    for _ in range(repeats):
        t0 = time.perf_counter()
        res = fn()
        dt = time.perf_counter() - t0
        best = dt if best is None else min(best, dt)
    return res, best


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--only-main", action="store_true", help="skip the other workloads")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle (no gates, no CPU baseline)")
    ap.add_argument("--force-variant", type=int, default=-1,
                    help="force this kernel variant index for the main workload (profiling a sweep candidate)")
    ap.add_argument("--force-batched-variant", type=int, default=-1,
                    help="force this kernel variant index for the two batched workloads")
    ap.add_argument("--force-attention-variant", type=int, default=-1,
                    help="time this attention variant instead of the library's choice")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 256 MiB device-to-device copy (a known-size reference for "
                         "scaling the profiler's FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--extras", action="store_true",
                    help="also time the operators beyond the five workloads (attention, matrix-vector, NCHW, memory-bound)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        return 2

    import torch
    from paper_2505_02146_amd import inputs, xp          # fails loudly if libxp.so is missing
    dev = xp.to_device
    oracle = None
    if not args.no_cpu:
        import oracle                                    # the checker: only this script's gates and CPU baseline use it

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    failed = []
    cores = oracle.num_threads() if oracle else None

    def cpu_entry(seconds, ops, sample):
        return {"seconds": round(seconds, 4), "cores": cores, "rate": round(ops / seconds / 1e9, 3), "unit": "G(FL)OP/s",
                "kind": "oracle", "sample": sample}

    # ---- what the matrix cores sustain with nothing else going on (register-resident MFMA loop)
    ceiling = {}
    for kind, gen in (("bf16", lambda n: inputs.to_bf16_bits(inputs.normal((n,), 0, 1))), ("i8", lambda n: inputs.int8_uniform((n,), 0, 1))):
        ops_buf = dev(gen(196608 // (2 if kind == "bf16" else 1)))
        sink = torch.zeros(256 * 512, dtype=torch.int32, device="cuda")
        iters = 1000
        m = _measure(torch, lambda: xp.xp_mfma_ceiling(kind, 16, 2, iters, ops_buf, sink), per_batch=4)
        ceiling[kind] = xp.xp_mfma_ceiling_ops(kind, 16, 2, iters) / (m["median_ms"] * 1e-3) / 1e12
        del ops_buf, sink

    # ---- main workload: bf16 GEMM 4096^3, NT
    w = inputs.workload("gemm_bf16_4096")
    M, N, K = w["M"], w["N"], w["K"]
    dA, dB = dev(w["A"].reshape(-1)), dev(w["B"].reshape(-1))
    dC = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    if args.force_variant >= 0:
        xp.xp_force_config(xp.XP_OP_GEMM, "bf16", args.force_variant)

    def step():
        xp.xp_gemm(M, N, K, 1.0, dA, "row", K, dB, "col", K, 0.0, dC, "row", N, a_type="bf16", b_type="bf16")

    preload_calls = _settle(torch, step, PRELOAD_MS)
    ev_ms, wall_ms = _region(torch, step, args.steps, args.warmup)
    spread = _spread(torch, step, per_batch=20)
    flops = 2.0 * M * N * K
    tflops = flops / (ev_ms * 1e-3) / 1e12
    variant = xp.xp_describe_config(0, "bf16", xp.xp_last_config(0, "bf16"))
    traffic, traffic_src = TRAFFIC.get(variant, (None, None))
    main_c = dC.cpu().numpy()                            # what the timed launches wrote
    xp.xp_force_config(xp.XP_OP_GEMM, "bf16", -1)
    del dA, dB, dC

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
        "preload_ms": PRELOAD_MS,
        "preload_calls": preload_calls,
        "pct_mfma_peak": round(100.0 * tflops / PEAK_BF16_TFLOPS, 2),
        "roofline": {"bound": "mfma", "achieved": round(tflops, 2), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(tflops / PEAK_BF16_TFLOPS, 4), "traffic": traffic, "traffic_source": traffic_src,
                     "kernel_ms": round(ev_ms, 5),
                     "measured_ceiling": round(ceiling["bf16"], 1),
                     "frac_of_measured_ceiling": round(tflops / ceiling["bf16"], 4),
                     "measured_ceiling_kernel": "xp_mfma_ceiling: 16x16x32 bf16 MFMAs in dependent pairs on N(0,1) operands held in registers, "
                                                "2 waves per SIMD on 256 compute units"},
        "timing": dict(spread, TFLOPs_at_median=round(flops / (spread["median_ms"] * 1e-3) / 1e12, 1),
                       TFLOPs_at_min=round(flops / (spread["min_ms"] * 1e-3) / 1e12, 1)),
    }

    if oracle:
        ref, dt = _timed_oracle(lambda: oracle.gemm_float(M, N, K, w["A"].reshape(-1), "row", w["B"].reshape(-1), "col"))
        out["gates"] = _gates(main_c, ref)
        if not out["gates"]["pass"]:
            failed.append("gemm_bf16_4096")
        out["cpu_baseline"] = {"value": round(flops / dt / 1e12, 5), "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
                               "sample": f"the whole 4096^3 workload (all rows of C), {dt:.1f} s; its result is the reference of `gates`",
                               "host_cpus": os.cpu_count()}
        del ref
    del main_c

    if args.calibrate_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    if not args.only_main:
        side = {}

        # ---- fp32 GEMM 256^3 (launch-latency bound: microseconds and TFLOP/s, no roofline claim)
        w1 = inputs.workload("gemm_f32_256")
        a1, b1 = dev(w1["A"].reshape(-1)), dev(w1["B"].reshape(-1))
        c1 = torch.full((256, 256), float("nan"), dtype=torch.float32, device="cuda")
        m = _measure(torch, lambda: xp.xp_gemm(256, 256, 256, 1.0, a1, "row", 256, b1, "row", 256, 0.0, c1, "row", 256),
                     per_batch=50, preload_ms=30.0)
        f1 = 2.0 * 256 ** 3
        side["gemm_f32_256"] = dict(m, us=round(m["median_ms"] * 1e3, 2), **{"TFLOP/s": round(f1 / (m["median_ms"] * 1e-3) / 1e12, 3)},
                                    bound="launch latency (33.6 MFLOP, 0.79 MB)",
                                    kernel=xp.xp_describe_config(0, "f32", xp.xp_last_config(0, "f32")))
        # the same call captured 50 times into a HIP graph: what the kernel costs without the host's share of a launch
        def call1():
            xp.xp_gemm(256, 256, 256, 1.0, a1, "row", 256, b1, "row", 256, 0.0, c1, "row", 256)
        cap_stream = torch.cuda.Stream()
        cap_stream.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(cap_stream):
            call1()
        torch.cuda.current_stream().wait_stream(cap_stream)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=cap_stream):
            for _ in range(50):
                call1()
        mg = _measure(torch, graph.replay, per_batch=4, preload_ms=30.0)
        side["gemm_f32_256"]["in_hip_graph_us_per_call"] = round(mg["median_ms"] * 1e3 / 50, 2)
        side["gemm_f32_256"]["in_hip_graph_TFLOP/s"] = round(f1 / (mg["median_ms"] * 1e-3 / 50) / 1e12, 3)
        if oracle:
            call = lambda: oracle.gemm_float(256, 256, 256, w1["A"].reshape(-1), "row", w1["B"].reshape(-1), "row")
            ref, dt = _timed_oracle(call, 3)
            side["gemm_f32_256"]["gates"] = _gates(c1.cpu().numpy(), ref)
            side["gemm_f32_256"]["cpu_oracle"] = cpu_entry(dt, f1, "whole workload, best of 3")
            oracle.set_num_threads(1)
            _, dt1 = _timed_oracle(call, 3)
            oracle.set_num_threads(0)
            side["gemm_f32_256"]["cpu_oracle_one_core"] = dict(cpu_entry(dt1, f1, "whole workload, best of 3"), cores=1)
        del a1, b1, c1

        # ---- int8 GEMM 4096 x 4096 x 8192
        w8 = inputs.workload("gemm_i8_4096x4096x8192")
        a8, b8 = dev(w8["A"].reshape(-1)), dev(w8["B"].reshape(-1))
        c8 = torch.full((4096, 4096), -1, dtype=torch.int32, device="cuda")
        m = _measure(torch, lambda: xp.xp_gemm(4096, 4096, 8192, 1.0, a8, "row", 8192, b8, "col", 8192, 0.0, c8, "row", 4096),
                     per_batch=20)
        ops8 = 2.0 * 4096 * 4096 * 8192
        tops = ops8 / (m["median_ms"] * 1e-3) / 1e12
        side["gemm_i8_4096x4096x8192"] = dict(m, TOPS=round(tops, 1), pct_int8_mfma_peak=round(100 * tops / PEAK_INT8_TOPS, 2),
                                              measured_ceiling_TOPS=round(ceiling["i8"], 1),
                                              frac_of_measured_ceiling=round(tops / ceiling["i8"], 4),
                                              kernel=xp.xp_describe_config(0, "i8", xp.xp_last_config(0, "i8")))
        if oracle:
            ref, dt = _timed_oracle(lambda: oracle.gemm_i8(4096, 4096, 8192, w8["A"].reshape(-1), "row", w8["B"].reshape(-1), "col"))
            side["gemm_i8_4096x4096x8192"]["gates"] = _exact(c8.cpu().numpy(), ref)
            side["gemm_i8_4096x4096x8192"]["cpu_oracle"] = cpu_entry(dt, ops8, "whole workload")
            del ref
        del a8, b8, c8

        # ---- convolution stage 32 x 56 x 56 x 256 -> 256, 3 x 3
        wc = inputs.workload("conv_bf16_56")
        xin, fil = dev(wc["input"].reshape(-1)), dev(wc["filter"].reshape(-1))
        oc = torch.full((32, 56, 56, 256), float("nan"), dtype=torch.float32, device="cuda")
        m = _measure(torch, lambda: xp.xp_conv2d_nhwc(32, 56, 56, 256, 256, 3, 3, 1, 1, 1, 1, xin, fil, "krsc", oc,
                                                      in_type="bf16", w_type="bf16"), per_batch=20)
        fc = 2.0 * 32 * 56 * 56 * 256 * 9 * 256
        tf = fc / (m["median_ms"] * 1e-3) / 1e12
        side["conv_bf16_56"] = dict(m, **{"TFLOP/s": round(tf, 1)}, pct_bf16_mfma_peak=round(100 * tf / PEAK_BF16_TFLOPS, 2),
                                    frac_of_measured_ceiling=round(tf / ceiling["bf16"], 4),
                                    ratio_to_gemm_fraction=round(tf / (flops / (spread["median_ms"] * 1e-3) / 1e12), 3),
                                    kernel=xp.xp_describe_config(2, "bf16", xp.xp_last_config(2, "bf16")))
        if oracle:
            ref, dt = _timed_oracle(lambda: oracle.conv2d_nhwc(wc["input"], wc["filter"], N=32, H=56, W=56, Cin=256, Cout=256, R=3, S=3,
                                                               pad=(1, 1)))
            side["conv_bf16_56"]["gates"] = _gates(oc.cpu().numpy(), ref)
            side["conv_bf16_56"]["cpu_oracle"] = cpu_entry(dt, fc, "whole workload (all 32 images)")
            del ref
        del xin, fil, oc

        # ---- the two batched stages, HBM-cold: rotating through buffer sets larger than the 256 MB last-level cache
        for name, alg_bytes in (("bgemm_bf16_qk", 113.2e6), ("bgemm_bf16_pv", 69.2e6)):
            wb = inputs.workload(name)
            b, m_, n, k = wb["batch"], wb["M"], wb["N"], wb["K"]
            lb = wb["b_layout"]
            ldb = n if lb == "row" else k
            sets = max(2, int(600e6 // alg_bytes) + 1)
            As = [dev(wb["A"].reshape(-1)) for _ in range(sets)]
            Bs = [dev(wb["B"].reshape(-1)) for _ in range(sets)]
            Cs = [torch.full((b, m_, n), float("nan"), dtype=torch.float32, device="cuda") for _ in range(sets)]
            it = {"i": 0}

            def call():
                i = it["i"] % sets
                it["i"] += 1
                xp.xp_gemm_batched(b, m_, n, k, 1.0, As[i], "row", k, m_ * k, Bs[i], lb, ldb, k * n, 0.0, Cs[i], "row", n,
                                   m_ * n, a_type="bf16", b_type="bf16")
            if args.force_batched_variant >= 0:
                xp.xp_force_config(xp.XP_OP_GEMM_BATCHED, "bf16", args.force_batched_variant)
            try:
                m = _measure(torch, call, per_batch=sets * 2)
            except xp.XpError:                       # the forced variant does not serve this layout
                xp.xp_force_config(xp.XP_OP_GEMM_BATCHED, "bf16", -1)
                m = _measure(torch, call, per_batch=sets * 2)
            finally:
                xp.xp_force_config(xp.XP_OP_GEMM_BATCHED, "bf16", -1)
            fb = 2.0 * b * m_ * n * k
            side[name] = dict(m, **{"TFLOP/s": round(fb / (m["median_ms"] * 1e-3) / 1e12, 1),
                                    "GB/s": round(alg_bytes / (m["median_ms"] * 1e-3) / 1e9, 1)},
                              pct_hbm_peak=round(100 * alg_bytes / (m["median_ms"] * 1e-3) / 1e9 / PEAK_HBM_GBS, 2),
                              buffers=f"{sets} rotating sets (HBM-cold)",
                              kernel=xp.xp_describe_config(1, "bf16", xp.xp_last_config(1, "bf16")))
            if oracle:
                ref, dt = _timed_oracle(lambda: oracle.gemm_float_batched(b, m_, n, k, wb["A"].reshape(-1), "row", wb["B"].reshape(-1), lb), 3)
                side[name]["gates"] = _gates(Cs[(it["i"] - 1) % sets].cpu().numpy(), ref)
                side[name]["cpu_oracle"] = cpu_entry(dt, fb, "whole workload, best of 3")
                del ref
            del As, Bs, Cs

        for name, entry in side.items():
            if "gates" in entry and not entry["gates"]["pass"]:
                failed.append(name)

        if args.extras:
            side.update(_extras(torch, xp, inputs, dev, args, side))
        out["other_workloads"] = side

    if failed:
        out["gate_failures"] = failed
    print(json.dumps(out))
    return 1 if failed else 0


def _extras(torch, xp, inputs, dev, args, side):
    """Operators beyond the five workloads: fused attention, matrix-vector, NCHW convolution, memory-bound operators."""
    extra = {}
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
        m = _measure(torch, call_attention, per_batch=sets)
    finally:
        xp.xp_force_config(xp.XP_OP_ATTENTION, "bf16", -1)
    ms = m["median_ms"]
    unfused = side["bgemm_bf16_qk"]["median_ms"] + side["bgemm_bf16_pv"]["median_ms"]
    extra["attention_bf16_512"] = dict(m, **{"TFLOP/s": round(4.0 * b * L * L * d / (ms * 1e-3) / 1e12, 1),
                                             "GB/s": round(alg_bytes / (ms * 1e-3) / 1e9, 1)},
                                       buffers=f"{sets} rotating sets (HBM-cold)",
                                       vs_two_batched_gemm_stages_without_softmax=round(unfused / ms, 2),
                                       kernel=xp.xp_describe_config(3, "bf16", xp.xp_last_config(3, "bf16")))
    del Qs, Ks, Vs, Os
    # the same operator at a decoder block's shape: 32 heads of 128 over 2048 positions (compute-bound)
    w2 = inputs.workload("attention_bf16_2048_d128")
    b2, L2, d2 = w2["batch"], w2["Lq"], w2["d"]
    Q2, K2, V2 = dev(w2["Q"].reshape(-1)), dev(w2["K"].reshape(-1)), dev(w2["V"].reshape(-1))
    O2 = torch.empty((b2 * L2 * d2,), dtype=torch.float32, device="cuda")
    m = _measure(torch, lambda: xp.xp_attention(b2, L2, L2, d2, d2, w2["scale"], Q2, d2, L2 * d2, K2, d2, L2 * d2, V2, d2,
                                                L2 * d2, O2, d2, L2 * d2, q_type="bf16", k_type="bf16", v_type="bf16"), per_batch=5)
    tf2 = 4.0 * b2 * L2 * L2 * d2 / (m["median_ms"] * 1e-3) / 1e12
    extra["attention_bf16_2048_d128"] = dict(m, **{"TFLOP/s": round(tf2, 1)}, pct_bf16_mfma_peak=round(100 * tf2 / PEAK_BF16_TFLOPS, 2),
                                             kernel=xp.xp_describe_config(3, "bf16", xp.xp_last_config(3, "bf16")))
    del Q2, K2, V2, O2
    # matrix-vector product: one pass over a 134 MB matrix, HBM-cold by rotation
    wv = inputs.workload("gemv_bf16_8192")
    mv, kv = wv["M"], wv["K"]
    alg_bytes = mv * kv * 2 + kv * 2 + mv * 4
    sets = 5
    Av = [dev(wv["A"].reshape(-1)) for _ in range(sets)]
    xv = dev(wv["B"].reshape(-1))
    yv = torch.empty((mv,), dtype=torch.float32, device="cuda")
    it2 = {"i": 0}

    def call_gemv():
        i = it2["i"] % sets
        it2["i"] += 1
        xp.xp_gemm(mv, 1, kv, 1.0, Av[i], "row", kv, xv, "col", kv, 0.0, yv, "row", 1, a_type="bf16", b_type="bf16")
    m = _measure(torch, call_gemv, per_batch=sets * 2)
    extra["gemv_bf16_8192"] = dict(m, **{"GB/s": round(alg_bytes / (m["median_ms"] * 1e-3) / 1e9, 1)},
                                   pct_hbm_peak=round(100 * alg_bytes / (m["median_ms"] * 1e-3) / 1e9 / PEAK_HBM_GBS, 2),
                                   buffers=f"{sets} rotating matrices (HBM-cold)",
                                   kernel=xp.xp_describe_config(0, "bf16", xp.xp_last_config(0, "bf16")))
    del Av, xv, yv
    # the convolution workload with NCHW tensors: two layout-change passes in front of the same kernels
    torch.manual_seed(0)
    xn = torch.randn(32, 256, 56, 56, device="cuda").bfloat16()
    wn = (torch.randn(256, 256, 3, 3, device="cuda") / 48.0).bfloat16()
    on = torch.empty(32, 256, 56, 56, device="cuda")
    wsn = torch.empty(xp.xp_conv2d_nchw_workspace_bytes(32, 56, 56, 256, 256, 3, 3, 1, 1, 1, 1, "bf16"), dtype=torch.uint8, device="cuda")
    m = _measure(torch, lambda: xp.xp_conv2d_nchw(32, 56, 56, 256, 256, 3, 3, 1, 1, 1, 1, xn, wn, on, wsn), per_batch=10)
    extra["conv_bf16_56_nchw"] = dict(m, **{"TFLOP/s": round(2.0 * 32 * 56 * 56 * 256 * 9 * 256 / (m["median_ms"] * 1e-3) / 1e12, 1)},
                                      note="input NCHW -> NHWC and filter KCRS -> KRSC passes included; the kernel writes NCHW directly")
    del xn, wn, on, wsn
    # operators that are not contractions: achieved algorithmic bytes/s against the HBM peak, HBM-cold
    from paper_2505_02146_amd import opbench
    mem = {}
    for op in opbench.BENCH_OPS:
        name, ms, nbytes, note = opbench.time_op(op, 200, 50)
        mem[name] = {"ms": round(ms, 5), "GB/s": round(nbytes / (ms * 1e-3) / 1e9, 1),
                     "pct_hbm_peak": round(100 * nbytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 2), "buffers": note}
    extra["memory_bound"] = mem
    return extra


if __name__ == "__main__":
    sys.exit(main())
