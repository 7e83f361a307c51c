"""Per-shape sweep over the kernel variants: the stand-in for the brute-force intra-pass
auto-tuning of the paper (Section 5.1), with its reward (Eq. 3-4): the throughput of a
candidate if it is valid, else 0; the best candidate wins.

A candidate is valid when the library accepts it for the call and its output agrees with the
general kernel's output for the same inputs (bit-exact for int8, within fp32 summation-order
noise otherwise; within the bf16 rounding of the probabilities for fused attention).  Parity against the CPU oracle is the test-suite's job, not the sweep's.

    python -m paper_2505_02146_amd.sweep [--workload NAME ...] [--steps 30] [--rounds 1] [--only IDX ...]
        [--json out.json] [--calibrate-copy]
"""
from __future__ import annotations

import argparse
import json
import sys

import numpy as np

from . import inputs


def _dev(a):
    import torch
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16).copy()).cuda()
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _prepare(name):
    """Returns (op, dtype, flops, call(out), make_out) for a named workload."""
    import torch
    from . import xp
    w = inputs.workload(name)
    kind = w["dtype"]
    if w["op"] == "gemm":
        M, N, K = w["M"], w["N"], w["K"]
        la, lb = w["a_layout"], w["b_layout"]
        lda = K if la == "row" else M
        ldb = N if lb == "row" else K
        A, B = _dev(w["A"].reshape(-1)), _dev(w["B"].reshape(-1))
        odt = torch.int32 if kind == "i8" else torch.float32

        def call(out):
            xp.xp_gemm(M, N, K, 1.0, A, la, lda, B, lb, ldb, 0.0, out, "row", N, a_type=kind, b_type=kind)
        return xp.XP_OP_GEMM, kind, 2.0 * M * N * K, call, lambda: torch.zeros((M, N), dtype=odt, device="cuda")
    if w["op"] == "gemm_batched":
        b, M, N, K = w["batch"], w["M"], w["N"], w["K"]
        lb = w["b_layout"]
        ldb = N if lb == "row" else K
        A, B = _dev(w["A"].reshape(-1)), _dev(w["B"].reshape(-1))

        def call(out):
            xp.xp_gemm_batched(b, M, N, K, 1.0, A, "row", K, M * K, B, lb, ldb, K * N, 0.0, out, "row", N, M * N,
                               a_type=kind, b_type=kind)
        return (xp.XP_OP_GEMM_BATCHED, kind, 2.0 * b * M * N * K, call,
                lambda: torch.zeros((b, M, N), dtype=torch.float32, device="cuda"))
    if w["op"] == "attention":
        b, lq, lk, d, dv = (w[k] for k in ("batch", "Lq", "Lk", "d", "dv"))
        Q, K, V = (_dev(w[t].reshape(-1)) for t in ("Q", "K", "V"))

        def call(out):
            xp.xp_attention(b, lq, lk, d, dv, w["scale"], Q, d, lq * d, K, d, lk * d, V, dv, lk * dv, out, dv, lq * dv,
                            q_type=kind, k_type=kind, v_type=kind)
        return (xp.XP_OP_ATTENTION, kind, 2.0 * b * lq * lk * (d + dv), call,
                lambda: torch.zeros((b, lq, dv), dtype=torch.float32, device="cuda"))
    n, h, wd, ci, co, r, s = (w[k] for k in ("N", "H", "W", "Cin", "Cout", "R", "S"))
    (sh, sw), (ph, pw) = w["stride"], w["pad"]
    p = (h + 2 * ph - r) // sh + 1
    q = (wd + 2 * pw - s) // sw + 1
    X, F = _dev(w["input"].reshape(-1)), _dev(w["filter"].reshape(-1))

    def call(out):
        xp.xp_conv2d_nhwc(n, h, wd, ci, co, r, s, sh, sw, ph, pw, X, F, w["filter_layout"], out,
                          in_type=kind, w_type=kind)
    return (xp.XP_OP_CONV2D, kind, 2.0 * n * p * q * co * r * s * ci, call,
            lambda: torch.zeros((n, p, q, co), dtype=torch.float32, device="cuda"))


def sweep(name: str, steps: int = 30, warmup: int = 5, rounds: int = 1, only=None) -> list[dict]:
    """Force every variant (or the indices in `only`) on workload `name`, gate it, time it.

    With rounds > 1 the valid candidates are timed round-robin `rounds` times and the median
    is reported, which takes clock drift under the power limit out of the comparison."""
    import torch
    from . import xp
    op, kind, flops, call, make_out = _prepare(name)
    xp.xp_force_config(op, kind, 0)
    ref = make_out()
    call(ref)
    torch.cuda.synchronize()
    rows = []
    outs = {}
    for v in range(xp.xp_num_configs(op, kind)):
        if only is not None and v not in only:
            continue
        row = {"workload": name, "variant": v, "name": xp.xp_describe_config(op, kind, v), "tflops": 0.0}
        rows.append(row)
        xp.xp_force_config(op, kind, v)
        out = make_out()
        try:
            call(out)
        except xp.XpError:
            row.update(valid=False, reason="cannot run this call")
            continue
        torch.cuda.synchronize()
        if kind == "i8":
            ok = bool(torch.equal(out, ref))
        else:
            d = (out.double() - ref.double()).norm() / ref.double().norm().clamp_min(1e-30)
            # attention variants may round the probabilities to bf16 (2^-9 each) before the second product
            ok = bool(torch.isfinite(out).all()) and float(d) < (5e-3 if op == xp.XP_OP_ATTENTION else 1e-5)
        if not ok:
            row.update(valid=False, reason="output differs from the general kernel")
            continue
        row.update(valid=True, samples=[])
        outs[v] = out
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for _ in range(rounds):
        for row in rows:
            if not row["valid"]:
                continue
            xp.xp_force_config(op, kind, row["variant"])
            out = outs[row["variant"]]
            for _ in range(warmup):
                call(out)
            torch.cuda.synchronize()
            e0.record()
            for _ in range(steps):
                call(out)
            e1.record()
            torch.cuda.synchronize()
            row["samples"].append(e0.elapsed_time(e1) / steps)
    for row in rows:
        if row["valid"]:
            ms = sorted(row["samples"])[len(row["samples"]) // 2]
            row.update(ms=round(ms, 5), tflops=round(flops / (ms * 1e-3) / 1e12, 2),
                       samples=[round(x, 5) for x in row["samples"]])
    xp.xp_force_config(op, kind, -1)
    out = make_out()
    call(out)
    torch.cuda.synchronize()
    chosen = xp.xp_last_config(op, kind)
    best = max(rows, key=lambda r: r["tflops"])
    for r in rows:
        r["selected_by_library"] = r["variant"] == chosen
        r["best"] = r is best
    return rows


def main(argv=None) -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", nargs="*", default=list(inputs.WORKLOADS + inputs.EXTRA_WORKLOADS))
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--rounds", type=int, default=1, help="time the candidates round-robin this many times, report medians")
    ap.add_argument("--only", type=int, nargs="*", default=None, help="variant indices to time (default: all)")
    ap.add_argument("--json", default=None)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one 256 MiB device copy: a known traffic for scaling profiler byte counters")
    args = ap.parse_args(argv)
    if args.calibrate_copy:
        import torch
        src = torch.zeros(256 << 20, dtype=torch.uint8, device="cuda")
        torch.empty_like(src).copy_(src)
        torch.cuda.synchronize()
    all_rows = []
    for name in args.workload:
        rows = sweep(name, args.steps, rounds=args.rounds, only=args.only)
        all_rows += rows
        print(f"== {name}")
        for r in rows:
            flag = ("*" if r["best"] else " ") + ("S" if r["selected_by_library"] else " ")
            if r["valid"]:
                print(f" {flag} {r['variant']:2d} {r['name']:55s} {r['ms']:9.4f} ms {r['tflops']:9.1f} T/s", flush=True)
            else:
                print(f" {flag} {r['variant']:2d} {r['name']:55s} invalid: {r['reason']}", flush=True)
    if args.json:
        with open(args.json, "w") as f:
            json.dump(all_rows, f, indent=1)
    return 0


if __name__ == "__main__":
    sys.exit(main())
