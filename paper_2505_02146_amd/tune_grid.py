"""Runs the library's run-time tuner (the brute-force search of Section 5.1 of the paper, reward of
Eq. 3-4: a variant that fails the comparison with the general kernel scores zero, the others by
their measured time) over a grid of common shapes and saves the winners as text.

    python -m paper_2505_02146_amd.tune_grid --out tuned.txt [--quick]

The text is what `xp_tune_load` reads back; `csrc/make_tuned_table.py` turns it into the table of
winners compiled into the library, which also serves shapes *near* a tuned one.
"""
from __future__ import annotations

import argparse
import itertools
import time


def _time(torch, fn, n=20):
    for _ in range(3):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(n):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / n * 1e3


def gemm_shapes(quick):
    """(type, A layout, B layout, M, N, K): bf16 with both operands contiguous along K on a grid with half
    steps (tile quantisation shows between powers of two), the other layouts and int8 on powers of two."""
    fine = (512, 2048, 8192) if quick else (256, 384, 512, 768, 1024, 1536, 2048, 3072, 4096, 6144, 8192)
    coarse = (512, 2048, 8192) if quick else (512, 1024, 2048, 4096, 8192)
    for M, N, K in itertools.product(fine, fine, (1024,) if quick else (256, 512, 1024, 2048, 4096, 8192)):
        yield "bf16", "row", "col", M, N, K
    for la, lb in (("row", "row"), ("col", "col"), ("col", "row")):
        for M, N, K in itertools.product(coarse, coarse, (1024,) if quick else (256, 1024, 4096)):
            yield "bf16", la, lb, M, N, K
    for M, N, K in itertools.product(coarse, coarse, (2048,) if quick else (512, 2048, 8192)):
        yield "i8", "row", "col", M, N, K


BATCHED = [  # batch, M, N, K, B layout
    (96, 512, 512, 64, "col"), (96, 512, 64, 512, "row"), (32, 1024, 1024, 128, "col"), (32, 1024, 128, 1024, "row"),
    (16, 2048, 2048, 64, "col"), (16, 2048, 64, 2048, "row"), (128, 128, 128, 64, "col"), (128, 128, 64, 128, "row"),
    (64, 256, 256, 256, "col"), (8, 1024, 1024, 1024, "col"), (48, 512, 512, 128, "col"), (48, 512, 128, 512, "row"),
    (192, 256, 256, 64, "col"), (192, 256, 64, 256, "row"), (24, 2048, 2048, 128, "col"), (24, 2048, 128, 2048, "row"),
]

CONVS = [  # N, H, W, Cin, Cout, R, S, stride, pad  (stages of residual image networks)
    (32, 56, 56, 64, 64, 3, 3, 1, 1), (32, 56, 56, 256, 256, 3, 3, 1, 1), (32, 28, 28, 128, 128, 3, 3, 1, 1),
    (32, 28, 28, 512, 512, 3, 3, 1, 1), (32, 14, 14, 256, 256, 3, 3, 1, 1), (32, 7, 7, 512, 512, 3, 3, 1, 1),
    (32, 56, 56, 64, 256, 1, 1, 1, 0), (32, 56, 56, 256, 64, 1, 1, 1, 0), (32, 28, 28, 128, 512, 1, 1, 1, 0),
    (32, 14, 14, 256, 1024, 1, 1, 1, 0), (32, 7, 7, 512, 2048, 1, 1, 1, 0), (32, 56, 56, 128, 128, 3, 3, 2, 1),
    (8, 112, 112, 64, 64, 3, 3, 1, 1), (64, 14, 14, 512, 512, 3, 3, 1, 1), (16, 56, 56, 128, 128, 3, 3, 1, 1),
    (32, 28, 28, 256, 256, 3, 3, 1, 1), (16, 28, 28, 256, 1024, 1, 1, 1, 0), (32, 14, 14, 512, 512, 3, 3, 1, 1),
    (8, 64, 64, 128, 128, 3, 3, 1, 1), (32, 28, 28, 256, 512, 3, 3, 2, 1), (32, 56, 56, 128, 256, 1, 1, 1, 0),
    (16, 32, 32, 320, 320, 3, 3, 1, 1), (8, 64, 64, 320, 320, 3, 3, 1, 1), (4, 128, 128, 128, 128, 3, 3, 1, 1),
]


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--out", required=True)
    ap.add_argument("--quick", action="store_true", help="a coarse grid (a minute instead of several)")
    ap.add_argument("--reps", type=int, default=20)
    args = ap.parse_args(argv)
    import torch
    from . import xp
    xp.xp_tune_clear()
    torch.manual_seed(0)
    t_start = time.time()
    gain = []

    chosen = {}                                     # shape key -> variant name, in the order of the grid
    tmp = args.out + ".tmp"

    def saved_keys():
        xp.xp_tune_save(tmp)
        with open(tmp) as f:
            return [line.split(" | ", 1)[0] for line in f if " | " in line and not line.startswith("#")]

    def report(what, fn, tune, op, kind):
        us0 = _time(torch, fn)
        v0 = xp.xp_last_config(op, kind)
        best, _ = tune()
        key = [k for k in saved_keys() if k not in chosen]
        assert len(key) == 1, (what, key)
        keep, us1 = best, _time(torch, fn)
        if best != v0:
            # A second look before the built-in choice is displaced: the tuner times each candidate once, and on a
            # power-limited part the clock that a candidate meets depends on what ran before it.  Both variants
            # in turns, three times; the newcomer has to win by 2 %.
            t = {v0: [], best: []}
            for _ in range(3):
                for v in (v0, best):
                    xp.xp_force_config(op, kind, v)
                    t[v].append(_time(torch, fn))
            xp.xp_force_config(op, kind, -1)
            us0, us1 = min(t[v0]), min(t[best])
            if us1 > 0.98 * us0:
                keep, us1 = v0, us0
        chosen[key[0]] = xp.xp_describe_config(op, kind, keep)
        gain.append(us0 / us1)
        print(f"{what}: default v{v0} {us0:8.1f} us -> tuned v{best} {us1:8.1f} us  x{us0 / us1:.2f}  kept v{keep} [{chosen[key[0]]}]",
              flush=True)

    for kind, a_layout, b_layout, M, N, K in gemm_shapes(args.quick):
        if kind == "bf16":
            A = (torch.randn(M, K, device="cuda") if a_layout == "row" else torch.randn(K, M, device="cuda")).bfloat16()
            B = (torch.randn(N, K, device="cuda") if b_layout == "col" else torch.randn(K, N, device="cuda")).bfloat16()
            C = torch.empty(M, N, device="cuda")
        else:
            A = torch.randint(-128, 128, (M, K) if a_layout == "row" else (K, M), device="cuda", dtype=torch.int8)
            B = torch.randint(-128, 128, (N, K) if b_layout == "col" else (K, N), device="cuda", dtype=torch.int8)
            C = torch.empty(M, N, device="cuda", dtype=torch.int32)
        lda = K if a_layout == "row" else M
        ldb = K if b_layout == "col" else N
        ws = torch.empty(xp.xp_tune_workspace_bytes(M * N), dtype=torch.uint8, device="cuda")
        call = lambda: xp.xp_gemm(M, N, K, 1.0, A, a_layout, lda, B, b_layout, ldb, 0.0, C, "row", N)
        tune = lambda: xp.xp_tune_gemm(M, N, K, 1.0, A, a_layout, lda, B, b_layout, ldb, 0.0, C, "row", N, ws, reps=args.reps)
        report(f"gemm {kind} A {a_layout} B {b_layout} {M}x{N}x{K}", call, tune, 0, kind)
        del A, B, C, ws
    for batch, M, N, K, b_layout in BATCHED:
        A = torch.randn(batch, M, K, device="cuda").bfloat16()
        B = (torch.randn(batch, N, K, device="cuda") if b_layout == "col" else torch.randn(batch, K, N, device="cuda")).bfloat16()
        C = torch.empty(batch, M, N, device="cuda")
        ldb = K if b_layout == "col" else N
        ws = torch.empty(xp.xp_tune_workspace_bytes(batch * M * N), dtype=torch.uint8, device="cuda")
        call = lambda: xp.xp_gemm_batched(batch, M, N, K, 1.0, A, "row", K, M * K, B, b_layout, ldb, N * K, 0.0, C, "row", N, M * N)
        tune = lambda: xp.xp_tune_gemm_batched(batch, M, N, K, 1.0, A, "row", K, M * K, B, b_layout, ldb, N * K, 0.0, C, "row", N,
                                               M * N, ws, reps=args.reps)
        report(f"batched bf16 B {b_layout} {batch}x{M}x{N}x{K}", call, tune, 1, "bf16")
        del A, B, C, ws
    for (n, H, W, Cin, Cout, R, S, stride, pad) in (CONVS[:4] if args.quick else CONVS):
        P, Q = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1
        x = torch.randn(n, H, W, Cin, device="cuda").bfloat16()
        w = (torch.randn(Cout, R, S, Cin, device="cuda") / (R * S * Cin) ** 0.5).bfloat16()
        out = torch.empty(n, P, Q, Cout, device="cuda")
        ws = torch.empty(xp.xp_tune_workspace_bytes(n * P * Q * Cout), dtype=torch.uint8, device="cuda")
        call = lambda: xp.xp_conv2d_nhwc(n, H, W, Cin, Cout, R, S, stride, stride, pad, pad, x, w, "krsc", out)
        tune = lambda: xp.xp_tune_conv2d_nhwc(n, H, W, Cin, Cout, R, S, stride, stride, pad, pad, x, w, "krsc", out, ws, reps=args.reps)
        report(f"conv bf16 {n}x{H}x{W}x{Cin}->{Cout} {R}x{S} s{stride} p{pad}", call, tune, 2, "bf16")
        del x, w, out, ws
    with open(tmp) as f:
        header = [line for line in f if line.startswith("#")]
    with open(args.out, "w") as f:                  # the format of xp_tune_save, shapes sorted by key as it writes them
        f.writelines(header)
        for k in sorted(chosen):
            f.write(f"{k} | {chosen[k]}\n")
    __import__("os").remove(tmp)
    g = sorted(gain)
    print(f"{len(g)} shapes tuned in {time.time() - t_start:.0f} s; default/tuned time: median x{g[len(g) // 2]:.2f}, "
          f"worst x{g[-1]:.2f}, geometric mean x{(__import__('math').prod(g)) ** (1 / len(g)):.3f}; saved to {args.out}")
    return 0


if __name__ == "__main__":
    raise SystemExit(main())
