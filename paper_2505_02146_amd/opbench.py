"""Workloads of the operators that are not contractions (Table 5: activations, element-wise, pooling,
normalisations, depthwise convolution, deformable attention), with a command line that times one of
them -- the command profilers are pointed at.

    python -m paper_2505_02146_amd.opbench --op layernorm [--steps 40] [--calibrate-copy]
    python -m paper_2505_02146_amd.opbench --list

Each workload is (callable, algorithmic bytes, buffer note): the callable runs the operator once on the
next of several identical buffer sets, which together exceed the 256 MB last-level cache, so that a
timing loop measures HBM-cold launches.  Timing inputs for the dense operators come from torch's seeded
generator on the device (the values do not influence their run time; parity is the tests' job);
deformable attention, whose memory behaviour depends on the sampling positions, uses the seeded
encoder-layer recipe of `inputs.py`.
"""
from __future__ import annotations

import argparse

import numpy as np

from . import inputs


def _rot(n):
    state = {"i": 0}

    def nxt():
        state["i"] += 1
        return state["i"] % n
    return nxt


def _dense_rows(torch):
    rows, cols = 16384, 4096
    xs = [torch.randn(rows, cols, device="cuda").bfloat16() for _ in range(3)]
    ys = [torch.empty(rows, cols, device="cuda", dtype=torch.bfloat16) for _ in range(3)]
    return rows, cols, xs, ys, _rot(3)


def make(op: str):
    """Returns (name, call, algorithmic_bytes, buffers_note, keep_alive)."""
    import torch
    from . import xp
    torch.manual_seed(0)
    if op in ("layernorm", "rmsnorm", "gelu", "relu", "sigmoid", "sign", "add", "softmax_bf16"):
        rows, cols, xs, ys, nxt = _dense_rows(torch)
        n, nb = rows * cols, 2 * rows * cols * 2
        note = "3 rotating sets of 268 MB"
        if op == "layernorm":
            gam, bet = torch.randn(cols, device="cuda").bfloat16(), torch.randn(cols, device="cuda").bfloat16()
            return ("layernorm_bf16_16384x4096", lambda: (lambda i: xp.xp_layernorm(rows, cols, xs[i], cols, gam, bet, 1e-5, ys[i], cols))(nxt()),
                    nb, note, (xs, ys, gam, bet))
        if op == "rmsnorm":
            gam = torch.randn(cols, device="cuda").bfloat16()
            return ("rmsnorm_bf16_16384x4096", lambda: (lambda i: xp.xp_rmsnorm(rows, cols, xs[i], cols, gam, 1e-6, ys[i], cols))(nxt()),
                    nb, note, (xs, ys, gam))
        if op == "softmax_bf16":
            return ("softmax_bf16_16384x4096", lambda: (lambda i: xp.xp_softmax(rows, cols, xs[i], cols, ys[i], cols))(nxt()), nb, note, (xs, ys))
        if op == "add":
            return ("add_bf16_64M", lambda: (lambda i: xp.xp_add(n, xs[i], xs[(i + 1) % 3], ys[i]))(nxt()), 3 * n * 2, "3 rotating sets", (xs, ys))
        return (f"{op}_bf16_64M", lambda: (lambda i: xp.xp_unary(op, n, xs[i], ys[i]))(nxt()), nb, note, (xs, ys))
    if op == "softmax":
        srows, scols = 96 * 512, 512
        sx = [torch.randn(srows, scols, device="cuda") for _ in range(4)]
        sy = [torch.empty(srows, scols, device="cuda") for _ in range(4)]
        nxt = _rot(4)
        return ("softmax_f32_49152x512", lambda: (lambda i: xp.xp_softmax(srows, scols, sx[i], scols, sy[i], scols))(nxt()),
                2 * srows * scols * 4, "4 rotating sets of 201 MB", (sx, sy))
    if op in ("maxpool", "avgpool"):
        pn, ph, pc = 64, 112, 64
        px = [torch.randn(pn, ph, ph, pc, device="cuda").bfloat16() for _ in range(4)]
        py = [torch.empty(pn, 56, 56, pc, device="cuda", dtype=torch.bfloat16) for _ in range(4)]
        nxt = _rot(4)
        nb = (pn * ph * ph * pc + pn * 56 * 56 * pc) * 2
        if op == "maxpool":
            return ("maxpool_bf16_64x112x112x64_3x3s2", lambda: (lambda i: xp.xp_pool2d_nhwc("max", pn, ph, ph, pc, 3, 3, 2, 2, 1, 1, px[i], py[i]))(nxt()),
                    nb, "4 rotating sets of 128 MB", (px, py))
        return ("avgpool_bf16_64x112x112x64_2x2s2", lambda: (lambda i: xp.xp_pool2d_nhwc("avg", pn, ph, ph, pc, 2, 2, 2, 2, 0, 0, px[i], py[i]))(nxt()),
                nb, "4 rotating sets of 128 MB", (px, py))
    if op == "depthwise":
        dn, dh, dc = 32, 112, 64
        px = [torch.randn(dn, dh, dh, dc, device="cuda").bfloat16() for _ in range(4)]
        py = [torch.empty(dn, dh, dh, dc, device="cuda", dtype=torch.bfloat16) for _ in range(4)]
        dwf = (0.3 * torch.randn(3, 3, dc, device="cuda")).bfloat16()
        nxt = _rot(4)
        return ("depthwise_bf16_32x112x112x64_3x3s1", lambda: (lambda i: xp.xp_depthwise_conv2d_nhwc(dn, dh, dh, dc, 3, 3, 1, 1, 1, 1, px[i], dwf, "rsck", py[i]))(nxt()),
                2 * dn * dh * dh * dc * 2, "4 rotating sets of 103 MB", (px, py, dwf))
    if op == "deformable":
        cfg = inputs.DEFORMABLE_WORKLOAD
        lev, b, hd, d, pt = cfg["levels"], cfg["batch"], cfg["heads"], cfg["d"], cfg["points"]
        S = sum(h * w for h, w in lev)
        v_np, loc_np, w_np = inputs.deformable_attention_inputs(b, S, hd, d, lev, pt, seed=5)
        dv = [torch.from_numpy(v_np.view(np.int16)).cuda().view(torch.bfloat16)]
        dloc, dwg = [torch.from_numpy(loc_np).cuda()], [torch.from_numpy(w_np).cuda()]
        for _ in range(3):                       # the same values at other addresses
            dv.append(dv[0].clone()); dloc.append(dloc[0].clone()); dwg.append(dwg[0].clone())
        dout = [torch.empty(b * S * hd * d, device="cuda") for _ in range(4)]
        nxt = _rot(4)
        nb = dv[0].numel() * 2 + dloc[0].numel() * 4 + dwg[0].numel() * 4 + dout[0].numel() * 4
        return ("deformable_attention_bf16_8x5440q_8h32_4l4p",
                lambda: (lambda i: xp.xp_deformable_attention(b, S, hd, d, pt, dv[i], lev, dloc[i], dwg[i], dout[i]))(nxt()),
                nb, "4 rotating sets of 134 MB", (dv, dloc, dwg, dout))
    if op == "conv_nchw":
        xn = torch.randn(32, 256, 56, 56, device="cuda").bfloat16()
        wn = (torch.randn(256, 256, 3, 3, device="cuda") / 48.0).bfloat16()
        on = torch.empty(32, 256, 56, 56, device="cuda")
        wsn = torch.empty(xp.xp_conv2d_nchw_workspace_bytes(32, 56, 56, 256, 256, 3, 3, 1, 1, 1, 1, "bf16"), dtype=torch.uint8, device="cuda")
        nb = xn.numel() * 2 + wn.numel() * 2 + on.numel() * 4
        return ("conv_bf16_56_nchw", lambda: xp.xp_conv2d_nchw(32, 56, 56, 256, 256, 3, 3, 1, 1, 1, 1, xn, wn, on, wsn), nb, "one set", (xn, wn, on, wsn))
    raise ValueError(f"unknown operator workload {op!r}")


OPS = ("layernorm", "rmsnorm", "gelu", "relu", "sigmoid", "sign", "add", "softmax", "softmax_bf16", "maxpool", "avgpool", "depthwise",
       "deformable", "conv_nchw")
# the ones bench.py reports
BENCH_OPS = ("layernorm", "rmsnorm", "gelu", "add", "softmax", "maxpool", "depthwise", "deformable")


def time_op(op: str, steps: int, warmup: int = 5):
    """(name, ms per call, algorithmic bytes, buffers note), timed with HIP events on the current stream."""
    import torch
    name, call, nbytes, note, keep = make(op)
    for _ in range(warmup):
        call()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        call()
    e1.record()
    torch.cuda.synchronize()
    del keep
    return name, e0.elapsed_time(e1) / steps, nbytes, note


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--op", action="append", choices=OPS)
    ap.add_argument("--list", action="store_true")
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one 256 MiB device copy: a known traffic for scaling profiler byte counters")
    args = ap.parse_args(argv)
    if args.list:
        print("\n".join(OPS))
        return 0
    import torch
    if args.calibrate_copy:
        src = torch.zeros(256 << 20, dtype=torch.uint8, device="cuda")
        torch.empty_like(src).copy_(src)
        torch.cuda.synchronize()
        del src
    for op in args.op or BENCH_OPS:
        name, ms, nbytes, note = time_op(op, args.steps)
        print(f"{name:48s} {ms * 1e3:9.1f} us {nbytes / ms / 1e6:9.1f} GB/s of algorithmic bytes   ({note})", flush=True)
    return 0


if __name__ == "__main__":
    raise SystemExit(main())
