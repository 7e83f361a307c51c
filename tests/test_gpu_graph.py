"""The entry points under HIP graph capture: they neither allocate nor synchronise, so a chain of
them can be captured once and replayed.  Every replay is compared bit for bit with the eager run on
the same inputs (the kernels are deterministic), with eager work and synchronisations between the
replays and the inputs changed in place between them."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def xp():
    import torch
    assert torch.cuda.is_available()
    from paper_2505_02146_amd import xp as m
    return m


def test_chain_of_entry_points_replays_like_eager(xp):
    import torch
    torch.manual_seed(3)
    dev = "cuda"
    M, K, N = 512, 1024, 1024
    b, L, d = 4, 256, 64
    levels, heads, dd, pts = [(16, 16), (8, 8)], 4, 32, 4
    S = sum(h * w for h, w in levels)
    bufs = {
        "x": torch.empty(M, K, device=dev, dtype=torch.bfloat16),
        "w": torch.empty(N, K, device=dev, dtype=torch.bfloat16),            # column-major B
        "g": torch.empty(N, device=dev), "beta": torch.empty(N, device=dev),
        "qkv": torch.empty(3, b, L, d, device=dev, dtype=torch.bfloat16),
        "img": torch.empty(2, 28, 28, 64, device=dev, dtype=torch.bfloat16),
        "dwf": torch.empty(3, 3, 64, device=dev, dtype=torch.bfloat16),
        "cw": torch.empty(64, 3, 3, 64, device=dev, dtype=torch.bfloat16),
        "nchw": torch.empty(2, 64, 28, 28, device=dev, dtype=torch.bfloat16),
        "cw_nchw": torch.empty(64, 64, 3, 3, device=dev, dtype=torch.bfloat16),
        "val": torch.empty(2, S, heads, dd, device=dev, dtype=torch.bfloat16),
        "loc": torch.empty(2, 400, heads, 2, pts, 2, device=dev),
        "aw": torch.empty(2, 400, heads, 2, pts, device=dev),
    }
    out = {
        "y": torch.empty(M, N, device=dev), "ln": torch.empty(M, N, device=dev), "act": torch.empty(M, N, device=dev, dtype=torch.bfloat16),
        "sm": torch.empty(M, N, device=dev), "sum": torch.empty(M, N, device=dev),
        "o": torch.empty(b, L, d, device=dev),
        "pool": torch.empty(2, 14, 14, 64, device=dev, dtype=torch.bfloat16),
        "dw": torch.empty(2, 28, 28, 64, device=dev), "conv": torch.empty(2, 28, 28, 64, device=dev),
        "conv_nchw": torch.empty(2, 64, 28, 28, device=dev),
        "da": torch.empty(2, 400, heads, dd, device=dev),
    }
    ws = torch.empty(xp.xp_conv2d_nchw_workspace_bytes(2, 28, 28, 64, 64, 3, 3, 1, 1, 1, 1, "bf16"), dtype=torch.uint8, device=dev)

    def fill(seed):
        gen = torch.Generator(device=dev)
        gen.manual_seed(seed)
        for name, t in bufs.items():
            if name == "loc":
                t.copy_(torch.rand(t.shape, device=dev, generator=gen) * 1.2 - 0.1)
            elif name == "aw":
                t.copy_(torch.rand(t.shape, device=dev, generator=gen) / 8)
            else:
                t.copy_((torch.randn(t.shape, device=dev, generator=gen) * (0.05 if name in ("w", "cw", "cw_nchw") else 1.0)).to(t.dtype))

    def chain():
        xp.xp_gemm(M, N, K, 1.0, bufs["x"], "row", K, bufs["w"], "col", K, 0.0, out["y"], "row", N)
        xp.xp_layernorm(M, N, out["y"], N, bufs["g"], bufs["beta"], 1e-5, out["ln"], N)
        xp.xp_unary("gelu", M * N, out["ln"], out["act"])
        xp.xp_softmax(M, N, out["ln"], N, out["sm"], N)
        xp.xp_add(M * N, out["sm"], out["ln"], out["sum"])
        q, k, v = bufs["qkv"][0], bufs["qkv"][1], bufs["qkv"][2]
        xp.xp_attention(b, L, L, d, d, 0.125, q, d, L * d, k, d, L * d, v, d, L * d, out["o"], d, L * d)
        xp.xp_pool2d_nhwc("max", 2, 28, 28, 64, 3, 3, 2, 2, 1, 1, bufs["img"], out["pool"])
        xp.xp_depthwise_conv2d_nhwc(2, 28, 28, 64, 3, 3, 1, 1, 1, 1, bufs["img"], bufs["dwf"], "rsck", out["dw"])
        xp.xp_conv2d_nhwc(2, 28, 28, 64, 64, 3, 3, 1, 1, 1, 1, bufs["img"], bufs["cw"], "krsc", out["conv"])
        xp.xp_conv2d_nchw(2, 28, 28, 64, 64, 3, 3, 1, 1, 1, 1, bufs["nchw"], bufs["cw_nchw"], out["conv_nchw"], ws)
        xp.xp_deformable_attention(2, 400, heads, dd, pts, bufs["val"], levels, bufs["loc"], bufs["aw"], out["da"])

    def snapshot():
        torch.cuda.synchronize()
        return {k: t.clone() for k, t in out.items()}

    def poison():
        for t in out.values():
            t.fill_(7.0)

    eager = {}
    for seed in (11, 12):
        fill(seed)
        poison()
        chain()
        eager[seed] = snapshot()
    for k in out:
        assert not torch.equal(eager[11][k], eager[12][k]), k            # the two input sets give different results

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        chain()                                                          # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        chain()
    for i, seed in enumerate((12, 11, 12, 11, 11)):
        fill(seed)
        poison()
        scratch = torch.randn(1 << 20, device=dev).sum().item()          # eager work and a synchronisation in between
        assert np.isfinite(scratch)
        graph.replay()
        got = snapshot()
        for k in out:
            assert torch.equal(got[k], eager[seed][k]), f"replay {i} (inputs {seed}): {k} differs from the eager run"
