"""Seeded synthetic input generators shared by the tests, the benchmark and the smoke check.

This module holds no operator arithmetic: it only produces deterministic host arrays
(numpy) with the value distributions of the benchmark workloads.  Every element is a
pure function of (seed, tensor_id, element_index) through the SplitMix64 finaliser
(Steele, Lea, Flood 2014; Vigna's public-domain formulation), so results do not depend on
array shape, chunking, thread count or library version.

bf16 tensors are returned as uint16 bit patterns (round-to-nearest-even from fp32), and
those bits are the input both to the GPU path and to the CPU oracle, so input rounding
never enters an error measurement.
"""
from __future__ import annotations

import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_TENSOR = np.uint64(0xD1B54A32D192ED03)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_SECOND_STREAM = np.uint64(1 << 40)
_CHUNK = 1 << 22


def _splitmix64(x: np.ndarray) -> np.ndarray:
    z = x + _GOLDEN
    z = (z ^ (z >> np.uint64(30))) * _M1
    z = (z ^ (z >> np.uint64(27))) * _M2
    return z ^ (z >> np.uint64(31))


def _raw(seed: int, tensor_id: int, start: int, count: int, second: bool = False) -> np.ndarray:
    with np.errstate(over="ignore"):
        base = np.uint64(seed & 0xFFFFFFFFFFFFFFFF) * _GOLDEN + np.uint64(tensor_id) * _TENSOR
        idx = np.arange(start, start + count, dtype=np.uint64)
        if second:
            idx = idx + _SECOND_STREAM
        return _splitmix64(base + idx)


def _chunks(n: int):
    for s in range(0, n, _CHUNK):
        yield s, min(_CHUNK, n - s)


def uniform_pm1(shape, seed: int, tensor_id: int) -> np.ndarray:
    """fp32 values uniform on [-1, 1): top 24 bits of the hash, scaled."""
    n = int(np.prod(shape, dtype=np.int64))
    out = np.empty(n, dtype=np.float32)
    for s, c in _chunks(n):
        top = (_raw(seed, tensor_id, s, c) >> np.uint64(40)).astype(np.float64)
        out[s:s + c] = (top / float(1 << 24) * 2.0 - 1.0).astype(np.float32)
    return out.reshape(shape)


def normal(shape, seed: int, tensor_id: int, sigma: float = 1.0) -> np.ndarray:
    """fp32 values N(0, sigma^2) by Box-Muller on two hash-derived uniforms."""
    n = int(np.prod(shape, dtype=np.int64))
    out = np.empty(n, dtype=np.float32)
    for s, c in _chunks(n):
        t1 = (_raw(seed, tensor_id, s, c) >> np.uint64(40)).astype(np.float64)
        t2 = (_raw(seed, tensor_id, s, c, second=True) >> np.uint64(40)).astype(np.float64)
        u1 = (t1 + 1.0) / float(1 << 24)          # (0, 1]
        u2 = t2 / float(1 << 24)                  # [0, 1)
        z = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
        out[s:s + c] = (z * sigma).astype(np.float32)
    return out.reshape(shape)


def int8_uniform(shape, seed: int, tensor_id: int) -> np.ndarray:
    """int8 values uniform on [-128, 127]: top 8 bits of the hash minus 128."""
    n = int(np.prod(shape, dtype=np.int64))
    out = np.empty(n, dtype=np.int8)
    for s, c in _chunks(n):
        top = (_raw(seed, tensor_id, s, c) >> np.uint64(56)).astype(np.int16)
        out[s:s + c] = (top - 128).astype(np.int8)
    return out.reshape(shape)


def small_integers(shape, seed: int, tensor_id: int, lo: int = -8, hi: int = 8) -> np.ndarray:
    """fp32 integer-valued entries in [lo, hi]; exact in bf16 and fp32."""
    n = int(np.prod(shape, dtype=np.int64))
    span = hi - lo + 1
    out = np.empty(n, dtype=np.float32)
    for s, c in _chunks(n):
        top = (_raw(seed, tensor_id, s, c) >> np.uint64(33)).astype(np.int64)
        out[s:s + c] = (top % span + lo).astype(np.float32)
    return out.reshape(shape)


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns (uint16), round to nearest, ties to even; NaN stays NaN."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = ((u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)).astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        r = np.where(nan, ((u >> np.uint32(16)) | np.uint32(0x40)).astype(np.uint16), r)
    return r


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> fp32, exact."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# Tensor ids: one independent stream per operand.
TID_A, TID_B, TID_C = 1, 2, 3


def workload(name: str, seed: int = 0) -> dict:
    """Host inputs and call parameters for the five named benchmark workloads.

    Returns a dict with the numpy operands (bf16 as uint16 bits) plus the shape and
    layout parameters the C-ABI calls take.  Layout strings: "row"/"col" refer to the
    logical M x K, K x N and M x N matrices.
    """
    if name == "gemm_f32_256":
        M = N = K = 256
        return dict(op="gemm", dtype="f32", M=M, N=N, K=K, a_layout="row", b_layout="row",
                    A=uniform_pm1((M, K), seed, TID_A), B=uniform_pm1((K, N), seed, TID_B))
    if name == "gemm_bf16_4096":
        M = N = K = 4096
        # B is column-major K x N: stored as an N x K row-major array (K contiguous).
        return dict(op="gemm", dtype="bf16", M=M, N=N, K=K, a_layout="row", b_layout="col",
                    A=to_bf16_bits(normal((M, K), seed, TID_A)),
                    B=to_bf16_bits(normal((N, K), seed, TID_B)))
    if name == "gemm_bf16_4096_rowb":
        # the same product with B stored row-major (K x N, N contiguous), the layout of C = A @ B in a framework
        M = N = K = 4096
        return dict(op="gemm", dtype="bf16", M=M, N=N, K=K, a_layout="row", b_layout="row",
                    A=to_bf16_bits(normal((M, K), seed, TID_A)),
                    B=to_bf16_bits(normal((K, N), seed, TID_B)))
    if name == "gemm_i8_4096x4096x8192":
        M, N, K = 4096, 4096, 8192
        return dict(op="gemm", dtype="i8", M=M, N=N, K=K, a_layout="row", b_layout="col",
                    A=int8_uniform((M, K), seed, TID_A), B=int8_uniform((N, K), seed, TID_B))
    if name == "bgemm_bf16_qk":
        b, M, N, K = 96, 512, 512, 64
        return dict(op="gemm_batched", dtype="bf16", batch=b, M=M, N=N, K=K,
                    a_layout="row", b_layout="col",
                    A=to_bf16_bits(normal((b, M, K), seed, TID_A, 0.125)),
                    B=to_bf16_bits(normal((b, N, K), seed, TID_B, 0.125)))
    if name == "bgemm_bf16_pv":
        b, M, N, K = 96, 512, 64, 512
        return dict(op="gemm_batched", dtype="bf16", batch=b, M=M, N=N, K=K,
                    a_layout="row", b_layout="row",
                    A=to_bf16_bits(normal((b, M, K), seed, TID_A, 0.125)),
                    B=to_bf16_bits(normal((b, K, N), seed, TID_B, 0.125)))
    if name == "conv_bf16_56":
        n, h, w, ci, co, r, s = 32, 56, 56, 256, 256, 3, 3
        return dict(op="conv2d_nhwc", dtype="bf16", N=n, H=h, W=w, Cin=ci, Cout=co, R=r, S=s,
                    stride=(1, 1), pad=(1, 1), filter_layout="krsc",
                    input=to_bf16_bits(normal((n, h, w, ci), seed, TID_A)),
                    filter=to_bf16_bits(normal((co, r, s, ci), seed, TID_B, 1.0 / 48.0)))
    if name == "attention_bf16_512":
        # the two batched stages above with a row softmax between them, as one operator: unit-variance
        # Q and K with scale 1/sqrt(d) give scores of unit variance, i.e. a softmax that is neither
        # flat nor one-hot
        b, L, d = 96, 512, 64
        return dict(op="attention", dtype="bf16", batch=b, Lq=L, Lk=L, d=d, dv=d, scale=1.0 / 8.0,
                    Q=to_bf16_bits(normal((b, L, d), seed, TID_A)),
                    K=to_bf16_bits(normal((b, L, d), seed, TID_B)),
                    V=to_bf16_bits(normal((b, L, d), seed, TID_C)))
    if name == "attention_bf16_2048_d128":
        # a decoder-style block: 32 heads of 128 over 2048 positions
        b, L, d = 32, 2048, 128
        return dict(op="attention", dtype="bf16", batch=b, Lq=L, Lk=L, d=d, dv=d, scale=1.0 / np.sqrt(128.0),
                    Q=to_bf16_bits(normal((b, L, d), seed, TID_A)),
                    K=to_bf16_bits(normal((b, L, d), seed, TID_B)),
                    V=to_bf16_bits(normal((b, L, d), seed, TID_C)))
    if name == "gemv_bf16_8192":
        # matrix-vector product: nothing is reused, the 134 MB matrix is read once
        M = K = 8192
        return dict(op="gemm", dtype="bf16", M=M, N=1, K=K, a_layout="row", b_layout="col",
                    A=to_bf16_bits(normal((M, K), seed, TID_A)),
                    B=to_bf16_bits(normal((1, K), seed, TID_B)))
    raise KeyError(name)


WORKLOADS = ("gemm_f32_256", "gemm_bf16_4096", "gemm_i8_4096x4096x8192",
             "bgemm_bf16_qk", "bgemm_bf16_pv", "conv_bf16_56")
# operators beyond the GEMM / convolution set, each served by its own entry point
EXTRA_WORKLOADS = ("attention_bf16_512", "attention_bf16_2048_d128", "gemv_bf16_8192", "gemm_bf16_4096_rowb")


# A detection-encoder layer's deformable attention: the queries are the pixels of the four feature
# levels themselves (64x64 down to 8x8 for a 512x512 image at strides 8..64), 8 heads of 32 channels.
DEFORMABLE_WORKLOAD = {"batch": 8, "levels": [(64, 64), (32, 32), (16, 16), (8, 8)], "heads": 8, "d": 32, "points": 4}


def deformable_attention_inputs(batch, Lq, heads, d, levels, points, seed: int):
    """(value as bf16 bits, locations fp32, weights fp32) with the structure of an encoder layer: query i
    is pixel i of the concatenated levels (wrapping round if Lq is larger), its sampling positions are
    its own normalised centre plus offsets of about two pixels of the sampled level, the weights of a
    (query, head) are positive and sum to one."""
    S = sum(h * w for h, w in levels)
    value = to_bf16_bits(normal((batch, S, heads, d), seed, 1))
    centres = np.concatenate([np.stack([(np.tile(np.arange(w), h) + 0.5) / w, (np.repeat(np.arange(h), w) + 0.5) / h], axis=-1)
                              for h, w in levels]).astype(np.float32)
    ref = centres[np.arange(Lq) % S]                                            # Lq x 2
    off = normal((batch, Lq, heads, len(levels), points, 2), seed, 2, 2.0)
    size = np.array([[w, h] for h, w in levels], dtype=np.float32)              # levels x (W, H)
    loc = (ref[None, :, None, None, None, :] + off / size[None, None, None, :, None, :]).astype(np.float32)
    u = np.abs(normal((batch, Lq, heads, len(levels), points), seed, 3)) + np.float32(1e-3)
    wgt = (u / u.sum(axis=(3, 4), keepdims=True)).astype(np.float32)
    return value, loc, wgt
