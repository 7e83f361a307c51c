"""Python face of the CPU oracle (TEST INFRASTRUCTURE ONLY).

Thin ctypes marshalling around oracle/liboracle.so; all arithmetic is in xp_oracle.c.
Only tests, the smoke check and the benchmark's CPU-baseline leg may import this package;
the GPU library never does.

bf16 operands are numpy uint16 arrays of bit patterns; fp32 operands are float32 arrays;
int8 operands are int8 arrays.  Matrices are described the way the C-ABI describes them:
a flat buffer, a layout ("row" or "col") of the logical matrix, and a leading dimension.
"""
from __future__ import annotations

import ctypes as C

import numpy as np

from .build import LIB, build

_lib = None

_LAYOUT = {"row": 0, "col": 1}
_FILTER = {"krsc": 0, "rsck": 1}


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        build(force=False)
        L = C.CDLL(str(LIB))
        i64, dbl, vp, i = C.c_int64, C.c_double, C.c_void_p, C.c_int
        L.oracle_gemm_float.argtypes = [i64, i64, i64, dbl, vp, i, i, i64, vp, i, i, i64,
                                        dbl, vp, i, i64, vp]
        L.oracle_gemm_i8.argtypes = [i64, i64, i64, vp, i, i64, vp, i, i64, vp]
        L.oracle_gemm_float_batched.argtypes = [i64, i64, i64, i64, dbl,
                                                vp, i, i, i64, i64, vp, i, i, i64, i64,
                                                dbl, vp, i, i64, i64, vp]
        L.oracle_conv2d_nhwc.argtypes = [i64] * 11 + [vp, i, vp, i, i, vp]
        L.oracle_attention.argtypes = [i64] * 5 + [dbl] + [vp, i, i64, i64] * 3 + [vp]
        L.oracle_softmax.argtypes = [i64, i64, vp, i, i64, vp]
        L.oracle_layernorm.argtypes = [i64, i64, vp, i, i64, vp, vp, dbl, vp]
        L.oracle_rmsnorm.argtypes = [i64, i64, vp, i, i64, vp, dbl, vp]
        L.oracle_unary.argtypes = [i, i64, vp, i, vp]
        L.oracle_add.argtypes = [i64, vp, vp, i, vp]
        L.oracle_pool2d_nhwc.argtypes = [i] + [i64] * 10 + [vp, i, vp]
        L.oracle_depthwise_conv2d_nhwc.argtypes = [i64] * 10 + [vp, i, vp, i, i, vp]
        L.oracle_depthwise_conv2d_nhwc.restype = i
        L.oracle_conv2d_nchw.argtypes = [i64] * 11 + [vp, i, vp, i, vp]
        L.oracle_conv2d_nchw.restype = i
        L.oracle_deformable_attention.argtypes = [i64] * 6 + [vp, i, vp, vp, vp, vp, vp]
        L.oracle_deformable_attention.restype = i
        for f in (L.oracle_gemm_float, L.oracle_gemm_i8, L.oracle_gemm_float_batched,
                  L.oracle_conv2d_nhwc, L.oracle_attention, L.oracle_softmax, L.oracle_layernorm,
                  L.oracle_rmsnorm, L.oracle_unary, L.oracle_add, L.oracle_pool2d_nhwc, L.oracle_num_threads):
            f.restype = i
        _lib = L
    return _lib


def num_threads() -> int:
    return lib().oracle_num_threads()


def set_num_threads(n: int) -> None:
    """Caps the OpenMP threads of the loops (n <= 0 restores the default): for timing the oracle on one core."""
    L = lib()
    L.oracle_set_num_threads.argtypes = [C.c_int]
    L.oracle_set_num_threads.restype = None
    L.oracle_set_num_threads(int(n))


def _ftype(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return 0
    if a.dtype == np.uint16:
        return 1
    raise TypeError(f"float operand must be float32 or uint16 (bf16 bits), got {a.dtype}")


def _ptr(a):
    if a is None:
        return None
    assert a.flags["C_CONTIGUOUS"], "oracle operands are flat contiguous buffers"
    return a.ctypes.data


def _min_ld(layout: str, rows: int, cols: int) -> int:
    return cols if layout == "row" else rows


def gemm_float(M, N, K, A, a_layout, B, b_layout, *, lda=None, ldb=None, alpha=1.0, beta=0.0,
               C0=None, c_layout="row", ldc=None) -> np.ndarray:
    """fp64 reference of alpha*A.B + beta*C0 as a dense row-major M x N float64 array."""
    lda = _min_ld(a_layout, M, K) if lda is None else lda
    ldb = _min_ld(b_layout, K, N) if ldb is None else ldb
    ldc = _min_ld(c_layout, M, N) if ldc is None else ldc
    ref = np.empty((M, N), dtype=np.float64)
    if C0 is not None:
        assert C0.dtype == np.float32
    rc = lib().oracle_gemm_float(M, N, K, float(alpha), _ptr(A), _ftype(A), _LAYOUT[a_layout], lda,
                                 _ptr(B), _ftype(B), _LAYOUT[b_layout], ldb,
                                 float(beta), _ptr(C0), _LAYOUT[c_layout], ldc, _ptr(ref))
    if rc:
        raise ValueError(f"oracle_gemm_float failed with code {rc}")
    return ref


def gemm_i8(M, N, K, A, a_layout, B, b_layout, *, lda=None, ldb=None) -> np.ndarray:
    """Exact int32 reference of A.B for int8 operands (raises if a sum leaves int32)."""
    lda = _min_ld(a_layout, M, K) if lda is None else lda
    ldb = _min_ld(b_layout, K, N) if ldb is None else ldb
    assert A.dtype == np.int8 and B.dtype == np.int8
    ref = np.empty((M, N), dtype=np.int32)
    rc = lib().oracle_gemm_i8(M, N, K, _ptr(A), _LAYOUT[a_layout], lda,
                              _ptr(B), _LAYOUT[b_layout], ldb, _ptr(ref))
    if rc == 100:
        raise OverflowError("int8 GEMM sum outside the int32 range")
    if rc:
        raise ValueError(f"oracle_gemm_i8 failed with code {rc}")
    return ref


def gemm_float_batched(batch, M, N, K, A, a_layout, B, b_layout, *, lda=None, ldb=None,
                       strideA=None, strideB=None, alpha=1.0, beta=0.0, C0=None,
                       c_layout="row", ldc=None, strideC=None) -> np.ndarray:
    """fp64 reference of the strided-batched GEMM, dense batch x M x N."""
    lda = _min_ld(a_layout, M, K) if lda is None else lda
    ldb = _min_ld(b_layout, K, N) if ldb is None else ldb
    ldc = _min_ld(c_layout, M, N) if ldc is None else ldc
    strideA = M * K if strideA is None else strideA
    strideB = K * N if strideB is None else strideB
    strideC = M * N if strideC is None else strideC
    ref = np.empty((batch, M, N), dtype=np.float64)
    rc = lib().oracle_gemm_float_batched(batch, M, N, K, float(alpha),
                                         _ptr(A), _ftype(A), _LAYOUT[a_layout], lda, strideA,
                                         _ptr(B), _ftype(B), _LAYOUT[b_layout], ldb, strideB,
                                         float(beta), _ptr(C0), _LAYOUT[c_layout], ldc, strideC,
                                         _ptr(ref))
    if rc:
        raise ValueError(f"oracle_gemm_float_batched failed with code {rc}")
    return ref


def conv_out_hw(H, W, R, S, stride, pad):
    P = (H + 2 * pad[0] - R) // stride[0] + 1 if H + 2 * pad[0] >= R else 0
    Q = (W + 2 * pad[1] - S) // stride[1] + 1 if W + 2 * pad[1] >= S else 0
    return P, Q


def conv2d_nhwc(x, w, *, N, H, W, Cin, Cout, R, S, stride=(1, 1), pad=(0, 0),
                filter_layout="krsc") -> np.ndarray:
    """fp64 reference of the NHWC cross-correlation, dense N x P x Q x Cout."""
    P, Q = conv_out_hw(H, W, R, S, stride, pad)
    ref = np.empty((N, P, Q, Cout), dtype=np.float64)
    rc = lib().oracle_conv2d_nhwc(N, H, W, Cin, Cout, R, S, stride[0], stride[1], pad[0], pad[1],
                                  _ptr(x), _ftype(x), _ptr(w), _ftype(w), _FILTER[filter_layout],
                                  _ptr(ref))
    if rc:
        raise ValueError(f"oracle_conv2d_nhwc failed with code {rc}")
    return ref


def attention(Q, K, V, *, batch, Lq, Lk, d, dv, scale, ldq=None, ldk=None, ldv=None,
              strideQ=None, strideK=None, strideV=None) -> np.ndarray:
    """fp64 reference of softmax(scale * Q.K^T).V per batch index, dense batch x Lq x dv."""
    ldq = d if ldq is None else ldq
    ldk = d if ldk is None else ldk
    ldv = dv if ldv is None else ldv
    strideQ = Lq * ldq if strideQ is None else strideQ
    strideK = Lk * ldk if strideK is None else strideK
    strideV = Lk * ldv if strideV is None else strideV
    ref = np.empty((batch, Lq, dv), dtype=np.float64)
    rc = lib().oracle_attention(batch, Lq, Lk, d, dv, float(scale),
                                _ptr(Q), _ftype(Q), ldq, strideQ, _ptr(K), _ftype(K), ldk, strideK,
                                _ptr(V), _ftype(V), ldv, strideV, _ptr(ref))
    if rc:
        raise ValueError(f"oracle_attention failed with code {rc}")
    return ref


UNARY = {"relu": 0, "gelu": 1, "sigmoid": 2, "sign": 3}
POOL = {"max": 0, "avg": 1, "min": 2, "sum": 3}


def _rc(rc, what):
    if rc:
        raise ValueError(f"{what} failed with code {rc}")


def softmax(x, *, rows, cols, ldx=None) -> np.ndarray:
    """fp64 softmax over the last dimension of a rows x cols matrix with row pitch ldx."""
    ref = np.empty((rows, cols), dtype=np.float64)
    _rc(lib().oracle_softmax(rows, cols, _ptr(x), _ftype(x), cols if ldx is None else ldx, _ptr(ref)), "oracle_softmax")
    return ref


def layernorm(x, *, rows, cols, gamma=None, beta=None, eps=1e-5, ldx=None) -> np.ndarray:
    ref = np.empty((rows, cols), dtype=np.float64)
    for v in (gamma, beta):
        assert v is None or v.dtype == x.dtype
    _rc(lib().oracle_layernorm(rows, cols, _ptr(x), _ftype(x), cols if ldx is None else ldx, _ptr(gamma), _ptr(beta),
                               float(eps), _ptr(ref)), "oracle_layernorm")
    return ref


def rmsnorm(x, *, rows, cols, gamma=None, eps=1e-6, ldx=None) -> np.ndarray:
    ref = np.empty((rows, cols), dtype=np.float64)
    assert gamma is None or gamma.dtype == x.dtype
    _rc(lib().oracle_rmsnorm(rows, cols, _ptr(x), _ftype(x), cols if ldx is None else ldx, _ptr(gamma), float(eps),
                             _ptr(ref)), "oracle_rmsnorm")
    return ref


def unary(op: str, x) -> np.ndarray:
    ref = np.empty(x.size, dtype=np.float64)
    _rc(lib().oracle_unary(UNARY[op], x.size, _ptr(x), _ftype(x), _ptr(ref)), "oracle_unary")
    return ref.reshape(x.shape)


def add(a, b) -> np.ndarray:
    assert a.dtype == b.dtype and a.size == b.size
    ref = np.empty(a.size, dtype=np.float64)
    _rc(lib().oracle_add(a.size, _ptr(a), _ptr(b), _ftype(a), _ptr(ref)), "oracle_add")
    return ref.reshape(a.shape)


def pool2d_nhwc(op: str, x, *, N, H, W, C, R, S, stride=(1, 1), pad=(0, 0)) -> np.ndarray:
    P, Q = conv_out_hw(H, W, R, S, stride, pad)
    ref = np.empty((N, P, Q, C), dtype=np.float64)
    _rc(lib().oracle_pool2d_nhwc(POOL[op], N, H, W, C, R, S, stride[0], stride[1], pad[0], pad[1], _ptr(x), _ftype(x),
                                 _ptr(ref)), "oracle_pool2d_nhwc")
    return ref


def depthwise_conv2d_nhwc(x, w, *, N, H, W, C, R, S, stride=(1, 1), pad=(0, 0), filter_layout="rsck") -> np.ndarray:
    """fp64 reference of the depthwise NHWC convolution, dense N x P x Q x C."""
    P, Q = conv_out_hw(H, W, R, S, stride, pad)
    ref = np.empty((N, P, Q, C), dtype=np.float64)
    _rc(lib().oracle_depthwise_conv2d_nhwc(N, H, W, C, R, S, stride[0], stride[1], pad[0], pad[1], _ptr(x), _ftype(x),
                                           _ptr(w), _ftype(w), _FILTER[filter_layout], _ptr(ref)), "oracle_depthwise_conv2d_nhwc")
    return ref


def conv2d_nchw(x, w, *, N, H, W, Cin, Cout, R, S, stride=(1, 1), pad=(0, 0)) -> np.ndarray:
    """fp64 reference of the NCHW cross-correlation with a KCRS filter, dense N x Cout x P x Q."""
    P, Q = conv_out_hw(H, W, R, S, stride, pad)
    ref = np.empty((N, Cout, P, Q), dtype=np.float64)
    _rc(lib().oracle_conv2d_nchw(N, H, W, Cin, Cout, R, S, stride[0], stride[1], pad[0], pad[1], _ptr(x), _ftype(x),
                                 _ptr(w), _ftype(w), _ptr(ref)), "oracle_conv2d_nchw")
    return ref


def deformable_attention(value, level_hw, locations, weights, *, batch, Lq, heads, d, points) -> np.ndarray:
    """fp64 reference of multi-scale deformable attention, dense batch x Lq x heads x d.
    level_hw: list of (H, W); locations float32 [batch, Lq, heads, levels, points, 2]; weights float32 without the last axis."""
    hs = np.array([h for h, _ in level_hw], dtype=np.int64)
    ws_ = np.array([w for _, w in level_hw], dtype=np.int64)
    assert locations.dtype == np.float32 and weights.dtype == np.float32
    ref = np.empty((batch, Lq, heads, d), dtype=np.float64)
    _rc(lib().oracle_deformable_attention(batch, Lq, heads, d, len(level_hw), points, _ptr(value), _ftype(value),
                                          _ptr(hs), _ptr(ws_), _ptr(locations), _ptr(weights), _ptr(ref)),
        "oracle_deformable_attention")
    return ref
