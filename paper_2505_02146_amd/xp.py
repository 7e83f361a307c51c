"""ctypes binding of libxp.so: the same entry points as include/xp.h, marshalling only.

Operands are torch tensors living on the GPU (torch is used for device memory and streams,
nothing else); every step of the computation runs in the library's HIP kernels.  If the
shared library has not been built the import of this module fails: there is no fallback.

bf16 operands may be torch.bfloat16 tensors or int16/uint16 tensors holding bf16 bit patterns.
"""
from __future__ import annotations

import ctypes as C
import pathlib

import torch

_HERE = pathlib.Path(__file__).resolve().parent
import os

# XP_LIBRARY selects another build of the same library (the LDS-poison debug build, say)
LIB_PATH = pathlib.Path(os.environ["XP_LIBRARY"]) if os.environ.get("XP_LIBRARY") else _HERE / "libxp.so"

if not LIB_PATH.exists():
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2505_02146_amd.build` "
                      "(or __graft_entry__.build()); there is no fallback path")

_lib = C.CDLL(str(LIB_PATH))

XP_F32, XP_BF16, XP_I8, XP_I32 = 0, 1, 2, 3
XP_ROW, XP_COL = 0, 1
XP_FILTER_KRSC, XP_FILTER_RSCK = 0, 1
XP_OP_GEMM, XP_OP_GEMM_BATCHED, XP_OP_CONV2D, XP_OP_ATTENTION = 0, 1, 2, 3
XP_OK = 0

_i64, _f, _vp, _i = C.c_int64, C.c_float, C.c_void_p, C.c_int
_lib.xp_gemm.argtypes = [_i64, _i64, _i64, _f, _vp, _i, _i, _i64, _vp, _i, _i, _i64, _f, _vp, _i, _i, _i64, _vp]
_lib.xp_gemm_batched.argtypes = [_i64, _i64, _i64, _i64, _f, _vp, _i, _i, _i64, _i64, _vp, _i, _i, _i64, _i64,
                                 _f, _vp, _i, _i, _i64, _i64, _vp]
_lib.xp_conv2d_nhwc.argtypes = [_i64] * 11 + [_vp, _i, _vp, _i, _i, _vp, _i, _vp]
_lib.xp_attention.argtypes = [_i64] * 5 + [_f] + [_vp, _i, _i64, _i64] * 4 + [_vp]
_ip, _fp = C.POINTER(C.c_int), C.POINTER(C.c_float)
_tune_tail = [_vp, C.c_size_t, _i, _ip, _fp, _vp]       # workspace, bytes, reps, best, best_us, stream
_lib.xp_tune_gemm.argtypes = _lib.xp_gemm.argtypes[:-1] + _tune_tail
_lib.xp_tune_gemm_batched.argtypes = _lib.xp_gemm_batched.argtypes[:-1] + _tune_tail
_lib.xp_tune_conv2d_nhwc.argtypes = _lib.xp_conv2d_nhwc.argtypes[:-1] + _tune_tail
_lib.xp_tune_workspace_bytes.argtypes = [_i64]
_lib.xp_tune_workspace_bytes.restype = C.c_size_t
_lib.xp_tune_save.argtypes = [C.c_char_p]
_lib.xp_tune_load.argtypes = [C.c_char_p]
_lib.xp_tune_clear.restype = None
_lib.xp_softmax.argtypes = [_i64, _i64, _vp, _i, _i64, _vp, _i, _i64, _vp]
_lib.xp_layernorm.argtypes = [_i64, _i64, _vp, _i, _i64, _vp, _vp, _f, _vp, _i, _i64, _vp]
_lib.xp_rmsnorm.argtypes = [_i64, _i64, _vp, _i, _i64, _vp, _f, _vp, _i, _i64, _vp]
_lib.xp_unary.argtypes = [_i, _i64, _vp, _i, _vp, _i, _vp]
_lib.xp_add.argtypes = [_i64, _vp, _vp, _i, _vp, _i, _vp]
_lib.xp_pool2d_nhwc.argtypes = [_i] + [_i64] * 10 + [_vp, _i, _vp, _i, _vp]
_lib.xp_conv2d_nchw_workspace_bytes.argtypes = [_i64] * 11 + [_i]
_lib.xp_conv2d_nchw_workspace_bytes.restype = C.c_size_t
_lib.xp_conv2d_nchw.argtypes = [_i64] * 11 + [_vp, _i, _vp, _i, _vp, _i, _vp, C.c_size_t, _vp]
_lib.xp_conv2d_nchw_static.argtypes = [_i64] * 11 + [_vp, _i, _vp, _i, _vp, _i, _vp]
_lib.xp_conv2d_nchw_static_max_bytes.argtypes = []
_lib.xp_conv2d_nchw_static_max_bytes.restype = C.c_size_t
_lib.xp_depthwise_conv2d_nhwc.argtypes = [_i64] * 10 + [_vp, _i, _vp, _i, _i, _vp, _i, _vp]
_lib.xp_deformable_attention.argtypes = [_i64] * 6 + [_vp, _i, _vp, _vp, _vp, _vp, _vp, _i, _vp]
_lib.xp_mfma_ceiling_ops.argtypes = [_i, _i, _i, _i64]
_lib.xp_mfma_ceiling_ops.restype = C.c_double
_lib.xp_mfma_ceiling.argtypes = [_i, _i, _i, _i64, _vp, C.c_size_t, _vp, C.c_size_t, _vp]
_lib.xp_mfma_ceiling.restype = _i
_lib.xp_num_configs.argtypes = [_i, _i]
_lib.xp_describe_config.argtypes = [_i, _i, _i, C.c_char_p, C.c_size_t]
_lib.xp_force_config.argtypes = [_i, _i, _i]
_lib.xp_last_config.argtypes = [_i, _i]
_lib.xp_status_string.argtypes = [_i]
_lib.xp_status_string.restype = C.c_char_p
_lib.xp_version.restype = C.c_char_p
for _name in ("xp_gemm", "xp_gemm_batched", "xp_conv2d_nhwc", "xp_attention", "xp_tune_gemm", "xp_tune_gemm_batched",
              "xp_tune_conv2d_nhwc", "xp_tune_save", "xp_tune_load", "xp_tune_count", "xp_softmax", "xp_layernorm",
              "xp_rmsnorm", "xp_unary", "xp_add", "xp_pool2d_nhwc", "xp_depthwise_conv2d_nhwc", "xp_conv2d_nchw",
              "xp_conv2d_nchw_static",
              "xp_deformable_attention", "xp_num_configs", "xp_describe_config",
              "xp_force_config", "xp_last_config"):
    getattr(_lib, _name).restype = _i

_LAYOUT = {"row": XP_ROW, "col": XP_COL, XP_ROW: XP_ROW, XP_COL: XP_COL}
_FILTER = {"krsc": XP_FILTER_KRSC, "rsck": XP_FILTER_RSCK, 0: 0, 1: 1}
_DTYPE = {torch.float32: XP_F32, torch.bfloat16: XP_BF16, torch.int16: XP_BF16, torch.uint16: XP_BF16,
          torch.int8: XP_I8, torch.int32: XP_I32}
DTYPE_BY_NAME = {"f32": XP_F32, "bf16": XP_BF16, "i8": XP_I8, "i32": XP_I32}


def to_device(a):
    """numpy host array -> torch tensor on the current GPU (uint16 bf16 bit patterns travel as int16)."""
    import numpy as np
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16).copy()).cuda()
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


class XpError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__(f"xp status {status}: {status_string(status)}")


def status_string(status: int) -> str:
    return _lib.xp_status_string(status).decode()


def version() -> str:
    return _lib.xp_version().decode()


def _ptr(t):
    return None if t is None else t.data_ptr()


def _dt(t, override=None):
    if override is not None:
        return DTYPE_BY_NAME.get(override, override)
    return _DTYPE[t.dtype]


# the raw handle of the current stream of the current device (torch.cuda.current_stream() builds a Python object
# for it: 2.7 us a call, more than half of what a small GEMM call costs)
_raw_current_stream = getattr(torch._C, "_cuda_getCurrentRawStream", None)


def _stream(stream):
    if stream is None:
        return _raw_current_stream(-1) if _raw_current_stream is not None else torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else stream


def _check(status: int):
    if status != XP_OK:
        raise XpError(status)


def xp_gemm(M, N, K, alpha, A, a_layout, lda, B, b_layout, ldb, beta, C_, c_layout, ldc, stream=None,
            a_type=None, b_type=None, c_type=None):
    """C = alpha * A.B + beta * C on the GPU (see include/xp.h: xp_gemm)."""
    _check(_lib.xp_gemm(M, N, K, alpha, _ptr(A), _dt(A, a_type), _LAYOUT[a_layout], lda,
                        _ptr(B), _dt(B, b_type), _LAYOUT[b_layout], ldb, beta,
                        _ptr(C_), _dt(C_, c_type), _LAYOUT[c_layout], ldc, _stream(stream)))


def xp_gemm_batched(batch, M, N, K, alpha, A, a_layout, lda, strideA, B, b_layout, ldb, strideB, beta,
                    C_, c_layout, ldc, strideC, stream=None, a_type=None, b_type=None, c_type=None):
    """Strided-batched GEMM on the GPU (see include/xp.h: xp_gemm_batched)."""
    _check(_lib.xp_gemm_batched(batch, M, N, K, alpha, _ptr(A), _dt(A, a_type), _LAYOUT[a_layout], lda, strideA,
                                _ptr(B), _dt(B, b_type), _LAYOUT[b_layout], ldb, strideB, beta,
                                _ptr(C_), _dt(C_, c_type), _LAYOUT[c_layout], ldc, strideC, _stream(stream)))


def xp_conv2d_nhwc(N, H, W, Cin, Cout, R, S, stride_h, stride_w, pad_h, pad_w, x, w, filter_layout, out,
                   stream=None, in_type=None, w_type=None, out_type=None):
    """NHWC convolution as an implicit GEMM on the GPU (see include/xp.h: xp_conv2d_nhwc)."""
    _check(_lib.xp_conv2d_nhwc(N, H, W, Cin, Cout, R, S, stride_h, stride_w, pad_h, pad_w,
                               _ptr(x), _dt(x, in_type), _ptr(w), _dt(w, w_type), _FILTER[filter_layout],
                               _ptr(out), _dt(out, out_type), _stream(stream)))


def xp_attention(batch, Lq, Lk, d, dv, scale, Q, ldq, strideQ, K, ldk, strideK, V, ldv, strideV, O, ldo, strideO,
                 stream=None, q_type=None, k_type=None, v_type=None, o_type=None):
    """O = softmax(scale * Q.K^T).V per batch index, fused on the GPU (see include/xp.h: xp_attention)."""
    _check(_lib.xp_attention(batch, Lq, Lk, d, dv, scale, _ptr(Q), _dt(Q, q_type), ldq, strideQ,
                             _ptr(K), _dt(K, k_type), ldk, strideK, _ptr(V), _dt(V, v_type), ldv, strideV,
                             _ptr(O), _dt(O, o_type), ldo, strideO, _stream(stream)))


def _tune_call(fn, args, workspace, reps, stream):
    best, best_us = C.c_int(-1), C.c_float(0.0)
    _check(fn(*args, _ptr(workspace), workspace.numel() * workspace.element_size(), reps, C.byref(best), C.byref(best_us),
              _stream(stream)))
    return best.value, best_us.value


def xp_tune_gemm(M, N, K, alpha, A, a_layout, lda, B, b_layout, ldb, beta, C_, c_layout, ldc, workspace, reps=20,
                 stream=None, a_type=None, b_type=None, c_type=None):
    """Brute-force search over the variants for this call's shape (see include/xp.h: xp_tune_gemm).
    Returns (index of the winner, microseconds per launch)."""
    args = (M, N, K, alpha, _ptr(A), _dt(A, a_type), _LAYOUT[a_layout], lda, _ptr(B), _dt(B, b_type), _LAYOUT[b_layout], ldb,
            beta, _ptr(C_), _dt(C_, c_type), _LAYOUT[c_layout], ldc)
    return _tune_call(_lib.xp_tune_gemm, args, workspace, reps, stream)


def xp_tune_gemm_batched(batch, M, N, K, alpha, A, a_layout, lda, strideA, B, b_layout, ldb, strideB, beta, C_, c_layout,
                         ldc, strideC, workspace, reps=20, stream=None, a_type=None, b_type=None, c_type=None):
    args = (batch, M, N, K, alpha, _ptr(A), _dt(A, a_type), _LAYOUT[a_layout], lda, strideA,
            _ptr(B), _dt(B, b_type), _LAYOUT[b_layout], ldb, strideB, beta,
            _ptr(C_), _dt(C_, c_type), _LAYOUT[c_layout], ldc, strideC)
    return _tune_call(_lib.xp_tune_gemm_batched, args, workspace, reps, stream)


def xp_tune_conv2d_nhwc(N, H, W, Cin, Cout, R, S, stride_h, stride_w, pad_h, pad_w, x, w, filter_layout, out, workspace,
                        reps=20, stream=None, in_type=None, w_type=None, out_type=None):
    args = (N, H, W, Cin, Cout, R, S, stride_h, stride_w, pad_h, pad_w, _ptr(x), _dt(x, in_type), _ptr(w), _dt(w, w_type),
            _FILTER[filter_layout], _ptr(out), _dt(out, out_type))
    return _tune_call(_lib.xp_tune_conv2d_nhwc, args, workspace, reps, stream)


def xp_tune_workspace_bytes(c_extent: int) -> int:
    return _lib.xp_tune_workspace_bytes(c_extent)


def xp_tune_save(path: str) -> None:
    _check(_lib.xp_tune_save(str(path).encode()))


def xp_tune_load(path: str) -> None:
    _check(_lib.xp_tune_load(str(path).encode()))


def xp_tune_clear() -> None:
    _lib.xp_tune_clear()


def xp_tune_count() -> int:
    return _lib.xp_tune_count()


UNARY = {"relu": 0, "gelu": 1, "sigmoid": 2, "sign": 3}
POOL = {"max": 0, "avg": 1, "min": 2, "sum": 3}


def xp_softmax(rows, cols, x, ldx, y, ldy, stream=None, x_type=None, y_type=None):
    """Row softmax on the GPU (see include/xp.h: xp_softmax)."""
    _check(_lib.xp_softmax(rows, cols, _ptr(x), _dt(x, x_type), ldx, _ptr(y), _dt(y, y_type), ldy, _stream(stream)))


def xp_layernorm(rows, cols, x, ldx, gamma, beta, eps, y, ldy, stream=None, x_type=None, y_type=None):
    _check(_lib.xp_layernorm(rows, cols, _ptr(x), _dt(x, x_type), ldx, _ptr(gamma), _ptr(beta), eps,
                             _ptr(y), _dt(y, y_type), ldy, _stream(stream)))


def xp_rmsnorm(rows, cols, x, ldx, gamma, eps, y, ldy, stream=None, x_type=None, y_type=None):
    _check(_lib.xp_rmsnorm(rows, cols, _ptr(x), _dt(x, x_type), ldx, _ptr(gamma), eps, _ptr(y), _dt(y, y_type), ldy,
                           _stream(stream)))


def xp_unary(op, n, x, y, stream=None, x_type=None, y_type=None):
    _check(_lib.xp_unary(UNARY.get(op, op), n, _ptr(x), _dt(x, x_type), _ptr(y), _dt(y, y_type), _stream(stream)))


def xp_add(n, a, b, y, stream=None, x_type=None, y_type=None):
    _check(_lib.xp_add(n, _ptr(a), _ptr(b), _dt(a, x_type), _ptr(y), _dt(y, y_type), _stream(stream)))


def xp_pool2d_nhwc(op, N, H, W, C, R, S, stride_h, stride_w, pad_h, pad_w, x, y, stream=None, x_type=None, y_type=None):
    _check(_lib.xp_pool2d_nhwc(POOL.get(op, op), N, H, W, C, R, S, stride_h, stride_w, pad_h, pad_w,
                               _ptr(x), _dt(x, x_type), _ptr(y), _dt(y, y_type), _stream(stream)))


def xp_conv2d_nchw_workspace_bytes(N, H, W, Cin, Cout, R, S, stride_h, stride_w, pad_h, pad_w, in_type) -> int:
    return _lib.xp_conv2d_nchw_workspace_bytes(N, H, W, Cin, Cout, R, S, stride_h, stride_w, pad_h, pad_w,
                                               DTYPE_BY_NAME.get(in_type, in_type))


def xp_conv2d_nchw(N, H, W, Cin, Cout, R, S, stride_h, stride_w, pad_h, pad_w, x, w, out, workspace, stream=None,
                   in_type=None, w_type=None, out_type=None):
    """NCHW convolution through NHWC in the workspace (see include/xp.h: xp_conv2d_nchw)."""
    _check(_lib.xp_conv2d_nchw(N, H, W, Cin, Cout, R, S, stride_h, stride_w, pad_h, pad_w, _ptr(x), _dt(x, in_type),
                               _ptr(w), _dt(w, w_type), _ptr(out), _dt(out, out_type), _ptr(workspace),
                               workspace.numel() * workspace.element_size(), _stream(stream)))


def xp_conv2d_nchw_static_max_bytes() -> int:
    return _lib.xp_conv2d_nchw_static_max_bytes()


def xp_conv2d_nchw_static(N, H, W, Cin, Cout, R, S, stride_h, stride_w, pad_h, pad_w, x, w, out, stream=None,
                          in_type=None, w_type=None, out_type=None):
    """xp_conv2d_nchw on the library's built-in layout-change buffer (see include/xp.h: xp_conv2d_nchw_static)."""
    _check(_lib.xp_conv2d_nchw_static(N, H, W, Cin, Cout, R, S, stride_h, stride_w, pad_h, pad_w, _ptr(x), _dt(x, in_type),
                                      _ptr(w), _dt(w, w_type), _ptr(out), _dt(out, out_type), _stream(stream)))


def xp_mfma_ceiling_ops(in_type, block, waves, iters) -> float:
    return _lib.xp_mfma_ceiling_ops(DTYPE_BY_NAME.get(in_type, in_type), block, waves, iters)


def xp_mfma_ceiling(in_type, block, waves, iters, operands, sink, stream=None):
    """Register-resident MFMA loop (see include/xp.h: xp_mfma_ceiling)."""
    _check(_lib.xp_mfma_ceiling(DTYPE_BY_NAME.get(in_type, in_type), block, waves, iters, _ptr(operands),
                                operands.numel() * operands.element_size(), _ptr(sink), sink.numel() * sink.element_size(),
                                _stream(stream)))


def xp_depthwise_conv2d_nhwc(N, H, W, C, R, S, stride_h, stride_w, pad_h, pad_w, x, w, filter_layout, y, stream=None,
                             x_type=None, w_type=None, y_type=None):
    _check(_lib.xp_depthwise_conv2d_nhwc(N, H, W, C, R, S, stride_h, stride_w, pad_h, pad_w, _ptr(x), _dt(x, x_type),
                                         _ptr(w), _dt(w, w_type), _FILTER[filter_layout], _ptr(y), _dt(y, y_type),
                                         _stream(stream)))


def xp_deformable_attention(batch, Lq, heads, d, points, value, level_hw, locations, weights, out, stream=None,
                            v_type=None, out_type=None):
    """level_hw: sequence of (H, W) per level (host side); locations / weights: float32 device tensors."""
    n = len(level_hw)
    hs = (C.c_int64 * max(n, 1))(*[int(h) for h, _ in level_hw])
    ws = (C.c_int64 * max(n, 1))(*[int(w) for _, w in level_hw])
    _check(_lib.xp_deformable_attention(batch, Lq, heads, d, n, points, _ptr(value), _dt(value, v_type),
                                        C.cast(hs, C.c_void_p), C.cast(ws, C.c_void_p), _ptr(locations), _ptr(weights),
                                        _ptr(out), _dt(out, out_type), _stream(stream)))


def xp_num_configs(op: int, in_type) -> int:
    return _lib.xp_num_configs(op, DTYPE_BY_NAME.get(in_type, in_type))


def xp_describe_config(op: int, in_type, idx: int) -> str:
    buf = C.create_string_buffer(256)
    _check(_lib.xp_describe_config(op, DTYPE_BY_NAME.get(in_type, in_type), idx, buf, 256))
    return buf.value.decode()


def xp_force_config(op: int, in_type, idx: int) -> None:
    _check(_lib.xp_force_config(op, DTYPE_BY_NAME.get(in_type, in_type), idx))


def xp_last_config(op: int, in_type) -> int:
    return _lib.xp_last_config(op, DTYPE_BY_NAME.get(in_type, in_type))


def raw() -> C.CDLL:
    """The ctypes handle itself, for tests of argument validation with raw pointers."""
    return _lib
