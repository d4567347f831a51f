"""CPU oracle: plain direct-loop conv2d / matmul / requantize in C (unit_oracle.c).

TEST INFRASTRUCTURE ONLY.  Nothing in the product package imports this module;
it is used by the tests, by the smoke check and by the benchmark's cpu_baseline
leg.  It shares no code with the GPU library and never calls it.

Every function takes and returns numpy arrays.  The definitions follow the
paper's statement of the problem (Section I: conv and matmul as series of
multiply-accumulates with low-precision products reduced into a high-precision
accumulator; Section III-A: int32 accumulation for byte products, fp32
accumulation for fp16 products; Section III-C.2: conv index forms without a
kernel flip).
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "unit_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force=False):
    """Compile unit_oracle.c with gcc (no fast-math, no FMA contraction)."""
    if (not force and os.path.exists(_LIB)
            and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC)):
        return _LIB
    cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp",
           "-ffp-contract=off", "-fno-fast-math", "-Wall", "-Wextra",
           _SRC, "-o", _LIB, "-lm"]
    subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build()
    L = ctypes.CDLL(_LIB)
    i, l, p = ctypes.c_int, ctypes.c_long, ctypes.c_void_p
    L.oracle_num_threads.restype = i
    L.oracle_set_num_threads.argtypes = [i]
    L.oracle_out_dim.restype = i
    L.oracle_out_dim.argtypes = [i, i, i, i]
    L.oracle_half_to_float.restype = ctypes.c_float
    L.oracle_half_to_float.argtypes = [ctypes.c_uint16]
    conv_args = [i] * 11 + [p, p, p]
    L.oracle_conv2d_i8.argtypes = conv_args
    L.oracle_conv2d_f16.argtypes = conv_args
    L.oracle_conv2d_f16_f64.argtypes = conv_args + [p]
    L.oracle_conv3d_i8.argtypes = [i] * 9 + [p, p, p, p, p]
    L.oracle_conv3d_f16.argtypes = [i] * 9 + [p, p, p, p, p, p, p]
    L.oracle_conv3d_i8.restype = None
    L.oracle_conv3d_f16.restype = None
    mm_args = [i, i, i, p, l, p, l, p, l]
    L.oracle_matmul_i8.argtypes = mm_args
    L.oracle_matmul_f16.argtypes = mm_args
    L.oracle_matmul_f16_f64.argtypes = [i, i, i, p, l, p, l, p, p, l]
    L.oracle_requant_one.restype = ctypes.c_int8
    L.oracle_requant_one.argtypes = [ctypes.c_int32, ctypes.c_float, i]
    L.oracle_requant.argtypes = [i, i, i, p, p, p, p, i, p]
    L.oracle_maxpool_i8.argtypes = [i] * 10 + [p, p]
    L.oracle_global_sumpool_requant_i8.argtypes = [i, i, i, p, p, p]
    L.oracle_widen_scale_i8.argtypes = [ctypes.c_size_t, p, ctypes.c_int32, p]
    L.oracle_bf16_to_float.restype = ctypes.c_float
    L.oracle_bf16_to_float.argtypes = [ctypes.c_uint16]
    L.oracle_conv2d_u8i8.argtypes = conv_args
    L.oracle_matmul_u8i8.argtypes = mm_args
    L.oracle_conv2d_bf16.argtypes = conv_args + [p, p]
    L.oracle_matmul_bf16.argtypes = [i, i, i, p, l, p, l, p, p, p, l]
    L.oracle_fp8_e4m3_to_float.restype = ctypes.c_float
    L.oracle_fp8_e4m3_to_float.argtypes = [ctypes.c_uint8]
    L.oracle_conv2d_fp8.argtypes = conv_args + [p, p]
    L.oracle_matmul_fp8.argtypes = [i, i, i, p, l, p, l, p, p, p, l]
    L.oracle_conv2d_fp8.restype = None
    L.oracle_matmul_fp8.restype = None
    for name in ("oracle_conv2d_u8i8", "oracle_matmul_u8i8", "oracle_conv2d_bf16", "oracle_matmul_bf16"):
        getattr(L, name).restype = None
    for name in ("oracle_conv2d_i8", "oracle_conv2d_f16", "oracle_conv2d_f16_f64",
                 "oracle_matmul_i8", "oracle_matmul_f16", "oracle_matmul_f16_f64",
                 "oracle_requant", "oracle_maxpool_i8", "oracle_global_sumpool_requant_i8",
                 "oracle_widen_scale_i8", "oracle_set_num_threads"):
        getattr(L, name).restype = None
    _lib = L
    return L


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _chk(a, dtype, shape=None):
    if not isinstance(a, np.ndarray) or a.dtype != dtype or not a.flags["C_CONTIGUOUS"]:
        raise TypeError(f"expected C-contiguous numpy array of {dtype}")
    if shape is not None and tuple(a.shape) != tuple(shape):
        raise ValueError(f"expected shape {tuple(shape)}, got {a.shape}")
    return a


def num_threads():
    return _load().oracle_num_threads()


def set_num_threads(n):
    _load().oracle_set_num_threads(int(n))


def out_dim(size, window, stride, pad):
    return _load().oracle_out_dim(size, window, stride, pad)


def half_to_float(bits):
    return float(_load().oracle_half_to_float(int(bits)))


def _conv_dims(x, w, stride, pad):
    N, C, H, W = x.shape
    K, C2, R, S = w.shape
    if C2 != C:
        raise ValueError("channel mismatch")
    sh, sw = stride
    ph, pw = pad
    P, Q = out_dim(H, R, sh, ph), out_dim(W, S, sw, pw)
    if P <= 0 or Q <= 0:
        raise ValueError("empty output")
    return (N, C, H, W, K, R, S, sh, sw, ph, pw), (N, K, P, Q)


def conv2d_i8(x, w, stride=(1, 1), pad=(0, 0)):
    """x int8 NCHW, w int8 KCRS -> int32 NKPQ."""
    _chk(x, np.int8), _chk(w, np.int8)
    dims, oshape = _conv_dims(x, w, stride, pad)
    y = np.empty(oshape, np.int32)
    _load().oracle_conv2d_i8(*dims, _ptr(x), _ptr(w), _ptr(y))
    return y


def conv2d_f16(x, w, stride=(1, 1), pad=(0, 0)):
    """x, w: binary16 bit patterns as uint16 (NCHW, KCRS) -> float32 NKPQ."""
    _chk(x, np.uint16), _chk(w, np.uint16)
    dims, oshape = _conv_dims(x, w, stride, pad)
    y = np.empty(oshape, np.float32)
    _load().oracle_conv2d_f16(*dims, _ptr(x), _ptr(w), _ptr(y))
    return y


def conv2d_f16_f64(x, w, stride=(1, 1), pad=(0, 0)):
    """fp64-accumulated value and sum of |products| for each output."""
    _chk(x, np.uint16), _chk(w, np.uint16)
    dims, oshape = _conv_dims(x, w, stride, pad)
    y = np.empty(oshape, np.float64)
    ya = np.empty(oshape, np.float64)
    _load().oracle_conv2d_f16_f64(*dims, _ptr(x), _ptr(w), _ptr(y), _ptr(ya))
    return y, ya


def _conv3_dims(x, w, stride, pad):
    N, C, D, H, W = x.shape
    K, C2, T, R, S = w.shape
    if C2 != C:
        raise ValueError("channel mismatch")
    O, P, Q = (out_dim(D, T, stride[0], pad[0]), out_dim(H, R, stride[1], pad[1]),
               out_dim(W, S, stride[2], pad[2]))
    if min(O, P, Q) <= 0:
        raise ValueError("empty output")
    st = np.asarray(stride, np.int32)
    pd = np.asarray(pad, np.int32)
    return (N, C, D, H, W, K, T, R, S), st, pd, (N, K, O, P, Q)


def conv3d_i8(x, w, stride=(1, 1, 1), pad=(0, 0, 0)):
    """x int8 NCDHW, w int8 KCTRS -> int32 NKOPQ."""
    _chk(x, np.int8), _chk(w, np.int8)
    dims, st, pd, oshape = _conv3_dims(x, w, stride, pad)
    y = np.empty(oshape, np.int32)
    _load().oracle_conv3d_i8(*dims, _ptr(st), _ptr(pd), _ptr(x), _ptr(w), _ptr(y))
    return y


def conv3d_f16(x, w, stride=(1, 1, 1), pad=(0, 0, 0)):
    """binary16 bit patterns -> (fp32 result, fp64-accumulated value, sum of |products|)."""
    _chk(x, np.uint16), _chk(w, np.uint16)
    dims, st, pd, oshape = _conv3_dims(x, w, stride, pad)
    y = np.empty(oshape, np.float32)
    y64 = np.empty(oshape, np.float64)
    ya = np.empty(oshape, np.float64)
    _load().oracle_conv3d_f16(*dims, _ptr(st), _ptr(pd), _ptr(x), _ptr(w), _ptr(y), _ptr(y64), _ptr(ya))
    return y, y64, ya


def _mm_dims(A, B):
    M, K = A.shape
    N, K2 = B.shape
    if K != K2:
        raise ValueError("inner dimension mismatch")
    return M, N, K


def matmul_i8(A, B):
    """A int8 [M,K] row-major; B int8 given as [N,K] (column-major K x N) -> int32 [M,N]."""
    _chk(A, np.int8), _chk(B, np.int8)
    M, N, K = _mm_dims(A, B)
    C = np.empty((M, N), np.int32)
    _load().oracle_matmul_i8(M, N, K, _ptr(A), K, _ptr(B), K, _ptr(C), N)
    return C


def matmul_f16(A, B):
    _chk(A, np.uint16), _chk(B, np.uint16)
    M, N, K = _mm_dims(A, B)
    C = np.empty((M, N), np.float32)
    _load().oracle_matmul_f16(M, N, K, _ptr(A), K, _ptr(B), K, _ptr(C), N)
    return C


def matmul_f16_f64(A, B):
    _chk(A, np.uint16), _chk(B, np.uint16)
    M, N, K = _mm_dims(A, B)
    C = np.empty((M, N), np.float64)
    Ca = np.empty((M, N), np.float64)
    _load().oracle_matmul_f16_f64(M, N, K, _ptr(A), K, _ptr(B), K, _ptr(C), _ptr(Ca), N)
    return C, Ca


def requant_one(t, scale, relu=False):
    return int(_load().oracle_requant_one(int(t), float(np.float32(scale)), int(bool(relu))))


def requant(acc, scale, bias=None, residual=None, relu=False):
    """acc int32 [N,K,...]; scale float32 [K]; bias int32 [K]; residual like acc -> int8."""
    _chk(acc, np.int32)
    N, K = acc.shape[0], acc.shape[1]
    PQ = int(np.prod(acc.shape[2:], dtype=np.int64)) if acc.ndim > 2 else 1
    _chk(scale, np.float32, (K,))
    if bias is not None:
        _chk(bias, np.int32, (K,))
    if residual is not None:
        _chk(residual, np.int32, acc.shape)
    out = np.empty(acc.shape, np.int8)
    _load().oracle_requant(N, K, PQ, _ptr(acc), _ptr(bias), _ptr(residual),
                           _ptr(scale), int(bool(relu)), _ptr(out))
    return out


def maxpool_i8(x, window=(3, 3), stride=(2, 2), pad=(1, 1)):
    _chk(x, np.int8)
    N, C, H, W = x.shape
    R, S = window
    P, Q = out_dim(H, R, stride[0], pad[0]), out_dim(W, S, stride[1], pad[1])
    y = np.empty((N, C, P, Q), np.int8)
    _load().oracle_maxpool_i8(N, C, H, W, R, S, stride[0], stride[1], pad[0], pad[1],
                              _ptr(x), _ptr(y))
    return y


def global_sumpool_requant_i8(x, scale):
    """int32 sum over H*W per (n,c), then requant with scale[c] (no ReLU) -> int8 [N,C]."""
    _chk(x, np.int8)
    N, C, H, W = x.shape
    _chk(scale, np.float32, (C,))
    y = np.empty((N, C), np.int8)
    _load().oracle_global_sumpool_requant_i8(N, C, H * W, _ptr(x), _ptr(scale), _ptr(y))
    return y


def widen_scale_i8(x, mult):
    _chk(x, np.int8)
    y = np.empty(x.shape, np.int32)
    _load().oracle_widen_scale_i8(x.size, _ptr(x), int(mult), _ptr(y))
    return y


# ------------------------------------------------------------------ other operand types

def bf16_to_float(bits):
    return float(_load().oracle_bf16_to_float(int(bits)))


def conv2d_u8i8(x, w, stride=(1, 1), pad=(0, 0)):
    """x uint8 NCHW, w int8 KCRS -> int32 NKPQ."""
    _chk(x, np.uint8), _chk(w, np.int8)
    dims, oshape = _conv_dims(x, w, stride, pad)
    y = np.empty(oshape, np.int32)
    _load().oracle_conv2d_u8i8(*dims, _ptr(x), _ptr(w), _ptr(y))
    return y


def matmul_u8i8(A, B):
    """A uint8 [M,K]; B int8 [N,K] -> int32 [M,N]."""
    _chk(A, np.uint8), _chk(B, np.int8)
    M, N, K = _mm_dims(A, B)
    C = np.empty((M, N), np.int32)
    _load().oracle_matmul_u8i8(M, N, K, _ptr(A), K, _ptr(B), K, _ptr(C), N)
    return C


def conv2d_bf16(x, w, stride=(1, 1), pad=(0, 0)):
    """bfloat16 bit patterns -> (fp32 result, fp64-accumulated value, sum of |products|)."""
    _chk(x, np.uint16), _chk(w, np.uint16)
    dims, oshape = _conv_dims(x, w, stride, pad)
    y = np.empty(oshape, np.float32)
    y64 = np.empty(oshape, np.float64)
    ya = np.empty(oshape, np.float64)
    _load().oracle_conv2d_bf16(*dims, _ptr(x), _ptr(w), _ptr(y), _ptr(y64), _ptr(ya))
    return y, y64, ya


def matmul_bf16(A, B):
    _chk(A, np.uint16), _chk(B, np.uint16)
    M, N, K = _mm_dims(A, B)
    C = np.empty((M, N), np.float32)
    C64 = np.empty((M, N), np.float64)
    Ca = np.empty((M, N), np.float64)
    _load().oracle_matmul_bf16(M, N, K, _ptr(A), K, _ptr(B), K, _ptr(C), _ptr(C64), _ptr(Ca), N)
    return C, C64, Ca


def fp8_e4m3_to_float(bits):
    return float(_load().oracle_fp8_e4m3_to_float(int(bits)))


def conv2d_fp8(x, w, stride=(1, 1), pad=(0, 0)):
    """E4M3 bit patterns (uint8) -> (fp32 result, fp64-accumulated value, sum of |products|)."""
    _chk(x, np.uint8), _chk(w, np.uint8)
    dims, oshape = _conv_dims(x, w, stride, pad)
    y = np.empty(oshape, np.float32)
    y64 = np.empty(oshape, np.float64)
    ya = np.empty(oshape, np.float64)
    _load().oracle_conv2d_fp8(*dims, _ptr(x), _ptr(w), _ptr(y), _ptr(y64), _ptr(ya))
    return y, y64, ya


def matmul_fp8(A, B):
    _chk(A, np.uint8), _chk(B, np.uint8)
    M, N, K = _mm_dims(A, B)
    C = np.empty((M, N), np.float32)
    C64 = np.empty((M, N), np.float64)
    Ca = np.empty((M, N), np.float64)
    _load().oracle_matmul_fp8(M, N, K, _ptr(A), K, _ptr(B), K, _ptr(C), _ptr(C64), _ptr(Ca), N)
    return C, C64, Ca
