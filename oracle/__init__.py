"""ctypes front end of the fp64 CPU oracle (oracle/anr_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests, the smoke check and the
benchmark's cpu_baseline leg.  The product package never imports it, and it
imports nothing from the product package.

Every function takes float32 numpy arrays (the same values the GPU sees),
and returns a float64 array holding the operator's mathematical definition
evaluated in double precision.  Operators follow arXiv 2006.06762 Sec. 4.1
(matmul), Sec. 7.1 with Appendix C (C2D, DEP) and Sec. 7.2 (ConvLayer, TBS).
"""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liborc.so")
_lib = None

_f32p = ctypes.POINTER(ctypes.c_float)
_f64p = ctypes.POINTER(ctypes.c_double)
_i64 = ctypes.c_int64
_int = ctypes.c_int


def _load():
    global _lib
    if _lib is not None:
        return _lib
    src = os.path.join(_HERE, "anr_oracle.c")
    if (not os.path.exists(_LIB_PATH)
            or os.path.getmtime(_LIB_PATH) < os.path.getmtime(src)):
        from .build import build
        build()
    lib = ctypes.CDLL(_LIB_PATH)
    lib.orc_max_threads.restype = _int
    lib.orc_set_threads.argtypes = [_int]
    lib.orc_set_threads.restype = None
    lib.orc_gemm.argtypes = [_i64, _i64, _i64, _f32p, _i64, _f32p, _i64, _f64p, _i64,
                             _i64, _i64, _i64, _i64]
    lib.orc_gemm.restype = None
    conv_args = [_int] * 11
    lib.orc_conv2d.argtypes = conv_args + [_f32p, _f32p, _f64p]
    lib.orc_conv2d.restype = None
    lib.orc_conv2d_general.argtypes = [_int] * 14 + [_f32p, _f32p, _f64p]
    lib.orc_conv2d_general.restype = _int
    lib.orc_conv_bn_relu.argtypes = conv_args + [_f32p, _f32p, _f32p, _f32p, _f32p, _f32p,
                                                 ctypes.c_float, _f64p]
    lib.orc_conv_bn_relu.restype = None
    lib.orc_dwconv.argtypes = [_int] * 10 + [_f32p, _f32p, _f64p]
    lib.orc_dwconv.restype = None
    lib.orc_nrm.argtypes = [_i64] * 5 + [_f32p, _f64p]
    lib.orc_nrm.restype = None
    lib.orc_tbg.argtypes = [_int] * 4 + [_f32p, _f32p, _f64p]
    lib.orc_tbg.restype = _int
    lib.orc_tbs.argtypes = [_int] * 4 + [_f32p, _f32p, _f64p]
    lib.orc_tbs.restype = _int
    _lib = lib
    return lib


def _f32(a, shape=None):
    a = np.ascontiguousarray(a)
    if a.dtype != np.float32:
        raise TypeError("oracle inputs must be float32 (the values the GPU sees), got %s" % a.dtype)
    if shape is not None and tuple(a.shape) != tuple(shape):
        raise ValueError("expected shape %s, got %s" % (tuple(shape), tuple(a.shape)))
    return a


def _p32(a):
    return a.ctypes.data_as(_f32p)


def _p64(a):
    return a.ctypes.data_as(_f64p)


def max_threads() -> int:
    return int(_load().orc_max_threads())


def set_threads(n: int) -> None:
    _load().orc_set_threads(int(n))


def out_extent(size: int, pad: int, kernel: int, stride: int) -> int:
    """floor((size + 2*pad - kernel)/stride) + 1."""
    return (size + 2 * pad - kernel) // stride + 1


def gemm(A, B):
    """C = A.B for A [M,K], B [K,N]; or batched for A [b,M,K], B [b,K,N]."""
    A = _f32(A)
    B = _f32(B)
    batched = A.ndim == 3
    if not batched:
        A = A[None]
        B = B[None]
    b, M, K = A.shape
    b2, K2, N = B.shape
    if b != b2 or K != K2:
        raise ValueError("shape mismatch %s x %s" % (A.shape, B.shape))
    C = np.empty((b, M, N), dtype=np.float64)
    _load().orc_gemm(M, N, K, _p32(A), K, _p32(B), N, _p64(C), N, b, M * K, K * N, M * N)
    return C if batched else C[0]


def conv2d(x, w, stride=(1, 1), pad=(0, 0)):
    x = _f32(x)
    w = _f32(w)
    N, C, H, W = x.shape
    K, C2, R, S = w.shape
    if C != C2:
        raise ValueError("channel mismatch")
    OH = out_extent(H, pad[0], R, stride[0])
    OW = out_extent(W, pad[1], S, stride[1])
    if OH <= 0 or OW <= 0:
        raise ValueError("empty output")
    y = np.empty((N, K, OH, OW), dtype=np.float64)
    _load().orc_conv2d(N, C, H, W, K, R, S, stride[0], stride[1], pad[0], pad[1],
                       _p32(x), _p32(w), _p64(y))
    return y


def conv2d_general(x, w, stride=(1, 1), pad=(0, 0), dil=(1, 1), groups=1):
    """Grouped and / or dilated convolution (the GRP and DIL operators): x [N,C,H,W],
    w [K, C/groups, R, S] -> y [N,K,OH,OW]."""
    x = _f32(x)
    w = _f32(w)
    N, C, H, W = x.shape
    K, Cg, R, S = w.shape
    if groups < 1 or C % groups or K % groups or Cg != C // groups:
        raise ValueError("channel counts do not match the group count")
    OH = out_extent(H, pad[0], dil[0] * (R - 1) + 1, stride[0])
    OW = out_extent(W, pad[1], dil[1] * (S - 1) + 1, stride[1])
    if OH <= 0 or OW <= 0:
        raise ValueError("empty output")
    y = np.empty((N, K, OH, OW), dtype=np.float64)
    rc = _load().orc_conv2d_general(N, C, H, W, K, R, S, stride[0], stride[1], pad[0], pad[1],
                                    dil[0], dil[1], groups, _p32(x), _p32(w), _p64(y))
    if rc != 0:
        raise ValueError("orc_conv2d_general rejected the shape")
    return y


def conv_bn_relu_general(x, w, gamma, beta, mean, var, eps, stride=(1, 1), pad=(0, 0), dil=(1, 1), groups=1):
    """ConvLayer (Sec. 7.2) over the grouped / dilated convolution: conv2d_general, then per output
    channel gamma * (v - mean) / sqrt(var + eps) + beta, then max(., 0), in float64 with every
    parameter widened from its float32 value."""
    v = conv2d_general(x, w, stride, pad, dil, groups)
    K = v.shape[1]
    g, b, m, s2 = (_f32(t, (K,)).astype(np.float64)[None, :, None, None] for t in (gamma, beta, mean, var))
    y = g * (v - m) / np.sqrt(s2 + np.float64(np.float32(eps))) + b
    return np.maximum(y, 0.0)


def conv_bn_relu(x, w, gamma, beta, mean, var, eps, stride=(1, 1), pad=(0, 0)):
    x = _f32(x)
    w = _f32(w)
    N, C, H, W = x.shape
    K, C2, R, S = w.shape
    if C != C2:
        raise ValueError("channel mismatch")
    gamma, beta, mean, var = (_f32(v, (K,)) for v in (gamma, beta, mean, var))
    OH = out_extent(H, pad[0], R, stride[0])
    OW = out_extent(W, pad[1], S, stride[1])
    if OH <= 0 or OW <= 0:
        raise ValueError("empty output")
    y = np.empty((N, K, OH, OW), dtype=np.float64)
    _load().orc_conv_bn_relu(N, C, H, W, K, R, S, stride[0], stride[1], pad[0], pad[1],
                             _p32(x), _p32(w), _p32(gamma), _p32(beta), _p32(mean), _p32(var),
                             np.float32(eps), _p64(y))
    return y


def dwconv(x, w, stride=(1, 1), pad=(0, 0)):
    x = _f32(x)
    w = _f32(w)
    N, C, H, W = x.shape
    C2, one, R, S = w.shape
    if C != C2 or one != 1:
        raise ValueError("depthwise weights must be [C,1,R,S]")
    OH = out_extent(H, pad[0], R, stride[0])
    OW = out_extent(W, pad[1], S, stride[1])
    if OH <= 0 or OW <= 0:
        raise ValueError("empty output")
    y = np.empty((N, C, OH, OW), dtype=np.float64)
    _load().orc_dwconv(N, C, H, W, R, S, stride[0], stride[1], pad[0], pad[1],
                       _p32(x), _p32(w), _p64(y))
    return y


def nrm(x):
    """Entrywise 2-norm of each matrix: x [N,M] -> scalar array [1]; x [b,N,M] -> [b]."""
    x = _f32(x)
    if x.ndim == 2:
        x = x[None]
    b, N, M = x.shape
    out = np.empty((b,), dtype=np.float64)
    _load().orc_nrm(b, N, M, M, N * M, _p32(x), _p64(out))
    return out


def tbg(q, k):
    """q, k [B,S,H,D] -> out [B,H,S,S] = transpose(q) . transpose(k)^T per (b,h)."""
    q = _f32(q)
    k = _f32(k, q.shape)
    B, S, H, D = q.shape
    out = np.empty((B, H, S, S), dtype=np.float64)
    if _load().orc_tbg(B, S, H, D, _p32(q), _p32(k), _p64(out)) != 0:
        raise MemoryError("orc_tbg")
    return out


def tbs(q, k):
    """tbg followed by a softmax over the last axis."""
    q = _f32(q)
    k = _f32(k, q.shape)
    B, S, H, D = q.shape
    out = np.empty((B, H, S, S), dtype=np.float64)
    if _load().orc_tbs(B, S, H, D, _p32(q), _p32(k), _p64(out)) != 0:
        raise MemoryError("orc_tbs")
    return out
