"""ctypes binding of libanr.so: argument marshalling only.

Function names and arguments mirror ``include/anr.h``.  Every tensor argument
is a torch CUDA tensor (float32); torch is used for device memory and for the
current HIP stream, nothing else.  There is no CPU path: if the library has not
been built, importing this module raises.
"""
import ctypes
import os

# torch ships its own HIP runtime (libamdhip64.so.7).  It must be in the process before
# libanr.so is opened, so that the library binds to that same runtime instance: streams
# and device pointers are only meaningful inside the runtime that created them.
import torch  # noqa: F401

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libanr.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        "%s is missing: build it with `python -m paper_2006_06762_amd.build` "
        "(there is no fallback path)" % LIB_PATH)

_lib = ctypes.CDLL(LIB_PATH)

ANR_OK, ANR_ERR_NULL, ANR_ERR_INVALID_ARG, ANR_ERR_UNSUPPORTED, ANR_ERR_WORKSPACE, ANR_ERR_LAUNCH = range(6)
ANR_LAYOUT_NCHW = 0
ANR_OP_GEMM, ANR_OP_CONV2D, ANR_OP_CONV_BN_RELU, ANR_OP_DWCONV, ANR_OP_TBG, ANR_OP_TBS, ANR_OP_NRM = range(7)

EXPORTS = ("anr_gemm", "anr_conv2d", "anr_conv2d_noalloc", "anr_conv2d_packed_size", "anr_conv2d_pack_weights",
           "anr_conv2d_packed", "anr_conv_bn_relu_packed", "anr_conv_bn_relu", "anr_dwconv", "anr_tbg", "anr_tbs", "anr_nrm",
           "anr_workspace_size", "anr_conv2d_route", "anr_status_string", "anr_version", "anr_last_hip_error",
           "anr_last_hip_error_string")


class GemmDesc(ctypes.Structure):
    _fields_ = [("M", ctypes.c_int64), ("N", ctypes.c_int64), ("K", ctypes.c_int64),
                ("lda", ctypes.c_int64), ("ldb", ctypes.c_int64), ("ldc", ctypes.c_int64),
                ("batch", ctypes.c_int64),
                ("strideA", ctypes.c_int64), ("strideB", ctypes.c_int64), ("strideC", ctypes.c_int64)]


class ConvDesc(ctypes.Structure):
    _fields_ = [("N", ctypes.c_int32), ("C", ctypes.c_int32), ("H", ctypes.c_int32), ("W", ctypes.c_int32),
                ("K", ctypes.c_int32), ("R", ctypes.c_int32), ("S", ctypes.c_int32),
                ("stride_h", ctypes.c_int32), ("stride_w", ctypes.c_int32),
                ("pad_h", ctypes.c_int32), ("pad_w", ctypes.c_int32),
                ("dil_h", ctypes.c_int32), ("dil_w", ctypes.c_int32),
                ("layout", ctypes.c_int32),
                ("x_stride", ctypes.c_int64 * 4), ("y_stride", ctypes.c_int64 * 4),
                ("groups", ctypes.c_int32), ("route", ctypes.c_int32)]


class ConvRoute(ctypes.Structure):
    _fields_ = [("kernel", ctypes.c_int32), ("tile_m", ctypes.c_int32), ("tile_n", ctypes.c_int32),
                ("ksplit", ctypes.c_int32), ("wave_groups", ctypes.c_int32), ("work_groups", ctypes.c_int32),
                ("workspace_bytes", ctypes.c_uint64)]


ANR_CONV_ROUTE_AUTO, ANR_CONV_ROUTE_PATCH, ANR_CONV_ROUTE_GENERAL = 0, 1, 2
ANR_CONV_KERNEL_PATCH, ANR_CONV_KERNEL_TAPS, ANR_CONV_KERNEL_BIGTAPS, ANR_CONV_KERNEL_GATHER, \
    ANR_CONV_KERNEL_DIRECT, ANR_CONV_KERNEL_POINTWISE = 1, 2, 3, 4, 5, 6


class NrmDesc(ctypes.Structure):
    _fields_ = [("N", ctypes.c_int64), ("M", ctypes.c_int64), ("ld", ctypes.c_int64),
                ("batch", ctypes.c_int64), ("stride", ctypes.c_int64)]


class TbgDesc(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("S", ctypes.c_int32), ("H", ctypes.c_int32), ("D", ctypes.c_int32),
                ("q_stride", ctypes.c_int64 * 4), ("k_stride", ctypes.c_int64 * 4),
                ("o_stride", ctypes.c_int64 * 4)]


_vp = ctypes.c_void_p
_lib.anr_gemm.argtypes = [ctypes.POINTER(GemmDesc), _vp, _vp, _vp, _vp, ctypes.c_size_t, _vp]
_lib.anr_conv2d.argtypes = [ctypes.POINTER(ConvDesc), _vp, _vp, _vp, _vp, ctypes.c_size_t, _vp]
_lib.anr_conv2d_noalloc.argtypes = [ctypes.POINTER(ConvDesc), _vp, _vp, _vp, _vp]
_lib.anr_conv2d_packed_size.argtypes = [ctypes.POINTER(ConvDesc), ctypes.POINTER(ctypes.c_size_t)]
_lib.anr_conv2d_pack_weights.argtypes = [ctypes.POINTER(ConvDesc), _vp, _vp, _vp, _vp, _vp, ctypes.c_float, _vp,
                                         ctypes.c_size_t, _vp]
_lib.anr_conv2d_packed.argtypes = [ctypes.POINTER(ConvDesc), _vp, _vp, _vp, _vp, ctypes.c_size_t, _vp]
_lib.anr_conv_bn_relu_packed.argtypes = [ctypes.POINTER(ConvDesc), _vp, _vp, _vp, _vp, ctypes.c_size_t, _vp]
_lib.anr_conv_bn_relu.argtypes = [ctypes.POINTER(ConvDesc), _vp, _vp, _vp, _vp, _vp, _vp, ctypes.c_float,
                                  _vp, _vp, ctypes.c_size_t, _vp]
_lib.anr_dwconv.argtypes = [ctypes.POINTER(ConvDesc), _vp, _vp, _vp, _vp, ctypes.c_size_t, _vp]
_lib.anr_tbg.argtypes = [ctypes.POINTER(TbgDesc), _vp, _vp, _vp, _vp, ctypes.c_size_t, _vp]
_lib.anr_tbs.argtypes = [ctypes.POINTER(TbgDesc), _vp, _vp, _vp, _vp, ctypes.c_size_t, _vp]
_lib.anr_nrm.argtypes = [ctypes.POINTER(NrmDesc), _vp, _vp, _vp, ctypes.c_size_t, _vp]
_lib.anr_workspace_size.argtypes = [ctypes.c_int, _vp, ctypes.POINTER(ctypes.c_size_t)]
_lib.anr_conv2d_route.argtypes = [ctypes.POINTER(ConvDesc), ctypes.POINTER(ConvRoute)]
for _name in ("anr_gemm", "anr_conv2d", "anr_conv2d_noalloc", "anr_conv2d_packed_size", "anr_conv2d_pack_weights",
              "anr_conv2d_packed", "anr_conv_bn_relu_packed", "anr_conv_bn_relu", "anr_dwconv", "anr_tbg", "anr_tbs",
              "anr_workspace_size"):
    getattr(_lib, _name).restype = ctypes.c_int
_lib.anr_status_string.argtypes = [ctypes.c_int]
_lib.anr_status_string.restype = ctypes.c_char_p
_lib.anr_version.argtypes = []
_lib.anr_version.restype = ctypes.c_int
_lib.anr_last_hip_error.argtypes = []
_lib.anr_last_hip_error.restype = ctypes.c_int
_lib.anr_last_hip_error_string.argtypes = []
_lib.anr_last_hip_error_string.restype = ctypes.c_char_p


class AnrError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        msg = "%s: %s (status %d)" % (where, status_string(status), status)
        if status == ANR_ERR_LAUNCH:
            msg += " [hip error %d: %s]" % (_lib.anr_last_hip_error(),
                                            _lib.anr_last_hip_error_string().decode())
        super().__init__(msg)


def raw():
    """The ctypes library handle, for tests that call the C ABI with hand-made arguments."""
    return _lib


def status_string(status: int) -> str:
    return _lib.anr_status_string(int(status)).decode()


def version() -> int:
    return int(_lib.anr_version())


def _check(status, where):
    if status != ANR_OK:
        raise AnrError(status, where)


def _ptr(t):
    if not isinstance(t, torch.Tensor) or t.dtype != torch.float32 or not t.is_cuda:
        raise TypeError("expected a float32 CUDA tensor")
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def conv_desc(x_shape, K, R, S, stride=(1, 1), pad=(0, 0), x_stride=None, y_stride=None, dil=(1, 1),
              layout=ANR_LAYOUT_NCHW, groups=1, route=ANR_CONV_ROUTE_AUTO) -> ConvDesc:
    N, C, H, W = x_shape
    d = ConvDesc(N, C, H, W, K, R, S, stride[0], stride[1], pad[0], pad[1], dil[0], dil[1], layout)
    d.groups = groups
    d.route = route
    if x_stride is not None:
        d.x_stride = (ctypes.c_int64 * 4)(*x_stride)
    if y_stride is not None:
        d.y_stride = (ctypes.c_int64 * 4)(*y_stride)
    return d


def _packed(t, shape):
    """True when tensor t is the packed row-major layout of `shape`."""
    return tuple(t.shape) == tuple(shape) and t.is_contiguous()


def workspace_size(op: int, desc) -> int:
    n = ctypes.c_size_t(0)
    _check(_lib.anr_workspace_size(op, ctypes.cast(ctypes.byref(desc), _vp), ctypes.byref(n)),
           "anr_workspace_size")
    return int(n.value)


def conv2d_route(desc: ConvDesc) -> ConvRoute:
    """Which kernel anr_conv2d would run for the descriptor (aligned pointers assumed), its tile,
    split and workspace need; host-side planning only."""
    r = ConvRoute()
    _check(_lib.anr_conv2d_route(ctypes.byref(desc), ctypes.byref(r)), "anr_conv2d_route")
    return r


_workspaces = {}


def _workspace(op: int, desc, ws):
    """(pointer, bytes) of the workspace for one call: the caller's tensor, else a buffer kept
    per (device, stream) and grown on demand (calls on one stream run in order, so they can
    share it; a call never synchronises)."""
    need = workspace_size(op, desc)
    if need == 0:
        return None, 0
    if ws is None:
        key = (torch.cuda.current_device(), torch.cuda.current_stream().cuda_stream)
        ws = _workspaces.get(key)
        if ws is None or ws.numel() < need:
            ws = torch.empty(need, dtype=torch.uint8, device="cuda")
            _workspaces[key] = ws
    if not ws.is_cuda or not ws.is_contiguous() or ws.numel() * ws.element_size() < need:
        raise ValueError("workspace must be a contiguous CUDA tensor of at least %d bytes" % need)
    return ctypes.c_void_p(ws.data_ptr()), ws.numel() * ws.element_size()


def gemm(A, B, C):
    """C = A.B.  A [M,K] / [b,M,K], B [K,N] / [b,K,N], C [M,N] / [b,M,N]; last dim contiguous."""
    if A.dim() == 2:
        M, K = A.shape
        N = B.shape[1]
        d = GemmDesc(M, N, K, A.stride(0), B.stride(0), C.stride(0), 1, 0, 0, 0)
    else:
        b, M, K = A.shape
        N = B.shape[2]
        d = GemmDesc(M, N, K, A.stride(1), B.stride(1), C.stride(1), b,
                     A.stride(0), B.stride(0), C.stride(0))
    if A.stride(-1) != 1 or B.stride(-1) != 1 or C.stride(-1) != 1:
        raise ValueError("innermost dimension must be contiguous")
    _check(_lib.anr_gemm(ctypes.byref(d), _ptr(A), _ptr(B), _ptr(C), None, 0, _stream()), "anr_gemm")
    return C


def _conv_strides(t):
    return None if t.is_contiguous() else tuple(t.stride())


def conv2d(x, w, y, stride=(1, 1), pad=(0, 0), ws=None, dil=(1, 1), groups=1, route=ANR_CONV_ROUTE_AUTO):
    """y = conv2d(x, w); x [N,C,H,W], w [K,C/groups,R,S] packed, y [N,K,OH,OW] (may be strided views).
    ws: optional workspace tensor of at least workspace_size(ANR_OP_CONV2D, desc) bytes."""
    K, _, R, S = w.shape
    if not w.is_contiguous():
        raise ValueError("weights must be packed")
    d = conv_desc(tuple(x.shape), K, R, S, stride, pad, _conv_strides(x), _conv_strides(y), dil=dil, groups=groups,
                  route=route)
    wp, wb = _workspace(ANR_OP_CONV2D, d, ws)
    _check(_lib.anr_conv2d(ctypes.byref(d), _ptr(x), _ptr(w), _ptr(y), wp, wb, _stream()), "anr_conv2d")
    return y


STATIC_SCRATCH_BYTES = 16 << 20


def conv2d_noalloc(x, w, y, stride=(1, 1), pad=(0, 0), dil=(1, 1), groups=1, route=ANR_CONV_ROUTE_AUTO):
    """conv2d without a workspace argument: split reductions use the library's static scratch array."""
    K, _, R, S = w.shape
    if not w.is_contiguous():
        raise ValueError("weights must be packed")
    d = conv_desc(tuple(x.shape), K, R, S, stride, pad, _conv_strides(x), _conv_strides(y), dil=dil, groups=groups,
                  route=route)
    _check(_lib.anr_conv2d_noalloc(ctypes.byref(d), _ptr(x), _ptr(w), _ptr(y), _stream()), "anr_conv2d_noalloc")
    return y


def conv2d_packed_size(desc: ConvDesc) -> int:
    n = ctypes.c_size_t(0)
    _check(_lib.anr_conv2d_packed_size(ctypes.byref(desc), ctypes.byref(n)), "anr_conv2d_packed_size")
    return int(n.value)


def conv2d_pack_weights(x_shape, w, stride=(1, 1), pad=(0, 0), bn=None, eps=0.0, dil=(1, 1), groups=1,
                        route=ANR_CONV_ROUTE_AUTO):
    """Packs w (and, with bn = (gamma, beta, mean, var), the folded batch norm) for the layer that
    x_shape, w and the geometry describe.  Returns (descriptor, pack): the pack is a new uint8 CUDA
    tensor (torch's allocations are 256-byte aligned) to hand to conv2d_packed / conv_bn_relu_packed."""
    K, _, R, S = w.shape
    if not w.is_contiguous():
        raise ValueError("weights must be packed OIHW")
    d = conv_desc(tuple(x_shape), K, R, S, stride, pad, dil=dil, groups=groups, route=route)
    pack = torch.empty(conv2d_packed_size(d), dtype=torch.uint8, device=w.device)
    vecs = [None] * 4 if bn is None else [_ptr(v) for v in bn]
    _check(_lib.anr_conv2d_pack_weights(ctypes.byref(d), _ptr(w), vecs[0], vecs[1], vecs[2], vecs[3],
                                        ctypes.c_float(eps), ctypes.c_void_p(pack.data_ptr()), pack.numel(), _stream()),
           "anr_conv2d_pack_weights")
    return d, pack


def _run_packed(fn, name, desc, x, pack, y, ws):
    d = ConvDesc.from_buffer_copy(desc)
    xs, ys = _conv_strides(x), _conv_strides(y)
    d.x_stride = (ctypes.c_int64 * 4)(*(xs or (0, 0, 0, 0)))
    d.y_stride = (ctypes.c_int64 * 4)(*(ys or (0, 0, 0, 0)))
    op = ANR_OP_CONV2D if fn is _lib.anr_conv2d_packed else ANR_OP_CONV_BN_RELU
    wp, wb = _workspace(op, d, ws)
    _check(fn(ctypes.byref(d), _ptr(x), ctypes.c_void_p(pack.data_ptr()), _ptr(y), wp, wb, _stream()), name)
    return y


def conv2d_packed(desc, x, pack, y, ws=None):
    """conv2d with weights from conv2d_pack_weights (desc: the descriptor it returned)."""
    return _run_packed(_lib.anr_conv2d_packed, "anr_conv2d_packed", desc, x, pack, y, ws)


def conv_bn_relu_packed(desc, x, pack, y, ws=None):
    """conv + batch norm + ReLU with a pack made with bn=(gamma, beta, mean, var)."""
    return _run_packed(_lib.anr_conv_bn_relu_packed, "anr_conv_bn_relu_packed", desc, x, pack, y, ws)


def conv_bn_relu(x, w, gamma, beta, mean, var, eps, y, stride=(1, 1), pad=(0, 0), ws=None, dil=(1, 1), groups=1,
                 route=ANR_CONV_ROUTE_AUTO):
    K, _, R, S = w.shape
    if not w.is_contiguous():
        raise ValueError("weights must be packed")
    for v in (gamma, beta, mean, var):
        if tuple(v.shape) != (K,) or not v.is_contiguous():
            raise ValueError("batch-norm vectors must be packed [K]")
    d = conv_desc(tuple(x.shape), K, R, S, stride, pad, _conv_strides(x), _conv_strides(y), dil=dil, groups=groups,
                  route=route)
    wp, wb = _workspace(ANR_OP_CONV_BN_RELU, d, ws)
    _check(_lib.anr_conv_bn_relu(ctypes.byref(d), _ptr(x), _ptr(w), _ptr(gamma), _ptr(beta), _ptr(mean),
                                 _ptr(var), ctypes.c_float(eps), _ptr(y), wp, wb, _stream()),
           "anr_conv_bn_relu")
    return y


def dwconv(x, w, y, stride=(1, 1), pad=(0, 0), dil=(1, 1)):
    C, _, R, S = w.shape
    if not w.is_contiguous():
        raise ValueError("weights must be packed")
    d = conv_desc(tuple(x.shape), C, R, S, stride, pad, _conv_strides(x), _conv_strides(y), dil=dil)
    _check(_lib.anr_dwconv(ctypes.byref(d), _ptr(x), _ptr(w), _ptr(y), None, 0, _stream()), "anr_dwconv")
    return y


def _tbg_desc(q, k, out) -> TbgDesc:
    B, S, H, D = q.shape
    d = TbgDesc(B, S, H, D)
    if not q.is_contiguous():
        d.q_stride = (ctypes.c_int64 * 4)(*q.stride())
    if not k.is_contiguous():
        d.k_stride = (ctypes.c_int64 * 4)(*k.stride())
    if not out.is_contiguous():
        d.o_stride = (ctypes.c_int64 * 4)(*out.stride())
    return d


def tbg(q, k, out):
    """out[b,h,i,j] = sum_d q[b,i,h,d] k[b,j,h,d]; q,k [B,S,H,D], out [B,H,S,S]."""
    d = _tbg_desc(q, k, out)
    _check(_lib.anr_tbg(ctypes.byref(d), _ptr(q), _ptr(k), _ptr(out), None, 0, _stream()), "anr_tbg")
    return out


def tbs(q, k, out):
    """tbg followed by a softmax over the last axis."""
    d = _tbg_desc(q, k, out)
    _check(_lib.anr_tbs(ctypes.byref(d), _ptr(q), _ptr(k), _ptr(out), None, 0, _stream()), "anr_tbs")
    return out


def nrm(x, out, ws=None):
    """out[b] = sqrt(sum of squares of x[b]).  x [N,M] or [b,N,M] with unit column stride, out [1] / [b]."""
    if x.dim() == 2:
        N, M = x.shape
        d = NrmDesc(N, M, x.stride(0), 1, 0)
    else:
        b, N, M = x.shape
        d = NrmDesc(N, M, x.stride(1), b, x.stride(0) if b > 1 else 0)
    if x.stride(-1) != 1 or not out.is_contiguous() or out.numel() != d.batch:
        raise ValueError("x needs unit column stride and out one packed float per matrix")
    wp, wb = _workspace(ANR_OP_NRM, d, ws)
    _check(_lib.anr_nrm(ctypes.byref(d), _ptr(x), _ptr(out), wp, wb, _stream()), "anr_nrm")
    return out
