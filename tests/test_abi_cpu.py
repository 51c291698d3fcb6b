"""CPU-only checks of the C-ABI library: it loads, exports every declared symbol, its
descriptor structs have the layout the binding assumes, and every argument error is
reported as a return code before anything could be launched (no GPU is touched)."""
import ctypes
import os
import re
import subprocess

import numpy as np
import pytest

from paper_2006_06762_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "anr.h")
DUMMY = ctypes.c_void_p(0x1000)       # never dereferenced: validation fails first


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(anr_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert set(names) == set(B.EXPORTS)
    lib = B.raw()
    for n in names:
        assert getattr(lib, n) is not None


def test_version_and_status_strings():
    assert B.version() >= 100
    seen = {B.status_string(s) for s in range(6)}
    assert len(seen) == 6 and "ok" in seen
    assert "unknown" in B.status_string(99)


def test_struct_layout_matches_c(tmp_path):
    # compile a tiny C program against the header and compare sizeof/offsetof with ctypes
    src = tmp_path / "layout.c"
    src.write_text(r'''
#include <stdio.h>
#include <stddef.h>
#include "anr.h"
int main(void) {
  printf("%zu %zu %zu\n", sizeof(anr_gemm_desc), sizeof(anr_conv_desc), sizeof(anr_tbg_desc));
  printf("%zu %zu %zu %zu\n", offsetof(anr_gemm_desc, strideC), offsetof(anr_conv_desc, layout),
         offsetof(anr_conv_desc, x_stride), offsetof(anr_conv_desc, y_stride));
  printf("%zu %zu %zu\n", offsetof(anr_tbg_desc, q_stride), offsetof(anr_tbg_desc, k_stride),
         offsetof(anr_tbg_desc, o_stride));
  printf("%zu %zu\n", offsetof(anr_conv_desc, groups), offsetof(anr_conv_desc, route));
  return 0; }''')
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()
    got = [int(v) for v in out]
    exp = [ctypes.sizeof(B.GemmDesc), ctypes.sizeof(B.ConvDesc), ctypes.sizeof(B.TbgDesc),
           B.GemmDesc.strideC.offset, B.ConvDesc.layout.offset, B.ConvDesc.x_stride.offset,
           B.ConvDesc.y_stride.offset, B.TbgDesc.q_stride.offset, B.TbgDesc.k_stride.offset,
           B.TbgDesc.o_stride.offset, B.ConvDesc.groups.offset, B.ConvDesc.route.offset]
    assert got == exp


def gemm_status(**kw):
    base = dict(M=4, N=4, K=4, lda=4, ldb=4, ldc=4, batch=1, strideA=0, strideB=0, strideC=0)
    base.update(kw)
    d = B.GemmDesc(**base)
    return B.raw().anr_gemm(ctypes.byref(d), DUMMY, DUMMY, DUMMY, None, 0, None)


def test_gemm_validation():
    assert gemm_status(M=0) == B.ANR_ERR_INVALID_ARG
    assert gemm_status(N=-1) == B.ANR_ERR_INVALID_ARG
    assert gemm_status(K=0) == B.ANR_ERR_INVALID_ARG
    assert gemm_status(batch=0) == B.ANR_ERR_INVALID_ARG
    assert gemm_status(lda=3) == B.ANR_ERR_INVALID_ARG
    assert gemm_status(ldb=3) == B.ANR_ERR_INVALID_ARG
    assert gemm_status(ldc=3) == B.ANR_ERR_INVALID_ARG
    assert gemm_status(batch=2, strideC=15) == B.ANR_ERR_INVALID_ARG     # overlapping outputs
    assert gemm_status(batch=70000, strideC=16) == B.ANR_ERR_UNSUPPORTED
    # extents and leading dimensions whose products would leave 64 bits are refused, not multiplied
    assert gemm_status(M=1 << 30, lda=4) == B.ANR_ERR_UNSUPPORTED
    assert gemm_status(ldc=1 << 62, batch=2, strideC=1 << 62) == B.ANR_ERR_UNSUPPORTED
    d = B.GemmDesc(4, 4, 4, 4, 4, 4, 1, 0, 0, 0)
    lib = B.raw()
    assert lib.anr_gemm(None, DUMMY, DUMMY, DUMMY, None, 0, None) == B.ANR_ERR_NULL
    assert lib.anr_gemm(ctypes.byref(d), None, DUMMY, DUMMY, None, 0, None) == B.ANR_ERR_NULL
    assert lib.anr_gemm(ctypes.byref(d), DUMMY, None, DUMMY, None, 0, None) == B.ANR_ERR_NULL
    assert lib.anr_gemm(ctypes.byref(d), DUMMY, DUMMY, None, None, 0, None) == B.ANR_ERR_NULL


def conv_status(fn="anr_conv2d", x_stride=None, y_stride=None, **kw):
    base = dict(N=1, C=4, H=8, W=8, K=4, R=3, S=3, stride_h=1, stride_w=1, pad_h=1, pad_w=1,
                dil_h=1, dil_w=1, layout=0)
    base.update(kw)
    d = B.ConvDesc(**base)
    if x_stride:
        d.x_stride = (ctypes.c_int64 * 4)(*x_stride)
    if y_stride:
        d.y_stride = (ctypes.c_int64 * 4)(*y_stride)
    lib = B.raw()
    if fn == "anr_conv_bn_relu":
        return lib.anr_conv_bn_relu(ctypes.byref(d), DUMMY, DUMMY, DUMMY, DUMMY, DUMMY, DUMMY,
                                    ctypes.c_float(1e-5), DUMMY, None, 0, None)
    return getattr(lib, fn)(ctypes.byref(d), DUMMY, DUMMY, DUMMY, None, 0, None)


@pytest.mark.parametrize("fn", ["anr_conv2d", "anr_conv_bn_relu", "anr_dwconv"])
def test_conv_validation(fn):
    for field in ("N", "C", "H", "W", "K", "R", "S", "stride_h", "stride_w"):
        assert conv_status(fn, **{field: 0}) == B.ANR_ERR_INVALID_ARG, field
    assert conv_status(fn, pad_h=-1) == B.ANR_ERR_INVALID_ARG
    assert conv_status(fn, dil_w=0) == B.ANR_ERR_INVALID_ARG
    assert conv_status(fn, H=4, R=3, dil_h=2, pad_h=0) == B.ANR_ERR_INVALID_ARG   # dilated kernel taller than the image
    assert conv_status(fn, groups=-1) == B.ANR_ERR_INVALID_ARG
    assert conv_status(fn, route=3) == B.ANR_ERR_INVALID_ARG
    assert conv_status(fn, route=-1) == B.ANR_ERR_INVALID_ARG
    if fn != "anr_dwconv":
        assert conv_status(fn, groups=3) == B.ANR_ERR_INVALID_ARG                 # channels not a multiple
    assert conv_status(fn, layout=1) == B.ANR_ERR_UNSUPPORTED
    assert conv_status(fn, H=2, R=5, pad_h=1) == B.ANR_ERR_INVALID_ARG          # empty output
    assert conv_status(fn, x_stride=(256, 64, 8, 2)) == B.ANR_ERR_UNSUPPORTED   # w stride != 1
    assert conv_status(fn, x_stride=(256, 64, 7, 1)) == B.ANR_ERR_INVALID_ARG   # rows overlap
    assert conv_status(fn, x_stride=(256, 60, 8, 1)) == B.ANR_ERR_INVALID_ARG   # planes overlap
    assert conv_status(fn, x_stride=(255, 64, 8, 1)) == B.ANR_ERR_INVALID_ARG   # images overlap
    assert conv_status(fn, y_stride=(256, 64, 8, -1)) == B.ANR_ERR_INVALID_ARG


def test_dwconv_requires_k_equals_c():
    assert conv_status("anr_dwconv", K=8) == B.ANR_ERR_INVALID_ARG


def test_conv_null_pointers():
    d = B.conv_desc((1, 4, 8, 8), 4, 3, 3, (1, 1), (1, 1))
    lib = B.raw()
    assert lib.anr_conv2d(None, DUMMY, DUMMY, DUMMY, None, 0, None) == B.ANR_ERR_NULL
    assert lib.anr_conv2d(ctypes.byref(d), None, DUMMY, DUMMY, None, 0, None) == B.ANR_ERR_NULL
    assert lib.anr_dwconv(ctypes.byref(d), DUMMY, None, DUMMY, None, 0, None) == B.ANR_ERR_NULL
    assert lib.anr_conv_bn_relu(ctypes.byref(d), DUMMY, DUMMY, DUMMY, None, DUMMY, DUMMY,
                                ctypes.c_float(1e-5), DUMMY, None, 0, None) == B.ANR_ERR_NULL
    assert lib.anr_conv_bn_relu(ctypes.byref(d), DUMMY, DUMMY, DUMMY, DUMMY, DUMMY, DUMMY,
                                ctypes.c_float(float("nan")), DUMMY, None, 0, None) == B.ANR_ERR_INVALID_ARG


def test_conv2d_noalloc_validation():
    # the entry point without a workspace argument validates as anr_conv2d does, before anything else
    lib = B.raw()
    d = B.conv_desc((1, 4, 8, 8), 4, 3, 3, (1, 1), (1, 1))
    assert lib.anr_conv2d_noalloc(None, DUMMY, DUMMY, DUMMY, None) == B.ANR_ERR_NULL
    assert lib.anr_conv2d_noalloc(ctypes.byref(d), None, DUMMY, DUMMY, None) == B.ANR_ERR_NULL
    assert lib.anr_conv2d_noalloc(ctypes.byref(d), DUMMY, DUMMY, None, None) == B.ANR_ERR_NULL
    d.stride_w = 0
    assert lib.anr_conv2d_noalloc(ctypes.byref(d), DUMMY, DUMMY, DUMMY, None) == B.ANR_ERR_INVALID_ARG
    text = open(HEADER).read()
    assert int(re.search(r"ANR_STATIC_SCRATCH_BYTES \(\(size_t\)(\d+) << 20\)", text).group(1)) << 20 == B.STATIC_SCRATCH_BYTES


def test_packed_weights_size_and_validation():
    lib = B.raw()
    n = ctypes.c_size_t(0)
    # patch-kernel plan: scale/shift block (2K floats rounded up to 64) + per channel tile and chunk an
    # LDS image of 32 rows x (8 channels x 9 taps + 4) floats for the 28x28 ConvLayer shape
    d = B.conv_desc((16, 128, 28, 28), 128, 3, 3, (1, 1), (1, 1))
    assert B.conv2d_packed_size(d) == 4 * (256 + 4 * 16 * 32 * (8 * 9 + 4))
    # the stride-2 layer: chunks of 8 channels, 16 channel tiles of 32
    d2 = B.conv_desc((16, 256, 28, 28), 512, 3, 3, (2, 2), (1, 1))
    assert B.conv2d_packed_size(d2) == 4 * (1024 + 16 * 32 * 32 * (8 * 9 + 4))
    # any other plan keeps OIHW order
    d3 = B.conv_desc((1, 3, 224, 224), 64, 7, 7, (2, 2), (3, 3))
    assert B.conv2d_packed_size(d3) == 4 * (128 + 64 * 3 * 49)
    # the route is part of the plan
    d4 = B.conv_desc((16, 128, 28, 28), 128, 3, 3, (1, 1), (1, 1), route=B.ANR_CONV_ROUTE_GENERAL)
    assert B.conv2d_packed_size(d4) == 4 * (256 + 128 * 128 * 9)
    assert lib.anr_conv2d_packed_size(ctypes.byref(d), None) == B.ANR_ERR_NULL
    assert lib.anr_conv2d_packed_size(None, ctypes.byref(n)) == B.ANR_ERR_NULL
    need = B.conv2d_packed_size(d)
    f = ctypes.c_float(1e-5)
    pack = ctypes.c_void_p(0x10000)
    assert lib.anr_conv2d_pack_weights(ctypes.byref(d), None, None, None, None, None, f, pack, need, None) == B.ANR_ERR_NULL
    assert lib.anr_conv2d_pack_weights(ctypes.byref(d), DUMMY, None, None, None, None, f, None, need, None) == B.ANR_ERR_NULL
    # batch-norm vectors: all four or none
    assert lib.anr_conv2d_pack_weights(ctypes.byref(d), DUMMY, DUMMY, None, None, None, f, pack, need, None) == B.ANR_ERR_NULL
    assert lib.anr_conv2d_pack_weights(ctypes.byref(d), DUMMY, DUMMY, DUMMY, DUMMY, DUMMY, ctypes.c_float(float("inf")),
                                       pack, need, None) == B.ANR_ERR_INVALID_ARG
    assert lib.anr_conv2d_pack_weights(ctypes.byref(d), DUMMY, None, None, None, None, f, pack, need - 1,
                                       None) == B.ANR_ERR_WORKSPACE
    assert lib.anr_conv2d_pack_weights(ctypes.byref(d), DUMMY, None, None, None, None, f, ctypes.c_void_p(0x10010), need,
                                       None) == B.ANR_ERR_INVALID_ARG          # pack not 256-byte aligned
    for fn in (lib.anr_conv2d_packed, lib.anr_conv_bn_relu_packed):
        assert fn(ctypes.byref(d), None, pack, DUMMY, None, 0, None) == B.ANR_ERR_NULL
        assert fn(ctypes.byref(d), DUMMY, None, DUMMY, None, 0, None) == B.ANR_ERR_NULL
        assert fn(ctypes.byref(d), DUMMY, ctypes.c_void_p(0x10010), DUMMY, None, 0, None) == B.ANR_ERR_INVALID_ARG
        assert fn(None, DUMMY, pack, DUMMY, None, 0, None) == B.ANR_ERR_NULL
        # a pack in the patch kernel's order and an x that kernel cannot read
        assert fn(ctypes.byref(d), ctypes.c_void_p(0x1004), pack, DUMMY, None, 0, None) == B.ANR_ERR_INVALID_ARG


@pytest.mark.parametrize("fn", ["anr_tbg", "anr_tbs"])
def test_tbg_validation(fn):
    lib = B.raw()
    f = getattr(lib, fn)
    for field in ("B", "S", "H", "D"):
        kw = dict(B=1, S=4, H=2, D=4)
        kw[field] = 0
        d = B.TbgDesc(**kw)
        assert f(ctypes.byref(d), DUMMY, DUMMY, DUMMY, None, 0, None) == B.ANR_ERR_INVALID_ARG
    d = B.TbgDesc(1, 4, 2, 4)
    assert f(None, DUMMY, DUMMY, DUMMY, None, 0, None) == B.ANR_ERR_NULL
    assert f(ctypes.byref(d), DUMMY, DUMMY, None, None, 0, None) == B.ANR_ERR_NULL
    d.q_stride = (ctypes.c_int64 * 4)(32, 8, 4, 2)
    assert f(ctypes.byref(d), DUMMY, DUMMY, DUMMY, None, 0, None) == B.ANR_ERR_UNSUPPORTED
    d = B.TbgDesc(1, 4, 2, 4)
    d.o_stride = (ctypes.c_int64 * 4)(32, 16, 3, 1)       # rows overlap
    assert f(ctypes.byref(d), DUMMY, DUMMY, DUMMY, None, 0, None) == B.ANR_ERR_INVALID_ARG
    d.o_stride = (ctypes.c_int64 * 4)(32, 15, 4, 1)       # heads overlap
    assert f(ctypes.byref(d), DUMMY, DUMMY, DUMMY, None, 0, None) == B.ANR_ERR_INVALID_ARG
    d.o_stride = (ctypes.c_int64 * 4)(31, 16, 4, 1)       # batches overlap
    assert f(ctypes.byref(d), DUMMY, DUMMY, DUMMY, None, 0, None) == B.ANR_ERR_INVALID_ARG
    if fn == "anr_tbs":
        d = B.TbgDesc(1, 2048, 1, 4)
        assert f(ctypes.byref(d), DUMMY, DUMMY, DUMMY, None, 0, None) == B.ANR_ERR_UNSUPPORTED


def test_nrm_validation():
    lib = B.raw()
    ok = dict(N=8, M=8, ld=8, batch=1, stride=0)
    for field, bad in (("N", 0), ("M", 0), ("batch", 0), ("ld", 7), ("stride", -1)):
        d = B.NrmDesc(**dict(ok, **{field: bad}))
        assert lib.anr_nrm(ctypes.byref(d), DUMMY, DUMMY, None, 0, None) == B.ANR_ERR_INVALID_ARG, field
    d = B.NrmDesc(**ok)
    assert lib.anr_nrm(None, DUMMY, DUMMY, None, 0, None) == B.ANR_ERR_NULL
    assert lib.anr_nrm(ctypes.byref(d), None, DUMMY, None, 0, None) == B.ANR_ERR_NULL
    assert lib.anr_nrm(ctypes.byref(d), DUMMY, None, None, 0, None) == B.ANR_ERR_NULL
    assert lib.anr_nrm(ctypes.byref(B.NrmDesc(8, 8, 8, 70000, 64)), DUMMY, DUMMY, None, 0, None) == B.ANR_ERR_UNSUPPORTED
    assert lib.anr_nrm(ctypes.byref(B.NrmDesc(8, 8, 8, 2, 63)), DUMMY, DUMMY, None, 0, None) == B.ANR_ERR_INVALID_ARG  # matrices overlap
    assert lib.anr_nrm(ctypes.byref(B.NrmDesc(8, 8, 1 << 40, 1, 0)), DUMMY, DUMMY, None, 0, None) == B.ANR_ERR_UNSUPPORTED
    assert B.workspace_size(B.ANR_OP_NRM, d) == 0                      # one slice: no partial sums
    big = B.NrmDesc(4096, 4096, 4096, 1, 0)
    need = B.workspace_size(B.ANR_OP_NRM, big)
    assert need == 4 * 1024                                             # 16 M elements in 1024 slices
    assert lib.anr_nrm(ctypes.byref(big), DUMMY, DUMMY, None, 0, None) == B.ANR_ERR_WORKSPACE


def test_workspace_size():
    g = B.GemmDesc(512, 512, 512, 512, 512, 512, 1, 0, 0, 0)
    assert B.workspace_size(B.ANR_OP_GEMM, g) == 0
    c = B.conv_desc((16, 64, 56, 56), 64, 3, 3, (1, 1), (1, 1))
    assert B.workspace_size(B.ANR_OP_CONV2D, c) == 0
    assert B.workspace_size(B.ANR_OP_CONV_BN_RELU, c) == 0
    assert B.workspace_size(B.ANR_OP_TBG, B.TbgDesc(16, 128, 12, 64)) == 0
    # few output tiles and a long reduction: the general kernel splits K over a workspace
    small = B.conv_desc((1, 512, 7, 7), 512, 3, 3, (1, 1), (1, 1))
    need = B.workspace_size(B.ANR_OP_CONV2D, small)
    assert need > 0 and need % 16 == 0
    assert B.workspace_size(B.ANR_OP_CONV_BN_RELU, small) == need
    lib = B.raw()
    # reported before anything is launched: missing, too small, misaligned
    assert lib.anr_conv2d(ctypes.byref(small), DUMMY, DUMMY, DUMMY, None, 0, None) == B.ANR_ERR_WORKSPACE
    assert lib.anr_conv2d(ctypes.byref(small), DUMMY, DUMMY, DUMMY, DUMMY, need - 1, None) == B.ANR_ERR_WORKSPACE
    assert lib.anr_conv2d(ctypes.byref(small), DUMMY, DUMMY, DUMMY, ctypes.c_void_p(0x1004), need,
                          None) == B.ANR_ERR_INVALID_ARG
    with pytest.raises(B.AnrError):
        B.workspace_size(B.ANR_OP_DWCONV, c.__class__(1, 4, 8, 8, 8, 3, 3, 1, 1, 1, 1, 1, 1, 0))
    with pytest.raises(B.AnrError):
        B.workspace_size(42, g)
    n = ctypes.c_size_t(0)
    assert B.raw().anr_workspace_size(0, None, ctypes.byref(n)) == B.ANR_ERR_NULL


# ------------------------------------------------------------------ which kernel a convolution takes
def route(x_shape, K, R, stride=1, pad=0, dil=1, groups=1):
    d = B.conv_desc(x_shape, K, R, R, (stride, stride), (pad, pad), dil=(dil, dil), groups=groups)
    return d, B.conv2d_route(d)


def test_conv_route_benchmark_configs_take_the_patch_kernel():
    # the three convolution launches of the benchmark step: tuned kernel, no split, no workspace
    for shape, K, stride, tile in [((16, 64, 56, 56), 64, 1, (224, 64)), ((16, 128, 28, 28), 128, 1, (224, 32)),
                                   ((16, 256, 28, 28), 512, 2, (224, 32))]:
        d, r = route(shape, K, 3, stride, 1)
        assert r.kernel == B.ANR_CONV_KERNEL_PATCH and (r.tile_m, r.tile_n) == tile
        assert r.ksplit == 1 and r.workspace_bytes == 0 and r.work_groups == 224
        assert B.workspace_size(B.ANR_OP_CONV2D, d) == 0 and B.workspace_size(B.ANR_OP_CONV_BN_RELU, d) == 0


def test_conv_route_follows_the_descriptor_field():
    # many output tiles: the library's choice is the patch kernel; route 2 keeps it out
    auto = B.conv_desc((16, 64, 56, 56), 64, 3, 3, (1, 1), (1, 1))
    gen = B.conv_desc((16, 64, 56, 56), 64, 3, 3, (1, 1), (1, 1), route=B.ANR_CONV_ROUTE_GENERAL)
    assert B.conv2d_route(auto).kernel == B.ANR_CONV_KERNEL_PATCH
    assert B.conv2d_route(gen).kernel == B.ANR_CONV_KERNEL_TAPS
    # few output tiles: the library's choice is the general kernel with a split reduction; route 1
    # forces the patch kernel, which needs no workspace
    auto = B.conv_desc((1, 64, 56, 56), 64, 3, 3, (1, 1), (1, 1))
    patch = B.conv_desc((1, 64, 56, 56), 64, 3, 3, (1, 1), (1, 1), route=B.ANR_CONV_ROUTE_PATCH)
    ra, rp = B.conv2d_route(auto), B.conv2d_route(patch)
    assert ra.kernel == B.ANR_CONV_KERNEL_TAPS and ra.ksplit > 1
    assert rp.kernel == B.ANR_CONV_KERNEL_PATCH and rp.workspace_bytes == 0
    # the workspace figure is the plan's own need, route by route
    assert B.workspace_size(B.ANR_OP_CONV2D, auto) == ra.workspace_bytes > 0
    assert B.workspace_size(B.ANR_OP_CONV2D, patch) == 0
    # a shape the patch kernel cannot run (width not a multiple of 4) takes the general one under any route
    odd = B.conv_desc((16, 64, 14, 14), 64, 3, 3, (1, 1), (1, 1), route=B.ANR_CONV_ROUTE_PATCH)
    assert B.conv2d_route(odd).kernel == B.ANR_CONV_KERNEL_TAPS


def test_no_environment_variable_steers_the_library():
    # what a call does follows from its arguments alone
    csrc = os.path.join(ROOT, "paper_2006_06762_amd", "csrc")
    for name in sorted(os.listdir(csrc)):
        text = open(os.path.join(csrc, name)).read()
        assert "getenv" not in text and "environ" not in text, name


def test_conv_route_large_batch_without_split_keeps_the_mfma_kernels():
    # a VGG-style stem at batch 32: 3 channels rule out the tap kernels, and the cap on the split-K
    # workspace must not apply to plans that do not split
    d, r = route((32, 3, 224, 224), 64, 3, 1, 1)
    assert r.kernel == B.ANR_CONV_KERNEL_GATHER and r.ksplit == 1 and r.workspace_bytes == 0


def test_conv_route_by_kernel_size_and_channels():
    K = B
    # few output tiles: the tuned kernel steps aside, the reduction is split through the workspace
    d, r = route((1, 64, 56, 56), 64, 3, 1, 1)
    assert r.kernel == K.ANR_CONV_KERNEL_TAPS and r.ksplit > 1 and r.workspace_bytes > 0
    assert r.workspace_bytes == K.workspace_size(K.ANR_OP_CONV2D, d)
    # 14x14 and 7x7 maps (width not a multiple of 4), pointwise layers: compile-time taps, 64x64 tiles
    for shape, Kout, R, pad in [((16, 256, 14, 14), 256, 3, 1), ((16, 512, 7, 7), 512, 3, 1), ((16, 64, 56, 56), 256, 1, 0),
                                ((16, 1024, 14, 14), 256, 1, 0)]:
        d, r = route(shape, Kout, R, 1, pad)
        assert r.kernel == K.ANR_CONV_KERNEL_TAPS and (r.tile_m, r.tile_n) == (64, 64)
        assert r.workspace_bytes == K.workspace_size(K.ANR_OP_CONV2D, d)
    # pointwise layers with few channels on dense images, grouped or not: the streaming kernel (no
    # workspace); not with more channels, groups that are not whole 16-byte units of a weight row, a
    # stride, too few tiles, or when the general family is ruled out by route 1
    d, r = route((16, 64, 56, 56), 64, 1)
    assert r.kernel == K.ANR_CONV_KERNEL_POINTWISE and r.work_groups == 16 * 49 and r.workspace_bytes == 0
    assert K.workspace_size(K.ANR_OP_CONV2D, d) == 0
    assert route((16, 128, 28, 28), 100, 1)[1].kernel == K.ANR_CONV_KERNEL_POINTWISE
    assert route((16, 256, 28, 28), 64, 1)[1].kernel == K.ANR_CONV_KERNEL_TAPS
    assert route((16, 64, 56, 56), 64, 1, stride=2)[1].kernel == K.ANR_CONV_KERNEL_TAPS
    assert route((1, 64, 56, 56), 64, 1)[1].kernel == K.ANR_CONV_KERNEL_TAPS
    assert route((16, 64, 56, 56), 64, 1, groups=4)[1].kernel == K.ANR_CONV_KERNEL_POINTWISE
    assert route((16, 96, 56, 56), 96, 1, groups=16)[1].kernel != K.ANR_CONV_KERNEL_POINTWISE      # 6 channels per group
    assert route((16, 64, 56, 56), 64, 1, dil=2)[1].kernel == K.ANR_CONV_KERNEL_POINTWISE      # one tap: dilation is moot
    # 7x7 stem and 5x5: one channel per chunk
    assert route((16, 3, 224, 224), 64, 7, 2, 3)[1].kernel == K.ANR_CONV_KERNEL_BIGTAPS
    assert route((2, 32, 28, 28), 64, 5, 1, 2)[1].kernel == K.ANR_CONV_KERNEL_BIGTAPS
    # channel counts the tap kernels do not divide, other kernel sizes: any-geometry kernel
    assert route((2, 6, 20, 20), 16, 3, 1, 1)[1].kernel == K.ANR_CONV_KERNEL_GATHER
    assert route((2, 48, 20, 20), 16, 1)[1].kernel == K.ANR_CONV_KERNEL_GATHER
    assert route((2, 8, 20, 20), 16, 4, 1, 1)[1].kernel == K.ANR_CONV_KERNEL_GATHER
    # dilation and groups never take the patch kernel
    assert route((16, 64, 56, 56), 64, 3, 1, 2, dil=2)[1].kernel == K.ANR_CONV_KERNEL_TAPS
    assert route((16, 64, 56, 56), 64, 3, 1, 1, groups=4)[1].kernel == K.ANR_CONV_KERNEL_TAPS


def test_conv_route_wave_groups_and_split():
    # about 200 tiles with a long chain and no split: two, then four groups of waves share it
    r = route((4, 512, 7, 7), 2048, 1)[1]
    assert (r.kernel, r.ksplit, r.wave_groups, r.work_groups) == (B.ANR_CONV_KERNEL_TAPS, 1, 2, 128)
    r = route((16, 1024, 14, 14), 256, 1)[1]
    assert (r.ksplit, r.wave_groups, r.work_groups) == (1, 4, 196)
    # many tiles: one group, no split
    r = route((16, 64, 56, 56), 256, 1)[1]
    assert (r.ksplit, r.wave_groups) == (1, 1) and r.work_groups == 784 * 4
    # the split never leaves a work-group without chunks and stays within the stated workspace
    for shape, Kout, R, pad in [((1, 256, 14, 14), 256, 3, 1), ((1, 512, 7, 7), 512, 3, 1), ((4, 512, 7, 7), 512, 3, 1),
                                ((1, 3, 224, 224), 64, 7, 3)]:
        d, r = route(shape, Kout, R, 1 if R == 3 else 2, pad)
        assert 1 <= r.ksplit <= 4608 and r.work_groups % r.ksplit == 0
        assert r.workspace_bytes == B.workspace_size(B.ANR_OP_CONV2D, d)
        assert (r.workspace_bytes > 0) == (r.ksplit > 1)


def test_conv_route_packs_small_groups_of_pointwise_layers():
    # 56x56, 256 -> 64, 1x1, 4 groups of 16 output channels: the four groups share one 64-wide column
    # tile (784 work-groups, as for an ungrouped layer) instead of taking a quarter-filled tile each
    r = route((16, 256, 56, 56), 64, 1, groups=4)[1]
    assert (r.kernel, r.tile_n, r.ksplit, r.wave_groups, r.work_groups) == (B.ANR_CONV_KERNEL_TAPS, 64, 1, 1, 784)
    # 32 groups of 4 output channels: two packs of 16 groups
    assert route((16, 256, 28, 28), 128, 1, groups=32)[1].work_groups == 196 * 2
    # groups of 64 output channels and more are not packed; neither are 12 groups (not a multiple of 4)
    assert route((16, 256, 28, 28), 256, 1, groups=4)[1].work_groups == 196 * 4
    r = route((1, 48, 5, 5), 48, 1, groups=12)[1]
    assert r.kernel == B.ANR_CONV_KERNEL_GATHER and r.work_groups % 12 == 0


def test_conv_route_beyond_32bit_offsets_is_the_direct_kernel():
    r = route((1, 2, 16400, 16400), 1, 3, 1, 1)[1]
    assert r.kernel == B.ANR_CONV_KERNEL_DIRECT and r.workspace_bytes == 0


def test_conv_planning_random_descriptors():
    """Host-side planning over a few thousand random layer descriptors, all three routes: every plan
    names a kernel, a tile and a work-group count, the workspace query agrees with it, the pack size
    is that of the weights or more, and forcing the general route never picks the patch kernel."""
    g = np.random.Generator(np.random.PCG64(20060676))
    kernels = {B.ANR_CONV_KERNEL_PATCH, B.ANR_CONV_KERNEL_GATHER, B.ANR_CONV_KERNEL_TAPS, B.ANR_CONV_KERNEL_BIGTAPS,
               B.ANR_CONV_KERNEL_DIRECT, B.ANR_CONV_KERNEL_POINTWISE}
    seen = set()
    for i in range(3000):
        R = int(g.choice([1, 3, 3, 3, 5, 7]))
        groups = int(g.choice([1, 1, 1, 2, 4]))
        C = groups * int(g.choice([1, 3, 4, 8, 16, 24, 32, 64, 96]))
        K = groups * int(g.choice([1, 8, 16, 32, 48, 64, 100]))
        H = int(g.choice([7, 8, 14, 16, 28, 30, 56, 57, 112]))
        W = int(g.choice([7, 8, 12, 14, 16, 28, 36, 56, 60, 112, 224]))
        N = int(g.choice([1, 2, 4, 16, 33]))
        stride = int(g.choice([1, 1, 2]))
        dil = int(g.choice([1, 1, 1, 2]))
        pad = int(g.choice([0, R // 2, R // 2, R - 1]))
        if (H + 2 * pad - dil * (R - 1) - 1) < 0 or (W + 2 * pad - dil * (R - 1) - 1) < 0:
            continue
        for rt in (B.ANR_CONV_ROUTE_AUTO, B.ANR_CONV_ROUTE_PATCH, B.ANR_CONV_ROUTE_GENERAL):
            d = B.conv_desc((N, C, H, W), K, R, R, (stride, stride), (pad, pad), dil=(dil, dil), groups=groups, route=rt)
            r = B.conv2d_route(d)
            assert r.kernel in kernels, (i, rt)
            assert r.tile_m > 0 and r.tile_n > 0 and r.work_groups > 0 and r.ksplit >= 1, (i, rt, r.kernel)
            assert r.workspace_bytes == B.workspace_size(B.ANR_OP_CONV2D, d) == B.workspace_size(B.ANR_OP_CONV_BN_RELU, d)
            assert (r.workspace_bytes > 0) == (r.ksplit > 1), (i, rt)
            assert B.conv2d_packed_size(d) >= 4 * K * (C // groups) * R * R
            if rt == B.ANR_CONV_ROUTE_GENERAL:
                assert r.kernel != B.ANR_CONV_KERNEL_PATCH
            seen.add(r.kernel)
    assert {B.ANR_CONV_KERNEL_PATCH, B.ANR_CONV_KERNEL_GATHER, B.ANR_CONV_KERNEL_TAPS, B.ANR_CONV_KERNEL_POINTWISE} <= seen


def test_conv_route_validation():
    r = B.ConvRoute()
    assert B.raw().anr_conv2d_route(None, ctypes.byref(r)) == B.ANR_ERR_NULL
    d = B.conv_desc((1, 4, 8, 8), 8, 3, 3, (1, 1), (1, 1))
    assert B.raw().anr_conv2d_route(ctypes.byref(d), None) == B.ANR_ERR_NULL
    d.stride_h = 0
    assert B.raw().anr_conv2d_route(ctypes.byref(d), ctypes.byref(r)) == B.ANR_ERR_INVALID_ARG
