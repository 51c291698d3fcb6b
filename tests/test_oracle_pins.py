"""Pins for the fp64 CPU oracle (CPU only).

The paper (arXiv 2006.06762) prints no numeric example for any operator, so
the oracle is pinned to what the mathematics fixes: closed forms, invariants,
reductions of one operator to another, and a second, differently written
evaluation (numpy einsum / explicit padding and window slicing) on small
shapes.  Each test names the plausible mistake it would catch.
"""
import math

import numpy as np
import pytest

import oracle
from paper_2006_06762_amd import inputs as I

F64 = np.float64


def rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


# ---------------------------------------------------------------- helpers
def ref_conv_windows(x, w, stride, pad):
    """Independent evaluation: explicit zero padding, then one einsum per tap."""
    x = x.astype(F64)
    w = w.astype(F64)
    N, C, H, W = x.shape
    K, _, R, S = w.shape
    xp = np.pad(x, ((0, 0), (0, 0), (pad[0], pad[0]), (pad[1], pad[1])))
    OH = (H + 2 * pad[0] - R) // stride[0] + 1
    OW = (W + 2 * pad[1] - S) // stride[1] + 1
    y = np.zeros((N, K, OH, OW), dtype=F64)
    for r in range(R):
        for s in range(S):
            win = xp[:, :, r:r + (OH - 1) * stride[0] + 1:stride[0],
                     s:s + (OW - 1) * stride[1] + 1:stride[1]]
            y += np.einsum("nchw,kc->nkhw", win, w[:, :, r, s])
    return y


def im2col(x, R, S, stride, pad):
    """[N*OH*OW, C*R*S] matrix of fp32 patches, built with plain loops."""
    N, C, H, W = x.shape
    OH = (H + 2 * pad[0] - R) // stride[0] + 1
    OW = (W + 2 * pad[1] - S) // stride[1] + 1
    cols = np.zeros((N * OH * OW, C * R * S), dtype=np.float32)
    for n in range(N):
        for oh in range(OH):
            for ow in range(OW):
                row = (n * OH + oh) * OW + ow
                for c in range(C):
                    for r in range(R):
                        for s in range(S):
                            ih = oh * stride[0] - pad[0] + r
                            iw = ow * stride[1] - pad[1] + s
                            if 0 <= ih < H and 0 <= iw < W:
                                cols[row, (c * R + r) * S + s] = x[n, c, ih, iw]
    return cols, OH, OW


# ---------------------------------------------------------------- GEMM
@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (5, 7, 3), (33, 17, 65), (64, 64, 64)])
def test_gemm_vs_einsum(M, N, K):
    # catches: transposed operand, wrong leading dimension, dropped k term
    A, B = I.gemm_inputs(I.GemmShape(M, N, K), 11)
    ref = np.einsum("ik,kj->ij", A.astype(F64), B.astype(F64))
    np.testing.assert_allclose(oracle.gemm(A, B), ref, rtol=0, atol=1e-12)


def test_gemm_batched_vs_einsum():
    A, B = I.gemm_inputs(I.GemmShape(6, 5, 9, batch=3), 12)
    ref = np.einsum("bik,bkj->bij", A.astype(F64), B.astype(F64))
    np.testing.assert_allclose(oracle.gemm(A, B), ref, rtol=0, atol=1e-12)


def test_gemm_identity_zero_permutation():
    # identity B returns A, zero B returns 0, permutation B permutes columns: all exact
    A, _ = I.gemm_inputs(I.GemmShape(13, 9, 9), 13)
    eye = np.eye(9, dtype=np.float32)
    assert np.array_equal(oracle.gemm(A, eye), A.astype(F64))
    assert np.array_equal(oracle.gemm(A, np.zeros((9, 9), np.float32)), np.zeros((13, 9)))
    perm = rng(3).permutation(9)
    P = np.zeros((9, 9), np.float32)
    P[perm, np.arange(9)] = 1.0          # column j of A.P is column perm[j] of A
    assert np.array_equal(oracle.gemm(A, P), A.astype(F64)[:, perm])


def test_gemm_is_not_symmetric_in_operands():
    # A.B != B.A in general: catches an oracle that swaps operands
    A, B = I.gemm_inputs(I.GemmShape(4, 4, 4), 14, ints=True)
    assert not np.array_equal(oracle.gemm(A, B), oracle.gemm(B, A))
    assert np.array_equal(oracle.gemm(A, B).T, oracle.gemm(B.T.copy(), A.T.copy()))


def test_gemm_outer_product_closed_form():
    # K = 1: C[i,j] = a_i * b_j
    a = np.arange(1, 6, dtype=np.float32).reshape(5, 1)
    b = np.arange(-2, 5, dtype=np.float32).reshape(1, 7)
    assert np.array_equal(oracle.gemm(a, b), a.astype(F64) * b.astype(F64))


# ---------------------------------------------------------------- conv2d
CONV_CASES = [
    I.ConvShape(2, 3, 7, 6, 4, 3, 3, (1, 1), (1, 1)),
    I.ConvShape(1, 2, 9, 9, 3, 3, 3, (2, 2), (1, 1)),
    I.ConvShape(2, 3, 8, 11, 2, 1, 1, (1, 1), (0, 0)),
    I.ConvShape(1, 4, 10, 7, 3, 1, 1, (2, 2), (0, 0)),
    I.ConvShape(1, 3, 15, 14, 5, 7, 7, (2, 2), (3, 3)),
    I.ConvShape(1, 2, 6, 8, 2, 3, 2, (2, 1), (0, 1)),      # asymmetric everything
    I.ConvShape(1, 1, 3, 3, 1, 3, 3, (1, 1), (0, 0)),      # single output pixel
]


@pytest.mark.parametrize("shape", CONV_CASES, ids=str)
def test_conv2d_vs_windows(shape):
    # catches: kernel flip, wrong pad sign, stride applied to the tap instead of the pixel
    x, w = I.conv_inputs(shape, 21)
    ref = ref_conv_windows(x, w, shape.stride, shape.pad)
    got = oracle.conv2d(x, w, shape.stride, shape.pad)
    assert got.shape == (shape.N, shape.K, shape.OH, shape.OW)
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-12)


@pytest.mark.parametrize("shape", CONV_CASES[:4], ids=str)
def test_conv2d_equals_im2col_gemm(shape):
    # conv == (im2col matrix) . (weights as [C*R*S, K]) through the GEMM oracle
    x, w = I.conv_inputs(shape, 22)
    cols, OH, OW = im2col(x, shape.R, shape.S, shape.stride, shape.pad)
    wm = np.ascontiguousarray(w.reshape(shape.K, -1).T)
    y = oracle.gemm(cols, wm).reshape(shape.N, OH, OW, shape.K).transpose(0, 3, 1, 2)
    np.testing.assert_allclose(oracle.conv2d(x, w, shape.stride, shape.pad), y, rtol=0, atol=1e-12)


@pytest.mark.parametrize("r0,s0", [(0, 0), (0, 2), (1, 1), (2, 0), (2, 2), (1, 0)])
def test_conv2d_delta_kernel_shifts_input(r0, s0):
    # a kernel that is 1 at tap (r0,s0) on the diagonal ci==co shifts the image by
    # (r0-pad, s0-pad) with zero fill, exactly.  Catches a flipped kernel (r0 <-> 2-r0).
    C, H, W, p = 3, 6, 7, 1
    x = I.small_ints(rng(5), (2, C, H, W))
    w = np.zeros((C, C, 3, 3), np.float32)
    for c in range(C):
        w[c, c, r0, s0] = 1.0
    y = oracle.conv2d(x, w, (1, 1), (p, p))
    exp = np.zeros_like(y)
    for oh in range(H):
        for ow in range(W):
            ih, iw = oh + r0 - p, ow + s0 - p
            if 0 <= ih < H and 0 <= iw < W:
                exp[:, :, oh, ow] = x[:, :, ih, iw]
    assert np.array_equal(y, exp)


def test_conv2d_all_ones_counts_valid_taps():
    # x = w = 1: y = Cin * (# taps inside the image): 9 interior, 6 edge, 4 corner
    C, H, W = 5, 6, 8
    x = np.ones((1, C, H, W), np.float32)
    w = np.ones((2, C, 3, 3), np.float32)
    y = oracle.conv2d(x, w, (1, 1), (1, 1))
    assert y[0, 0, 2, 3] == 9 * C and y[0, 1, 0, 3] == 6 * C and y[0, 0, 3, 0] == 6 * C
    for (a, b) in [(0, 0), (0, W - 1), (H - 1, 0), (H - 1, W - 1)]:
        assert y[0, 0, a, b] == 4 * C
    assert y.sum() == 2 * C * ((H - 2) * (W - 2) * 9 + 2 * (H - 2 + W - 2) * 6 + 16)


def test_conv2d_stride2_samples_stride1():
    # k=3, pad=1: stride-2 output equals the stride-1 output at even positions
    shape = I.ConvShape(2, 3, 9, 8, 4, 3, 3, (1, 1), (1, 1))
    x, w = I.conv_inputs(shape, 23)
    y1 = oracle.conv2d(x, w, (1, 1), (1, 1))
    y2 = oracle.conv2d(x, w, (2, 2), (1, 1))
    assert y2.shape == (2, 4, 5, 4)
    assert np.array_equal(y2, y1[:, :, ::2, ::2])


def test_conv2d_channel_and_weight_indexing():
    # one-hot weight W[k0,c0,r0,s0] = 1 picks exactly input channel c0 into output channel k0
    x = I.small_ints(rng(6), (1, 4, 5, 5))
    w = np.zeros((3, 4, 3, 3), np.float32)
    w[2, 1, 1, 1] = 1.0
    y = oracle.conv2d(x, w, (1, 1), (1, 1))
    assert np.array_equal(y[0, 2], x[0, 1].astype(F64))
    assert not y[0, 0].any() and not y[0, 1].any()


def test_conv2d_linearity():
    shape = I.ConvShape(1, 3, 6, 6, 2, 3, 3, (1, 1), (1, 1))
    x1, w = I.conv_inputs(shape, 24, ints=True)
    x2, _ = I.conv_inputs(shape, 25, ints=True)
    a = np.float32(2.0)
    lhs = oracle.conv2d(a * x1 + x2, w, (1, 1), (1, 1))
    rhs = 2.0 * oracle.conv2d(x1, w, (1, 1), (1, 1)) + oracle.conv2d(x2, w, (1, 1), (1, 1))
    assert np.array_equal(lhs, rhs)


# ---------------------------------------------------------------- depthwise
DW_CASES = [
    I.ConvShape(2, 5, 7, 8, 5, 3, 3, (1, 1), (1, 1)),
    I.ConvShape(1, 4, 9, 9, 4, 3, 3, (2, 2), (1, 1)),
    I.ConvShape(1, 3, 6, 5, 3, 5, 5, (1, 1), (2, 2)),
]


# ---------------------------------------------------------------- grouped / dilated conv2d
def expand_kernel(w, dil):
    """The dilated kernel written out: zeros between the taps."""
    K, C, R, S = w.shape
    e = np.zeros((K, C, dil[0] * (R - 1) + 1, dil[1] * (S - 1) + 1), w.dtype)
    e[:, :, ::dil[0], ::dil[1]] = w
    return e


GENERAL_CASES = [   # N, C, H, W, K, R, S, stride, pad, dil, groups
    (2, 4, 9, 8, 6, 3, 3, (1, 1), (2, 2), (2, 2), 1),
    (1, 3, 15, 14, 4, 3, 2, (2, 1), (1, 3), (3, 2), 1),
    (2, 6, 7, 7, 4, 3, 3, (1, 1), (1, 1), (1, 1), 2),
    (1, 8, 6, 9, 12, 1, 1, (1, 1), (0, 0), (1, 1), 4),
    (1, 4, 11, 10, 8, 3, 3, (2, 2), (2, 2), (2, 2), 4),
]


def general_inputs(case, seed):
    N, C, H, W, K, R, S, stride, pad, dil, groups = case
    g = rng(seed)
    return I.uniform(g, (N, C, H, W)), I.normal(g, (K, C // groups, R, S), 0.5)


@pytest.mark.parametrize("case", GENERAL_CASES, ids=str)
def test_conv2d_general_vs_windows(case):
    # second derivation: pad explicitly, take the strided, dilated window of each output pixel
    # from the channels of its group, contract with einsum.  Catches dilation applied to the
    # pixel instead of the tap, a wrong group of input channels, a wrong output extent.
    N, C, H, W, K, R, S, stride, pad, dil, groups = case
    x, w = general_inputs(case, 31)
    got = oracle.conv2d_general(x, w, stride, pad, dil, groups)
    xp = np.pad(x.astype(np.float64), ((0, 0), (0, 0), (pad[0], pad[0]), (pad[1], pad[1])))
    OH = (H + 2 * pad[0] - dil[0] * (R - 1) - 1) // stride[0] + 1
    OW = (W + 2 * pad[1] - dil[1] * (S - 1) - 1) // stride[1] + 1
    assert got.shape == (N, K, OH, OW)
    Cg, Kg = C // groups, K // groups
    ref = np.zeros((N, K, OH, OW))
    for g in range(groups):
        for oh in range(OH):
            for ow in range(OW):
                win = xp[:, g * Cg:(g + 1) * Cg,
                         oh * stride[0]:oh * stride[0] + dil[0] * (R - 1) + 1:dil[0],
                         ow * stride[1]:ow * stride[1] + dil[1] * (S - 1) + 1:dil[1]]
                ref[:, g * Kg:(g + 1) * Kg, oh, ow] = np.einsum("ncrs,kcrs->nk", win,
                                                                w[g * Kg:(g + 1) * Kg].astype(np.float64))
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-12)


@pytest.mark.parametrize("shape", CONV_CASES, ids=str)
def test_conv2d_general_reduces_to_conv2d(shape):
    # one group, no dilation: the same loops in the same order as the C2D oracle
    x, w = I.conv_inputs(shape, 32)
    assert np.array_equal(oracle.conv2d_general(x, w, shape.stride, shape.pad, (1, 1), 1),
                          oracle.conv2d(x, w, shape.stride, shape.pad))


@pytest.mark.parametrize("case", GENERAL_CASES[:2], ids=str)
def test_dilated_conv_is_conv_with_zero_filled_kernel(case):
    # the dilated kernel written out with zeros between its taps, through the C2D oracle: the
    # zero products add nothing, so the sums agree exactly
    N, C, H, W, K, R, S, stride, pad, dil, groups = case
    x, w = general_inputs(case, 33)
    assert np.array_equal(oracle.conv2d_general(x, w, stride, pad, dil, 1),
                          oracle.conv2d(x, expand_kernel(w, dil), stride, pad))


def test_dilated_delta_kernel_shifts_by_dilated_tap():
    # 1 at tap (r0,s0): the image shifted by (r0*d - pad, s0*d - pad), exactly
    C, H, W, p, d = 2, 8, 9, 2, 2
    x = I.small_ints(rng(34), (1, C, H, W))
    for r0, s0 in [(0, 0), (2, 1), (1, 2)]:
        w = np.zeros((C, C, 3, 3), np.float32)
        for c in range(C):
            w[c, c, r0, s0] = 1.0
        y = oracle.conv2d_general(x, w, (1, 1), (p, p), (d, d), 1)
        assert y.shape == (1, C, H, W)
        exp = np.zeros_like(y)
        for oh in range(H):
            for ow in range(W):
                ih, iw = oh + r0 * d - p, ow + s0 * d - p
                if 0 <= ih < H and 0 <= iw < W:
                    exp[:, :, oh, ow] = x[:, :, ih, iw]
        assert np.array_equal(y, exp)


def test_dilated_all_ones_counts_valid_taps_and_extent():
    # dilation 2, pad 2, 3x3: taps at -2, 0, +2; corner 4, edge 6, interior 9 per channel
    C = 3
    x = np.ones((1, C, 7, 7), np.float32)
    w = np.ones((1, C, 3, 3), np.float32)
    y = oracle.conv2d_general(x, w, (1, 1), (2, 2), (2, 2), 1)
    assert y.shape == (1, 1, 7, 7)
    assert y[0, 0, 0, 0] == 4 * C and y[0, 0, 0, 3] == 6 * C and y[0, 0, 3, 3] == 9 * C
    assert y[0, 0, 1, 1] == 4 * C      # row 1: taps at -1 (out), 1, 3
    # the stem shape of the appendix with dilation 2: (224 + 6 - 13) // 2 + 1
    xs = np.zeros((1, 1, 224, 224), np.float32)
    assert oracle.conv2d_general(xs, np.zeros((1, 1, 7, 7), np.float32), (2, 2), (3, 3), (2, 2), 1).shape[2:] == (109, 109)


@pytest.mark.parametrize("case", GENERAL_CASES[2:], ids=str)
def test_grouped_conv_is_block_diagonal_conv(case):
    # the grouped weights placed on the diagonal blocks of a dense [K,C,R,S] kernel, through the
    # dilated single-group path: catches k % groups instead of k / (K/groups), a shifted run
    N, C, H, W, K, R, S, stride, pad, dil, groups = case
    x, w = general_inputs(case, 35)
    Cg, Kg = C // groups, K // groups
    dense = np.zeros((K, C, R, S), np.float32)
    for g in range(groups):
        dense[g * Kg:(g + 1) * Kg, g * Cg:(g + 1) * Cg] = w[g * Kg:(g + 1) * Kg]
    assert np.array_equal(oracle.conv2d_general(x, w, stride, pad, dil, groups),
                          oracle.conv2d_general(x, dense, stride, pad, dil, 1))


def test_convlayer_general_reduces_to_convlayer():
    # one group, no dilation: the ConvLayer oracle (C loops) and the general one agree
    s = I.ConvShape(2, 3, 7, 6, 4, 3, 3, (1, 1), (1, 1))
    x, w = I.conv_inputs(s, 38)
    gamma, beta, mean, var = I.bn_inputs(s.K, 39)
    a = oracle.conv_bn_relu(x, w, gamma, beta, mean, var, I.BN_EPS, s.stride, s.pad)
    b = oracle.conv_bn_relu_general(x, w, gamma, beta, mean, var, I.BN_EPS, s.stride, s.pad)
    np.testing.assert_allclose(a, b, rtol=0, atol=1e-14)
    assert (b >= 0).all() and (b == 0).any() and (b > 0).any()


def test_grouped_conv_with_one_channel_per_group_is_depthwise():
    s = I.ConvShape(2, 5, 8, 7, 5, 3, 3, (1, 1), (1, 1))
    x, w = I.dwconv_inputs(s, 36)
    assert np.array_equal(oracle.conv2d_general(x, w, s.stride, s.pad, (1, 1), s.C),
                          oracle.dwconv(x, w, s.stride, s.pad))


def test_grouped_conv_groups_do_not_mix():
    case = GENERAL_CASES[2]
    x, w = general_inputs(case, 37)
    y = oracle.conv2d_general(x, w, case[7], case[8], case[9], 2)
    x2 = x.copy()
    x2[:, 3:] += 1.0                     # second group's input channels only
    y2 = oracle.conv2d_general(x2, w, case[7], case[8], case[9], 2)
    assert np.array_equal(y[:, :2], y2[:, :2]) and not np.array_equal(y[:, 2:], y2[:, 2:])
    with pytest.raises(ValueError):
        oracle.conv2d_general(x, w[:, :2], case[7], case[8], case[9], 4)


# ---------------------------------------------------------------- dwconv
@pytest.mark.parametrize("shape", DW_CASES, ids=str)
def test_dwconv_equals_block_diagonal_conv2d(shape):
    # depthwise == dense conv whose weights are zero off the channel diagonal
    x, w = I.dwconv_inputs(shape, 31)
    wd = np.zeros((shape.C, shape.C, shape.R, shape.S), np.float32)
    for c in range(shape.C):
        wd[c, c] = w[c, 0]
    np.testing.assert_allclose(oracle.dwconv(x, w, shape.stride, shape.pad),
                               oracle.conv2d(x, wd, shape.stride, shape.pad), rtol=0, atol=1e-13)


@pytest.mark.parametrize("shape", DW_CASES, ids=str)
def test_dwconv_vs_windows(shape):
    x, w = I.dwconv_inputs(shape, 32)
    xs = x.astype(F64)
    p = shape.pad
    xp = np.pad(xs, ((0, 0), (0, 0), (p[0], p[0]), (p[1], p[1])))
    y = np.zeros((shape.N, shape.C, shape.OH, shape.OW))
    for r in range(shape.R):
        for s in range(shape.S):
            win = xp[:, :, r:r + (shape.OH - 1) * shape.stride[0] + 1:shape.stride[0],
                     s:s + (shape.OW - 1) * shape.stride[1] + 1:shape.stride[1]]
            y += win * w[:, 0, r, s].astype(F64)[None, :, None, None]
    np.testing.assert_allclose(oracle.dwconv(x, w, shape.stride, shape.pad), y, rtol=0, atol=1e-13)


def test_dwconv_all_ones_and_delta():
    x = np.ones((1, 3, 5, 6), np.float32)
    w = np.ones((3, 1, 3, 3), np.float32)
    y = oracle.dwconv(x, w, (1, 1), (1, 1))
    assert y[0, 1, 2, 2] == 9 and y[0, 2, 0, 2] == 6 and y[0, 0, 4, 5] == 4
    xi = I.small_ints(rng(7), (1, 3, 5, 6))
    wd = np.zeros((3, 1, 3, 3), np.float32)
    wd[:, 0, 0, 2] = 1.0                       # tap (0,2): y[oh,ow] = x[oh-1, ow+1]
    yd = oracle.dwconv(xi, wd, (1, 1), (1, 1))
    exp = np.zeros_like(yd)
    exp[:, :, 1:, :-1] = xi[:, :, :-1, 1:]
    assert np.array_equal(yd, exp)


# ---------------------------------------------------------------- ConvLayer
def test_convlayer_identity_bn_is_relu_of_conv():
    shape = I.ConvShape(2, 3, 6, 6, 4, 3, 3, (1, 1), (1, 1))
    x, w = I.conv_inputs(shape, 41, ints=True)
    K = shape.K
    eps = np.float32(0.25)
    one, zero = np.ones(K, np.float32), np.zeros(K, np.float32)
    var = np.full(K, 0.75, np.float32)           # var + eps == 1 exactly
    y = oracle.conv_bn_relu(x, w, one, zero, zero, var, eps, (1, 1), (1, 1))
    c = oracle.conv2d(x, w, (1, 1), (1, 1))
    assert np.array_equal(y, np.maximum(c, 0.0))
    assert (c < 0).any() and (y >= 0).all()


def test_convlayer_affine_by_hand():
    # large beta keeps everything positive: output is the affine map of the conv, by hand
    shape = I.ConvShape(1, 2, 5, 5, 3, 3, 3, (1, 1), (1, 1))
    x, w = I.conv_inputs(shape, 42)
    gamma, _, mean, var = I.bn_inputs(3, 43)
    beta = np.full(3, 100.0, np.float32)
    eps = 1e-5
    y = oracle.conv_bn_relu(x, w, gamma, beta, mean, var, eps, (1, 1), (1, 1))
    c = ref_conv_windows(x, w, (1, 1), (1, 1))
    g, b, m, v = (t.astype(F64)[None, :, None, None] for t in (gamma, beta, mean, var))
    exp = g * (c - m) / np.sqrt(v + F64(np.float32(eps))) + b
    np.testing.assert_allclose(y, exp, rtol=1e-14, atol=1e-12)


def test_convlayer_each_bn_parameter_matters():
    # catches a swapped or dropped parameter: perturbing each one moves the output the right way
    shape = I.ConvShape(1, 2, 4, 4, 2, 3, 3, (1, 1), (1, 1))
    x, w = I.conv_inputs(shape, 44)
    gamma = np.array([1.5, 0.5], np.float32)
    beta = np.array([50.0, 60.0], np.float32)
    mean = np.array([0.25, -0.5], np.float32)
    var = np.array([3.0, 0.5], np.float32)
    eps = 1.0
    base = oracle.conv_bn_relu(x, w, gamma, beta, mean, var, eps, (1, 1), (1, 1))
    c = oracle.conv2d(x, w, (1, 1), (1, 1))
    # channel 0: gamma/sqrt(var+eps) = 1.5/2 = 0.75 exactly
    np.testing.assert_allclose(base[0, 0], 0.75 * (c[0, 0] - 0.25) + 50.0, rtol=1e-15, atol=1e-13)
    # channel 1: 0.5/sqrt(1.5)
    np.testing.assert_allclose(base[0, 1], 0.5 / np.sqrt(1.5) * (c[0, 1] + 0.5) + 60.0,
                               rtol=1e-15, atol=1e-13)


# ---------------------------------------------------------------- TBG / TBS
def test_tbg_vs_einsum():
    # catches: reading q as [B,H,S,D], contracting over the wrong axis, i/j swapped
    q, k = I.tbg_inputs(I.TbgShape(2, 5, 3, 4), 51)
    ref = np.einsum("bihd,bjhd->bhij", q.astype(F64), k.astype(F64))
    np.testing.assert_allclose(oracle.tbg(q, k), ref, rtol=0, atol=1e-12)


def test_tbg_equals_gemm_on_permuted_copies():
    q, k = I.tbg_inputs(I.TbgShape(2, 6, 3, 5), 52)
    B, S, H, D = q.shape
    qt = np.ascontiguousarray(q.transpose(0, 2, 1, 3)).reshape(B * H, S, D)
    ktT = np.ascontiguousarray(k.transpose(0, 2, 3, 1)).reshape(B * H, D, S)
    ref = oracle.gemm(qt, ktT).reshape(B, H, S, S)
    np.testing.assert_allclose(oracle.tbg(q, k), ref, rtol=0, atol=1e-13)


def test_tbg_symmetric_when_k_is_q():
    q, _ = I.tbg_inputs(I.TbgShape(2, 7, 2, 3), 53)
    out = oracle.tbg(q, q)
    assert np.array_equal(out, out.transpose(0, 1, 3, 2))
    diag = np.einsum("bhii->bhi", out)
    norms = (q.astype(F64) ** 2).sum(-1).transpose(0, 2, 1)
    np.testing.assert_allclose(diag, norms, rtol=1e-14)
    assert (diag >= 0).all()


def test_tbg_one_hot_index_code():
    # q[b,i,h,:] = e_(i mod D), k[b,j,h,:] = (1+b+10h) e_(j mod D): the output says who met whom
    B, S, H, D = 2, 4, 3, 4
    q = np.zeros((B, S, H, D), np.float32)
    k = np.zeros((B, S, H, D), np.float32)
    for b in range(B):
        for s in range(S):
            for h in range(H):
                q[b, s, h, s % D] = 1.0
                k[b, s, h, (s + 1) % D] = 1.0 + b + 10 * h
    out = oracle.tbg(q, k)
    for b in range(B):
        for h in range(H):
            for i in range(S):
                for j in range(S):
                    exp = (1.0 + b + 10 * h) if i % D == (j + 1) % D else 0.0
                    assert out[b, h, i, j] == exp


def test_tbs_rows_are_softmax_of_tbg():
    q, k = I.tbg_inputs(I.TbgShape(1, 6, 2, 4), 54)
    p = oracle.tbs(q, k)
    s = oracle.tbg(q, k)
    e = np.exp(s - s.max(-1, keepdims=True))
    np.testing.assert_allclose(p, e / e.sum(-1, keepdims=True), rtol=1e-14)
    np.testing.assert_allclose(p.sum(-1), 1.0, rtol=1e-14)
    assert np.array_equal(p.argmax(-1), s.argmax(-1))
    # softmax is invariant to a per-row shift: scale q's contribution by adding a constant column
    # (closed form) -- uniform scores give exactly 1/S
    z = np.zeros_like(q)
    assert np.array_equal(oracle.tbs(z, k), np.full_like(p, 1.0 / 6))


def test_tbs_two_keys_is_the_logistic_function():
    # S = 2: softmax over two scores is 1 / (1 + exp(-(s_j - s_other))), written out by hand
    B, S, H, D = 1, 2, 1, 3
    q = np.array([[[[1.0, 2.0, -1.0]], [[0.5, 0.0, 2.0]]]], dtype=np.float32).reshape(B, S, H, D)
    k = np.array([[[[0.25, -1.0, 0.5]], [[1.0, 1.0, 1.0]]]], dtype=np.float32).reshape(B, S, H, D)
    p = oracle.tbs(q, k)
    for i in range(S):
        s0 = float(sum(float(q[0, i, 0, d]) * float(k[0, 0, 0, d]) for d in range(D)))
        s1 = float(sum(float(q[0, i, 0, d]) * float(k[0, 1, 0, d]) for d in range(D)))
        assert abs(p[0, 0, i, 0] - 1.0 / (1.0 + math.exp(s1 - s0))) < 1e-15
        assert abs(p[0, 0, i, 1] - 1.0 / (1.0 + math.exp(s0 - s1))) < 1e-15


def test_tbs_large_scores_do_not_overflow():
    # scores near 1600: exp overflows a double unless the row maximum is subtracted first; the
    # softmax of (1600, 1599, 0) is (1, e^-1, e^-1600) / (1 + e^-1 + e^-1600); all inputs exact in fp32
    B, S, H, D = 1, 3, 1, 2
    q = np.zeros((B, S, H, D), dtype=np.float32)
    q[0, :, 0, 0] = 32.0
    k = np.zeros((B, S, H, D), dtype=np.float32)
    k[0, :, 0, 0] = [50.0, 49.96875, 0.0]
    p = oracle.tbs(q, k)
    assert np.isfinite(p).all()
    z = 1.0 + math.exp(-1.0)
    want = np.array([1.0 / z, math.exp(-1.0) / z, 0.0])
    for i in range(S):
        np.testing.assert_allclose(p[0, 0, i], want, rtol=0, atol=1e-15)


# ---------------------------------------------------------------- NRM
def test_nrm_vs_library_frobenius_norm():
    # the entrywise 2-norm of a matrix is the Frobenius norm: numpy's routine on the same values
    x = I.uniform(rng(51), (3, 37, 53))
    ref = np.array([np.linalg.norm(x[b].astype(np.float64), "fro") for b in range(3)])
    np.testing.assert_allclose(oracle.nrm(x), ref, rtol=1e-14)
    np.testing.assert_allclose(oracle.nrm(x[1]), ref[1:2], rtol=1e-14)


def test_nrm_closed_forms():
    assert oracle.nrm(np.ones((6, 24), np.float32))[0] == 12.0                 # sqrt(N*M)
    x = np.zeros((5, 7), np.float32)
    x[3, 2] = -2.5
    assert oracle.nrm(x)[0] == 2.5                                             # one entry: |a|, sign lost
    x[0, 6] = 6.0
    assert oracle.nrm(x)[0] == 6.5                                             # 2.5, 6, 6.5 triple
    assert oracle.nrm(np.zeros((4, 4), np.float32))[0] == 0.0
    # every entry counts once: an N x M ramp, sum of squares 1..n = n(n+1)(2n+1)/6
    n = 12 * 9
    ramp = np.arange(1, n + 1, dtype=np.float32).reshape(12, 9)
    assert oracle.nrm(ramp)[0] == np.sqrt(n * (n + 1) * (2 * n + 1) / 6.0)


def test_nrm_invariants():
    x = I.uniform(rng(52), (2, 16, 10))
    base = oracle.nrm(x)
    # batch entries are independent; transposing or permuting entries changes nothing
    np.testing.assert_allclose(oracle.nrm(np.ascontiguousarray(x.transpose(0, 2, 1))), base, rtol=1e-14)
    np.testing.assert_allclose(oracle.nrm(x[::-1].copy()), base[::-1], rtol=0)
    # homogeneity with an exactly representable factor
    np.testing.assert_allclose(oracle.nrm((x * np.float32(-4.0))), 4.0 * base, rtol=1e-15)
    # Pythagoras for matrices with disjoint supports
    a = x.copy(); a[:, :, 5:] = 0
    b = x.copy(); b[:, :, :5] = 0
    np.testing.assert_allclose(np.sqrt(oracle.nrm(a) ** 2 + oracle.nrm(b) ** 2), base, rtol=1e-14)


def test_oracle_thread_count_does_not_change_results():
    shape = I.ConvShape(2, 3, 7, 6, 4, 3, 3, (1, 1), (1, 1))
    x, w = I.conv_inputs(shape, 61)
    n = oracle.max_threads()
    oracle.set_threads(1)
    y1 = oracle.conv2d(x, w, (1, 1), (1, 1))
    oracle.set_threads(n)
    yn = oracle.conv2d(x, w, (1, 1), (1, 1))
    assert np.array_equal(y1, yn)


def test_golden_shape_list_parses(golden_dir):
    import os
    ops = {}
    for line in open(os.path.join(golden_dir, "appendix_c_shapes.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        name, *vals = line.split()
        ops.setdefault(name, []).append(tuple(int(v) for v in vals))
    assert {k: len(v) for k, v in ops.items()} == {"C2D": 4, "GMM": 4, "DEP": 4, "ConvLayer": 4, "TBS": 4,
                                                   "GRP": 4, "DIL": 4, "NRM": 4}
    assert (512, 512, 512) in ops["GMM"] and (128, 12, 64) in ops["TBS"]
    # the list the benchmark walks is the same list
    from paper_2006_06762_amd import inputs as I
    assert ops == I.APPENDIX_C
    s = I.appendix_shape("ConvLayer", I.APPENDIX_C["ConvLayer"][2], 16)
    assert (s.N, s.C, s.K, s.R, s.stride, s.pad, s.OH, s.OW) == (16, 128, 256, 1, (2, 2), (0, 0), 14, 14)
    s = I.appendix_shape("DIL", I.APPENDIX_C["DIL"][0], 1)
    assert (s.dil, s.groups, s.OH, s.OW) == ((2, 2), 1, 109, 109)
    assert I.appendix_shape("GRP", I.APPENDIX_C["GRP"][0], 1) is None       # 3 channels, 4 groups
    assert I.appendix_shape("GRP", I.APPENDIX_C["GRP"][2], 16).groups == 4
