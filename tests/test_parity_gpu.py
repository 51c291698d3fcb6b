"""GPU parity: every C-ABI entry point against the fp64 CPU oracle, element by element,
on the same seeded fp32 inputs.

Bar (floating point): max_e |gpu_e - oracle_e| / max(1, |oracle_e|) <= 1e-4.
Bar (index / layout handling): with small-integer inputs every partial sum is exact in
fp32, so the GPU result must equal the oracle bit for bit.
"""
import numpy as np
import pytest

import oracle
from paper_2006_06762_amd import inputs as I

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

TOL = 1e-4
CANARY = 12345.0


@pytest.fixture(scope="module")
def anr():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2006_06762_amd import binding
    return binding


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def rel_err(got, ref):
    got = got.astype(np.float64)
    return float(np.max(np.abs(got - ref) / np.maximum(1.0, np.abs(ref))))


def guarded(shape):
    """Output tensor with a canary band before and after it (catches out-of-bounds stores)."""
    n = int(np.prod(shape))
    buf = torch.full((n + 2 * 64,), CANARY, dtype=torch.float32, device="cuda")
    return buf, buf[64:64 + n].view(*shape)


def check_guard(buf):
    torch.cuda.synchronize()
    assert bool((buf[:64] == CANARY).all()) and bool((buf[-64:] == CANARY).all()), "store out of bounds"


def assert_parity(got_t, ref, exact=False, what=""):
    got = got_t.cpu().numpy()
    assert not np.isnan(got).any(), what + ": NaN in output"
    if exact:
        assert np.array_equal(got.astype(np.float64), ref), what + ": not bit-exact"
    else:
        e = rel_err(got, ref)
        assert e <= TOL, "%s: rel err %.3e" % (what, e)


# ------------------------------------------------------------------ GEMM
GEMM_SHAPES = [(1, 1, 1), (5, 7, 3), (33, 17, 65), (64, 64, 64), (100, 132, 72), (257, 129, 33),
               (128, 128, 128), (512, 32, 512), (130, 260, 16)]


@pytest.mark.parametrize("M,N,K", GEMM_SHAPES)
@pytest.mark.parametrize("ints", [False, True])
def test_gemm_small(anr, M, N, K, ints):
    A, B = I.gemm_inputs(I.GemmShape(M, N, K), 100 + M, ints=ints)
    buf, C = guarded((M, N))
    anr.gemm(dev(A), dev(B), C)
    check_guard(buf)
    assert_parity(C, oracle.gemm(A, B), exact=ints, what="gemm %dx%dx%d" % (M, N, K))


def test_gemm_config_512(anr):
    cfg = I.config_inputs("GMM")
    C = torch.empty((512, 512), dtype=torch.float32, device="cuda")
    anr.gemm(dev(cfg["A"]), dev(cfg["B"]), C)
    assert_parity(C, oracle.gemm(cfg["A"], cfg["B"]), what="GMM 512^3")


def test_gemm_1024_and_big_tiles(anr):
    # large enough for the 128x128 tile variant; ragged in M and N
    for (M, N, K) in [(1024, 1024, 1024), (1920, 1670, 96)]:
        A, B = I.gemm_inputs(I.GemmShape(M, N, K), 7)
        C = torch.empty((M, N), dtype=torch.float32, device="cuda")
        anr.gemm(dev(A), dev(B), C)
        assert_parity(C, oracle.gemm(A, B), what="gemm %dx%dx%d" % (M, N, K))


def test_gemm_batched_and_strided(anr):
    A, B = I.gemm_inputs(I.GemmShape(70, 52, 40, batch=3), 8)
    C = torch.empty((3, 70, 52), dtype=torch.float32, device="cuda")
    anr.gemm(dev(A), dev(B), C)
    assert_parity(C, oracle.gemm(A, B), what="batched gemm")
    # leading dimensions larger than the row length (views into wider matrices), odd offsets
    Aw = torch.zeros((70, 47), device="cuda")
    Bw = torch.zeros((40, 59), device="cuda")
    Cw = torch.full((70, 61), CANARY, device="cuda")
    Aw[:, 3:43] = dev(A[0])
    Bw[:, 5:57] = dev(B[0])
    anr.gemm(Aw[:, 3:43], Bw[:, 5:57], Cw[:, 2:54])
    assert_parity(Cw[:, 2:54].contiguous(), oracle.gemm(A[0], B[0]), what="strided gemm")
    assert bool((Cw[:, :2] == CANARY).all()) and bool((Cw[:, 54:] == CANARY).all())


@pytest.mark.parametrize("M,N,K,batch", [(1024, 1024, 64, 8),      # 128 x 128 tiles of the pipelined kernel
                                          (1000, 1000, 100, 4),     # 128 x 64 tiles, ragged rows and columns
                                          (300, 200, 36, 3),        # 64 x 64 tiles, two chunks, ragged
                                          (64, 64, 4, 1),           # a single short chunk
                                          (640, 600, 388, 1),       # few tiles, 13 chunks: two groups of waves, one with a chunk fewer
                                          (300, 500, 1000, 1),      # few tiles, 32 chunks with a K tail: four groups
                                          (200, 260, 2048, 2)])     # four groups, batched
@pytest.mark.parametrize("ints", [False, True])
def test_gemm_pipelined_tiles(anr, M, N, K, batch, ints):
    A, B = I.gemm_inputs(I.GemmShape(M, N, K, batch), 110, ints=ints)
    shape = (batch, M, N) if batch > 1 else (M, N)
    buf, C = guarded(shape)
    anr.gemm(dev(A), dev(B), C)
    check_guard(buf)
    assert_parity(C, oracle.gemm(A, B), exact=ints, what="gemm %dx%dx%d b%d" % (M, N, K, batch))


@pytest.mark.parametrize("M,N,K,batch", [(64, 96, 128, 1), (32, 32, 256, 1), (96, 160, 256, 3), (160, 64, 512, 2),
                                         (32, 512, 512, 1), (256, 256, 128, 4)])
@pytest.mark.parametrize("ints", [False, True])
def test_gemm_wave_split_k_tiles(anr, M, N, K, batch, ints):
    """Few 32x32 tiles and K of 128, 256 or 512: one tile per work-group, its 4, 8 or 16 waves split K."""
    A, B = I.gemm_inputs(I.GemmShape(M, N, K, batch), 120 + K, ints=ints)
    shape = (batch, M, N) if batch > 1 else (M, N)
    buf, C = guarded(shape)
    anr.gemm(dev(A), dev(B), C)
    check_guard(buf)
    assert_parity(C, oracle.gemm(A, B), exact=ints, what="gemm %dx%dx%d b%d" % (M, N, K, batch))


def test_gemm_wave_split_k_strided_views(anr):
    """The same kernel on views into wider matrices (leading dimensions that are multiples of 4)."""
    A, B = I.gemm_inputs(I.GemmShape(64, 96, 256), 131)
    Aw = torch.zeros((64, 264), device="cuda")
    Bw = torch.zeros((256, 104), device="cuda")
    Cw = torch.full((64, 100), CANARY, device="cuda")
    Aw[:, 4:260] = dev(A)
    Bw[:, 8:104] = dev(B)
    anr.gemm(Aw[:, 4:260], Bw[:, 8:104], Cw[:, 1:97])
    assert_parity(Cw[:, 1:97].contiguous(), oracle.gemm(A, B), what="strided split-K gemm")
    Cw[:, 1:97] = CANARY
    assert bool((Cw == CANARY).all()), "store outside the output view"


def test_gemm_identity_returns_a(anr):
    A, _ = I.gemm_inputs(I.GemmShape(96, 96, 96), 9)
    C = torch.empty((96, 96), device="cuda")
    anr.gemm(dev(A), torch.eye(96, device="cuda"), C)
    assert np.array_equal(C.cpu().numpy(), A)


# ------------------------------------------------------------------ conv2d
# MFMA path: 3x3, W % 4 == 0, C % 8 == 0.  Ragged pixel tiles, K not a multiple of the
# channel tile, tiles that straddle images, stride 2.
CONV_FAST = [
    I.ConvShape(1, 8, 8, 8, 16, 3, 3, (1, 1), (1, 1)),
    I.ConvShape(3, 16, 12, 20, 40, 3, 3, (1, 1), (1, 1)),
    I.ConvShape(2, 8, 28, 28, 70, 3, 3, (1, 1), (1, 1)),
    I.ConvShape(5, 24, 9, 12, 33, 3, 3, (1, 1), (1, 1)),
    I.ConvShape(3, 16, 28, 28, 64, 3, 3, (2, 2), (1, 1)),
    I.ConvShape(2, 8, 17, 16, 20, 3, 3, (2, 2), (1, 1)),
    I.ConvShape(2, 8, 10, 12, 8, 3, 3, (1, 1), (0, 0)),
    I.ConvShape(2, 8, 10, 12, 8, 3, 3, (1, 2), (2, 1)),
    I.ConvShape(1, 32, 56, 56, 64, 3, 3, (1, 1), (1, 1)),
    # pointwise (1x1) MFMA path: C % 32 == 0 and C >= 256, W % 4 == 0
    I.ConvShape(2, 256, 12, 12, 40, 1, 1, (1, 1), (0, 0)),
    I.ConvShape(3, 288, 8, 8, 70, 1, 1, (1, 1), (0, 0)),
    I.ConvShape(1, 256, 28, 28, 64, 1, 1, (1, 1), (0, 0)),
    I.ConvShape(2, 256, 12, 16, 16, 1, 1, (2, 2), (0, 0)),
    I.ConvShape(1, 320, 9, 8, 33, 1, 1, (1, 1), (1, 1)),
    # narrower pointwise layers always take the general kernel
    I.ConvShape(2, 32, 12, 12, 40, 1, 1, (1, 1), (0, 0)),
    I.ConvShape(1, 64, 56, 56, 64, 1, 1, (1, 1), (0, 0)),
    I.ConvShape(1, 96, 9, 8, 33, 1, 1, (1, 1), (1, 1)),
]
# everything else goes through the general gather kernel
CONV_GENERIC = [
    I.ConvShape(2, 3, 7, 6, 4, 3, 3, (1, 1), (1, 1)),
    I.ConvShape(1, 3, 30, 30, 8, 7, 7, (2, 2), (3, 3)),
    I.ConvShape(2, 16, 14, 14, 12, 1, 1, (1, 1), (0, 0)),
    I.ConvShape(2, 16, 14, 14, 12, 1, 1, (2, 2), (0, 0)),
    I.ConvShape(1, 12, 7, 7, 9, 3, 3, (1, 1), (1, 1)),
    I.ConvShape(1, 2, 6, 8, 2, 3, 2, (2, 1), (0, 1)),
    # several pixel tiles and a ragged last one, reduction length not a multiple of 4 or 32
    I.ConvShape(3, 5, 15, 13, 70, 3, 3, (1, 1), (1, 1)),
    I.ConvShape(2, 3, 37, 41, 64, 7, 7, (2, 2), (3, 3)),
    I.ConvShape(1, 7, 9, 9, 130, 5, 5, (1, 1), (2, 2)),
    # few output tiles, long reduction: split-K through the workspace
    I.ConvShape(1, 256, 14, 14, 64, 3, 3, (1, 1), (1, 1)),
    I.ConvShape(1, 512, 7, 7, 96, 3, 3, (1, 1), (1, 1)),
    I.ConvShape(2, 128, 14, 14, 80, 1, 1, (2, 2), (0, 0)),
    I.ConvShape(1, 101, 5, 6, 33, 3, 3, (1, 1), (1, 1)),
    # more output channels than pixels, kernel larger than the padded image allows in places
    I.ConvShape(1, 16, 3, 3, 200, 3, 3, (1, 1), (1, 1)),
    I.ConvShape(4, 6, 8, 5, 10, 4, 2, (3, 2), (2, 1)),
]


@pytest.fixture(params=["tuned", "general"])
def conv_route(request):
    """Runs a test once with the tuned patch-staging kernel wherever it can take the shape
    and once with the general gather kernel for everything: the value for the descriptor's
    `route` field (left at 0, the choice depends on the number of output tiles)."""
    return 1 if request.param == "tuned" else 2


@pytest.mark.parametrize("shape", CONV_FAST + CONV_GENERIC, ids=str)
@pytest.mark.parametrize("ints", [False, True])
def test_conv2d_small(anr, conv_route, shape, ints):
    x, w = I.conv_inputs(shape, 200, ints=ints)
    buf, y = guarded((shape.N, shape.K, shape.OH, shape.OW))
    anr.conv2d(dev(x), dev(w), y, shape.stride, shape.pad, route=conv_route)
    check_guard(buf)
    assert_parity(y, oracle.conv2d(x, w, shape.stride, shape.pad), exact=ints, what=str(shape))


# ------------------------------------------------------------------ streaming pointwise kernel
POINTWISE_SHAPES = [
    I.ConvShape(16, 64, 56, 56, 64, 1, 1, (1, 1), (0, 0)),       # the Appendix C layer
    I.ConvShape(18, 32, 30, 30, 24, 1, 1, (1, 1), (0, 0)),       # 900 pixels: ragged pixel tile, channels past K
    I.ConvShape(10, 96, 26, 34, 100, 1, 1, (1, 1), (0, 0)),      # two channel tiles, the second ragged
    I.ConvShape(32, 128, 14, 14, 128, 1, 1, (1, 1), (0, 0)),     # 196 pixels: three whole tiles and four pixels
]


@pytest.mark.parametrize("shape", POINTWISE_SHAPES, ids=str)
def test_conv2d_pointwise_stream(anr, shape):
    """1x1 layers with few channels run the streaming kernel: integer values bit for bit, then the
    ConvLayer epilogue within the bar, on dense tensors and on images spaced apart in x and y."""
    s = shape
    d = anr.conv_desc((s.N, s.C, s.H, s.W), s.K, 1, 1)
    assert anr.conv2d_route(d).kernel == anr.ANR_CONV_KERNEL_POINTWISE
    x, w = I.conv_inputs(s, 1500, ints=True)
    buf, y = guarded((s.N, s.K, s.OH, s.OW))
    anr.conv2d(dev(x), dev(w), y, s.stride, s.pad)
    check_guard(buf)
    ref = oracle.conv2d(x, w, s.stride, s.pad)
    assert_parity(y, ref, exact=True, what="pointwise %s" % (s,))
    # images 8 floats further apart than dense, in x and in y
    xw = torch.zeros((s.N, s.C * s.H * s.W + 8), device="cuda")
    xw[:, :s.C * s.H * s.W] = dev(x).reshape(s.N, -1)
    yw = torch.full((s.N, s.K * s.OH * s.OW + 8), CANARY, device="cuda")
    xv = xw[:, :s.C * s.H * s.W].view(s.N, s.C, s.H, s.W)
    yv = yw[:, :s.K * s.OH * s.OW].view(s.N, s.K, s.OH, s.OW)
    anr.conv2d(xv, dev(w), yv, s.stride, s.pad)
    assert_parity(yv.contiguous(), ref, exact=True, what="pointwise, spaced images %s" % (s,))
    assert bool((yw[:, s.K * s.OH * s.OW:] == CANARY).all()), "store between the images"
    x, w = I.conv_inputs(s, 1501)
    gamma, beta, mean, var = I.bn_inputs(s.K, 1502)
    w = (w * 4).astype(np.float32)
    anr.conv_bn_relu(dev(x), dev(w), dev(gamma), dev(beta), dev(mean), dev(var), I.BN_EPS, y, s.stride, s.pad)
    check_guard(buf)
    assert_parity(y, oracle.conv_bn_relu(x, w, gamma, beta, mean, var, I.BN_EPS, s.stride, s.pad), what="pointwise ConvLayer %s" % (s,))
    got = y.cpu().numpy()
    assert (got >= 0).all() and (got == 0).any() and (got > 0).any()


RING_GEOMETRIES = [          # the layer geometries whose instantiations run the ring of three staging buffers
    (4, 56, 56, 64, (1, 1)),     # 56x56 maps, stride 1: 224 x 64 tiles
    (4, 28, 28, 32, (1, 1)),     # 28x28 maps, stride 1: 224 x 32 tiles
    (4, 28, 28, 32, (2, 2)),     # 28x28 maps, stride 2
]


@pytest.mark.parametrize("geom", RING_GEOMETRIES, ids=str)
@pytest.mark.parametrize("C", [8, 16, 24, 32, 40])
def test_conv2d_patch_kernel_few_chunks(anr, geom, C):
    """The tuned instantiations of the patch kernel keep three staging buffers in rotation, with chunk
    c + 1 stored and chunk c + 2 requested while chunk c is multiplied: one to five chunks of eight
    channels cover a reduction shorter than the ring, every buffer's first use and the first wrap-around.
    Integer values bit for bit, unpacked and packed, then the fused epilogue within the bar."""
    N, H, W, K, stride = geom
    s = I.ConvShape(N, C, H, W, K, 3, 3, stride, (1, 1))
    d = anr.conv_desc((s.N, s.C, s.H, s.W), s.K, 3, 3, s.stride, s.pad, route=1)
    assert anr.conv2d_route(d).kernel == anr.ANR_CONV_KERNEL_PATCH
    x, w = I.conv_inputs(s, 1600 + C, ints=True)
    ref = oracle.conv2d(x, w, s.stride, s.pad)
    buf, y = guarded((s.N, s.K, s.OH, s.OW))
    anr.conv2d(dev(x), dev(w), y, s.stride, s.pad, route=1)
    check_guard(buf)
    assert_parity(y, ref, exact=True, what="patch kernel, %d chunks %s" % (C // 8, geom))
    d, pack = anr.conv2d_pack_weights((s.N, s.C, s.H, s.W), dev(w), s.stride, s.pad, route=1)
    y.fill_(CANARY)
    anr.conv2d_packed(d, dev(x), pack, y)
    check_guard(buf)
    assert_parity(y, ref, exact=True, what="patch kernel packed, %d chunks %s" % (C // 8, geom))
    x, w = I.conv_inputs(s, 1650 + C)
    gamma, beta, mean, var = I.bn_inputs(s.K, 1651 + C)
    w = (w * 4).astype(np.float32)
    anr.conv_bn_relu(dev(x), dev(w), dev(gamma), dev(beta), dev(mean), dev(var), I.BN_EPS, y, s.stride, s.pad, route=1)
    check_guard(buf)
    assert_parity(y, oracle.conv_bn_relu(x, w, gamma, beta, mean, var, I.BN_EPS, s.stride, s.pad),
                  what="patch kernel ConvLayer, %d chunks %s" % (C // 8, geom))


GROUPED_POINTWISE_SHAPES = [     # grouped 1x1 layers the streaming kernel takes: a block-diagonal weight tile
    I.ConvShape(16, 64, 56, 56, 64, 1, 1, (1, 1), (0, 0), (1, 1), 4),     # the GRP layer of Appendix C at batch 16
    I.ConvShape(20, 128, 30, 30, 96, 1, 1, (1, 1), (0, 0), (1, 1), 8),     # 16 -> 12 channels per group, two channel tiles, ragged pixels
    I.ConvShape(64, 32, 14, 14, 64, 1, 1, (1, 1), (0, 0), (1, 1), 8),      # 4 -> 8 channels per group: one 16-byte unit per row
    I.ConvShape(20, 96, 26, 34, 48, 1, 1, (1, 1), (0, 0), (1, 1), 2),      # channels past K in the tile
]


@pytest.mark.parametrize("shape", GROUPED_POINTWISE_SHAPES, ids=str)
def test_conv2d_pointwise_stream_groups(anr, shape):
    s = shape
    d = anr.conv_desc((s.N, s.C, s.H, s.W), s.K, 1, 1, groups=s.groups)
    assert anr.conv2d_route(d).kernel == anr.ANR_CONV_KERNEL_POINTWISE
    x, w = I.conv_inputs(s, 1520, ints=True)
    buf, y = guarded((s.N, s.K, s.OH, s.OW))
    anr.conv2d(dev(x), dev(w), y, s.stride, s.pad, groups=s.groups)
    check_guard(buf)
    assert_parity(y, oracle.conv2d_general(x, w, s.stride, s.pad, s.dil, s.groups), exact=True, what="grouped pointwise %s" % (s,))
    x, w = I.conv_inputs(s, 1521)
    gamma, beta, mean, var = I.bn_inputs(s.K, 1522)
    w = (w * 4).astype(np.float32)
    anr.conv_bn_relu(dev(x), dev(w), dev(gamma), dev(beta), dev(mean), dev(var), I.BN_EPS, y, s.stride, s.pad, groups=s.groups)
    check_guard(buf)
    ref = oracle.conv_bn_relu_general(x, w, gamma, beta, mean, var, I.BN_EPS, s.stride, s.pad, s.dil, s.groups)
    assert_parity(y, ref, what="grouped pointwise ConvLayer %s" % (s,))


# ------------------------------------------------------------------ pre-packed weights
@pytest.mark.parametrize("name", ["C2D", "C2D_S2"])
def test_conv2d_packed_configs(anr, name):
    """The benchmark convolutions with pre-packed weights: within the bar of the oracle, and bit for
    bit what the unpacked call gives (same products, same order)."""
    cfg = I.config_inputs(name)
    s = cfg["shape"]
    xd, wd = dev(cfg["x"]), dev(cfg["w"])
    d, pack = anr.conv2d_pack_weights((s.N, s.C, s.H, s.W), wd, s.stride, s.pad)
    assert anr.conv2d_route(d).kernel == anr.ANR_CONV_KERNEL_PATCH
    buf, y = guarded((s.N, s.K, s.OH, s.OW))
    anr.conv2d_packed(d, xd, pack, y)
    check_guard(buf)
    assert_parity(y, oracle.conv2d(cfg["x"], cfg["w"], s.stride, s.pad), what=name + " packed")
    y2 = torch.empty_like(y)
    anr.conv2d(xd, wd, y2, s.stride, s.pad)
    assert torch.equal(y, y2), "packed and unpacked results differ"


def test_conv_bn_relu_packed_config(anr):
    cfg = I.config_inputs("ConvLayer")
    s = cfg["shape"]
    xd, wd = dev(cfg["x"]), dev(cfg["w"])
    bn = [dev(cfg[k]) for k in ("gamma", "beta", "mean", "var")]
    d, pack = anr.conv2d_pack_weights((s.N, s.C, s.H, s.W), wd, s.stride, s.pad, bn=bn, eps=cfg["eps"])
    buf, y = guarded((s.N, s.K, s.OH, s.OW))
    anr.conv_bn_relu_packed(d, xd, pack, y)
    check_guard(buf)
    ref = oracle.conv_bn_relu(cfg["x"], cfg["w"], cfg["gamma"], cfg["beta"], cfg["mean"], cfg["var"], cfg["eps"],
                              s.stride, s.pad)
    assert_parity(y, ref, what="ConvLayer packed")
    y2 = torch.empty_like(y)
    anr.conv_bn_relu(xd, wd, *bn, cfg["eps"], y2, s.stride, s.pad)
    assert torch.equal(y, y2), "packed and unpacked results differ"
    # the same pack without the fused epilogue is the plain convolution
    anr.conv2d_packed(d, xd, pack, y)
    assert_parity(y, oracle.conv2d(cfg["x"], cfg["w"], s.stride, s.pad), what="ConvLayer pack, plain conv")


PACKED_SHAPES = [
    (I.ConvShape(3, 16, 20, 24, 40, 3, 3, (1, 1), (1, 1)), 1),        # patch kernel, channel tile past K, ragged pixel tile
    (I.ConvShape(2, 24, 17, 12, 70, 3, 3, (2, 2), (1, 1)), 1),        # patch kernel, stride 2, three chunks
    (I.ConvShape(8, 32, 28, 28, 32, 3, 3, (1, 1), (1, 1)), 0),        # library's choice
    (I.ConvShape(1, 64, 14, 14, 96, 3, 3, (1, 1), (1, 1)), 0),        # general kernel, split reduction
    (I.ConvShape(2, 3, 30, 30, 16, 7, 7, (2, 2), (3, 3)), 0),         # 7x7
    (I.ConvShape(2, 32, 9, 9, 24, 1, 1, (1, 1), (0, 0)), 0),          # 1x1
    (I.ConvShape(8, 64, 48, 48, 64, 1, 1, (1, 1), (0, 0)), 0),        # 1x1, streaming kernel
    (I.ConvShape(2, 16, 14, 14, 24, 3, 3, (1, 1), (2, 2), (2, 2), 4), 0),   # grouped, dilated
]


@pytest.mark.parametrize("shape,route", PACKED_SHAPES, ids=str)
def test_conv2d_packed_small(anr, shape, route):
    """Integer-valued inputs: the packed call equals the oracle bit for bit, with and without the
    fused batch norm + ReLU, whatever kernel the descriptor is planned for."""
    s = shape
    x, w = I.conv_inputs(s, 1400, ints=True)
    xd, wd = dev(x), dev(w)
    gamma, beta, mean, var = I.bn_inputs(s.K, 1401)
    bn = [dev(v) for v in (gamma, beta, mean, var)]
    d, pack = anr.conv2d_pack_weights((s.N, s.C, s.H, s.W), wd, s.stride, s.pad, bn=bn, eps=I.BN_EPS, dil=s.dil,
                                      groups=s.groups, route=route)
    buf, y = guarded((s.N, s.K, s.OH, s.OW))
    anr.conv2d_packed(d, xd, pack, y)
    check_guard(buf)
    assert_parity(y, oracle.conv2d_general(x, w, s.stride, s.pad, s.dil, s.groups), exact=True, what="packed %s" % (s,))
    y2 = torch.empty_like(y)
    anr.conv_bn_relu_packed(d, xd, pack, y)
    anr.conv_bn_relu(xd, wd, *bn, I.BN_EPS, y2, s.stride, s.pad, dil=s.dil, groups=s.groups, route=route)
    assert torch.equal(y, y2), "packed and unpacked ConvLayer differ"
    ref = oracle.conv_bn_relu_general(x, w, gamma, beta, mean, var, I.BN_EPS, s.stride, s.pad, s.dil, s.groups)
    assert_parity(y, ref, what="packed ConvLayer %s" % (s,))


def test_conv2d_packed_refuses_an_input_the_pack_was_not_planned_for(anr):
    """A pack in the patch kernel's order cannot serve a view of x that kernel cannot read."""
    import ctypes
    s = I.ConvShape(8, 16, 56, 56, 64, 3, 3, (1, 1), (1, 1))
    x, w = I.conv_inputs(s, 1410, ints=True)
    d, pack = anr.conv2d_pack_weights((s.N, s.C, s.H, s.W), dev(w), s.stride, s.pad)
    assert anr.conv2d_route(d).kernel == anr.ANR_CONV_KERNEL_PATCH
    xbuf = torch.zeros((x.size + 1,), device="cuda")
    xbuf[1:] = dev(x).reshape(-1)
    xv = xbuf[1:].view(*x.shape)                       # 4-byte aligned only
    y = torch.empty((s.N, s.K, s.OH, s.OW), device="cuda")
    st = anr.raw().anr_conv2d_packed(ctypes.byref(d), ctypes.c_void_p(xv.data_ptr()), ctypes.c_void_p(pack.data_ptr()),
                                     ctypes.c_void_p(y.data_ptr()), None, 0, None)
    assert st == anr.ANR_ERR_INVALID_ARG


def test_conv2d_split_k_workspace(anr):
    """A split-K shape with the caller's own workspace, twice: the partial tiles are summed in
    a fixed order, so both runs agree bit for bit; too small a workspace is an error."""
    from paper_2006_06762_amd import binding as B
    s = I.ConvShape(1, 512, 7, 7, 512, 3, 3, (1, 1), (1, 1))
    x, w = I.conv_inputs(s, 210)
    d = B.conv_desc((s.N, s.C, s.H, s.W), s.K, s.R, s.S, s.stride, s.pad)
    need = B.workspace_size(B.ANR_OP_CONV2D, d)
    assert need > 0
    ws = torch.full((need + 256,), 0x7f, dtype=torch.uint8, device="cuda")    # NaN-ish garbage
    xd, wd = dev(x), dev(w)
    y1 = torch.empty((1, s.K, s.OH, s.OW), device="cuda")
    y2 = torch.empty_like(y1)
    anr.conv2d(xd, wd, y1, s.stride, s.pad, ws=ws)
    anr.conv2d(xd, wd, y2, s.stride, s.pad)             # the binding's own workspace
    assert_parity(y1, oracle.conv2d(x, w, s.stride, s.pad), what="split-K conv")
    assert torch.equal(y1, y2)
    assert bool((ws[need:] == 0x7f).all()), "wrote past the stated workspace size"
    with pytest.raises(ValueError):
        anr.conv2d(xd, wd, y2, s.stride, s.pad, ws=ws[:need // 2])
    st = B.raw().anr_conv2d(__import__("ctypes").byref(d), B._ptr(xd), B._ptr(wd), B._ptr(y2), None, 0,
                            B._stream())
    assert st == B.ANR_ERR_WORKSPACE


def test_conv_bn_relu_split_k(anr):
    """The fused epilogue runs in the reduce kernel when the reduction is split."""
    s = I.ConvShape(1, 256, 14, 14, 256, 3, 3, (1, 1), (1, 1))
    x, w = I.conv_inputs(s, 211)
    gamma, beta, mean, var = I.bn_inputs(s.K, 212)
    buf, y = guarded((1, s.K, s.OH, s.OW))
    anr.conv_bn_relu(dev(x), dev(w), dev(gamma), dev(beta), dev(mean), dev(var), I.BN_EPS, y, s.stride, s.pad)
    check_guard(buf)
    ref = oracle.conv_bn_relu(x, w, gamma, beta, mean, var, I.BN_EPS, s.stride, s.pad)
    assert_parity(y, ref, what="split-K ConvLayer")
    assert float(y.min()) >= 0.0


def test_conv2d_gather_strided_views(anr):
    """Odd-width, unaligned views (one float into a wider buffer) take the general kernel."""
    s = I.ConvShape(2, 6, 9, 7, 10, 3, 3, (1, 1), (1, 1))
    x, w = I.conv_inputs(s, 213)
    xw = torch.zeros((2, 8, 11, 10), device="cuda")
    xw[:, 1:7, 1:10, 1:8] = dev(x)
    yw = torch.full((2, 12, s.OH + 1, s.OW + 3), CANARY, device="cuda")
    yv = yw[:, 1:11, :s.OH, 2:2 + s.OW]
    anr.conv2d(xw[:, 1:7, 1:10, 1:8], dev(w), yv, s.stride, s.pad)
    assert_parity(yv.contiguous(), oracle.conv2d(x, w, s.stride, s.pad), what="gather strided views")
    yw[:, 1:11, :s.OH, 2:2 + s.OW] = CANARY
    assert bool((yw == CANARY).all()), "store outside the output view"


# ------------------------------------------------------------------ GRP and DIL (grouped, dilated)
GENERAL_SHAPES = [
    I.ConvShape(2, 8, 12, 12, 8, 3, 3, (1, 1), (2, 2), (2, 2), 1),
    I.ConvShape(1, 3, 41, 37, 20, 7, 7, (2, 2), (3, 3), (2, 2), 1),
    I.ConvShape(2, 16, 9, 11, 12, 3, 2, (2, 1), (1, 3), (3, 2), 1),
    I.ConvShape(2, 12, 14, 14, 40, 3, 3, (1, 1), (1, 1), (1, 1), 4),
    I.ConvShape(1, 64, 9, 9, 96, 1, 1, (1, 1), (0, 0), (1, 1), 4),
    I.ConvShape(1, 256, 7, 7, 256, 3, 3, (1, 1), (1, 1), (1, 1), 4),      # split-K inside each group
    I.ConvShape(3, 10, 13, 10, 130, 3, 3, (2, 2), (2, 2), (2, 2), 2),      # 65 channels per group: ragged tiles
    I.ConvShape(2, 6, 8, 8, 6, 3, 3, (1, 1), (1, 1), (1, 1), 6),           # one channel per group
]


@pytest.mark.parametrize("shape", GENERAL_SHAPES, ids=str)
@pytest.mark.parametrize("ints", [False, True])
def test_conv2d_grouped_dilated(anr, shape, ints):
    x, w = I.conv_inputs(shape, 220, ints=ints)
    buf, y = guarded((shape.N, shape.K, shape.OH, shape.OW))
    anr.conv2d(dev(x), dev(w), y, shape.stride, shape.pad, dil=shape.dil, groups=shape.groups)
    check_guard(buf)
    ref = oracle.conv2d_general(x, w, shape.stride, shape.pad, shape.dil, shape.groups)
    assert_parity(y, ref, exact=ints, what=str(shape))


# 1 x 1 kernels of small groups: 64 / Kg groups share a column tile with a block-diagonal weight tile.
# Packs of 8, 16, 4 and 2 groups, several packs, several chunks per pack, stride and padding (a 1 x 1
# tap that leaves the image), a pixel count that is not a multiple of the tile, and a case whose few
# tiles make the planner split the reduction.
PACKED_GROUP_SHAPES = [
    I.ConvShape(2, 64, 9, 11, 64, 1, 1, (1, 1), (0, 0), (1, 1), 8),
    I.ConvShape(1, 128, 13, 7, 64, 1, 1, (1, 1), (0, 0), (1, 1), 16),
    I.ConvShape(3, 64, 10, 10, 64, 1, 1, (2, 2), (1, 1), (1, 1), 4),
    I.ConvShape(1, 96, 8, 9, 192, 1, 1, (1, 1), (0, 0), (1, 1), 6),
    I.ConvShape(2, 256, 6, 6, 128, 1, 1, (1, 1), (0, 0), (1, 1), 32),
    I.ConvShape(1, 512, 7, 7, 128, 1, 1, (1, 1), (0, 0), (1, 1), 8),
    I.ConvShape(1, 48, 5, 5, 48, 1, 1, (1, 1), (0, 0), (1, 1), 12),      # 3 packs of 4 groups would need 48 % 32 == 0: general kernel
]


@pytest.mark.parametrize("shape", PACKED_GROUP_SHAPES, ids=str)
@pytest.mark.parametrize("ints", [False, True])
def test_conv2d_packed_groups(anr, shape, ints):
    x, w = I.conv_inputs(shape, 230, ints=ints)
    buf, y = guarded((shape.N, shape.K, shape.OH, shape.OW))
    anr.conv2d(dev(x), dev(w), y, shape.stride, shape.pad, dil=shape.dil, groups=shape.groups)
    check_guard(buf)
    ref = oracle.conv2d_general(x, w, shape.stride, shape.pad, shape.dil, shape.groups)
    assert_parity(y, ref, exact=ints, what=str(shape))


def test_conv_bn_relu_packed_groups(anr):
    s = I.ConvShape(2, 64, 12, 12, 64, 1, 1, (1, 1), (0, 0), (1, 1), 4)
    x, w = I.conv_inputs(s, 231)
    gamma, beta, mean, var = I.bn_inputs(s.K, 232)
    y = torch.empty((s.N, s.K, s.OH, s.OW), device="cuda")
    anr.conv_bn_relu(dev(x), dev(w), dev(gamma), dev(beta), dev(mean), dev(var), I.BN_EPS, y, s.stride, s.pad,
                     dil=s.dil, groups=s.groups)
    ref = oracle.conv_bn_relu_general(x, w, gamma, beta, mean, var, I.BN_EPS, s.stride, s.pad, s.dil, s.groups)
    assert_parity(y, ref, what="packed-group ConvLayer")


def test_conv_bn_relu_grouped_dilated(anr):
    s = I.ConvShape(2, 16, 10, 10, 24, 3, 3, (1, 1), (2, 2), (2, 2), 4)
    x, w = I.conv_inputs(s, 221)
    gamma, beta, mean, var = I.bn_inputs(s.K, 222)
    y = torch.empty((s.N, s.K, s.OH, s.OW), device="cuda")
    anr.conv_bn_relu(dev(x), dev(w), dev(gamma), dev(beta), dev(mean), dev(var), I.BN_EPS, y, s.stride, s.pad,
                     dil=s.dil, groups=s.groups)
    ref = oracle.conv_bn_relu_general(x, w, gamma, beta, mean, var, I.BN_EPS, s.stride, s.pad, s.dil, s.groups)
    assert_parity(y, ref, what="grouped dilated ConvLayer")


def test_dwconv_dilated(anr):
    s = I.ConvShape(2, 5, 12, 9, 5, 3, 3, (1, 1), (2, 2), (2, 2))
    x, w = I.dwconv_inputs(s, 223)
    buf, y = guarded((s.N, s.C, s.OH, s.OW))
    anr.dwconv(dev(x), dev(w), y, s.stride, s.pad, dil=s.dil)
    check_guard(buf)
    # depthwise = one channel per group
    assert_parity(y, oracle.conv2d_general(x, w, s.stride, s.pad, s.dil, s.C), what="dilated depthwise")


@pytest.mark.parametrize("name", ["C2D", "C2D_S2"])
def test_conv2d_configs(anr, conv_route, name):
    cfg = I.config_inputs(name)
    s = cfg["shape"]
    buf, y = guarded((s.N, s.K, s.OH, s.OW))
    anr.conv2d(dev(cfg["x"]), dev(cfg["w"]), y, s.stride, s.pad, route=conv_route)
    check_guard(buf)
    assert_parity(y, oracle.conv2d(cfg["x"], cfg["w"], s.stride, s.pad), what=name)


@pytest.mark.parametrize("name", ["C2D", "C2D_S2"])
def test_conv2d_configs_integer_exact(anr, name):
    s = I.config_inputs(name)["shape"]
    x, w = I.conv_inputs(s, 201, ints=True)
    y = torch.empty((s.N, s.K, s.OH, s.OW), device="cuda")
    anr.conv2d(dev(x), dev(w), y, s.stride, s.pad)
    assert_parity(y, oracle.conv2d(x, w, s.stride, s.pad), exact=True, what=name + " ints")


def test_conv2d_delta_kernel_is_shift(anr, conv_route):
    C, H, W = 8, 12, 16
    x = I.small_ints(np.random.Generator(np.random.PCG64(5)), (2, C, H, W))
    for (r0, s0) in [(0, 0), (0, 2), (2, 1), (1, 1)]:
        w = np.zeros((C, C, 3, 3), np.float32)
        for c in range(C):
            w[c, c, r0, s0] = 1.0
        y = torch.empty((2, C, H, W), device="cuda")
        anr.conv2d(dev(x), dev(w), y, (1, 1), (1, 1), route=conv_route)
        exp = np.zeros((2, C, H, W), np.float32)
        for oh in range(H):
            for ow in range(W):
                ih, iw = oh + r0 - 1, ow + s0 - 1
                if 0 <= ih < H and 0 <= iw < W:
                    exp[:, :, oh, ow] = x[:, :, ih, iw]
        assert np.array_equal(y.cpu().numpy(), exp)


def test_conv2d_strided_views(anr, conv_route):
    # x is a window of a larger tensor and y is written into a larger tensor
    s = I.ConvShape(2, 8, 12, 16, 16, 3, 3, (1, 1), (1, 1))
    x, w = I.conv_inputs(s, 202)
    xw = torch.zeros((2, 10, 14, 24), device="cuda")
    xw[:, 1:9, 1:13, 4:20] = dev(x)
    yw = torch.full((2, 18, 13, 20), CANARY, device="cuda")
    anr.conv2d(xw[:, 1:9, 1:13, 4:20], dev(w), yw[:, 1:17, 0:12, 4:20], s.stride, s.pad, route=conv_route)
    ref = oracle.conv2d(x, w, s.stride, s.pad)
    assert_parity(yw[:, 1:17, 0:12, 4:20].contiguous(), ref, what="strided conv (aligned)")
    assert float((yw == CANARY).sum()) == yw.numel() - ref.size
    # an unaligned window (offset 1 in w) must give the same values through the generic kernel
    xw2 = torch.zeros((2, 10, 14, 24), device="cuda")
    xw2[:, 1:9, 1:13, 1:17] = dev(x)
    y2 = torch.empty((2, 16, 12, 16), device="cuda")
    anr.conv2d(xw2[:, 1:9, 1:13, 1:17], dev(w), y2, s.stride, s.pad)
    assert_parity(y2, ref, what="strided conv (unaligned)")


def test_conv2d_is_deterministic(anr):
    s = I.ConvShape(2, 16, 28, 28, 64, 3, 3, (1, 1), (1, 1))
    x, w = I.conv_inputs(s, 203)
    xd, wd = dev(x), dev(w)
    y1 = torch.empty((2, 64, 28, 28), device="cuda")
    y2 = torch.full((2, 64, 28, 28), float("nan"), device="cuda")
    anr.conv2d(xd, wd, y1, s.stride, s.pad)
    anr.conv2d(xd, wd, y2, s.stride, s.pad)
    assert torch.equal(y1, y2)


# ------------------------------------------------------------------ ConvLayer
CONVLAYER_SHAPES = [
    I.ConvShape(2, 8, 12, 12, 24, 3, 3, (1, 1), (1, 1)),
    I.ConvShape(3, 16, 28, 28, 40, 3, 3, (2, 2), (1, 1)),
    I.ConvShape(1, 3, 16, 16, 8, 7, 7, (2, 2), (3, 3)),
    I.ConvShape(2, 16, 10, 10, 12, 1, 1, (2, 2), (0, 0)),
]


@pytest.mark.parametrize("shape", CONVLAYER_SHAPES, ids=str)
def test_conv_bn_relu_small(anr, conv_route, shape):
    x, w = I.conv_inputs(shape, 300)
    w = (w * 4).astype(np.float32)     # spread the pre-activation so that both ReLU branches are hit
    gamma, beta, mean, var = I.bn_inputs(shape.K, 301)
    buf, y = guarded((shape.N, shape.K, shape.OH, shape.OW))
    anr.conv_bn_relu(dev(x), dev(w), dev(gamma), dev(beta), dev(mean), dev(var), I.BN_EPS, y,
                     shape.stride, shape.pad, route=conv_route)
    check_guard(buf)
    ref = oracle.conv_bn_relu(x, w, gamma, beta, mean, var, I.BN_EPS, shape.stride, shape.pad)
    assert_parity(y, ref, what=str(shape))
    got = y.cpu().numpy()
    assert (got >= 0).all() and (got == 0).any() and (got > 0).any()


def test_conv_bn_relu_config(anr):
    cfg = I.config_inputs("ConvLayer")
    s = cfg["shape"]
    buf, y = guarded((s.N, s.K, s.OH, s.OW))
    anr.conv_bn_relu(dev(cfg["x"]), dev(cfg["w"]), dev(cfg["gamma"]), dev(cfg["beta"]), dev(cfg["mean"]),
                     dev(cfg["var"]), cfg["eps"], y, s.stride, s.pad)
    check_guard(buf)
    ref = oracle.conv_bn_relu(cfg["x"], cfg["w"], cfg["gamma"], cfg["beta"], cfg["mean"], cfg["var"],
                              cfg["eps"], s.stride, s.pad)
    assert_parity(y, ref, what="ConvLayer")
    assert (y >= 0).all()


def test_conv_bn_relu_identity_bn_exact(anr):
    # gamma=1, beta=0, mean=0, var+eps=1: the layer is exactly ReLU(conv) on integer inputs
    s = I.ConvShape(2, 8, 12, 12, 16, 3, 3, (1, 1), (1, 1))
    x, w = I.conv_inputs(s, 302, ints=True)
    K = s.K
    one, zero = torch.ones(K, device="cuda"), torch.zeros(K, device="cuda")
    var = torch.full((K,), 0.75, device="cuda")
    y = torch.empty((2, K, 12, 12), device="cuda")
    anr.conv_bn_relu(dev(x), dev(w), one, zero, zero, var, 0.25, y, s.stride, s.pad)
    ref = np.maximum(oracle.conv2d(x, w, s.stride, s.pad), 0.0)
    assert_parity(y, ref, exact=True, what="identity BN")


# ------------------------------------------------------------------ depthwise
DW_SHAPES = [
    I.ConvShape(2, 5, 8, 8, 5, 3, 3, (1, 1), (1, 1)),
    I.ConvShape(3, 20, 28, 28, 20, 3, 3, (1, 1), (1, 1)),
    I.ConvShape(1, 7, 13, 16, 7, 3, 3, (1, 1), (1, 1)),
    I.ConvShape(1, 3, 30, 112, 3, 3, 3, (1, 1), (1, 1)),
    I.ConvShape(2, 4, 7, 7, 4, 3, 3, (1, 1), (1, 1)),
    I.ConvShape(1, 6, 14, 14, 6, 3, 3, (2, 2), (1, 1)),
    I.ConvShape(1, 4, 17, 20, 4, 3, 3, (2, 2), (1, 1)),
    I.ConvShape(1, 3, 9, 10, 3, 5, 5, (1, 1), (2, 2)),
    I.ConvShape(1, 2, 6, 260, 2, 3, 3, (1, 1), (1, 1)),
    # general kernel: small planes, rows wider than a wave, tall images, asymmetric stride and
    # padding, kernels that hang over the image edge
    I.ConvShape(3, 67, 7, 7, 67, 3, 3, (1, 1), (1, 1)),
    I.ConvShape(2, 9, 14, 14, 9, 3, 3, (2, 2), (1, 1)),
    I.ConvShape(1, 3, 112, 112, 3, 3, 3, (2, 2), (1, 1)),
    I.ConvShape(1, 2, 150, 70, 2, 3, 3, (1, 1), (1, 1)),
    I.ConvShape(2, 3, 40, 130, 3, 5, 3, (2, 1), (2, 0)),
    I.ConvShape(1, 5, 9, 11, 5, 7, 7, (1, 1), (3, 3)),
    I.ConvShape(1, 4, 5, 5, 4, 5, 5, (1, 1), (4, 4)),
    I.ConvShape(1, 1, 64, 64, 1, 1, 1, (1, 1), (0, 0)),
    I.ConvShape(1, 3, 20, 65, 3, 2, 4, (3, 2), (1, 2)),
    # stride-2 register-sliding kernel (width a multiple of 8): odd height, a ragged row chunk,
    # planes that do not fill the last wave
    I.ConvShape(2, 5, 16, 24, 5, 3, 3, (2, 2), (1, 1)),
    I.ConvShape(1, 3, 9, 8, 3, 3, 3, (2, 2), (1, 1)),
    I.ConvShape(3, 7, 30, 56, 7, 3, 3, (2, 2), (1, 1)),
]


@pytest.mark.parametrize("shape", DW_SHAPES, ids=str)
@pytest.mark.parametrize("ints", [False, True])
def test_dwconv_small(anr, shape, ints):
    x, w = I.dwconv_inputs(shape, 400, ints=ints)
    buf, y = guarded((shape.N, shape.C, shape.OH, shape.OW))
    anr.dwconv(dev(x), dev(w), y, shape.stride, shape.pad)
    check_guard(buf)
    assert_parity(y, oracle.dwconv(x, w, shape.stride, shape.pad), exact=ints, what=str(shape))


def test_dwconv_small_planes_many_planes(anr):
    """Small maps with enough planes that a work-group stages several of them through LDS, the last
    work-group with fewer (plane count not a multiple of the group); 3x3, 5x5 and a 5x2 kernel.
    Then plane sizes that allow groups of one plane (H*W and OH*OW multiples of 4) and of two
    (both even), with few planes, so that the smallest group is the one taken."""
    for s in [I.ConvShape(2, 3101, 7, 7, 3101, 3, 3, (1, 1), (1, 1)),
              I.ConvShape(1, 6150, 14, 14, 6150, 3, 3, (2, 2), (1, 1)),
              I.ConvShape(3, 2051, 6, 5, 2051, 5, 2, (1, 2), (2, 0)),
              I.ConvShape(2, 1543, 14, 14, 1543, 5, 5, (1, 1), (2, 2)),
              I.ConvShape(1, 3079, 14, 14, 3079, 5, 5, (2, 2), (2, 2)),
              I.ConvShape(1, 37, 28, 28, 37, 3, 3, (2, 2), (1, 1)),
              I.ConvShape(3, 11, 30, 30, 11, 3, 3, (1, 1), (1, 1)),
              I.ConvShape(1, 45, 10, 9, 45, 3, 3, (1, 1), (1, 1)),
              I.ConvShape(2, 19, 22, 18, 19, 5, 5, (1, 1), (2, 2)),
              I.ConvShape(1, 5, 44, 44, 5, 5, 5, (1, 1), (0, 0))]:
        x, w = I.dwconv_inputs(s, 470, ints=True)
        buf, y = guarded((s.N, s.C, s.OH, s.OW))
        anr.dwconv(dev(x), dev(w), y, s.stride, s.pad)
        check_guard(buf)
        assert_parity(y, oracle.dwconv(x, w, s.stride, s.pad), exact=True, what=str(s))


def test_dwconv_config(anr):
    cfg = I.config_inputs("DEP")
    s = cfg["shape"]
    buf, y = guarded((s.N, s.C, s.OH, s.OW))
    anr.dwconv(dev(cfg["x"]), dev(cfg["w"]), y, s.stride, s.pad)
    check_guard(buf)
    assert_parity(y, oracle.dwconv(cfg["x"], cfg["w"], s.stride, s.pad), what="DEP")
    x, w = I.dwconv_inputs(s, 401, ints=True)
    anr.dwconv(dev(x), dev(w), y, s.stride, s.pad)
    assert_parity(y, oracle.dwconv(x, w, s.stride, s.pad), exact=True, what="DEP ints")


def test_dwconv_strided_views(anr):
    s = I.ConvShape(2, 6, 12, 16, 6, 3, 3, (1, 1), (1, 1))
    x, w = I.dwconv_inputs(s, 402)
    xw = torch.zeros((2, 8, 14, 24), device="cuda")
    xw[:, 1:7, 1:13, 4:20] = dev(x)
    yw = torch.full((2, 7, 13, 20), CANARY, device="cuda")
    anr.dwconv(xw[:, 1:7, 1:13, 4:20], dev(w), yw[:, 1:7, 0:12, 4:20], s.stride, s.pad)
    ref = oracle.dwconv(x, w, s.stride, s.pad)
    assert_parity(yw[:, 1:7, 0:12, 4:20].contiguous(), ref, what="strided dwconv")
    assert float((yw == CANARY).sum()) == yw.numel() - ref.size


# ------------------------------------------------------------------ TBG / TBS
TBG_SHAPES = [I.TbgShape(1, 1, 1, 1), I.TbgShape(2, 5, 3, 4), I.TbgShape(2, 70, 3, 20),
              I.TbgShape(1, 128, 2, 64), I.TbgShape(2, 64, 3, 128), I.TbgShape(1, 130, 2, 33)]


@pytest.mark.parametrize("shape", TBG_SHAPES, ids=str)
@pytest.mark.parametrize("ints", [False, True])
def test_tbg_small(anr, shape, ints):
    q, k = I.tbg_inputs(shape, 500, ints=ints)
    buf, out = guarded((shape.B, shape.H, shape.S, shape.S))
    anr.tbg(dev(q), dev(k), out)
    check_guard(buf)
    assert_parity(out, oracle.tbg(q, k), exact=ints, what=str(shape))


def test_tbg_config(anr):
    cfg = I.config_inputs("TBG")
    s = cfg["shape"]
    buf, out = guarded((s.B, s.H, s.S, s.S))
    anr.tbg(dev(cfg["q"]), dev(cfg["k"]), out)
    check_guard(buf)
    assert_parity(out, oracle.tbg(cfg["q"], cfg["k"]), what="TBG")


def test_tbg_q_equals_k_is_symmetric(anr):
    q, _ = I.tbg_inputs(I.TbgShape(2, 128, 3, 64), 501)
    qd = dev(q)
    out = torch.empty((2, 3, 128, 128), device="cuda")
    anr.tbg(qd, qd, out)
    o = out.cpu().numpy().astype(np.float64)
    assert np.max(np.abs(o - o.transpose(0, 1, 3, 2)) / np.maximum(1.0, np.abs(o))) <= 1e-6
    assert (np.einsum("bhii->bhi", o) >= 0).all()


def test_tbg_one_hot_index_code(anr):
    # which (b, h, i) met which j: catches a wrong transpose folded into the addressing
    B, S, H, D = 2, 64, 3, 64
    q = np.zeros((B, S, H, D), np.float32)
    k = np.zeros((B, S, H, D), np.float32)
    for b in range(B):
        for s in range(S):
            for h in range(H):
                q[b, s, h, s % D] = 1.0
                k[b, s, h, (s + 1) % D] = 1.0 + b + 10 * h
    out = torch.empty((B, H, S, S), device="cuda")
    anr.tbg(dev(q), dev(k), out)
    assert np.array_equal(out.cpu().numpy().astype(np.float64), oracle.tbg(q, k))


def test_tbg_strided_views(anr):
    # q and k as the two halves of one fused [B,S,2,H,D] projection output
    s = I.TbgShape(2, 40, 3, 16)
    q, k = I.tbg_inputs(s, 502)
    fused = torch.zeros((2, 40, 2, 3, 16), device="cuda")
    fused[:, :, 0] = dev(q)
    fused[:, :, 1] = dev(k)
    out = torch.empty((2, 3, 40, 40), device="cuda")
    anr.tbg(fused[:, :, 0], fused[:, :, 1], out)
    assert_parity(out, oracle.tbg(q, k), what="strided tbg")


def assert_softmax_parity(got_t, ref, what=""):
    """Probabilities are at most 1, where the general bar is an absolute one; here the error is
    taken relative to the largest probability of the row, which is what 1e-4 relative means for
    a row of softmax outputs (fp32 scores carry ~1e-6 absolute error, exp turns it relative)."""
    assert_parity(got_t, ref, what=what)
    got = got_t.cpu().numpy().astype(np.float64)
    e = float(np.max(np.abs(got - ref) / ref.max(axis=-1, keepdims=True)))
    assert e <= TOL, "%s: row-relative err %.3e" % (what, e)


# S <= 128 with D a multiple of 8 (up to 1024) takes the fused kernel, the rest the two-kernel path
TBS_SHAPES = [I.TbgShape(2, 5, 3, 4), I.TbgShape(1, 128, 2, 64), I.TbgShape(1, 130, 2, 33),
              I.TbgShape(2, 64, 12, 128), I.TbgShape(1, 1, 1, 8), I.TbgShape(3, 65, 2, 8),
              I.TbgShape(1, 100, 5, 32), I.TbgShape(2, 96, 3, 24), I.TbgShape(1, 128, 3, 128),
              I.TbgShape(1, 127, 2, 72), I.TbgShape(1, 129, 2, 64), I.TbgShape(1, 33, 2, 136),
              # short sequences: two key blocks x two query blocks, one key block x four query blocks
              I.TbgShape(2, 64, 3, 64), I.TbgShape(1, 48, 5, 40), I.TbgShape(2, 32, 3, 128),
              I.TbgShape(3, 20, 2, 16), I.TbgShape(1, 33, 2, 8),
              # reductions longer than one 64-column chunk, the last chunk partial
              I.TbgShape(1, 128, 2, 256), I.TbgShape(2, 50, 3, 200), I.TbgShape(1, 100, 2, 72)]


@pytest.mark.parametrize("shape", TBS_SHAPES, ids=str)
def test_tbs_small(anr, shape):
    q, k = I.tbg_inputs(shape, 503)
    q = (q * 0.35).astype(np.float32)
    buf, out = guarded((shape.B, shape.H, shape.S, shape.S))
    anr.tbs(dev(q), dev(k), out)
    check_guard(buf)
    ref = oracle.tbs(q, k)
    assert_softmax_parity(out, ref, what="tbs " + str(shape))
    np.testing.assert_allclose(out.cpu().numpy().sum(-1), 1.0, atol=1e-5)


def test_tbs_large_scores(anr):
    """Scores far from zero: the row maximum must be subtracted before exponentiation."""
    shape = I.TbgShape(1, 96, 2, 64)
    q, k = I.tbg_inputs(shape, 504)
    q = (q * 6.0).astype(np.float32)
    out = torch.empty((1, 2, 96, 96), device="cuda")
    anr.tbs(dev(q), dev(k), out)
    ref = oracle.tbs(q, k)
    got = out.cpu().numpy()
    assert np.isfinite(got).all()
    assert_softmax_parity(out, ref, what="tbs large scores")


def test_tbs_strided_views(anr):
    """q and k as slices of one fused [B, S, 2, H, D] projection, on the fused-kernel shape."""
    s = I.TbgShape(2, 72, 3, 16)
    q, k = I.tbg_inputs(s, 505)
    fused = torch.zeros((2, 72, 2, 3, 16), device="cuda")
    fused[:, :, 0] = dev(q)
    fused[:, :, 1] = dev(k)
    buf, out = guarded((2, 3, 72, 72))
    anr.tbs(fused[:, :, 0], fused[:, :, 1], out)
    check_guard(buf)
    assert_softmax_parity(out, oracle.tbs(q, k), what="strided tbs")


def test_tbs_config_shape(anr):
    cfg = I.config_inputs("TBG")
    s = cfg["shape"]
    out = torch.empty((s.B, s.H, s.S, s.S), device="cuda")
    anr.tbs(dev(cfg["q"]), dev(cfg["k"]), out)
    assert_softmax_parity(out, oracle.tbs(cfg["q"], cfg["k"]), what="TBS config")


# ------------------------------------------------------------------ seeded random geometries
def _random_conv_shapes(count, seed):
    g = np.random.Generator(np.random.PCG64(seed))
    shapes = []
    while len(shapes) < count:
        groups = int(g.choice([1, 1, 1, 2, 3, 4]))
        C = groups * int(g.integers(1, 13))
        K = groups * int(g.integers(1, 41))
        R, S = int(g.integers(1, 6)), int(g.integers(1, 6))
        dil = (int(g.integers(1, 4)), int(g.integers(1, 4)))
        stride = (int(g.integers(1, 4)), int(g.integers(1, 4)))
        pad = (int(g.integers(0, 4)), int(g.integers(0, 4)))
        H, W = int(g.integers(1, 24)), int(g.integers(1, 24))
        s = I.ConvShape(int(g.integers(1, 4)), C, H, W, K, R, S, stride, pad, dil, groups)
        if s.OH >= 1 and s.OW >= 1:
            shapes.append(s)
    return shapes


def test_conv2d_random_geometries(anr):
    """Forty seeded random geometries (kernel, stride, padding, dilation, groups, odd sizes) with
    small-integer values: the general kernel must agree with the oracle bit for bit."""
    for i, s in enumerate(_random_conv_shapes(40, 900)):
        x, w = I.conv_inputs(s, 901 + i, ints=True)
        buf, y = guarded((s.N, s.K, s.OH, s.OW))
        anr.conv2d(dev(x), dev(w), y, s.stride, s.pad, dil=s.dil, groups=s.groups)
        check_guard(buf)
        ref = oracle.conv2d_general(x, w, s.stride, s.pad, s.dil, s.groups)
        assert_parity(y, ref, exact=True, what="random conv %d %s" % (i, s))



def _random_tap_shapes(count, seed):
    """Geometries of the kernels with compile-time taps: 3x3 with channels per group a multiple of
    4, 1x1 with a multiple of 32, 5x5 and 7x7 with any channel count; everything else random."""
    g = np.random.Generator(np.random.PCG64(seed))
    shapes = []
    while len(shapes) < count:
        kind = int(g.choice([1, 3, 3, 5, 7]))
        groups = int(g.choice([1, 1, 2, 3]))
        cg = {1: 32 * int(g.integers(1, 4)), 3: 4 * int(g.integers(1, 9)), 5: int(g.integers(1, 9)),
              7: int(g.integers(1, 7))}[kind]
        K = groups * int(g.integers(1, 90))
        dil = (int(g.integers(1, 3)), int(g.integers(1, 3)))
        stride = (int(g.integers(1, 3)), int(g.integers(1, 3)))
        pad = (int(g.integers(0, 4)), int(g.integers(0, 4)))
        H, W = int(g.integers(1, 30)), int(g.integers(1, 30))
        s = I.ConvShape(int(g.integers(1, 4)), groups * cg, H, W, K, kind, kind, stride, pad, dil, groups)
        if s.OH >= 1 and s.OW >= 1:
            shapes.append(s)
    return shapes


def test_conv2d_random_geometries_tap_kernels(anr):
    """Seeded random geometries for the 3x3 / 1x1 / 5x5 / 7x7 forms of the general kernel (whole-channel
    chunks, one byte offset per tap), small-integer values, bit for bit; every third case passes its
    weights at an address that is only 4-byte aligned (the 3x3 and 1x1 forms then hand over to the
    any-geometry kernel, the 5x5 / 7x7 form reads its 16-byte units unaligned)."""
    for i, s in enumerate(_random_tap_shapes(48, 950)):
        x, w = I.conv_inputs(s, 951 + i, ints=True)
        wd = dev(w)
        if i % 3 == 2:
            wbuf = torch.empty((wd.numel() + 1,), device="cuda")
            wbuf[1:] = wd.reshape(-1)
            wd = wbuf[1:].view(wd.shape)
            assert wd.data_ptr() % 16 == 4
        buf, y = guarded((s.N, s.K, s.OH, s.OW))
        anr.conv2d(dev(x), wd, y, s.stride, s.pad, dil=s.dil, groups=s.groups)
        check_guard(buf)
        ref = oracle.conv2d_general(x, w, s.stride, s.pad, s.dil, s.groups)
        assert_parity(y, ref, exact=True, what="random tap-kernel conv %d %s" % (i, s))


def test_conv2d_large_batch_without_split_keeps_the_mfma_kernel(anr):
    """A VGG-style stem at batch 24 (3 channels rule out the tap kernels; 77 M outputs): the plan does
    not split the reduction, so the cap on the split-K workspace must not push it to the
    one-thread-per-output kernel.  Checked on the first and the last image (an image's outputs depend
    on that image alone)."""
    s = I.ConvShape(24, 3, 224, 224, 64, 3, 3, (1, 1), (1, 1))
    d = anr.conv_desc((s.N, s.C, s.H, s.W), s.K, 3, 3, s.stride, s.pad)
    r = anr.conv2d_route(d)
    assert r.kernel == anr.ANR_CONV_KERNEL_GATHER and r.ksplit == 1
    x, w = I.conv_inputs(s, 1600)
    y = torch.empty((s.N, s.K, s.OH, s.OW), device="cuda")
    anr.conv2d(dev(x), dev(w), y, s.stride, s.pad)
    for n in (0, s.N - 1):
        ref = oracle.conv2d(x[n:n + 1], w, s.stride, s.pad)
        assert_parity(y[n:n + 1], ref, what="stem at batch 24, image %d" % n)


def test_conv2d_wave_groups_share_a_chain(anr):
    """About 200 output tiles with 16 and with 32 chunks each and no split-K: the work-groups of
    the compile-time-tap kernel then run two and four groups of waves that take alternate chunks
    and add their accumulators in LDS."""
    for s in [I.ConvShape(4, 64, 56, 56, 64, 3, 3, (1, 1), (1, 1)),
              I.ConvShape(8, 1024, 14, 14, 512, 1, 1, (1, 1), (0, 0)),
              I.ConvShape(2, 36, 40, 40, 100, 3, 3, (1, 1), (1, 1), (2, 2), 1)]:
        x, w = I.conv_inputs(s, 995, ints=True)
        buf, y = guarded((s.N, s.K, s.OH, s.OW))
        anr.conv2d(dev(x), dev(w), y, s.stride, s.pad, dil=s.dil, groups=s.groups)
        check_guard(buf)
        ref = oracle.conv2d_general(x, w, s.stride, s.pad, s.dil, s.groups)
        assert_parity(y, ref, exact=True, what=str(s))


def test_conv_bn_relu_stem_split_k(anr):
    """7x7 stride-2 layer on a small image: the three channel chunks are split over work-groups and
    the fused epilogue runs in the reduce kernel."""
    s = I.ConvShape(1, 3, 40, 44, 64, 7, 7, (2, 2), (3, 3))
    x, w = I.conv_inputs(s, 990)
    gamma, beta, mean, var = I.bn_inputs(s.K, 991)
    buf, y = guarded((1, s.K, s.OH, s.OW))
    anr.conv_bn_relu(dev(x), dev(w), dev(gamma), dev(beta), dev(mean), dev(var), I.BN_EPS, y, s.stride, s.pad)
    check_guard(buf)
    ref = oracle.conv_bn_relu(x, w, gamma, beta, mean, var, I.BN_EPS, s.stride, s.pad)
    assert_parity(y, ref, what="7x7 ConvLayer")


def test_conv2d_random_geometries_tuned_kernel(anr):
    """Seeded random geometries inside what the tuned patch-staging kernel takes (3x3 with C % 8 == 0,
    1x1 with C % 32 == 0 and C >= 256, W % 4 == 0), forced onto it whatever the tile count."""
    g = np.random.Generator(np.random.PCG64(980))
    for i in range(40):
        if g.random() < 0.75:
            R, C = 3, 8 * int(g.integers(1, 6))
        else:
            R, C = 1, 32 * int(g.integers(8, 11))
        st = int(g.integers(1, 3))
        pad = (int(g.integers(0, 3)), int(g.integers(0, 3)))
        H, W = int(g.integers(3, 40)), 4 * int(g.integers(1, 16))
        s = I.ConvShape(int(g.integers(1, 5)), C, H, W, int(g.integers(1, 100)), R, R, (st, st), pad)
        if s.OH < 1 or s.OW < 1:
            continue
        x, w = I.conv_inputs(s, 981 + i, ints=True)
        buf, y = guarded((s.N, s.K, s.OH, s.OW))
        anr.conv2d(dev(x), dev(w), y, s.stride, s.pad, route=1)
        check_guard(buf)
        assert_parity(y, oracle.conv2d(x, w, s.stride, s.pad), exact=True, what="random tuned conv %d %s" % (i, s))


def test_dwconv_random_geometries(anr):
    g = np.random.Generator(np.random.PCG64(950))
    for i in range(30):
        C = int(g.integers(1, 20))
        R, S = int(g.integers(1, 5)), int(g.integers(1, 5))
        stride = (int(g.integers(1, 3)), int(g.integers(1, 3)))
        pad = (int(g.integers(0, 3)), int(g.integers(0, 3)))
        dil = (int(g.integers(1, 3)), int(g.integers(1, 3)))
        H, W = int(g.integers(1, 40)), int(g.choice([4, 7, 8, 12, 14, 16, 24, 28, 33, 56]))
        s = I.ConvShape(int(g.integers(1, 4)), C, H, W, C, R, S, stride, pad, dil)
        if s.OH < 1 or s.OW < 1:
            continue
        x, w = I.dwconv_inputs(s, 951 + i, ints=True)
        buf, y = guarded((s.N, s.C, s.OH, s.OW))
        anr.dwconv(dev(x), dev(w), y, s.stride, s.pad, dil=s.dil)
        check_guard(buf)
        ref = oracle.conv2d_general(x, w, s.stride, s.pad, s.dil, s.C)
        assert_parity(y, ref, exact=True, what="random dwconv %d %s" % (i, s))


def test_dwconv_stream_kernel_runs_of_rows(anr):
    """Stride-1 3x3 layers on dense tensors take the streaming kernel.  Planes taller than its rounds
    of rows are cut into runs with halo rows, four or eight rounds each (eight once that still makes
    4096 waves); widths whose rows fill 64, 56, 48 or 33 lanes of a round; single-row and two-row planes.
    Small-integer values: bit for bit."""
    shapes = [I.ConvShape(2, 5, 100, 64, 5, 3, 3, (1, 1), (1, 1)),        # 16 rows per run: 14 + halo
              I.ConvShape(8, 128, 60, 128, 128, 3, 3, (1, 1), (1, 1)),    # eight rounds: 1024 planes x 5 runs
              I.ConvShape(1, 3, 37, 256, 3, 3, 3, (1, 1), (1, 1)),        # one row per round
              I.ConvShape(3, 4, 29, 44, 4, 3, 3, (1, 1), (1, 1)),         # 11 units per row: 55 lanes
              I.ConvShape(2, 3, 1, 28, 3, 3, 3, (1, 1), (1, 1)),
              I.ConvShape(2, 3, 2, 12, 3, 3, 3, (1, 1), (1, 1)),
              I.ConvShape(1, 2, 70, 132, 2, 3, 3, (1, 1), (1, 1))]        # 33 units per row: one row per round
    for i, s in enumerate(shapes):
        x, w = I.dwconv_inputs(s, 1300 + i, ints=True)
        buf, y = guarded((s.N, s.C, s.OH, s.OW))
        anr.dwconv(dev(x), dev(w), y, s.stride, s.pad)
        check_guard(buf)
        assert_parity(y, oracle.dwconv(x, w, s.stride, s.pad), exact=True, what="stream dwconv %s" % (s,))


def test_dwconv_taps_across_the_plane_edge_are_not_multiplied(anr):
    """Zero padding means a tap outside the plane contributes nothing, whatever lies next to it in
    memory: an infinite value in the last column of a row must not reach the first column of the rows
    below it (nor one in the first column the last column of the rows above)."""
    s = I.ConvShape(1, 2, 28, 28, 2, 3, 3, (1, 1), (1, 1))
    x, w = I.dwconv_inputs(s, 1310)
    x[0, 0, 10, 27] = np.inf
    x[0, 1, 20, 0] = np.inf
    y = torch.empty((s.N, s.C, s.OH, s.OW), device="cuda")
    anr.dwconv(dev(x), dev(w), y, s.stride, s.pad)
    got = y.cpu().numpy()
    with np.errstate(invalid="ignore", over="ignore"):
        ref = oracle.dwconv(x, w, s.stride, s.pad)
    finite = np.isfinite(ref)
    assert finite[0, 0, 11, 0] and finite[0, 0, 12, 0] and finite[0, 1, 19, 27]     # the oracle agrees these are untouched
    assert np.array_equal(np.isfinite(got), finite)
    assert rel_err(got[finite], ref[finite]) <= TOL


def test_gemm_random_shapes(anr):
    g = np.random.Generator(np.random.PCG64(960))
    for i in range(30):
        M, N, K = int(g.integers(1, 200)), int(g.integers(1, 200)), int(g.integers(1, 200))
        if g.random() < 0.5:            # the aligned kernels
            N, K = 4 * ((N + 3) // 4), 4 * ((K + 3) // 4)
        batch = int(g.choice([1, 1, 2, 5]))
        A, B = I.gemm_inputs(I.GemmShape(M, N, K, batch), 961 + i, ints=True)
        shape = (batch, M, N) if batch > 1 else (M, N)
        buf, C = guarded(shape)
        anr.gemm(dev(A), dev(B), C)
        check_guard(buf)
        assert_parity(C, oracle.gemm(A, B), exact=True, what="random gemm %d %s" % (i, (M, N, K, batch)))


def test_tbs_random_shapes(anr):
    g = np.random.Generator(np.random.PCG64(970))
    for i in range(20):
        s = I.TbgShape(int(g.integers(1, 3)), int(g.integers(1, 140)), int(g.integers(1, 4)),
                       int(g.choice([4, 8, 12, 16, 24, 40, 64, 72, 128])))
        q, k = I.tbg_inputs(s, 971 + i)
        q = (q * 0.35).astype(np.float32)
        buf, out = guarded((s.B, s.H, s.S, s.S))
        anr.tbs(dev(q), dev(k), out)
        check_guard(buf)
        assert_softmax_parity(out, oracle.tbs(q, k), what="random tbs %d %s" % (i, s))
        anr.tbg(dev(q), dev(k), out)
        assert_parity(out, oracle.tbg(q, k), what="random tbg %d %s" % (i, s))


# ------------------------------------------------------------------ NRM
NRM_TOL = 2e-6      # relative: fp32 partial sums of at most a few thousand squares each, then a tree


@pytest.mark.parametrize("shape", [(1, 1, 1), (1, 33, 7), (1, 256, 256), (3, 100, 37), (16, 512, 512),
                                   (1, 1000, 1000), (2, 2048, 1024), (1, 4096, 4096), (16, 256, 256), (64, 256, 256),
                                   (256, 250, 260)], ids=str)
def test_nrm(anr, shape):
    b, N, M = shape
    x = I.uniform(np.random.Generator(np.random.PCG64(700 + N)), (b, N, M))
    out = torch.full((b + 2,), CANARY, device="cuda")
    anr.nrm(dev(x) if b > 1 else dev(x[0]), out[1:1 + b])
    ref = oracle.nrm(x)
    got = out.cpu().numpy().astype(np.float64)
    assert got[0] == CANARY and got[-1] == CANARY
    assert float(np.max(np.abs(got[1:-1] - ref) / ref)) <= NRM_TOL
    assert_parity(out[1:1 + b], ref, what="nrm %s" % (shape,))


def test_nrm_strided_rows_and_exact_small_integers(anr):
    # a view into a wider matrix (row stride > M, unaligned start) takes the element-wise path;
    # small integers: the sum of squares is exact in fp32, so the result is the rounded root
    x = I.small_ints(np.random.Generator(np.random.PCG64(710)), (2, 50, 30))
    wide = torch.zeros((2, 50, 41), device="cuda")
    wide[:, :, 3:33] = dev(x)
    out = torch.empty((2,), device="cuda")
    anr.nrm(wide[:, :, 3:33], out)
    ref = oracle.nrm(x)
    assert np.array_equal(out.cpu().numpy(), ref.astype(np.float32))
    out2 = torch.empty((2,), device="cuda")
    anr.nrm(dev(x), out2)
    assert torch.equal(out, out2)


# ------------------------------------------------------------------ paper shape lists (Appendix C)
def appendix_c(golden_dir):
    import os
    ops = {}
    for line in open(os.path.join(golden_dir, "appendix_c_shapes.txt")):
        line = line.strip()
        if line and not line.startswith("#"):
            name, *vals = line.split()
            ops.setdefault(name, []).append(tuple(int(v) for v in vals))
    return ops


def test_appendix_c_shapes_batch1(anr, golden_dir):
    """Every GMM / C2D / DEP / ConvLayer / TBS shape of the paper's list at batch 1."""
    ops = appendix_c(golden_dir)
    for (n, m, k) in ops["GMM"]:
        A, B = I.gemm_inputs(I.GemmShape(m, n, k), 600)
        C = torch.empty((m, n), device="cuda")
        anr.gemm(dev(A), dev(B), C)
        assert_parity(C, oracle.gemm(A, B), what="GMM %s" % ((n, m, k),))
    for (h, w_, ci, co, ks, st, pd) in ops["C2D"]:
        s = I.ConvShape(1, ci, h, w_, co, ks, ks, (st, st), (pd, pd))
        x, w = I.conv_inputs(s, 601)
        y = torch.empty((1, co, s.OH, s.OW), device="cuda")
        anr.conv2d(dev(x), dev(w), y, s.stride, s.pad)
        assert_parity(y, oracle.conv2d(x, w, s.stride, s.pad), what="C2D " + str(s))
    for (h, w_, c, ks, st, pd) in ops["DEP"]:
        s = I.ConvShape(1, c, h, w_, c, ks, ks, (st, st), (pd, pd))
        x, w = I.dwconv_inputs(s, 602)
        y = torch.empty((1, c, s.OH, s.OW), device="cuda")
        anr.dwconv(dev(x), dev(w), y, s.stride, s.pad)
        assert_parity(y, oracle.dwconv(x, w, s.stride, s.pad), what="DEP " + str(s))
    for (h, w_, ci, co, ks, st, pd) in ops["ConvLayer"]:
        s = I.ConvShape(1, ci, h, w_, co, ks, ks, (st, st), (pd, pd))
        x, w = I.conv_inputs(s, 603)
        gamma, beta, mean, var = I.bn_inputs(co, 604)
        y = torch.empty((1, co, s.OH, s.OW), device="cuda")
        anr.conv_bn_relu(dev(x), dev(w), dev(gamma), dev(beta), dev(mean), dev(var), I.BN_EPS, y,
                         s.stride, s.pad)
        ref = oracle.conv_bn_relu(x, w, gamma, beta, mean, var, I.BN_EPS, s.stride, s.pad)
        assert_parity(y, ref, what="ConvLayer " + str(s))
    for (n, m) in ops["NRM"]:
        x = I.uniform(np.random.Generator(np.random.PCG64(607)), (n, m))
        out = torch.empty((1,), device="cuda")
        anr.nrm(dev(x), out)
        ref = oracle.nrm(x)
        assert abs(float(out[0]) - ref[0]) / ref[0] <= NRM_TOL, "NRM %s" % ((n, m),)
    for op in ("GRP", "DIL"):
        for fields in ops[op]:
            s = I.appendix_shape(op, fields, 1)
            if s is None:          # 3 input channels in 4 groups, as printed in the appendix
                continue
            x, w = I.conv_inputs(s, 606)
            y = torch.empty((1, s.K, s.OH, s.OW), device="cuda")
            anr.conv2d(dev(x), dev(w), y, s.stride, s.pad, dil=s.dil, groups=s.groups)
            ref = oracle.conv2d_general(x, w, s.stride, s.pad, s.dil, s.groups)
            assert_parity(y, ref, what=op + " " + str(s))
    for (S, H, D) in ops["TBS"]:
        s = I.TbgShape(1, S, H, D)
        q, k = I.tbg_inputs(s, 605)
        q = (q * 0.35).astype(np.float32)
        out = torch.empty((1, H, S, S), device="cuda")
        anr.tbg(dev(q), dev(k), out)
        assert_parity(out, oracle.tbg(q, k), what="TBG " + str(s))
        anr.tbs(dev(q), dev(k), out)
        assert_parity(out, oracle.tbs(q, k), what="TBS " + str(s))


def test_appendix_c_gmm_batch16(anr, golden_dir):
    """The GMM list at batch 16 (the paper's second batch size), full outputs against the oracle."""
    for (n, m, k) in appendix_c(golden_dir)["GMM"]:
        A, B = I.gemm_inputs(I.GemmShape(m, n, k, batch=16), 610)
        C = torch.empty((16, m, n), device="cuda")
        anr.gemm(dev(A), dev(B), C)
        assert_parity(C, oracle.gemm(A, B), what="GMM x16 %s" % ((n, m, k),))


def test_appendix_c_convolutions_batch16(anr, golden_dir):
    """C2D, ConvLayer, GRP and DIL lists at batch 16, full outputs against the oracle."""
    ops = appendix_c(golden_dir)
    for (h, w_, ci, co, ks, st, pd) in ops["C2D"]:
        s = I.ConvShape(16, ci, h, w_, co, ks, ks, (st, st), (pd, pd))
        x, w = I.conv_inputs(s, 611)
        y = torch.empty((16, co, s.OH, s.OW), device="cuda")
        anr.conv2d(dev(x), dev(w), y, s.stride, s.pad)
        assert_parity(y, oracle.conv2d(x, w, s.stride, s.pad), what="C2D x16 " + str(s))
    for (h, w_, ci, co, ks, st, pd) in ops["ConvLayer"]:
        s = I.ConvShape(16, ci, h, w_, co, ks, ks, (st, st), (pd, pd))
        x, w = I.conv_inputs(s, 613)
        gamma, beta, mean, var = I.bn_inputs(co, 614)
        y = torch.empty((16, co, s.OH, s.OW), device="cuda")
        anr.conv_bn_relu(dev(x), dev(w), dev(gamma), dev(beta), dev(mean), dev(var), I.BN_EPS, y,
                         s.stride, s.pad)
        ref = oracle.conv_bn_relu(x, w, gamma, beta, mean, var, I.BN_EPS, s.stride, s.pad)
        assert_parity(y, ref, what="ConvLayer x16 " + str(s))
    for op in ("GRP", "DIL"):
        for fields in ops[op]:
            s = I.appendix_shape(op, fields, 16)
            if s is None:          # 3 input channels in 4 groups, as printed in the appendix
                continue
            x, w = I.conv_inputs(s, 616)
            y = torch.empty((16, s.K, s.OH, s.OW), device="cuda")
            anr.conv2d(dev(x), dev(w), y, s.stride, s.pad, dil=s.dil, groups=s.groups)
            ref = oracle.conv2d_general(x, w, s.stride, s.pad, s.dil, s.groups)
            assert_parity(y, ref, what=op + " x16 " + str(s))


def test_appendix_c_dep_tbs_nrm_batch16(anr, golden_dir):
    """DEP, TBS and NRM lists at batch 16 (the 4096 x 4096 NRM at batch 2: 16 of them are a gigabyte
    of host input), full outputs against the oracle."""
    ops = appendix_c(golden_dir)
    for (h, w_, c, ks, st, pd) in ops["DEP"]:
        s = I.ConvShape(16, c, h, w_, c, ks, ks, (st, st), (pd, pd))
        x, w = I.dwconv_inputs(s, 612)
        y = torch.empty((16, c, s.OH, s.OW), device="cuda")
        anr.dwconv(dev(x), dev(w), y, s.stride, s.pad)
        assert_parity(y, oracle.dwconv(x, w, s.stride, s.pad), what="DEP x16 " + str(s))
    for (S, H, D) in ops["TBS"]:
        s = I.TbgShape(16, S, H, D)
        q, k = I.tbg_inputs(s, 615)
        q = (q * 0.35).astype(np.float32)
        out = torch.empty((16, H, S, S), device="cuda")
        anr.tbg(dev(q), dev(k), out)
        assert_parity(out, oracle.tbg(q, k), what="TBG x16 " + str(s))
        anr.tbs(dev(q), dev(k), out)
        assert_parity(out, oracle.tbs(q, k), what="TBS x16 " + str(s))
    for (n, m) in ops["NRM"]:
        batch = 16 if n * m <= 1024 * 1024 else 2
        x = I.uniform(np.random.Generator(np.random.PCG64(617)), (batch, n, m))
        out = torch.empty((batch,), device="cuda")
        anr.nrm(dev(x), out)
        ref = oracle.nrm(x)
        got = out.cpu().numpy().astype(np.float64)
        assert float(np.max(np.abs(got - ref) / ref)) <= NRM_TOL, "NRM x%d %s" % (batch, (n, m))


# ------------------------------------------------------------------ extents beyond 32-bit byte offsets
def test_conv2d_extent_beyond_32bit_offsets(anr):
    """An input of 2.15 GB (more than 2^29 floats): the kernels with 32-bit byte offsets step aside and
    the call still has to index correctly.  Checked against the oracle on crops at the image's corners
    and in its middle (the last rows are where a wrapped offset would show)."""
    H = W = 16400
    gen = torch.Generator(device="cuda")
    gen.manual_seed(1234)
    x = torch.rand((1, 2, H, W), generator=gen, device="cuda") * 2 - 1
    w = (torch.rand((1, 2, 3, 3), generator=gen, device="cuda") * 2 - 1) * 0.25
    y = torch.empty((1, 1, H, W), device="cuda")
    anr.conv2d(x, w, y, (1, 1), (1, 1))
    wh = w.cpu().numpy()
    c = 40
    # top-left and bottom-right corners: the crop's own padding is the image's on two sides
    ref = oracle.conv2d(x[:, :, :c, :c].cpu().numpy(), wh, (1, 1), (1, 1))
    assert_parity(y[:, :, :c - 1, :c - 1].contiguous(), ref[:, :, :c - 1, :c - 1], what="top-left crop")
    ref = oracle.conv2d(x[:, :, H - c:, W - c:].cpu().numpy(), wh, (1, 1), (1, 1))
    assert_parity(y[:, :, H - c + 1:, W - c + 1:].contiguous(), ref[:, :, 1:, 1:], what="bottom-right crop")
    # interior crops: no padding, outputs of the crop's interior
    for r0, c0 in [(H // 2, W // 2), (H - 3000, 17), (9000, W - 500)]:
        ref = oracle.conv2d(x[:, :, r0:r0 + c, c0:c0 + c].cpu().numpy(), wh, (1, 1), (0, 0))
        assert_parity(y[:, :, r0 + 1:r0 + c - 1, c0 + 1:c0 + c - 1].contiguous(), ref, what="crop at %d,%d" % (r0, c0))


def test_gemm_extent_beyond_32bit_offsets(anr):
    """A of 70000 x 8192 floats (2.3 GB): the pipelined kernel's 32-bit offsets do not reach, the
    fallback must; rows at the start, in the middle and at the very end against the oracle."""
    M, K, N = 70000, 8192, 8
    gen = torch.Generator(device="cuda")
    gen.manual_seed(4321)
    A = torch.rand((M, K), generator=gen, device="cuda") * 2 - 1
    Bm = torch.rand((K, N), generator=gen, device="cuda") * 2 - 1
    C = torch.empty((M, N), device="cuda")
    anr.gemm(A, Bm, C)
    Bh = Bm.cpu().numpy()
    for r0 in (0, M // 2 - 7, M - 33):
        rows = slice(r0, r0 + 33)
        assert_parity(C[rows].contiguous(), oracle.gemm(A[rows].cpu().numpy(), Bh), what="rows from %d" % r0)


def test_nrm_more_than_2_to_29_elements(anr):
    """One 24000 x 24000 matrix (2.3 GB): slice offsets are 64-bit."""
    gen = torch.Generator(device="cuda")
    gen.manual_seed(99)
    x = torch.rand((24000, 24000), generator=gen, device="cuda") * 2 - 1
    out = torch.empty((1,), device="cuda")
    anr.nrm(x, out)
    ref = oracle.nrm(x.cpu().numpy())
    assert abs(float(out[0]) - ref[0]) / ref[0] <= NRM_TOL


def test_tbg_tbs_tensors_beyond_32bit_offsets(anr):
    """q, k and the scores are 2.1 GB each (B 8, S 1024, H 64, D 1024; S 128 for the fused softmax):
    the (b, h) base offsets are 64-bit; sampled heads against the oracle."""
    gen = torch.Generator(device="cuda")
    gen.manual_seed(77)
    B_, S, H, D = 8, 1024, 64, 1024
    q = (torch.rand((B_, S, H, D), generator=gen, device="cuda") * 2 - 1) * 0.1
    k = torch.rand((B_, S, H, D), generator=gen, device="cuda") * 2 - 1
    out = torch.empty((B_, H, S, S), device="cuda")
    anr.tbg(q, k, out)
    for b, h in [(0, 0), (7, 63), (4, 31)]:
        ref = oracle.tbg(q[b:b + 1, :, h:h + 1].cpu().numpy(), k[b:b + 1, :, h:h + 1].cpu().numpy())
        assert_parity(out[b:b + 1, h:h + 1].contiguous(), ref, what="TBG head %d,%d" % (b, h))
    del out
    # the fused kernel on the same tensors, first 128 positions of every sequence (a strided view)
    qv, kv = q[:, :128], k[:, :128]
    outs = torch.empty((B_, H, 128, 128), device="cuda")
    anr.tbs(qv, kv, outs)
    for b, h in [(0, 0), (7, 63), (5, 17)]:
        ref = oracle.tbs(qv[b:b + 1, :, h:h + 1].cpu().numpy(), kv[b:b + 1, :, h:h + 1].cpu().numpy())
        assert_softmax_parity(outs[b:b + 1, h:h + 1].contiguous(), ref, what="TBS head %d,%d" % (b, h))


def test_dwconv_tensor_beyond_32bit_offsets(anr):
    """16 x 2048 planes of 128 x 128 (2.1 GB in, 2.1 GB out) through the row kernel, and of 14 x 14
    with 700000 channels through the small-plane kernel: sampled planes against the oracle."""
    gen = torch.Generator(device="cuda")
    gen.manual_seed(55)
    N, C, H = 16, 2048, 128
    x = torch.rand((N, C, H, H), generator=gen, device="cuda") * 2 - 1
    w = (torch.rand((C, 1, 3, 3), generator=gen, device="cuda") * 2 - 1) * 0.3
    y = torch.empty((N, C, H, H), device="cuda")
    anr.dwconv(x, w, y, (1, 1), (1, 1))
    for n, c in [(0, 0), (15, 2047), (9, 1000)]:
        ref = oracle.dwconv(x[n:n + 1, c:c + 1].cpu().numpy(), w[c:c + 1].cpu().numpy(), (1, 1), (1, 1))
        assert_parity(y[n:n + 1, c:c + 1].contiguous(), ref, what="DEP plane %d,%d" % (n, c))
    del x, y
    N, C, H = 4, 700000, 14
    x = torch.rand((N, C, H, H), generator=gen, device="cuda") * 2 - 1
    w = (torch.rand((C, 1, 3, 3), generator=gen, device="cuda") * 2 - 1) * 0.3
    y = torch.empty((N, C, 7, 7), device="cuda")
    anr.dwconv(x, w, y, (2, 2), (1, 1))
    for n, c in [(0, 0), (3, 699999), (2, 123457)]:
        ref = oracle.dwconv(x[n:n + 1, c:c + 1].cpu().numpy(), w[c:c + 1].cpu().numpy(), (2, 2), (1, 1))
        assert_parity(y[n:n + 1, c:c + 1].contiguous(), ref, what="DEP small plane %d,%d" % (n, c))


# ------------------------------------------------------------------ the step on several streams
def test_step_on_three_streams_in_one_graph_matches_the_one_stream_step(anr):
    """bench.py's overlapped step: the six launches forked onto three streams inside one HIP graph.
    Replayed three times with eager work and synchronisation in between; after every replay all six
    outputs must equal the one-stream step's bit for bit (same kernels, same inputs)."""
    import os
    import sys
    sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
    import bench
    host = {name: I.config_inputs(name) for name in I.CONFIG_NAMES}
    sets = [bench.OpSet(anr, I, torch, host) for _ in range(4)]
    sets[0].step()
    torch.cuda.synchronize()
    want = {n: sets[0].output(n).clone() for n in I.CONFIG_NAMES}
    for rep in range(3):
        for s in sets:
            for n in I.CONFIG_NAMES:
                s.output(n).fill_(CANARY)            # eager work between the replays
        torch.cuda.synchronize()
        ms = bench.overlapped_steps(torch, sets, 4, 4)
        torch.cuda.synchronize()
        assert ms > 0
        for s in sets:
            for n in I.CONFIG_NAMES:
                assert torch.equal(s.output(n), want[n]), "replay %d: %s differs" % (rep, n)
