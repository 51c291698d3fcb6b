"""The entry point that allocates nothing (anr_conv2d_noalloc): through the C ABI, against
anr_conv2d with a caller's workspace (same kernels, so bit for bit) and against the oracle,
on two calls in a row, the second with a smaller input, so that whatever the first call left
in the library's static scratch array is there when the second one runs."""
import ctypes

import numpy as np
import pytest

import oracle
from paper_2006_06762_amd import inputs as I

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

TOL = 1e-4


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def run_pair(B, s, seed):
    """(output of anr_conv2d_noalloc, output of anr_conv2d with its own workspace, oracle)."""
    lib = B.raw()
    x, w = I.conv_inputs(s, seed)
    xd, wd = dev(x), dev(w)
    d = B.conv_desc((s.N, s.C, s.H, s.W), s.K, s.R, s.S, s.stride, s.pad)
    need = B.workspace_size(B.ANR_OP_CONV2D, d)
    assert 0 < need <= B.STATIC_SCRATCH_BYTES, "the case must split its reduction through a workspace"
    y_ref = torch.empty((s.N, s.K, s.OH, s.OW), device="cuda")
    y_new = torch.full_like(y_ref, float("nan"))
    ws = torch.full((need,), 0x7f, dtype=torch.uint8, device="cuda")
    stream = B._stream()
    st = lib.anr_conv2d(ctypes.byref(d), B._ptr(xd), B._ptr(wd), B._ptr(y_ref), ctypes.c_void_p(ws.data_ptr()), need,
                        stream)
    assert st == B.ANR_OK, B.status_string(st)
    st = lib.anr_conv2d_noalloc(ctypes.byref(d), B._ptr(xd), B._ptr(wd), B._ptr(y_new), stream)
    assert st == B.ANR_OK, B.status_string(st)
    torch.cuda.synchronize()
    return y_new.cpu().numpy(), y_ref.cpu().numpy(), oracle.conv2d(x, w, s.stride, s.pad)


def test_noalloc_conv_matches_the_workspace_entry_point_twice_in_a_row():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2006_06762_amd import binding as B
    big = I.ConvShape(1, 512, 7, 7, 512, 3, 3, (1, 1), (1, 1))       # 4 MiB of partial tiles
    small = I.ConvShape(1, 96, 9, 11, 40, 3, 3, (1, 1), (1, 1))      # fewer, smaller partial tiles
    for s, seed in ((big, 1210), (small, 1211)):
        print("noalloc case", s, flush=True)
        got, ref, orc = run_pair(B, s, seed)
        assert not np.isnan(got).any()
        assert np.array_equal(got, ref), "differs from anr_conv2d"
        err = float(np.max(np.abs(got.astype(np.float64) - orc) / np.maximum(1.0, np.abs(orc))))
        assert err <= TOL, "rel err %.3e" % err


def test_noalloc_conv_without_a_split_and_beyond_the_limit():
    from paper_2006_06762_amd import binding as B
    lib = B.raw()
    # a plan that needs no workspace runs as anr_conv2d does
    s = I.ConvShape(2, 16, 28, 28, 32, 3, 3, (1, 1), (1, 1))
    x, w = I.conv_inputs(s, 1212, ints=True)
    y = torch.empty((s.N, s.K, s.OH, s.OW), device="cuda")
    B.conv2d_noalloc(dev(x), dev(w), y, s.stride, s.pad)
    assert np.array_equal(y.cpu().numpy().astype(np.float64), oracle.conv2d(x, w, s.stride, s.pad))
    # a plan beyond the static array is refused before anything is launched
    d = None
    for n in range(2, 65):
        cand = B.conv_desc((n, 512, 14, 14), 2048, 3, 3, (1, 1), (1, 1))
        if B.workspace_size(B.ANR_OP_CONV2D, cand) > B.STATIC_SCRATCH_BYTES:
            d = cand
            break
    assert d is not None, "no shape found whose plan exceeds the static scratch array"
    dummy = ctypes.c_void_p(0x1000)
    assert lib.anr_conv2d_noalloc(ctypes.byref(d), dummy, dummy, dummy, None) == B.ANR_ERR_WORKSPACE
