// Launch logic of the depthwise convolution (kernel in dwconv_kernel.h).
#include "dwconv_kernel.h"

namespace anr {
namespace {

using dw::dwconv3x3_kernel;

template <int ROWS>
hipError_t launch_rows(const ConvArgs& a, hipStream_t stream)
{
    const int lpr = a.W / 4;
    const int ppw = 64 / lpr;
    const int64_t planes = (int64_t)a.N * a.C;
    const int row_chunks = (a.OH + ROWS - 1) / ROWS;
    const int64_t waves = ((planes + ppw - 1) / ppw) * row_chunks;
    // A partly filled last work-group still runs: its surplus waves see plane >= planes.
    return launch_kernel(dwconv3x3_kernel<ROWS>, dim3((unsigned)((waves + 3) / 4)), dim3(256), 0, stream,
                         a, lpr, ppw, planes, row_chunks);
}

template <int ROWS>
hipError_t launch_rows_s2(const ConvArgs& a, hipStream_t stream)
{
    const int lpr = a.OW / 4;
    const int ppw = 64 / lpr;
    const int64_t planes = (int64_t)a.N * a.C;
    const int row_chunks = (a.OH + ROWS - 1) / ROWS;
    const int64_t waves = ((planes + ppw - 1) / ppw) * row_chunks;
    return launch_kernel(dw::dwconv3x3s2_kernel<ROWS>, dim3((unsigned)((waves + 3) / 4)), dim3(256), 0, stream,
                         a, lpr, ppw, planes, row_chunks);
}

}  // namespace

hipError_t launch_dwconv3x3(const ConvArgs& a, hipStream_t stream, bool* taken)
{
    const bool common = a.R == 3 && a.S == 3 && a.dil_h == 1 && a.dil_w == 1 && a.pad_h == 1 && a.pad_w == 1 &&
                        is_aligned16(a.x) && is_aligned16(a.y) && (a.xs[0] % 4 == 0) && (a.xs[1] % 4 == 0) &&
                        (a.xs[2] % 4 == 0) && (a.ys[0] % 4 == 0) && (a.ys[1] % 4 == 0) && (a.ys[2] % 4 == 0);
    const bool s2 = common && a.stride_h == 2 && a.stride_w == 2 && (a.W % 8 == 0) && a.W <= 512;
    if (s2) {
        *taken = true;
        return launch_rows_s2<4>(a, stream);
    }
    const bool ok = common && a.stride_h == 1 && a.stride_w == 1 && (a.W % 4 == 0) && a.W <= 256;
    *taken = ok;
    if (!ok) return hipSuccess;
    // 14 rows per wave re-read fewer halo rows (2 in 16 instead of 2 in 9) but make half as many
    // waves; below about four waves per SIMD the shorter strips win (measured on 16x256x28x28:
    // 8.4 us against 9.5 us)
    const int ppw = 64 / (a.W / 4);
    const int64_t waves14 = (((int64_t)a.N * a.C + ppw - 1) / ppw) * ((a.OH + 13) / 14);
    if (waves14 >= 4096) return launch_rows<14>(a, stream);
    return launch_rows<7>(a, stream);
}

hipError_t launch_dwconv(const ConvArgs& a, hipStream_t stream)
{
    bool taken = false;
    hipError_t err = launch_dwconv3x3(a, stream, &taken);
    if (taken || err != hipSuccess) return err;
    return launch_dwconv_direct(a, stream);
}

}  // namespace anr
