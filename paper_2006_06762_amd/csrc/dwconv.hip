// Launch logic of the depthwise convolution (kernel in dwconv_kernel.h).
#include <algorithm>
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
    const dw::RowDivs dv{make_fastdiv(row_chunks), make_fastdiv(lpr), make_fastdiv(a.C)};
    // A partly filled last work-group still runs: its surplus waves see plane >= planes.
    return launch_kernel(dwconv3x3_kernel<ROWS>, dim3((unsigned)((waves + 3) / 4)), dim3(256), 0, stream,
                         a, lpr, ppw, planes, row_chunks, dv);
}

template <int ROWS>
hipError_t launch_rows_s2(const ConvArgs& a, hipStream_t stream)
{
    const int lpr = a.OW / 4;
    const int ppw = 64 / lpr;
    const int64_t planes = (int64_t)a.N * a.C;
    const int row_chunks = (a.OH + ROWS - 1) / ROWS;
    const int64_t waves = ((planes + ppw - 1) / ppw) * row_chunks;
    const dw::RowDivs dv{make_fastdiv(row_chunks), make_fastdiv(lpr), make_fastdiv(a.C)};
    return launch_kernel(dw::dwconv3x3s2_kernel<ROWS>, dim3((unsigned)((waves + 3) / 4)), dim3(256), 0, stream,
                         a, lpr, ppw, planes, row_chunks, dv);
}

// Stride 1 on dense tensors: see dwconv3x3_stream_kernel.  NI rounds of RPR rows hold an item's
// input rows: a whole plane if it fits, else equal runs of rows with their two halo rows.
template <int W4_T, int NI>
hipError_t launch_stream_as(const ConvArgs& a, hipStream_t stream)
{
    dw::StreamGeom g{};
    g.W4 = a.W / 4;
    g.RPR = 64 / g.W4;
    g.LPR = g.RPR * g.W4;
    const int rows_in = NI * g.RPR;
    int rc = a.H;
    if (rows_in < a.H) {
        rc = rows_in - 2;
        const int chunks = (a.H + rc - 1) / rc;
        rc = (a.H + chunks - 1) / chunks;
    }
    g.RC = rc;
    g.chunks = (a.H + rc - 1) / rc;
    g.hw = a.H * a.W;
    g.slice = ((rc + 2) * a.W + 8 + 3) / 4 * 4;
    g.items = a.N * a.C * g.chunks;
    g.d_chunks = make_fastdiv(g.chunks);
    g.d_w4 = make_fastdiv(g.W4);
    g.d_c = make_fastdiv(a.C);
    const size_t lds_bytes = sizeof(float) * (4 * (size_t)g.slice + 4);
    return launch_kernel(dw::dwconv3x3_stream_kernel<W4_T, NI>, dim3((unsigned)((g.items + 3) / 4)), dim3(256),
                         lds_bytes, stream, a, g);
}

template <int NI>
hipError_t launch_stream(const ConvArgs& a, hipStream_t stream)
{
    switch (a.W) {
        case 28: return launch_stream_as<7, NI>(a, stream);
        case 56: return launch_stream_as<14, NI>(a, stream);
        case 112: return launch_stream_as<28, NI>(a, stream);
        default: return launch_stream_as<0, NI>(a, stream);
    }
}

// Small planes of dense tensors: see dwconv_small_planes_kernel.
hipError_t launch_small_planes(const ConvArgs& a, hipStream_t stream, bool* taken)
{
    *taken = false;
    const int64_t hw = (int64_t)a.H * a.W, ohw = (int64_t)a.OH * a.OW;
    const bool dense = a.xs[2] == a.W && a.xs[1] == hw && a.xs[0] == a.C * hw && a.ys[2] == a.OW && a.ys[1] == ohw &&
                       a.ys[0] == a.C * ohw && is_aligned16(a.x) && is_aligned16(a.y);
    // at most about eight outputs per thread, ranges that start 16-byte aligned (G a multiple of
    // `unit`), and at least three work-groups per CU where the tensor has that many planes
    const int64_t planes = (int64_t)a.N * a.C;
    if (!dense || ohw > 2048 || a.C >= (1 << 30)) return hipSuccess;
    const int unit = ((hw | ohw) % 4 == 0) ? 1 : ((hw | ohw) % 2 == 0) ? 2 : 4;
    const int g_max = (int)std::min<int64_t>(256, 2048 / ohw) / unit * unit;
    if (g_max == 0) return hipSuccess;
    int G = (int)std::min<int64_t>(g_max, planes / 768 / unit * unit);
    if (G < unit) G = unit;
    const int64_t rs = (int64_t)a.R * a.S;
    const int64_t lds_floats = ((G * hw + 3) & ~(int64_t)3) + ((G * ohw + 3) & ~(int64_t)3) + G * rs;
    if (lds_floats * 4 > 48 * 1024 || planes >= ((int64_t)1 << 31) || (planes + G - 1) / G >= ((int64_t)1 << 31))
        return hipSuccess;
    dw::SmallPlanes g;
    g.G = G;
    g.hw = (int)hw;
    g.ohw = (int)ohw;
    g.rs = (int)rs;
    g.planes = planes;
    g.d_ohw = make_fastdiv((int)ohw);
    g.d_ow = make_fastdiv(a.OW);
    g.d_c = make_fastdiv(a.C);
    *taken = true;
    const dim3 grid((unsigned)((planes + G - 1) / G));
    if (a.R == 3 && a.S == 3)
        return launch_kernel(dw::dwconv_small_planes_kernel<3, 3>, grid, dim3(256), (size_t)lds_floats * 4, stream, a, g);
    if (a.R == 5 && a.S == 5)
        return launch_kernel(dw::dwconv_small_planes_kernel<5, 5>, grid, dim3(256), (size_t)lds_floats * 4, stream, a, g);
    return launch_kernel(dw::dwconv_small_planes_kernel<0, 0>, grid, dim3(256), (size_t)lds_floats * 4, stream, a, g);
}

}  // namespace

hipError_t launch_dwconv3x3(const ConvArgs& a, hipStream_t stream, bool* taken)
{
    const bool common = a.R == 3 && a.S == 3 && a.dil_h == 1 && a.dil_w == 1 && a.pad_h == 1 && a.pad_w == 1 &&
                        is_aligned16(a.x) && is_aligned16(a.y) && (a.xs[0] % 4 == 0) && (a.xs[1] % 4 == 0) &&
                        (a.xs[2] % 4 == 0) && (a.ys[0] % 4 == 0) && (a.ys[1] % 4 == 0) && (a.ys[2] % 4 == 0) &&
                        // wave and plane indices are divided as 31-bit numbers
                        (int64_t)a.N * a.C * a.OH < ((int64_t)1 << 31);
    const bool s2 = common && a.stride_h == 2 && a.stride_w == 2 && (a.W % 8 == 0) && a.W <= 512;
    if (s2) {
        *taken = true;
        return launch_rows_s2<4>(a, stream);
    }
    const bool ok = common && a.stride_h == 1 && a.stride_w == 1 && (a.W % 4 == 0) && a.W <= 256;
    *taken = ok;
    if (!ok) return hipSuccess;
    // dense x and y (planes and rows back to back): the streaming kernel
    const int64_t hw = (int64_t)a.H * a.W;
    const bool dense = a.xs[2] == a.W && a.xs[1] == hw && a.xs[0] == a.C * hw && a.ys[2] == a.W && a.ys[1] == hw &&
                       a.ys[0] == a.C * hw && hw < ((int64_t)1 << 30) && a.H >= 3 &&
                       (int64_t)a.N * a.C * a.H < ((int64_t)1 << 30);
    if (dense) {
        // Planes taller than four rounds of rows are cut into runs with two halo rows each: eight
        // rounds per run re-read less (112x112x32 at batch 16: 9.9 against 11.8 us) as long as that
        // still makes some 16 waves per CU (at batch 1: 4.0 against 3.1 us)
        const int rpr = 64 / (a.W / 4);
        const int64_t items8 = (int64_t)a.N * a.C * ((a.H + 8 * rpr - 3) / (8 * rpr - 2));
        if (a.H > 4 * rpr && items8 >= 4096) return launch_stream<8>(a, stream);
        return launch_stream<4>(a, stream);
    }
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
    err = launch_small_planes(a, stream, &taken);
    if (taken || err != hipSuccess) return err;
    return launch_dwconv_direct(a, stream);
}

}  // namespace anr
