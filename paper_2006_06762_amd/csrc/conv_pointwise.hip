// Selection and launch of the streaming pointwise convolution (kernel in conv_pointwise_kernel.h).
#include "conv_pointwise_kernel.h"

namespace anr {
namespace {

// What the kernel takes: 1 x 1, stride 1, no padding (a dilation means nothing to one tap); C one
// of 32, 64, 96, 128, in groups of a multiple of 4 channels;
// images whose planes are dense and follow each other (x and y are then [C or K][H*W] matrices per
// image) with H*W a multiple of 4; 16-byte aligned pointers.  It is chosen where the layer is
// bound by traffic rather than by the matrix pipes: K <= 128 as well.
bool takes(const ConvArgs& a)
{
    if (a.route == 1) return false;
    const int64_t hw = (int64_t)a.H * a.W;
    const bool geom = a.R == 1 && a.S == 1 && a.stride_h == 1 && a.stride_w == 1 && a.pad_h == 0 && a.pad_w == 0 &&
                      a.groups >= 1 && (a.C % a.groups == 0) && (a.K % a.groups == 0) && ((a.C / a.groups) % 4 == 0);
    const bool chans = (a.C == 32 || a.C == 64 || a.C == 96 || a.C == 128) && a.K <= 128;
    const bool dense = a.xs[2] == a.W && a.xs[1] == hw && a.ys[2] == a.W && a.ys[1] == hw && (a.xs[0] % 4 == 0) &&
                       (a.ys[0] % 4 == 0) && (hw % 4 == 0) && is_aligned16(a.x) && is_aligned16(a.y) && is_aligned16(a.w);
    const int64_t tiles = (int64_t)a.N * ((hw + 63) / 64) * ((a.K + 63) / 64);
    return geom && chans && dense && hw < ((int64_t)1 << 30) && tiles < ((int64_t)1 << 31) && tiles >= 256;
}

template <int C_T>
hipError_t launch_as(const ConvArgs& a, hipStream_t stream)
{
    pw::Geom g{};
    g.hw = a.H * a.W;
    g.tiles_p = (g.hw + 63) / 64;
    g.tiles_k = (a.K + 63) / 64;
    const int64_t tiles = (int64_t)a.N * g.tiles_p * g.tiles_k;
    g.xcd_chunk = tiles % 8 == 0 ? (int)(tiles / 8) : 0;
    g.d_tiles_k = make_fastdiv(g.tiles_k);
    g.d_tiles_p = make_fastdiv(g.tiles_p);
    g.cg = a.C / a.groups;
    g.d_kg = make_fastdiv(a.K / a.groups);
    return launch_kernel(pw::conv1x1_stream_kernel<C_T>, dim3((unsigned)tiles), dim3(256), 0, stream, a, g);
}

}  // namespace

bool describe_conv2d_pointwise(const ConvArgs& a, ConvRoute* r)
{
    if (!takes(a)) return false;
    const int64_t hw = (int64_t)a.H * a.W;
    *r = ConvRoute{6, 64, 64, 1, 1, (int)((int64_t)a.N * ((hw + 63) / 64) * ((a.K + 63) / 64)), 0};
    return true;
}

hipError_t launch_conv2d_pointwise(const ConvArgs& a, hipStream_t stream, bool* taken)
{
    *taken = takes(a);
    if (!*taken) return hipSuccess;
    switch (a.C) {
        case 32: return launch_as<32>(a, stream);
        case 64: return launch_as<64>(a, stream);
        case 96: return launch_as<96>(a, stream);
        default: return launch_as<128>(a, stream);
    }
}

}  // namespace anr
