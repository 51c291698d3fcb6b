// DEP (depthwise convolution, Sec. 7.1 / Appendix C of arXiv 2006.06762), the
// bandwidth-bound operator: 2.25 flop per byte, so the kernel is built around
// moving each input and output element through HBM exactly once.
//
// Stride 1: 3x3, pad 1, width a multiple of 4.  A lane owns a strip of four
// adjacent columns of one plane and walks down ROWS output rows; W/4 lanes
// cover the width and floor(64 / (W/4)) planes sit side by side in one wave.
// Each input row is one 16-byte load per lane; the two columns a strip needs
// from its neighbours come from the adjacent lanes by lane shuffle, so nothing
// is read twice and no LDS memory is used.  All ROWS+2 row loads of a lane are
// issued before the first use to keep many bytes in flight.
#pragma once
#include "anr_device.h"
#include "conv_internal.h"

namespace anr {
namespace dw {

template <int ROWS, int WPB = 4>
__global__ __launch_bounds__(64 * WPB) void dwconv3x3_kernel(const ConvArgs p, int lanes_per_row,
                                                        int planes_per_wave, int64_t planes,
                                                        int row_chunks)
{
    const int lane = threadIdx.x & 63;
    const int64_t wave = (int64_t)blockIdx.x * WPB + (threadIdx.x >> 6);
    const int64_t pgroup = wave / row_chunks;
    const int oh0 = (int)(wave % row_chunks) * ROWS;

    const int pl = lane / lanes_per_row, ch = lane % lanes_per_row;
    const int64_t plane = pgroup * planes_per_wave + pl;
    const bool active = (pl < planes_per_wave) && (plane < planes);
    const int n = active ? (int)(plane / p.C) : 0;
    const int c = active ? (int)(plane % p.C) : 0;
    const float* __restrict__ xp = p.x + n * p.xs[0] + c * p.xs[1] + 4 * ch;
    float* __restrict__ yp = p.y + n * p.ys[0] + c * p.ys[1] + 4 * ch;
    const bool first = ch == 0, last = ch == lanes_per_row - 1;

    float wt[9];
#pragma unroll
    for (int i = 0; i < 9; ++i) wt[i] = active ? p.w[(int64_t)c * 9 + i] : 0.f;

    // input rows oh0-1 .. oh0+ROWS, zero outside the image
    f32x4 v[ROWS + 2];
#pragma unroll
    for (int i = 0; i < ROWS + 2; ++i) {
        const int ih = oh0 - 1 + i;
        v[i] = (active && ih >= 0 && ih < p.H) ? ldg4(xp + ih * p.xs[2]) : zero4();
    }

    float lft[ROWS + 2], rgt[ROWS + 2];
#pragma unroll
    for (int i = 0; i < ROWS + 2; ++i) {
        const float l = __shfl_up(v[i][3], 1);
        const float r = __shfl_down(v[i][0], 1);
        lft[i] = first ? 0.f : l;
        rgt[i] = last ? 0.f : r;
    }

#pragma unroll
    for (int o = 0; o < ROWS; ++o) {
        const int oh = oh0 + o;
        f32x4 acc = zero4();
#pragma unroll
        for (int r = 0; r < 3; ++r) {
            const f32x4 m = v[o + r];
            const float w0 = wt[3 * r], w1 = wt[3 * r + 1], w2 = wt[3 * r + 2];
            acc[0] += w0 * lft[o + r] + w1 * m[0] + w2 * m[1];
            acc[1] += w0 * m[0] + w1 * m[1] + w2 * m[2];
            acc[2] += w0 * m[1] + w1 * m[2] + w2 * m[3];
            acc[3] += w0 * m[2] + w1 * m[3] + w2 * rgt[o + r];
        }
        if (active && oh < p.OH) stg4(yp + oh * p.ys[2], acc);
    }
}

// The stride-2 form (3x3, pad 1, width a multiple of 8): a lane owns four adjacent OUTPUT
// columns, i.e. input columns 8*ch - 1 .. 8*ch + 7: two 16-byte loads per input row plus the
// last column of the lane to its left.  ROWS output rows need 2*ROWS + 1 input rows.
template <int ROWS, int WPB = 4>
__global__ __launch_bounds__(64 * WPB) void dwconv3x3s2_kernel(const ConvArgs p, int lanes_per_row,
                                                          int planes_per_wave, int64_t planes,
                                                          int row_chunks)
{
    constexpr int IN = 2 * ROWS + 1;
    const int lane = threadIdx.x & 63;
    const int64_t wave = (int64_t)blockIdx.x * WPB + (threadIdx.x >> 6);
    const int64_t pgroup = wave / row_chunks;
    const int oh0 = (int)(wave % row_chunks) * ROWS;

    const int pl = lane / lanes_per_row, ch = lane % lanes_per_row;
    const int64_t plane = pgroup * planes_per_wave + pl;
    const bool active = (pl < planes_per_wave) && (plane < planes);
    const int n = active ? (int)(plane / p.C) : 0;
    const int c = active ? (int)(plane % p.C) : 0;
    const float* __restrict__ xp = p.x + n * p.xs[0] + c * p.xs[1] + 8 * ch;
    float* __restrict__ yp = p.y + n * p.ys[0] + c * p.ys[1] + 4 * ch;
    const bool first = ch == 0;

    float wt[9];
#pragma unroll
    for (int i = 0; i < 9; ++i) wt[i] = active ? p.w[(int64_t)c * 9 + i] : 0.f;

    // input rows 2*oh0 - 1 .. 2*oh0 + 2*ROWS - 1, zero outside the image
    f32x4 va[IN], vb[IN];
#pragma unroll
    for (int i = 0; i < IN; ++i) {
        const int ih = 2 * oh0 - 1 + i;
        const bool in = active && ih >= 0 && ih < p.H;
        va[i] = in ? ldg4(xp + ih * p.xs[2]) : zero4();
        vb[i] = in ? ldg4(xp + ih * p.xs[2] + 4) : zero4();
    }
    float lft[IN];
#pragma unroll
    for (int i = 0; i < IN; ++i) {
        const float l = __shfl_up(vb[i][3], 1);
        lft[i] = first ? 0.f : l;
    }

#pragma unroll
    for (int o = 0; o < ROWS; ++o) {
        const int oh = oh0 + o;
        f32x4 acc = zero4();
#pragma unroll
        for (int r = 0; r < 3; ++r) {
            const f32x4 a = va[2 * o + r], b = vb[2 * o + r];
            const float w0 = wt[3 * r], w1 = wt[3 * r + 1], w2 = wt[3 * r + 2];
            acc[0] += w0 * lft[2 * o + r] + w1 * a[0] + w2 * a[1];
            acc[1] += w0 * a[1] + w1 * a[2] + w2 * a[3];
            acc[2] += w0 * a[3] + w1 * b[0] + w2 * b[1];
            acc[3] += w0 * b[1] + w1 * b[2] + w2 * b[3];
        }
        if (active && oh < p.OH) stg4(yp + oh * p.ys[2], acc);
    }
}

}  // namespace dw
}  // namespace anr
