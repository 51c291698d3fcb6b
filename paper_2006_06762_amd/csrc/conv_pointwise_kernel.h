// Pointwise (1 x 1, stride 1) convolutions with few channels, e.g. the 56x56 64 -> 64 layer of the
// C2D / GRP / DIL shape lists (Appendix C of arXiv 2006.06762): y[n,k,p] = sum_c w[k,c] x[n,c,p]
// over the pixels p of an image.  With C and K around 64 this is 16 FLOP per byte, below the
// machine's ridge (19.7): like the TBS batch matmul it is bound by moving x and y through HBM
// once, and it is built the same way, as a stream: 9.4 us for the 25.7 MB of that layer at batch 16
// against 11.7 us in the general kernel (per work-group: data in LDS 3.8 us after the start, 32
// MFMAs per wave with three work-groups on a CU 2.2 us, sixteen stores 1 us).
//
// A work-group owns 64 pixels x 64 output channels of one image (four waves, a 32 x 32 block each)
// and the whole reduction (C <= 128).  The block is computed transposed -- output channels are the
// MFMA rows, pixels the columns -- so that in the accumulator layout a register holds, across the
// 32 lanes of a half-wave, 32 consecutive pixels of one channel: results leave straight from the
// registers in whole 128-byte lines, non-temporally (y is not read again), with no transposition.
// x comes in with non-temporal 16-byte loads, four rows of the tile per instruction (a row is 64
// consecutive pixels of a channel, 256 bytes), and sits in LDS unpadded: the B operand of a k-step
// is 32 consecutive floats of such a row, free of bank conflicts.  (Direct-to-LDS loads measured the
// same, 9.5 against 9.4 us; tiles of 128 pixels x 32 channels, for 512-byte runs: 10.7 us.)  The k-steps pair channel s with channel s + C/2
// (the two halves of the wave), so the A operand of a lane is a contiguous half row of w, which it
// reads from LDS once and keeps in registers for the whole tile.
#pragma once
#include "anr_device.h"
#include "conv_internal.h"

namespace anr {
namespace pw {

struct Geom {
    int hw;              // pixels per image
    int tiles_p;         // ceil(hw / 64)
    int tiles_k;         // ceil(K / 64)
    int xcd_chunk;       // work-groups per XCD when their count is a multiple of 8, else 0
    int cg;              // input channels per group (C for an ungrouped layer; a multiple of 4)
    FastDiv d_tiles_k, d_tiles_p, d_kg;   // d_kg: divisor K / groups
};

template <int C_T>
__global__ __launch_bounds__(256) void conv1x1_stream_kernel(const ConvArgs p, const Geom g)
{
    constexpr int HC = C_T / 2;                       // k-steps: channel s with channel s + HC
    __shared__ __attribute__((aligned(16))) float xs[C_T * 64];
    __shared__ __attribute__((aligned(16))) float ws[64 * (C_T + 4)];
    __shared__ float bn[4][64];                       // per wave: scale, then shift of its 32 channels

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r32 = lane & 31, h = lane >> 5;
    const int wk = wave >> 1, wp = wave & 1;          // channel block, pixel block of the wave
    // work-group id -> (image, pixel tile, channel tile); ids are dealt round-robin over the 8 XCDs,
    // so every XCD gets a contiguous range: the channel tiles of a pixel tile share its x in one L2
    int t = blockIdx.x;
    if (g.xcd_chunk > 0) t = (t & 7) * g.xcd_chunk + (t >> 3);
    const int q1 = g.d_tiles_k.div(t), tk = t - q1 * g.tiles_k;
    const int n = g.d_tiles_p.div(q1), tp = q1 - n * g.tiles_p;
    const int p0 = tp * 64, k0 = tk * 64;

    // ---- ConvLayer: the batch-norm constants of the wave's 32 channels, one channel per lane, once
    if (p.gamma && lane < 32) {
        int k = k0 + 32 * wk + lane;
        k = k < p.K ? k : p.K - 1;
        float scale, shift;
        if (p.scale_shift) {         // folded ahead of time (pre-packed call)
            scale = p.scale_shift[k];
            shift = p.scale_shift[p.K + k];
        } else {
            scale = p.gamma[k] / sqrtf(p.var[k] + p.eps);
            shift = p.beta[k] - p.mean[k] * scale;
        }
        bn[wave][lane] = scale;
        bn[wave][32 + lane] = shift;
    }
    // ---- x tile: channel c, pixels p0 .. p0+63; instruction i of a wave brings rows 4 * (4 i + wave) ..+3
    const float* __restrict__ xb = p.x + n * p.xs[0] + p0;
    f32x4 rx[C_T / 16];
    const int xrow = lane >> 4, xunit = lane & 15;
    {
        int pu = p0 + 4 * xunit < g.hw ? 4 * xunit : 0;     // hw is a multiple of 4: a unit is all in or all out
#pragma unroll
        for (int i = 0; i < C_T / 16; ++i) {
            const int c = 4 * (4 * i + wave) + xrow;
            rx[i] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(xb + (int64_t)c * g.hw + pu));
        }
    }
    // ---- w tile: rows k0 .. k0+63 of w (rows past K repeat the last one) as a 64 x C_T matrix: the cg
    //      weights of a row at the columns of its own group, zero elsewhere (a grouped layer is a
    //      block-diagonal matrix; the products with the zeros cost matrix time that this
    //      traffic-bound kernel has to spare: 56x56, 64 -> 64 in 4 groups at batch 16 12.0 -> 9.4 us).  Fetched
    //      with coalesced 16-byte loads (loading a lane's half row straight from global memory makes a
    //      request touch 32 lines for 16 bytes each: 11.6 us for the 56x56x64 layer, no better than the
    //      general kernel) and kept in LDS at a row stride of C_T + 4 floats, from where a lane takes
    //      its half row -- the A operand of all its k-steps -- into registers
    constexpr int WLD = C_T + 4;
    {
        constexpr int UPR = C_T / 4;                   // 16-byte units per row
#pragma unroll
        for (int i = 0; i < (64 * UPR) / 256; ++i) {
            const int u = tid + 256 * i;
            const int row = u / UPR, col = u - row * UPR;
            int k = k0 + row;
            k = k < p.K ? k : p.K - 1;
            const int lc = 4 * col - g.d_kg.div(k) * g.cg;          // the unit's first channel inside the row's group
            const bool in = (unsigned)lc < (unsigned)g.cg;
            const f32x4 v = ldg4(p.w + (int64_t)k * g.cg + (in ? lc : 0));
            *reinterpret_cast<f32x4*>(ws + row * WLD + 4 * col) = in ? v : zero4();
        }
    }
#pragma unroll
    for (int i = 0; i < C_T / 16; ++i)
        *reinterpret_cast<f32x4*>(xs + 256 * (4 * i + wave) + 64 * xrow + 4 * xunit) = rx[i];
    __syncthreads();
    f32x4 av[HC / 4];
#pragma unroll
    for (int u = 0; u < HC / 4; ++u) av[u] = *reinterpret_cast<const f32x4*>(ws + (32 * wk + r32) * WLD + h * HC + 4 * u);

    f32x16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    const float* bp = xs + (h * HC) * 64 + 32 * wp + r32;
#pragma unroll
    for (int u = 0; u < HC / 4; ++u)
#pragma unroll
        for (int e = 0; e < 4; ++e) acc = mfma32(av[u][e], bp[(4 * u + e) * 64], acc);

    // ---- register r of lane (h, r32): channel k0 + 32 wk + 8 (r/4) + 4 h + r%4, pixel p0 + 32 wp + r32.
    //      Buffer stores whose descriptor ends with the last channel row of y that exists, so that rows
    //      past K fall outside it and are dropped by the hardware; pixels past the image are masked
    //      once for all sixteen stores (inside the descriptor they would land in the next row).
    const int pix = p0 + 32 * wp + r32;
    const int rows_left = p.K - (k0 + 32 * wk);                   // <= 0: all of the wave's channels are past K
    const int rows = rows_left < 0 ? 0 : (rows_left < 32 ? rows_left : 32);
    const __amdgpu_buffer_rsrc_t yrsrc = __builtin_amdgcn_make_buffer_rsrc(
        p.y + n * p.ys[0] + (int64_t)(k0 + 32 * wk) * g.hw + p0, 0, rows > 0 ? 4 * (rows * g.hw - p0) : 0, 0x00020000);
    const int voff = 4 * ((4 * h) * g.hw + 32 * wp + r32);
    if (pix < g.hw) {
        // two separate store loops: with the fused epilogue's selects inside one loop the compiler
        // made every store wait for the one before it
        if (p.gamma) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int i = 8 * (r / 4) + 4 * h + (r % 4);
                const float v = fmaxf(fmaf(acc[r], bn[wave][i], bn[wave][32 + i]), 0.f);
                __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v), yrsrc, voff + 4 * ((8 * (r / 4) + (r % 4)) * g.hw), 0,
                                                      kBufferNonTemporal);
            }
        } else {
#pragma unroll
            for (int r = 0; r < 16; ++r)
                __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(acc[r]), yrsrc,
                                                      voff + 4 * ((8 * (r / 4) + (r % 4)) * g.hw), 0, kBufferNonTemporal);
        }
    }
}

}  // namespace pw
}  // namespace anr
