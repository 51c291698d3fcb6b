// The batch matmul of the TBS subgraph (Sec. 7.2 of arXiv 2006.06762) with its two
// transposes folded into addressing: out[b,h,i,j] = sum_d q[b,i,h,d] * k[b,j,h,d].
//
// 16 FLOP per byte of compulsory traffic puts this operator below the machine's ridge
// (19.7 FLOP/B): it is bound by moving q, k and out through HBM once, not by the MFMA
// units.  The kernel is therefore built for memory parallelism rather than register
// blocking: one work-group per 64 x 64 tile of one (b,h) score matrix (768 work-groups
// for the benchmark shape, three resident per CU so that the load, MFMA and store phases
// of different tiles overlap), every thread issues all its global loads at once, the
// whole reduction length (chunks of 64) sits in LDS at a time, and each of the four waves
// multiplies one 32 x 32 block with v_mfma_f32_32x32x2_f32, reading both operands from
// LDS with 16-byte reads (rows of q and k are both contiguous in d, so A and B use the
// same layout and a half-wave takes four consecutive d per read).
//
// Two restructurings were measured and dropped: one persistent work-group per CU that
// prefetches tile t+1 while multiplying tile t (11.9 us against 8.8 us: a single tile of
// look-ahead does not cover the ~2 us loaded memory latency), and one work-group per CU
// that requests the panels of its three tiles at once and shares panels between them
// (10.8 us: a CU ingests only ~10 bytes per clock from cold HBM, and a wave that is stuck
// issuing loads cannot multiply).  Three independent work-groups per CU keep more requests
// in flight and win.
#pragma once
#include "anr_device.h"
#include "anr_kernels.h"

namespace anr {
namespace tbg {

constexpr int kTile = 64;            // output tile edge
constexpr int kChunk = 64;           // reduction elements staged per pass
constexpr int kLds = kChunk + 4;     // LDS row stride in floats (272 B: 16-byte reads stay conflict free)

struct Args {
    const float* q;
    const float* k;
    float* out;
    int S, D, H;
    int64_t qs_b, qs_s, qs_h;   // element strides of q [b, s, h, d] (d stride 1)
    int64_t ks_b, ks_s, ks_h;
    int64_t os_b, os_h, os_i;   // element strides of out [b, h, i, j] (j stride 1)
    int tiles_i, tiles_j;       // ceil(S / 64) each
    int xcd_chunk;              // tiles per XCD when the tile count is a multiple of 8, else 0
};

#ifdef ANR_TBG_TRACE
__device__ long long* anr_tbg_trace = nullptr;
#define TT(slot) do { if (threadIdx.x == 0 && anr_tbg_trace) anr_tbg_trace[blockIdx.x * 8 + (slot)] = wall_clock64(); } while (0)
#define TT_END(slot) do { __builtin_amdgcn_s_waitcnt(0); TT(slot); } while (0)
#else
#define TT(slot) do { } while (0)
#define TT_END(slot) do { } while (0)
#endif

__global__ __launch_bounds__(256) void tbg_tile_kernel(const Args p)
{
    TT(0);
    __shared__ __attribute__((aligned(16))) float qs[kTile * kLds];
    __shared__ __attribute__((aligned(16))) float ks[kTile * kLds];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int r32 = lane & 31, h2 = lane >> 5;
    // tile id = ((b*H + h) * tiles_i + ti) * tiles_j + tj.  Work-group ids are dealt round-robin
    // over the 8 XCDs; give every XCD a contiguous range of tile ids, so that the tiles of one
    // score matrix, which share their q and k panels, meet in one L2.
    int t = blockIdx.x;
    if (p.xcd_chunk > 0) t = (t & 7) * p.xcd_chunk + (t >> 3);
    const int tj = t % p.tiles_j; t /= p.tiles_j;
    const int ti = t % p.tiles_i; t /= p.tiles_i;
    const int hh = t % p.H, b = t / p.H;
    const int i0 = ti * kTile, j0 = tj * kTile;

    const float* __restrict__ qb = p.q + b * p.qs_b + hh * p.qs_h;
    const float* __restrict__ kb = p.k + b * p.ks_b + hh * p.ks_h;

    // staging: thread -> (row = tid / 16 + 16*u, 16 bytes at d = 4 * (tid % 16)), u = 0..3
    const int srow = tid >> 4, sd = (tid & 15) * 4;
    const int wi = (wave >> 1) * 32, wj = (wave & 1) * 32;   // this wave's 32 x 32 block

    // two accumulators: consecutive MFMAs never wait on each other's result
    f32x16 acc, acc2;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = acc2[r] = 0.f;

    for (int d0 = 0; d0 < p.D; d0 += kChunk) {
        f32x4 rq[4], rk[4];
        const bool din = d0 + sd < p.D;          // D is a multiple of 4: the 16 bytes are all in or all out
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            // rows past S re-read row S-1 (their products are never stored); d past D must be zero
            int ri = i0 + srow + 16 * u, rj = j0 + srow + 16 * u;
            ri = ri < p.S ? ri : p.S - 1;
            rj = rj < p.S ? rj : p.S - 1;
            const int dd = din ? d0 + sd : 0;
            rq[u] = ldg4(qb + ri * p.qs_s + dd);
            rk[u] = ldg4(kb + rj * p.ks_s + dd);
        }
        TT(1);
        if (d0 > 0) __syncthreads();             // previous chunk fully consumed
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            *reinterpret_cast<f32x4*>(&qs[(srow + 16 * u) * kLds + sd]) = din ? rq[u] : zero4();
            *reinterpret_cast<f32x4*>(&ks[(srow + 16 * u) * kLds + sd]) = din ? rk[u] : zero4();
        }
        __syncthreads();
        TT(2);

        f32x4 a[8], bb[8];
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) {
            a[kk] = *reinterpret_cast<const f32x4*>(&qs[(wi + r32) * kLds + kk * 8 + 4 * h2]);
            bb[kk] = *reinterpret_cast<const f32x4*>(&ks[(wj + r32) * kLds + kk * 8 + 4 * h2]);
        }
#pragma unroll
        for (int kk = 0; kk < 8; ++kk)
#pragma unroll
            for (int e = 0; e < 4; e += 2) {
                acc = mfma32(a[kk][e], bb[kk][e], acc);
                acc2 = mfma32(a[kk][e + 1], bb[kk][e + 1], acc2);
            }
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] += acc2[r];
    TT(3);

    // register r of lane (h2, r32): row 8*(r/4) + 4*h2 + r%4, column r32 of the block
    float* __restrict__ ob = p.out + b * p.os_b + hh * p.os_h;
    const int col = j0 + wj + r32;
    if (col < p.S) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int row = i0 + wi + 8 * (r / 4) + 4 * h2 + (r % 4);
            if (row < p.S) ob[row * p.os_i + col] = acc[r];
        }
    }
    TT_END(4);
}

}  // namespace tbg
}  // namespace anr
