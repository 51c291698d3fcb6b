// C2D and the ConvLayer subgraph (Sec. 7.1, Sec. 7.2 and Appendix C of arXiv 2006.06762)
// for every geometry: any kernel size, stride, padding, dilation, channel count and image
// width, any strided NCHW view.  The shape lists of the paper hold layers the tuned
// patch-staging kernel cannot take (7x7 stride-2 stem with 3 channels, 14x14 and 7x7 maps,
// 1x1 stride 2) and run every shape at batch 1, where one image has too few pixels to fill
// the chip.
//
// Implicit GEMM with an explicit gather: rows m = output pixels (n, oh, ow), columns =
// output channels, reduction index k = (c, r, s) in the order of the OIHW weights.  A
// work-group owns BM pixels x BN channels and a range of reduction chunks of KC = 32.
//   A tile  [BM][KC]: thread t gathers pixel t % BM; the k it fetches is uniform over the
//           wave, so the split of k into (c, r, s) and the offset of that tap are scalar
//           work, and the lane adds its pixel's base offset and tests its own bounds.
//           Taps that fall outside the image get a buffer offset beyond the descriptor's
//           extent: the load returns zero without a branch.  Lanes are consecutive pixels,
//           so for stride 1 a load covers whole cache lines.
//   B tile  [BN][KC]: rows of the weight matrix [K][C*R*S] are contiguous in k: 16-byte
//           loads when C*R*S is a multiple of 4, single floats otherwise.
// Both tiles sit in LDS row-major in k with a row stride of KC + 2 floats (operand reads of
// 32 consecutive rows hit 32 different banks), double buffered, one barrier per chunk.  The
// MFMA is v_mfma_f32_32x32x2_f32; a lane reads two k values at a time (8-byte LDS reads)
// and feeds them to two consecutive MFMAs: half-wave h takes k = 4j + 2h and 4j + 2h + 1,
// which is a valid reduction order because A and B use the same one.
//
// Split-K: with few output tiles (batch 1, 7x7 maps) the reduction chunks of a tile are dealt
// to `ksplit` work-groups, which write partial tiles to a workspace; a second kernel sums them
// in fixed order (deterministic, no float atomics) and runs the epilogue.
#pragma once
#include <type_traits>

#include "anr_device.h"
#include "conv_internal.h"

namespace anr {
namespace gconv {

constexpr int KC = 32;           // reduction elements per chunk
constexpr int WS = KC + 2;       // LDS row stride, floats
constexpr uint32_t kOutOfRange = 0x80000000u;   // byte offset beyond any descriptor extent used here
constexpr int kNoRow = 0x7fff;                  // row displacement of a reduction index past the end
constexpr int kMaxExtent = 16000;               // image height/width and kernel extents the tap table packs

struct Plan {
    int Mtot, ohow, RS;
    int Ktot;                    // reduction length: (C / groups) * R * S
    int Cg, Kg;                  // input / output channels per group (per pack of groups when pack_cg > 0)
    int groups;                  // groups, or packs of groups
    int pack_cg, pack_kg;        // conv_taps_kernel with packed groups: channels of ONE group; else 0
    FastDiv d_pack_kg;
    int tiles_ng;                // column tiles per group (a tile never straddles two groups)
    int tiles_m, tiles_n, ksplit, nchunks, chunks_per_split;
    int Mpad, Kpad;              // tile-padded extents of the workspace
    int w_vec;                   // weight rows allow 16-byte loads
    int vec_store;               // 4 consecutive pixels of a lane are 16 contiguous, aligned bytes of y
    uint32_t x_bytes, w_bytes;
    FastDiv d_ow, d_oh, d_rs, d_s, d_ohow, d_tiles_m, d_tiles, d_tiles_ng, d_kg;
    int bm, bn;                  // chosen tile (host side)
    int kc;                      // reduction elements per chunk: KC, or 36 for the 3 x 3 form of conv_taps_kernel
    int tstore;                  // tap kernels: the tile is stored through LDS in runs of 64 pixels per channel
    int taps;                    // 0: conv_gather_kernel; 9 or 1: conv_taps_kernel for 3 x 3 / 1 x 1; 49 or 25: conv_bigtaps_kernel
    int nwg;                     // conv_taps_kernel: groups of four waves per work-group (1, 2 or 4)
    int rblocks;                 // work-groups per output channel in the split-K reduction
    FastDiv d_rblocks;
};

// Inference batch norm of output channel co as one multiply-add: y = v * scale + shift.
__device__ __forceinline__ void bn_constants(const ConvArgs& p, int co, float* scale, float* shift)
{
    if (p.scale_shift) {            // folded ahead of time (pre-packed call)
        *scale = p.scale_shift[co];
        *shift = p.scale_shift[p.K + co];
        return;
    }
    *scale = p.gamma[co] / sqrtf(p.var[co] + p.eps);
    *shift = p.beta[co] - p.mean[co] * *scale;
}

// Epilogue of one accumulator quad: registers 4q .. 4q+3 of a lane are pixels mq .. mq+3 of
// output channel co; scale and shift are that channel's batch-norm constants (used when the
// call has a fused epilogue).
__device__ __forceinline__ void store_quad_plain(const ConvArgs& p, const Plan& g, int mq, int co, f32x4 v);

__device__ __forceinline__ void store_quad(const ConvArgs& p, const Plan& g, int mq, int co, f32x4 v, float scale,
                                           float shift)
{
    if (p.gamma) {
#pragma unroll
        for (int r = 0; r < 4; ++r) v[r] = fmaxf(fmaf(v[r], scale, shift), 0.f);
    }
    store_quad_plain(p, g, mq, co, v);
}

// The four values as they are: pixels mq .. mq+3 of output channel co.  (Ordinary stores: storing
// the 256-byte runs of store_tile_runs non-temporally changed none of the Appendix C layers by
// more than the run-to-run spread.)
__device__ __forceinline__ void store_quad_plain(const ConvArgs& p, const Plan& g, int mq, int co, f32x4 v)
{
    if (g.vec_store) {
        if (mq < g.Mtot) {
            const int n = g.d_ohow.div(mq), pix = mq - n * g.ohow;
            stg4(p.y + n * p.ys[0] + co * p.ys[1] + pix, v);
        }
    } else {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int m = mq + r;
            if (m < g.Mtot) {
                const int gr = g.d_ow.div(m), ow = m - gr * p.OW;
                const int n = g.d_oh.div(gr), oh = gr - n * p.OH;
                p.y[n * p.ys[0] + co * p.ys[1] + oh * p.ys[2] + ow] = v[r];
            }
        }
    }
}

// Epilogue of a work-group's tile.  Accumulator register r of lane (h, r32) is pixel
// 8*(r/4) + 4*h + r%4 and channel r32 of its 32 x 32 block; waves are 2 x 2 with MB x NB blocks
// each.  With a split reduction the partial tile goes to the workspace, which is padded to
// whole tiles: no bounds to test.
template <int MB, int NB>
__device__ __forceinline__ void store_tile(const ConvArgs& p, const Plan& g, const f32x16 (&acc)[MB][NB], int split,
                                           int tile_n, int m0, int cl0, int cog, int wm, int wn, int r32, int h)
{
    constexpr int BN = 64 * NB;
    float* const wsp = p.ws + ((int64_t)split * g.Kpad + tile_n * BN + wn * NB * 32 + r32) * g.Mpad + m0 +
                       wm * MB * 32 + 4 * h;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const int tcol = (wn * NB + nb) * 32 + r32;             // column inside the tile: one channel per lane
        const bool col_ok = cl0 + tcol < g.Kg;
        // the channel's batch-norm constants once per lane, not once per quad (the division and
        // square root are a dozen vector-ALU instructions each time)
        float scale = 1.f, shift = 0.f;
        if (g.ksplit == 1 && p.gamma && col_ok) bn_constants(p, cog + cl0 + tcol, &scale, &shift);
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const f32x4 v = {acc[mb][nb][4 * q], acc[mb][nb][4 * q + 1], acc[mb][nb][4 * q + 2],
                                 acc[mb][nb][4 * q + 3]};
                if (g.ksplit > 1) {
                    stg4(wsp + (int64_t)(nb * 32) * g.Mpad + mb * 32 + 8 * q, v);
                } else if (col_ok) {
                    store_quad(p, g, m0 + (wm * MB + mb) * 32 + 8 * q + 4 * h, cog + cl0 + tcol, v, scale, shift);
                }
            }
    }
}

// The same epilogue for one 64 x 64 tile of four waves, through LDS: the tile is written
// transposed into `t` (64 x 68 floats that no wave reads any more) and leaves in runs of 64
// consecutive pixels of a channel (256 bytes from 16 lanes) instead of 64 separate 16-byte pieces
// per store instruction, one per lane and channel.
constexpr int kRunTileFloats = 64 * 68;

__device__ __forceinline__ void store_tile_runs(const ConvArgs& p, const Plan& g, const f32x16& acc, float* t, int split,
                                                int tile_n, int m0, int cl0, int cog, int wm, int wn, int r32, int h,
                                                int tid)
{
    constexpr int TS = 68;
    // the fused epilogue here, where a lane is one channel: its constants once per lane
    const bool fused = g.ksplit == 1 && p.gamma;
    float scale = 1.f, shift = 0.f;
    if (fused) {
        const int col = cl0 + wn * 32 + r32;
        bn_constants(p, cog + (col < g.Kg ? col : g.Kg - 1), &scale, &shift);
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        f32x4 v = {acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]};
        if (fused) {
#pragma unroll
            for (int r = 0; r < 4; ++r) v[r] = fmaxf(fmaf(v[r], scale, shift), 0.f);
        }
        *reinterpret_cast<f32x4*>(t + (wn * 32 + r32) * TS + wm * 32 + 8 * q + 4 * h) = v;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int ch = (tid >> 4) + 16 * k, quad = tid & 15;
        const f32x4 v = *reinterpret_cast<const f32x4*>(t + ch * TS + 4 * quad);
        if (g.ksplit > 1) {
            // partial tile: the workspace is padded to whole tiles
            stg4(p.ws + ((int64_t)split * g.Kpad + tile_n * 64 + ch) * g.Mpad + m0 + 4 * quad, v);
        } else if (cl0 + ch < g.Kg) {
            store_quad_plain(p, g, m0 + 4 * quad, cog + cl0 + ch, v);
        }
    }
}

// MASK: the kernel has at most 31 taps, so which taps of a pixel fall outside the image fits one
// register per lane and a gather load costs three vector-ALU instructions (bit test, add,
// and-or) instead of the two displacement adds, two compares and a select of the general form.
// Between MFMAs every vector-ALU instruction of any wave on the SIMD costs matrix time, and with
// 64 x 64 tiles the general form spends more of it on the gather than on the MFMAs.
template <int BM, int BN, bool MASK>
__global__ __launch_bounds__(256) void conv_gather_kernel(const ConvArgs p, const Plan g)
{
    constexpr int MB = BM / 64, NB = BN / 64;       // 32x32 blocks per wave (waves are 2 x 2)
    constexpr int KG = 256 / BM;                    // threads per pixel in the A gather
    constexpr int AU = KC / KG;                     // A elements per thread and chunk
    static_assert(AU % 8 == 0, "gather loads are issued in groups of eight");
    constexpr int BU4 = BN / 32;                    // B 16-byte units per thread and chunk
    constexpr int BU1 = BN / 8;                     // B single floats per thread and chunk
    constexpr int A_SZ = BM * WS, B_SZ = BN * WS;   // floats per buffer

    typedef int i32x2 __attribute__((ext_vector_type(2)));
    extern __shared__ __attribute__((aligned(16))) float glds[];   // A[2][BM][WS], then B[2][BN][WS]
    __shared__ i32x2 ktab[2 * KC];                                 // tap tables of two chunks
    float* const lds_a = glds;
    float* const lds_b = glds + 2 * A_SZ;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int r32 = lane & 31, h = lane >> 5;
    const int wm = wave >> 1, wn = wave & 1;

    // blockIdx.x = (split * tiles_n + tile_n) * tiles_m + tile_m
    const int tiles = g.tiles_m * g.tiles_n;
    const int split = g.d_tiles.div((int)blockIdx.x);
    const int trem = (int)blockIdx.x - split * tiles;
    const int tile_n = g.d_tiles_m.div(trem), tile_m = trem - tile_n * g.tiles_m;
    const int grp = g.d_tiles_ng.div(tile_n);                        // channel group of this tile
    const int m0 = tile_m * BM, cl0 = (tile_n - grp * g.tiles_ng) * BN;  // first column inside the group
    const int cog = grp * g.Kg;                                      // first output channel of the group
    const int c_begin = split * g.chunks_per_split;
    const int c_end = c_begin + g.chunks_per_split < g.nchunks ? c_begin + g.chunks_per_split : g.nchunks;

    // ---- the pixel this thread gathers for
    const int am = tid % BM;
    const int akg = __builtin_amdgcn_readfirstlane(tid / BM);    // uniform over the wave
    int m = m0 + am;
    m = m < g.Mtot ? m : g.Mtot - 1;          // rows past the end repeat the last pixel, never stored
    int ihb, iwb, xbase;
    {
        const int gr = g.d_ow.div(m), ow = m - gr * p.OW;
        const int n = g.d_oh.div(gr), oh = gr - n * p.OH;
        ihb = oh * p.stride_h - p.pad_h;
        iwb = ow * p.stride_w - p.pad_w;
        // may be negative; valid taps make it >= 0.  The group's first input channel is folded in.
        xbase = (int)(n * p.xs[0] + (int64_t)grp * g.Cg * p.xs[1] + ihb * p.xs[2] + iwb);
    }
    // bit t set: tap t of this pixel lies outside the image; bit 31 (no kernel has a tap 31
    // here) stands for the reduction indices past the end
    uint32_t notmask = 0x80000000u;
    if (MASK) {
        for (int r = 0; r < p.R; ++r)
            for (int s = 0; s < p.S; ++s) {
                const bool ok = ((unsigned)(ihb + r * p.dil_h) < (unsigned)p.H) &
                                ((unsigned)(iwb + s * p.dil_w) < (unsigned)p.W);
                notmask |= ok ? 0u : 1u << (r * p.S + s);
            }
    }
    const int xbase4 = 4 * xbase;
    const __amdgpu_buffer_rsrc_t xrsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(p.x), 0, (int)g.x_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t wrsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(p.w), 0, (int)g.w_bytes, 0x00020000);

    // Two chunks of look-ahead in registers: while chunk c is multiplied out of LDS, chunk c+1
    // waits in one register set and the loads of chunk c+2 go out into the other, so a load has
    // two chunks of MFMA time to come back.
    float ra[2][AU];
    float rb[2][BU1];                     // BU4 16-byte units or BU1 single floats: the same registers

    // byte offsets of this lane's 16-byte weight units inside a chunk (columns past the group
    // repeat its last one, never stored)
    uint32_t wvoff[BU4];
#pragma unroll
    for (int j = 0; j < BU4; ++j) {
        int co = cl0 + (tid >> 3) + 32 * j;
        co = cog + (co < g.Kg ? co : g.Kg - 1);
        wvoff[j] = 4u * (uint32_t)(co * g.Ktot + 4 * (tid & 7));
    }

    // The tap table of one chunk: for each of its KC reduction indices the offset of the tap
    // (c, r, s) inside an image and its row and column displacement.  32 threads fill it a chunk
    // ahead, so a gather load costs one broadcast LDS read instead of two scalar divisions.
    // The waves take turns at it: the divisions are vector-ALU work of one SIMD.
    auto fill_taps = [&](int chunk, int slot) {
        if (wave == (chunk & 3) && lane < KC) {
            const int k = chunk * KC + lane;
            const int c = g.d_rs.div(k), tap = k - c * g.RS;
            const int r = g.d_s.div(tap), s = tap - r * p.S;
            const int koff = (int)(c * p.xs[1] + (r * p.dil_h) * p.xs[2] + s * p.dil_w);
            i32x2 e;
            if (MASK) {
                // byte offset of the tap and its number
                e[0] = 4 * koff;
                e[1] = k < g.Ktot ? tap : 31;
            } else {
                // offset of the tap, then row and column displacement packed as two 16-bit fields; a
                // k past the end gets a row displacement no pixel can be in bounds with
                const int dr = k < g.Ktot ? r * p.dil_h : kNoRow;
                e[0] = koff;
                e[1] = (dr << 16) | (s * p.dil_w);
            }
            ktab[slot * KC + lane] = e;
        }
    };
    auto load_chunk = [&](int chunk, int slot, auto set_c) {
        constexpr int set = decltype(set_c)::value;
        const int k0 = chunk * KC;
#pragma unroll
        for (int j0 = 0; j0 < AU; j0 += 8) {
            // the table reads of eight loads go out together: one LDS round trip, not eight
            i32x2 e[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) e[j] = ktab[slot * KC + akg + KG * (j0 + j)];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                uint32_t off;
                if (MASK) {
                    // -1 if the tap is outside the image: the offset then gets its top bit set
                    const int out = __builtin_amdgcn_sbfe((int)notmask, (unsigned)e[j][1], 1u);
                    off = (uint32_t)(xbase4 + e[j][0]) | ((uint32_t)out & kOutOfRange);
                } else {
                    const int dr = e[j][1] >> 16, ds = e[j][1] & 0xffff;
                    const bool ok = ((unsigned)(ihb + dr) < (unsigned)p.H) & ((unsigned)(iwb + ds) < (unsigned)p.W);
                    off = ok ? 4u * (uint32_t)(xbase + e[j][0]) : kOutOfRange;
                }
                ra[set][j0 + j] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(xrsrc, (int)off, 0, 0));
            }
        }
        // weights: the lane's part of the offset is fixed (wvoff), the chunk's part is uniform and
        // rides in the scalar offset; only the last chunk can reach past the end of a row
        if (g.w_vec) {
            const bool past = k0 + 4 * (tid & 7) >= g.Ktot;
#pragma unroll
            for (int j = 0; j < BU4; ++j) {
                const uint32_t off = past ? kOutOfRange : wvoff[j];
                const f32x4 v = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(wrsrc, (int)off, 4 * k0, 0));
#pragma unroll
                for (int i = 0; i < 4; ++i) rb[set][4 * j + i] = v[i];
            }
        } else {
#pragma unroll
            for (int j = 0; j < BU1; ++j) {
                const int col = (tid >> 5) + 8 * j, k = k0 + (tid & 31);
                int co = cl0 + col;
                co = cog + (co < g.Kg ? co : g.Kg - 1);
                const uint32_t off = k < g.Ktot ? 4u * (uint32_t)(co * g.Ktot + k) : kOutOfRange;
                rb[set][j] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(wrsrc, (int)off, 0, 0));
            }
        }
    };
    auto store_chunk = [&](int buf, auto set_c) {
        constexpr int set = decltype(set_c)::value;
        float* const a = lds_a + buf * A_SZ;
        float* const b = lds_b + buf * B_SZ;
#pragma unroll
        for (int j = 0; j < AU; ++j) a[am * WS + akg + KG * j] = ra[set][j];
        if (g.w_vec) {
#pragma unroll
            for (int j = 0; j < BU4; ++j) {
                f32x2* dst = reinterpret_cast<f32x2*>(&b[((tid >> 3) + 32 * j) * WS + 4 * (tid & 7)]);
                const f32x2 lo = {rb[set][4 * j], rb[set][4 * j + 1]}, hi = {rb[set][4 * j + 2], rb[set][4 * j + 3]};
                dst[0] = lo;
                dst[1] = hi;
            }
        } else {
#pragma unroll
            for (int j = 0; j < BU1; ++j) b[((tid >> 5) + 8 * j) * WS + (tid & 31)] = rb[set][j];
        }
    };

    f32x16 acc[MB][NB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mb][nb][r] = 0.f;

    // chunks past the end of the range are the last chunk again: loaded, never multiplied (no
    // branch around the loads)
    auto clampc = [&](int c) { return c < c_end ? c : c_end - 1; };
    using S0 = std::integral_constant<int, 0>;
    using S1 = std::integral_constant<int, 1>;

    fill_taps(c_begin, 0);
    fill_taps(clampc(c_begin + 1), 1);
    __syncthreads();
    load_chunk(c_begin, 0, S0{});
    load_chunk(clampc(c_begin + 1), 1, S1{});
    __syncthreads();                       // every wave has read both tap tables
    fill_taps(clampc(c_begin + 2), 0);
    store_chunk(0, S0{});
    __syncthreads();

    // Iteration c: LDS buffer and tap slot of parity P hold chunk c and the taps of chunk c+2;
    // register set P is free, set P^1 holds chunk c+1.
    auto iteration = [&](int c, auto par_c) {
        constexpr int P = decltype(par_c)::value;
        load_chunk(clampc(c + 2), P, std::integral_constant<int, P>{});
        // keep the loads ahead of the MFMAs (the scheduler would sink them to their first use)
        __builtin_amdgcn_sched_barrier(0);
        const float* a = lds_a + P * A_SZ + (wm * MB * 32 + r32) * WS + 2 * h;
        const float* b = lds_b + P * B_SZ + (wn * NB * 32 + r32) * WS + 2 * h;
#pragma unroll
        for (int j = 0; j < KC / 4; ++j) {
            f32x2 av[MB], bv[NB];
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) av[mb] = *reinterpret_cast<const f32x2*>(a + mb * 32 * WS + 4 * j);
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) bv[nb] = *reinterpret_cast<const f32x2*>(b + nb * 32 * WS + 4 * j);
#pragma unroll
            for (int e = 0; e < 2; ++e)
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) acc[mb][nb] = mfma32(av[mb][e], bv[nb][e], acc[mb][nb]);
        }
        store_chunk(P ^ 1, std::integral_constant<int, P ^ 1>{});
        // slot P^1 held the taps of chunk c+1, last read before the previous barrier
        fill_taps(clampc(c + 3), P ^ 1);
        __syncthreads();
    };
    for (int c = c_begin; c < c_end; c += 2) {
        iteration(c, S0{});
        if (c + 1 < c_end) iteration(c + 1, S1{});
    }

    if (MB == 1 && NB == 1 && g.tstore) {
        // the last iteration ended with a barrier: the staging buffers are free
        store_tile_runs(p, g, acc[0][0], glds, split, tile_n, m0, cl0, cog, wm, wn, r32, h, tid);
        return;
    }
    store_tile<MB, NB>(p, g, acc, split, tile_n, m0, cl0, cog, wm, wn, r32, h);
}

// The same convolution for 3 x 3 and 1 x 1 kernels whose channel count fills whole chunks: a
// chunk is CPC whole input channels (4 x 9 or 32 x 1 reduction indices), so which tap a gather
// load fetches is known at compile time.  A lane keeps one byte offset per tap (its pixel's
// base plus the tap's displacement, or the out-of-range marker where the tap leaves the image)
// and the channel rides in the scalar offset of the buffer load: the loop between two barriers
// holds no vector-ALU instruction for addresses or bounds, no tap table and no tail handling.
// On this hardware every vector-ALU instruction of any wave on a SIMD takes about eight cycles
// from the matrix pipe, and counters show the general kernel above spending 35-40 % of its
// SIMD time on them.  Weights: a chunk of a row is KC consecutive floats of the OIHW order.
//
// NWG > 1: the work-group has NWG groups of four waves; group w takes every NWG-th chunk of the
// work-group's range through staging buffers of its own, and the groups' accumulators meet in LDS
// at the end.  For launches with one work-group per CU (batch 1: the chain of a work-group's
// chunks is what takes the time, and the matrix pipes idle between its barriers) this shortens the
// chain NWG-fold without more partial tiles in the workspace.
//
// PACK (1 x 1 kernels of grouped convolutions whose groups have fewer than 64 output channels): a
// column tile takes 64 / Kg consecutive groups at once as ONE group with a block-diagonal weight
// matrix.  The pixel gather, the tile and the stores are those of a convolution with that many
// fewer, larger groups; only the weight units differ: a unit of row co is real inside the channel
// range of co's own group and zero (an out-of-range load) elsewhere.  The extra products are
// zeros on matrix pipes that idle anyway; what is saved is one work-group, one pixel gather and
// three quarters of a column tile per group (56 x 56, 64 -> 64, 4 groups, batch 16: 22 -> 12 us).
template <int BM, int BN, int R_, int S_, int NWG, bool PACK = false>
__global__ __launch_bounds__(256 * NWG) void conv_taps_kernel(const ConvArgs p, const Plan g)
{
    static_assert(!PACK || (R_ == 1 && S_ == 1 && NWG == 1), "packed groups: 1 x 1 kernels, one wave group");
    constexpr int T = R_ * S_;
    constexpr int CPC = T == 1 ? 32 : 4;            // channels per chunk
    constexpr int KCT = CPC * T;                    // reduction elements per chunk
    constexpr int WST = KCT + 2;                    // LDS row stride, floats
    constexpr int MB = BM / 64, NB = BN / 64;
    constexpr int KG = 256 / BM;                    // threads per pixel in the A gather
    constexpr int CPT = CPC / KG;                   // channels of a chunk one thread gathers
    constexpr int AU = CPT * T;                     // A elements per thread and chunk
    constexpr int UPR = KCT / 4;                    // 16-byte units per weight row and chunk
    constexpr int BUNITS = BN * UPR;
    constexpr int BU = (BUNITS + 255) / 256;        // B units per thread and chunk
    constexpr int A_SZ = BM * WST, B_SZ = BN * WST;
    static_assert(KCT % 4 == 0 && CPC % KG == 0, "chunk geometry");
    static_assert(NWG == 1 || (MB == 1 && NB == 1), "wave groups share 64 x 64 tiles only");
    constexpr int REGION = 2 * (A_SZ + B_SZ);       // floats of staging per wave group

    extern __shared__ __attribute__((aligned(16))) float glds[];   // per group: A[2][BM][WST], then B[2][BN][WST]
    const int wgrp = NWG > 1 ? __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 8) : 0;
    float* const lds_a = glds + wgrp * REGION;
    float* const lds_b = lds_a + 2 * A_SZ;

    const int tid = (int)threadIdx.x & 255;         // thread inside its wave group
    const int lane = tid & 63, wave = tid >> 6;
    const int r32 = lane & 31, h = lane >> 5;
    const int wm = wave >> 1, wn = wave & 1;

    const int tiles = g.tiles_m * g.tiles_n;
    const int split = g.d_tiles.div((int)blockIdx.x);
    const int trem = (int)blockIdx.x - split * tiles;
    const int tile_n = g.d_tiles_m.div(trem), tile_m = trem - tile_n * g.tiles_m;
    const int grp = g.d_tiles_ng.div(tile_n);
    const int m0 = tile_m * BM, cl0 = (tile_n - grp * g.tiles_ng) * BN;
    const int cog = grp * g.Kg;
    const int c_begin = split * g.chunks_per_split;
    const int c_end = c_begin + g.chunks_per_split < g.nchunks ? c_begin + g.chunks_per_split : g.nchunks;

    // ---- the pixel this thread gathers for, and its byte offset for every tap
    const int am = tid % BM;
    const int akg = __builtin_amdgcn_readfirstlane(tid / BM);
    uint32_t voff[T];
    {
        int m = m0 + am;
        m = m < g.Mtot ? m : g.Mtot - 1;      // rows past the end repeat the last pixel, never stored
        const int gr = g.d_ow.div(m), ow = m - gr * p.OW;
        const int n = g.d_oh.div(gr), oh = gr - n * p.OH;
        const int ihb = oh * p.stride_h - p.pad_h, iwb = ow * p.stride_w - p.pad_w;
        const int xbase = (int)(n * p.xs[0] + (int64_t)grp * g.Cg * p.xs[1] + ihb * p.xs[2] + iwb);
        const int xs2 = (int)p.xs[2];
#pragma unroll
        for (int r = 0; r < R_; ++r)
#pragma unroll
            for (int s = 0; s < S_; ++s) {
                const bool ok = ((unsigned)(ihb + r * p.dil_h) < (unsigned)p.H) &
                                ((unsigned)(iwb + s * p.dil_w) < (unsigned)p.W);
                voff[r * S_ + s] = ok ? 4u * (uint32_t)(xbase + r * p.dil_h * xs2 + s * p.dil_w) : kOutOfRange;
            }
    }
    // ---- this thread's weight units: unit u is 16 bytes of row u / UPR; slots past the tile's
    //      units duplicate an earlier one (same data to the same place), columns past the group
    //      repeat its last (never stored)
    //      PACK: a weight row holds the pack_cg channels of its own group; wk is the unit's first
    //      channel of the FIRST chunk relative to that group's first channel (negative before it)
    uint32_t wvoff[BU], wlds[BU];
    int wk[BU];
#pragma unroll
    for (int j = 0; j < BU; ++j) {
        const int u = (tid + 256 * j) % BUNITS;
        const int row = u / UPR, q = u - row * UPR;
        int co = cl0 + row;
        co = co < g.Kg ? co : g.Kg - 1;
        if (PACK) {
            wk[j] = 4 * q - g.d_pack_kg.div(co) * g.pack_cg;
            wvoff[j] = 4u * (uint32_t)((cog + co) * g.pack_cg + wk[j]);     // never negative: co >= its group index
        } else {
            wk[j] = 0;
            wvoff[j] = 4u * (uint32_t)((cog + co) * g.Ktot + 4 * q);
        }
        wlds[j] = (uint32_t)(row * WST + 4 * q);
    }
    const __amdgpu_buffer_rsrc_t xrsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(p.x), 0, (int)g.x_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t wrsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(p.w), 0, (int)g.w_bytes, 0x00020000);
    const int xs1 = (int)p.xs[1];

    // two chunks of look-ahead in registers, as in the general kernel
    float ra[2][AU];
    f32x4 rb[2][BU];
    auto load_chunk = [&](int chunk, auto set_c) {
        constexpr int set = decltype(set_c)::value;
        const int c0 = chunk * CPC + akg * CPT;                  // uniform over the wave
#pragma unroll
        for (int cc = 0; cc < CPT; ++cc)
#pragma unroll
            for (int t = 0; t < T; ++t)
                ra[set][cc * T + t] = __builtin_bit_cast(
                    float, __builtin_amdgcn_raw_buffer_load_b32(xrsrc, (int)voff[t], 4 * (c0 + cc) * xs1, 0));
#pragma unroll
        for (int j = 0; j < BU; ++j) {
            // PACK: the unit is inside its group's block of this chunk or it is zero
            const uint32_t off =
                (!PACK || (unsigned)(chunk * KCT + wk[j]) < (unsigned)g.pack_cg) ? wvoff[j] : kOutOfRange;
            rb[set][j] = __builtin_bit_cast(
                f32x4, __builtin_amdgcn_raw_buffer_load_b128(wrsrc, (int)off, 4 * chunk * KCT, 0));
        }
    };
    auto store_chunk = [&](int buf, auto set_c) {
        constexpr int set = decltype(set_c)::value;
        float* const a = lds_a + buf * A_SZ + am * WST + akg * AU;
        float* const b = lds_b + buf * B_SZ;
#pragma unroll
        for (int i = 0; i < AU; ++i) a[i] = ra[set][i];
#pragma unroll
        for (int j = 0; j < BU; ++j) {
            f32x2* dst = reinterpret_cast<f32x2*>(b + wlds[j]);
            const f32x2 lo = {rb[set][j][0], rb[set][j][1]}, hi = {rb[set][j][2], rb[set][j][3]};
            dst[0] = lo;
            dst[1] = hi;
        }
    };

    f32x16 acc[MB][NB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mb][nb][r] = 0.f;

    // in the prologue a chunk past the end of the range is the last chunk again: loaded, never multiplied
    auto clampc = [&](int c) { return c < c_end ? c : c_end - 1; };
    using S0 = std::integral_constant<int, 0>;
    using S1 = std::integral_constant<int, 1>;

    // this group's chunks: first, first + NWG, ...; every group runs the same number of iterations
    // (the barriers are the work-group's)
    const int first = c_begin + wgrp;
    const int iters = (c_end - c_begin + NWG - 1) / NWG;
    load_chunk(clampc(first), S0{});
    load_chunk(clampc(first + NWG), S1{});
    store_chunk(0, S0{});
    __syncthreads();

    // Iteration c: LDS buffer P holds chunk c, register set P^1 the group's next chunk, set P is free.
    auto iteration = [&](int c, auto par_c) {
        constexpr int P = decltype(par_c)::value;
        // the last two iterations have nothing left to request (a uniform branch; requesting the last
        // chunk again instead cost 1 x 1 layers of two to four chunks 1-4 %)
        if (c + 2 * NWG < c_end) load_chunk(c + 2 * NWG, std::integral_constant<int, P>{});
        __builtin_amdgcn_sched_barrier(0);
        const float* a = lds_a + P * A_SZ + (wm * MB * 32 + r32) * WST + 2 * h;
        const float* b = lds_b + P * B_SZ + (wn * NB * 32 + r32) * WST + 2 * h;
        if (NWG == 1 || c < c_end) {          // a group may have one chunk fewer than the others
#pragma unroll
            for (int j = 0; j < KCT / 4; ++j) {
                f32x2 av[MB], bv[NB];
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
                    av[mb] = *reinterpret_cast<const f32x2*>(a + mb * 32 * WST + 4 * j);
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
                    bv[nb] = *reinterpret_cast<const f32x2*>(b + nb * 32 * WST + 4 * j);
#pragma unroll
                for (int e = 0; e < 2; ++e)
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                        for (int nb = 0; nb < NB; ++nb) acc[mb][nb] = mfma32(av[mb][e], bv[nb][e], acc[mb][nb]);
            }
        }
        store_chunk(P ^ 1, std::integral_constant<int, P ^ 1>{});
        __syncthreads();
    };
    for (int i = 0; i < iters; i += 2) {
        iteration(first + i * NWG, S0{});
        if (i + 1 < iters) iteration(first + (i + 1) * NWG, S1{});
    }
    if (NWG > 1) {
        // the last iteration ended with a barrier: every staging region is free.  Groups 1 .. NWG-1
        // leave their accumulators in their own regions, group 0 adds them in group order.
        if (wgrp > 0) {
#pragma unroll
            for (int r = 0; r < 16; ++r) lds_a[(wave * 16 + r) * 64 + lane] = acc[0][0][r];
        }
        __syncthreads();
        if (wgrp > 0) return;
#pragma unroll
        for (int o = 1; o < NWG; ++o)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[0][0][r] += glds[o * REGION + (wave * 16 + r) * 64 + lane];
    }
    if (NWG == 1 && MB == 1 && NB == 1 && g.tstore) {
        store_tile_runs(p, g, acc[0][0], glds, split, tile_n, m0, cl0, cog, wm, wn, r32, h, tid);
        return;
    }
    store_tile<MB, NB>(p, g, acc, split, tile_n, m0, cl0, cog, wm, wn, r32, h);
}

// Large kernels (7 x 7 and 5 x 5; the 7 x 7 stem of the shape lists has 3 channels, 49 taps): a chunk
// is ONE input channel, its T taps padded to a multiple of four.  The four threads of a pixel
// take taps akg, akg + 4, ...: which tap a load fetches is fixed for the thread, so its byte
// offset (or the out-of-range marker where the tap leaves the image, and for the padding) sits
// in a register and the channel rides in the scalar offset, as in conv_taps_kernel.  The general
// kernel spends two thirds of its SIMD time on gather arithmetic for this layer.  Weight rows
// are read as 16-byte units at 4-byte alignment (buffer loads of several dwords need dword
// alignment only) plus single floats for the T % 4 taps left over, so nothing past a row's
// chunk is ever multiplied.  One LDS buffer, two barriers per chunk, the next chunk's loads in
// flight meanwhile: a work-group has only as many chunks as the layer has channels, and the
// smaller footprint keeps four work-groups on a CU.
template <int R_, int S_>
__global__ __launch_bounds__(256) void conv_bigtaps_kernel(const ConvArgs p, const Plan g)
{
    constexpr int BM = 64, BN = 64;
    constexpr int T = R_ * S_;
    constexpr int KCT = (T + 3) / 4 * 4;            // reduction elements per chunk, padding included
    constexpr int WST = KCT + 2;                    // LDS row stride, floats
    constexpr int AU = KCT / 4;                     // A elements per thread and chunk
    constexpr int FU = T / 4, REM = T % 4;          // whole 16-byte units and left-over floats per weight row
    constexpr int BUNITS = BN * FU;
    constexpr int BU = (BUNITS + 255) / 256;
    constexpr int A_SZ = BM * WST;

    extern __shared__ __attribute__((aligned(16))) float glds[];   // A[BM][WST], then B[BN][WST]
    float* const lds_a = glds;
    float* const lds_b = glds + A_SZ;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int r32 = lane & 31, h = lane >> 5;
    const int wm = wave >> 1, wn = wave & 1;

    const int tiles = g.tiles_m * g.tiles_n;
    const int split = g.d_tiles.div((int)blockIdx.x);
    const int trem = (int)blockIdx.x - split * tiles;
    const int tile_n = g.d_tiles_m.div(trem), tile_m = trem - tile_n * g.tiles_m;
    const int grp = g.d_tiles_ng.div(tile_n);
    const int m0 = tile_m * BM, cl0 = (tile_n - grp * g.tiles_ng) * BN;
    const int cog = grp * g.Kg;
    const int c_begin = split * g.chunks_per_split;
    const int c_end = c_begin + g.chunks_per_split < g.nchunks ? c_begin + g.chunks_per_split : g.nchunks;

    // ---- the pixel this thread gathers for and the byte offsets of its taps akg + 4 i
    const int am = tid % BM;
    const int akg = __builtin_amdgcn_readfirstlane(tid / BM);
    uint32_t voff[AU];
    {
        int m = m0 + am;
        m = m < g.Mtot ? m : g.Mtot - 1;      // rows past the end repeat the last pixel, never stored
        const int gr = g.d_ow.div(m), ow = m - gr * p.OW;
        const int n = g.d_oh.div(gr), oh = gr - n * p.OH;
        const int ihb = oh * p.stride_h - p.pad_h, iwb = ow * p.stride_w - p.pad_w;
        const int xbase = (int)(n * p.xs[0] + (int64_t)grp * g.Cg * p.xs[1] + ihb * p.xs[2] + iwb);
        const int xs2 = (int)p.xs[2];
#pragma unroll
        for (int i = 0; i < AU; ++i) {
            const int t = akg + 4 * i;            // uniform over the wave
            const int r = t / S_, s = t - r * S_;
            const bool ok = (t < T) & ((unsigned)(ihb + r * p.dil_h) < (unsigned)p.H) &
                            ((unsigned)(iwb + s * p.dil_w) < (unsigned)p.W);
            voff[i] = ok ? 4u * (uint32_t)(xbase + r * p.dil_h * xs2 + s * p.dil_w) : kOutOfRange;
        }
    }
    // ---- weight units of this thread: unit u is floats 4q .. 4q+3 of the chunk of row u / FU;
    //      slots past the tile's units duplicate an earlier one, columns past the group repeat its
    //      last (never stored).  Left-over float e of row tid % BN goes to thread tid (e = tid / BN).
    uint32_t wvoff[BU], wlds[BU];
#pragma unroll
    for (int j = 0; j < BU; ++j) {
        const int u = (tid + 256 * j) % BUNITS;
        const int row = u / FU, q = u - row * FU;
        int co = cl0 + row;
        co = cog + (co < g.Kg ? co : g.Kg - 1);
        wvoff[j] = 4u * (uint32_t)(co * g.Ktot + 4 * q);
        wlds[j] = (uint32_t)(row * WST + 4 * q);
    }
    uint32_t rvoff = 0, rlds = 0;
    if (REM > 0) {
        const int row = tid % BN, e = (tid / BN) % REM;
        int co = cl0 + row;
        co = cog + (co < g.Kg ? co : g.Kg - 1);
        rvoff = 4u * (uint32_t)(co * g.Ktot + 4 * FU + e);
        rlds = (uint32_t)(row * WST + 4 * FU + e);
    }
    // the padding columns of the weight tile are never written again; the pixel tile's are
    // rewritten with the zeros its out-of-range loads return
    if (KCT > T)
        for (int i = tid; i < BN * (KCT - T); i += 256) lds_b[(i / (KCT - T)) * WST + T + i % (KCT - T)] = 0.f;

    const __amdgpu_buffer_rsrc_t xrsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(p.x), 0, (int)g.x_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t wrsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(p.w), 0, (int)g.w_bytes, 0x00020000);
    const int xs1 = (int)p.xs[1];

    float ra[2][AU], rr[2];
    f32x4 rb[2][BU];
    auto load_chunk = [&](int c, auto set_c) {
        constexpr int set = decltype(set_c)::value;
#pragma unroll
        for (int i = 0; i < AU; ++i)
            ra[set][i] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(xrsrc, (int)voff[i], 4 * c * xs1, 0));
#pragma unroll
        for (int j = 0; j < BU; ++j)
            rb[set][j] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(wrsrc, (int)wvoff[j], 4 * c * T, 0));
        if (REM > 0)
            rr[set] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(wrsrc, (int)rvoff, 4 * c * T, 0));
    };
    auto store_chunk = [&](auto set_c) {
        constexpr int set = decltype(set_c)::value;
        float* const a = lds_a + am * WST + akg;
#pragma unroll
        for (int i = 0; i < AU; ++i) a[4 * i] = ra[set][i];
#pragma unroll
        for (int j = 0; j < BU; ++j) {
            f32x2* dst = reinterpret_cast<f32x2*>(lds_b + wlds[j]);
            const f32x2 lo = {rb[set][j][0], rb[set][j][1]}, hi = {rb[set][j][2], rb[set][j][3]};
            dst[0] = lo;
            dst[1] = hi;
        }
        if (REM > 0) lds_b[rlds] = rr[set];
    };

    f32x16 acc[1][1];
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[0][0][r] = 0.f;

    using S0 = std::integral_constant<int, 0>;
    using S1 = std::integral_constant<int, 1>;
    auto clampc = [&](int c) { return c < c_end ? c : c_end - 1; };
    // Iteration c: register set P holds chunk c; chunk c+1 is requested into set P^1 before
    // chunk c is staged and multiplied.
    auto iteration = [&](int c, auto par_c) {
        constexpr int P = decltype(par_c)::value;
        load_chunk(clampc(c + 1), std::integral_constant<int, P ^ 1>{});
        __builtin_amdgcn_sched_barrier(0);
        store_chunk(std::integral_constant<int, P>{});
        __syncthreads();
        const float* a = lds_a + (wm * 32 + r32) * WST + 2 * h;
        const float* b = lds_b + (wn * 32 + r32) * WST + 2 * h;
#pragma unroll
        for (int j = 0; j < KCT / 4; ++j) {
            const f32x2 av = *reinterpret_cast<const f32x2*>(a + 4 * j);
            const f32x2 bv = *reinterpret_cast<const f32x2*>(b + 4 * j);
            acc[0][0] = mfma32(av[0], bv[0], acc[0][0]);
            acc[0][0] = mfma32(av[1], bv[1], acc[0][0]);
        }
        __syncthreads();                       // the tile is overwritten by the next chunk
    };
    load_chunk(c_begin, S0{});
    for (int c = c_begin; c < c_end; c += 2) {
        iteration(c, S0{});
        if (c + 1 < c_end) iteration(c + 1, S1{});
    }
    if (g.tstore) {
        // the last iteration ended with a barrier: the staging tile is free
        store_tile_runs(p, g, acc[0][0], glds, split, tile_n, m0, cl0, cog, wm, wn, r32, h, tid);
        return;
    }
    store_tile<1, 1>(p, g, acc, split, tile_n, m0, cl0, cog, wm, wn, r32, h);
}

// Sums the ksplit partial tiles and runs the epilogue.  LANES lanes share one (output channel,
// four consecutive pixels): lane j adds the partials of splits j, j + LANES, ... (all its loads in
// flight at once, up to four per lane), then the sums are combined by a fixed shuffle tree, so
// the result does not depend on scheduling.  One memory round trip however many splits there
// are; with few splits fewer lanes per quad, so that a launch is not eight times the waves its
// loads need (five splits of 14x14x256 at batch 16: 25088 waves of one load per lane with eight
// lanes, 6272 of three with two).
inline int reduce_lanes(int ksplit) { return ksplit > 16 ? 8 : ksplit > 8 ? 4 : ksplit > 4 ? 2 : 1; }

template <int LANES>
__global__ __launch_bounds__(256) void conv_splitk_reduce_kernel(const ConvArgs p, const Plan g)
{
    constexpr int kReduceLanes = LANES;
    // a work-group stays inside one output channel (blocks_per_co of them per channel), so the
    // channel, its workspace column and its batch-norm constants are scalar work
    const int co = g.d_rblocks.div((int)blockIdx.x);
    const int rblock = (int)blockIdx.x - co * g.rblocks;
    const int t = rblock * 256 + (int)threadIdx.x;
    const int sub = t & (kReduceLanes - 1);
    const int mq = 4 * (t / kReduceLanes);
    const bool live = mq < g.Mtot;
    // channel co sits in column (its group's first tile) * bn + (index inside the group)
    const int grp = g.d_kg.div(co);
    const float* src = p.ws + ((int64_t)grp * g.tiles_ng * g.bn + (co - grp * g.Kg)) * g.Mpad + (mq < g.Mpad ? mq : 0);
    const int64_t step = (int64_t)g.Kpad * g.Mpad;
    f32x4 v = zero4();
    // four loads in flight per round, none under a branch: a round's surplus slots re-read the
    // lane's first split (LANES <= ksplit, so that one exists) and are left out of the sum
    for (int s = sub; s < g.ksplit; s += 4 * kReduceLanes) {
        f32x4 u[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int idx = s + i * kReduceLanes;
            u[i] = ldg4(src + (idx < g.ksplit ? idx : sub) * step);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const bool in = s + i * kReduceLanes < g.ksplit;
#pragma unroll
            for (int r = 0; r < 4; ++r) v[r] += in ? u[i][r] : 0.f;
        }
    }
#pragma unroll
    for (int o = 1; o < kReduceLanes; o <<= 1)
#pragma unroll
        for (int r = 0; r < 4; ++r) v[r] += __shfl_xor(v[r], o);
    if (live && sub == 0) {
        float scale = 1.f, shift = 0.f;
        if (p.gamma) bn_constants(p, co, &scale, &shift);
        store_quad(p, g, mq, co, v, scale, shift);
    }
}

}  // namespace gconv
}  // namespace anr
