// GMM (C = A.B, Sec. 4.1 and Appendix C of arXiv 2006.06762) and its A.B^T form for operands
// that allow 16-byte loads (K, and N for the A.B form, multiples of 4; aligned bases and
// leading dimensions), any M, N, K otherwise.
//
// Work-group tile BM x BN, 4 waves in a 2 x 2 grid, reduction in chunks of 32.  A chunk of a
// work-group that has a CU to itself costs one memory round trip unless more than one chunk
// is in flight, so the operands travel global -> registers -> LDS with TWO chunks of
// look-ahead in registers and a double-buffered LDS tile: while chunk c is multiplied,
// chunk c+1 waits in one register set and the loads of chunk c+2 go out into the other.
// The loads are buffer loads: rows past M / N re-read the last row (never stored), and a
// reduction index past K gets an offset beyond the descriptor's extent, which loads zero
// without a branch.
//
// LDS: A (and B of the A.B^T form) row-major in k with a row stride of 36 floats (a staging unit is
// then one 16-byte store; with 34, conflict-free 8-byte operand reads but two stores per unit,
// 1024^3 x16 and 4096^3 ran 3 % slower), read two k
// at a time (8-byte reads, half-wave h takes k = 4j + 2h, 4j + 2h + 1: any order is a valid
// reduction order as long as both operands use it); B of the A.B form stays k-major as it is
// in memory, row stride BN + 16 floats (rows 4j + 2h of the two half-waves then fall into
// different halves of the LDS banks), read one float per MFMA.
#pragma once
#include <type_traits>

#include "anr_device.h"
#include "anr_kernels.h"

namespace anr {
namespace gpipe {

constexpr int KC = 32;
constexpr int WS = KC + 4;       // LDS row stride of the k-contiguous tiles: a staging unit is one 16-byte store
constexpr uint32_t kOutOfRange = 0x80000000u;

template <int BM, int BN, bool NT>
struct Tiles {
    static constexpr int A_SZ = BM * WS;
    static constexpr int LDB = BN + 16;
    static constexpr int B_SZ = NT ? BN * WS : KC * LDB;
    static constexpr size_t lds_bytes = sizeof(float) * 2 * (size_t)(A_SZ + B_SZ);
};

// NWG > 1 (64 x 64 tiles only): the work-group has NWG groups of four waves; group w takes every
// NWG-th chunk through staging buffers of its own and the groups' accumulators meet in LDS at the
// end.  For launches with at most one work-group per CU the chain of a work-group's chunks is what
// takes the time (the matrix pipes idle between its barriers); sharing it among groups shortens it.
template <int BM, int BN, bool NT, int NWG = 1>
__global__ __launch_bounds__(256 * NWG) void gemm_pipe_kernel(const GemmArgs p, int tiles_m, int tiles_n)
{
    using T = Tiles<BM, BN, NT>;
    constexpr int MB = BM / 64, NB = BN / 64;
    constexpr int AU = BM / 32;                 // 16-byte units of A per thread and chunk
    constexpr int BU = BN / 32;                 // 16-byte units of B per thread and chunk
    constexpr int A_SZ = T::A_SZ, B_SZ = T::B_SZ, LDB = T::LDB;

    static_assert(NWG == 1 || (MB == 1 && NB == 1), "wave groups share 64 x 64 tiles only");
    constexpr int REGION = 2 * (A_SZ + B_SZ);   // floats of staging per wave group

    extern __shared__ __attribute__((aligned(16))) float plds[];   // per group: A[2][A_SZ], then B[2][B_SZ]
    const int wgrp = NWG > 1 ? __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 8) : 0;
    float* const lds_a = plds + wgrp * REGION;
    float* const lds_b = lds_a + 2 * A_SZ;

    const int tid = (int)threadIdx.x & 255;     // thread inside its wave group
    const int lane = tid & 63, wave = tid >> 6;
    const int r32 = lane & 31, h = lane >> 5;
    const int wm = wave >> 1, wn = wave & 1;
    // consecutive work-groups walk down a column of tiles: they share the B panel
    const int tile_m = blockIdx.x % tiles_m, tile_n = blockIdx.x / tiles_m;
    const int m0 = tile_m * BM, n0 = tile_n * BN;
    const int zo = blockIdx.z / p.batch_inner, zi = blockIdx.z % p.batch_inner;
    const float* A = p.A + zo * p.sAo + zi * p.sAi;
    const float* B = p.B + zo * p.sBo + zi * p.sBi;
    float* __restrict__ C = p.C + zo * p.sCo + zi * p.sCi;
    const int M = p.M, N = p.N, K = p.K;

    const uint32_t a_bytes = 4u * (uint32_t)((int64_t)(M - 1) * p.lda + K);
    const uint32_t b_bytes = NT ? 4u * (uint32_t)((int64_t)(N - 1) * p.ldb + K)
                                : 4u * (uint32_t)((int64_t)(K - 1) * p.ldb + N);
    const __amdgpu_buffer_rsrc_t arsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(A), 0, (int)a_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t brsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(B), 0, (int)b_bytes, 0x00020000);

    // per-thread staging offsets (bytes), fixed over chunks except for the k term
    uint32_t aoff[AU], boff[BU];
    const int ak = 4 * (tid & 7);               // k offset of this thread's A units inside a chunk
#pragma unroll
    for (int j = 0; j < AU; ++j) {
        int row = m0 + (tid >> 3) + 32 * j;
        row = row < M ? row : M - 1;
        aoff[j] = 4u * (uint32_t)((int64_t)row * p.lda + ak);
    }
    constexpr int BQ = BN / 4;                  // A.B form: 16-byte units per k row of the B tile
    const int bk = NT ? ak : tid / BQ;          // k offset of this thread's first B unit
    bool bcol_ok = true;
#pragma unroll
    for (int j = 0; j < BU; ++j) {
        if (NT) {
            int row = n0 + (tid >> 3) + 32 * j;
            row = row < N ? row : N - 1;
            boff[j] = 4u * (uint32_t)((int64_t)row * p.ldb + ak);
        } else {
            const int col = n0 + 4 * (tid % BQ);
            bcol_ok = col < N;                  // N is a multiple of 4: a unit is in or out as a whole
            // a column past N keeps the out-of-range marker whatever is added to it for the chunk
            // (extents are below 2^29 floats)
            boff[j] = bcol_ok ? 4u * (uint32_t)((int64_t)(bk + (256 / BQ) * j) * p.ldb + col) : kOutOfRange;
        }
    }

    f32x4 ra[2][AU], rb[2][BU];
    auto load_chunk = [&](int chunk, auto set_c) {
        constexpr int set = decltype(set_c)::value;
        const int k0 = chunk * KC;
        if (k0 + KC <= K) {
            // a whole chunk: the chunk's part of the offset is uniform and rides in the scalar
            // offset of the load, so no vector-ALU instruction sits between the MFMAs for it
            // (each one costs the matrix pipe about eight cycles)
#pragma unroll
            for (int j = 0; j < AU; ++j)
                ra[set][j] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(arsrc, (int)aoff[j], 4 * k0, 0));
            const int bs = NT ? 4 * k0 : 4 * k0 * p.ldb;
#pragma unroll
            for (int j = 0; j < BU; ++j)
                rb[set][j] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(brsrc, (int)boff[j], bs, 0));
        } else {
            const bool a_in = k0 + ak < K;          // K is a multiple of 4
#pragma unroll
            for (int j = 0; j < AU; ++j) {
                const uint32_t off = a_in ? aoff[j] + 4u * (uint32_t)k0 : kOutOfRange;
                ra[set][j] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(arsrc, (int)off, 0, 0));
            }
#pragma unroll
            for (int j = 0; j < BU; ++j) {
                uint32_t off;
                if (NT) {
                    off = a_in ? boff[j] + 4u * (uint32_t)k0 : kOutOfRange;
                } else {
                    const bool in = k0 + bk + (256 / BQ) * j < K;
                    off = in ? boff[j] + 4u * (uint32_t)((int64_t)k0 * p.ldb) : kOutOfRange;
                }
                rb[set][j] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(brsrc, (int)off, 0, 0));
            }
        }
    };
    auto store_rows = [&](float* tile, const auto& reg) {
        constexpr int count = sizeof(reg) / sizeof(f32x4);
#pragma unroll
        for (int j = 0; j < count; ++j) {
            *reinterpret_cast<f32x4*>(&tile[((tid >> 3) + 32 * j) * WS + ak]) = reg[j];
        }
    };
    auto store_chunk = [&](int buf, auto set_c) {
        constexpr int set = decltype(set_c)::value;
        store_rows(lds_a + buf * A_SZ, ra[set]);
        if (NT) {
            store_rows(lds_b + buf * B_SZ, rb[set]);
        } else {
            float* b = lds_b + buf * B_SZ;
#pragma unroll
            for (int j = 0; j < BU; ++j)
                *reinterpret_cast<f32x4*>(&b[(bk + (256 / BQ) * j) * LDB + 4 * (tid % BQ)]) = rb[set][j];
        }
    };

    f32x16 acc[MB][NB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mb][nb][r] = 0.f;

    const int nchunks = (K + KC - 1) / KC;
    // chunks past the end are the last chunk again: loaded, never multiplied
    auto clampc = [&](int c) { return c < nchunks ? c : nchunks - 1; };
    using S0 = std::integral_constant<int, 0>;
    using S1 = std::integral_constant<int, 1>;

    // this group's chunks: wgrp, wgrp + NWG, ...; every group runs the same number of iterations
    // (the barriers are the work-group's)
    const int iters = (nchunks + NWG - 1) / NWG;
    load_chunk(clampc(wgrp), S0{});
    load_chunk(clampc(wgrp + NWG), S1{});
    store_chunk(0, S0{});
    __syncthreads();

    // Iteration c: LDS buffer P holds chunk c, register set P is free, set P^1 holds the group's next chunk.
    auto iteration = [&](int c, auto par_c) {
        constexpr int P = decltype(par_c)::value;
        load_chunk(clampc(c + 2 * NWG), std::integral_constant<int, P>{});
        // keep the loads ahead of the MFMAs (the scheduler would sink them to their first use)
        __builtin_amdgcn_sched_barrier(0);
        const float* a = lds_a + P * A_SZ + (wm * MB * 32 + r32) * WS + 2 * h;
        const float* b = NT ? lds_b + P * B_SZ + (wn * NB * 32 + r32) * WS + 2 * h
                            : lds_b + P * B_SZ + (2 * h) * LDB + wn * NB * 32 + r32;
        if (NWG == 1 || c < nchunks) {          // a group may have one chunk fewer than the others
#pragma unroll
            for (int j = 0; j < KC / 4; ++j) {
                f32x2 av[MB], bv[NB];
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
                    av[mb] = *reinterpret_cast<const f32x2*>(a + mb * 32 * WS + 4 * j);
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    if (NT) {
                        bv[nb] = *reinterpret_cast<const f32x2*>(b + nb * 32 * WS + 4 * j);
                    } else {
                        bv[nb][0] = b[(4 * j) * LDB + nb * 32];
                        bv[nb][1] = b[(4 * j + 1) * LDB + nb * 32];
                    }
                }
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
        iteration(wgrp + i * NWG, S0{});
        if (i + 1 < iters) iteration(wgrp + (i + 1) * NWG, S1{});
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
            for (int r = 0; r < 16; ++r) acc[0][0][r] += plds[o * REGION + (wave * 16 + r) * 64 + lane];
    }

    // accumulator register r of lane (h, r32): row 8*(r/4) + 4*h + r%4, column r32 of the block
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            const int col = n0 + (wn * NB + nb) * 32 + r32;
            if (col >= N) continue;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = m0 + (wm * MB + mb) * 32 + 8 * (r / 4) + 4 * h + (r % 4);
                // 32 lanes write one whole 128-byte run of a row; C is not read again (non-temporal:
                // no dirty lines left for the end of the kernel)
                if (row < M) __builtin_nontemporal_store(acc[mb][nb][r], &C[(int64_t)row * p.ldc + col]);
            }
        }
}

}  // namespace gpipe
}  // namespace anr
