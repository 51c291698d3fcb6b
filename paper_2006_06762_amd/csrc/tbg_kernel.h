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
// (10.8 us: a wave that is stuck issuing a long run of loads cannot multiply).  Three independent work-groups per CU keep more requests
// in flight and win.  Writing the tile through LDS so that every store instruction covers four
// whole 256-byte rows instead of two 128-byte pieces was also slower (8.7 against 8.4 us).
#pragma once
#include "anr_device.h"
#include "anr_kernels.h"

namespace anr {
namespace tbg {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

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
    FastDiv d_tiles_j, d_tiles_i, d_h;   // divisors tiles_j, tiles_i, H (tbg_tile64_kernel)
};


__global__ __launch_bounds__(256) void tbg_tile_kernel(const Args p)
{
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
        if (d0 > 0) __syncthreads();             // previous chunk fully consumed
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            *reinterpret_cast<f32x4*>(&qs[(srow + 16 * u) * kLds + sd]) = din ? rq[u] : zero4();
            *reinterpret_cast<f32x4*>(&ks[(srow + 16 * u) * kLds + sd]) = din ? rk[u] : zero4();
        }
        __syncthreads();

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
}

// The same tile for whole tiles and whole chunks (S and D multiples of 64: every shape of the
// paper's list) with the address arithmetic taken out of the vector ALU.  Counted on the kernel
// above, a wave spent about as many cycles on vector-ALU instructions (64-bit addresses of 8
// loads and 16 stores, bounds, the tile index's divisions, two accumulators to initialise and
// add) as on its 32 MFMAs, and with three waves per SIMD that is matrix time lost.  Here a lane
// holds one byte offset per operand and one for the output; tile, row group and chunk ride in
// the scalar offset of buffer loads and stores; one accumulator (consecutive MFMAs on one
// accumulator do not stall on this hardware).
__global__ __launch_bounds__(256) void tbg_tile64_kernel(const Args p)
{
    __shared__ __attribute__((aligned(16))) float qs[kTile * kLds];
    __shared__ __attribute__((aligned(16))) float ks[kTile * kLds];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int r32 = lane & 31, h2 = lane >> 5;
    int t = blockIdx.x;
    if (p.xcd_chunk > 0) t = (t & 7) * p.xcd_chunk + (t >> 3);
    int q1 = p.d_tiles_j.div(t);
    const int tj = t - q1 * p.tiles_j;
    int q2 = p.d_tiles_i.div(q1);
    const int ti = q1 - q2 * p.tiles_i;
    const int b = p.d_h.div(q2), hh = q2 - b * p.H;
    const int i0 = ti * kTile, j0 = tj * kTile;

    const float* qb = p.q + b * p.qs_b + hh * p.qs_h;
    const float* kb = p.k + b * p.ks_b + hh * p.ks_h;
    float* ob = p.out + b * p.os_b + hh * p.os_h;
    const int qs_s = (int)p.qs_s, ks_s = (int)p.ks_s, os_i = (int)p.os_i;
    const __amdgpu_buffer_rsrc_t qrsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float*>(qb), 0, 4 * ((p.S - 1) * qs_s + p.D), 0x00020000);
    const __amdgpu_buffer_rsrc_t krsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float*>(kb), 0, 4 * ((p.S - 1) * ks_s + p.D), 0x00020000);
    const __amdgpu_buffer_rsrc_t orsrc = __builtin_amdgcn_make_buffer_rsrc(
        ob, 0, 4 * ((p.S - 1) * os_i + p.S), 0x00020000);

    // staging: thread -> (row = tid / 16 + 16*u, 16 bytes at d = 4 * (tid % 16)), u = 0..3
    const int srow = tid >> 4, sd = (tid & 15) * 4;
    const int wi = (wave >> 1) * 32, wj = (wave & 1) * 32;   // this wave's 32 x 32 block
    const int voffq = 4 * (srow * qs_s + sd), voffk = 4 * (srow * ks_s + sd);

    f32x16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;

    for (int d0 = 0; d0 < p.D; d0 += kChunk) {
        f32x4 rq[4], rk[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            rq[u] = __builtin_bit_cast(
                f32x4, __builtin_amdgcn_raw_buffer_load_b128(qrsrc, voffq, 4 * ((i0 + 16 * u) * qs_s + d0), 0));
            rk[u] = __builtin_bit_cast(
                f32x4, __builtin_amdgcn_raw_buffer_load_b128(krsrc, voffk, 4 * ((j0 + 16 * u) * ks_s + d0), 0));
        }
        if (d0 > 0) __syncthreads();             // previous chunk fully consumed
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            *reinterpret_cast<f32x4*>(&qs[(srow + 16 * u) * kLds + sd]) = rq[u];
            *reinterpret_cast<f32x4*>(&ks[(srow + 16 * u) * kLds + sd]) = rk[u];
        }
        __syncthreads();

        f32x4 a[8], bb[8];
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) {
            a[kk] = *reinterpret_cast<const f32x4*>(&qs[(wi + r32) * kLds + kk * 8 + 4 * h2]);
            bb[kk] = *reinterpret_cast<const f32x4*>(&ks[(wj + r32) * kLds + kk * 8 + 4 * h2]);
        }
#pragma unroll
        for (int kk = 0; kk < 8; ++kk)
#pragma unroll
            for (int e = 0; e < 4; ++e) acc = mfma32(a[kk][e], bb[kk][e], acc);
    }

    // register r of lane (h2, r32): row 8*(r/4) + 4*h2 + r%4, column r32 of the block.  A store
    // instruction writes two whole 128-byte lines; the scores are not read again, so the stores are
    // non-temporal (9.4 -> 7.0 us with cold buffers: the lines need no write-back at the kernel's end)
    const int voffo = 4 * ((wi + 4 * h2) * os_i + wj + r32);
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const float v = acc[r];
        __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v), orsrc, voffo,
                                              4 * ((i0 + 8 * (r / 4) + (r % 4)) * os_i + j0), kBufferNonTemporal);
    }
}

// ---------------------------------------------------------------------------------------
// Full TBS for S <= 128: the batch matmul with the row softmax fused (Sec. 7.2: two
// transposes, one batch matmul, one softmax), so a row of scores never leaves the chip
// before it is normalised.
//
// Work-group = a block of queries x ALL keys of one (b, h); a wave owns 32 keys.  The benchmark
// shape (S = 128: 32 queries per work-group, wave w owns keys 32w .. 32w + 31) gives 768
// work-groups = 3 per CU, 3 waves on every SIMD.  The q rows and
// the k panel are staged in LDS with fully coalesced 16-byte loads (loading the MFMA operand
// registers straight from global memory was measured at 14.3 us for the matmul alone: a lane
// is a matrix row there, so every request touches 32 cache lines for 32 bytes each).
//
// The wave computes the TRANSPOSED block  T = k_blk . q_blk^T  (keys are MFMA rows, queries
// MFMA columns).  In the accumulator layout of v_mfma_f32_32x32x2_f32 a lane then holds 16
// keys of ONE query, so a softmax row reduces inside the lane: 15 max / add operations, one
// exchange with the other half-wave, one exchange through LDS between the four waves.  The
// probabilities go back through LDS (over the k panel) so that each store instruction writes
// two complete output rows.
//
// The four waves are KB key blocks x 4/KB query blocks of 32: KB = 4 for S <= 128 (32 queries
// per work-group), 2 for S <= 64 (64 queries), 1 for S <= 32 (128 queries), so a short sequence
// neither loads nor multiplies key rows it does not have.
// UT = 16-byte staging units per thread: ceil((32 * 4/KB + 32 * KB) * (min(D, 64)/4) / 256).
constexpr int kMaxKeys = 128;

template <int KB>
struct TbsShape {
    static constexpr int QBK = 4 / KB;            // query blocks per work-group
    static constexpr int rows_q = 32 * QBK, rows_k = 32 * KB;
    static constexpr int ldp = rows_k + 4;        // row stride of the staged probabilities
};

//
// WHOLE: S == 32 * KB, a multiple of the work-group's query rows, and D a multiple of 64 (every
// shape of the paper's list).  Nothing is then
// clamped or masked, a thread's staging units are whole q units followed by whole k units, and
// the loads are buffer loads with one byte offset per unit in a register and the chunk in the
// scalar offset; the tile index is decoded with multiply-shift divisions.  Vector-ALU
// instructions of any wave on a SIMD cost matrix time (about eight cycles each), and the general
// form spends more of them on addresses than the softmax needs.
template <int UT, bool SOFTMAX, int KB, bool WHOLE>
__global__ __launch_bounds__(256) void tbs_rows32_kernel(const Args p, int ld, int vec_store)
{
    using T = TbsShape<KB>;
    constexpr int QBK = T::QBK, kRowsQ = T::rows_q, kRowsK = T::rows_k, kLdP = T::ldp;
    extern __shared__ __attribute__((aligned(16))) float panel[];   // q rows, then k rows
    __shared__ float red[2][QBK][KB][32];
    float* const qs = panel;
    float* const ks = panel + kRowsQ * ld;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wv = tid >> 6;
    const int wave = wv % KB, qblk = wv / KB;   // key block, query block
    const int r32 = lane & 31, h2 = lane >> 5;
    // work item = (b*H + h) * tiles_i + ti, tiles_i = ceil(S / rows_q).  Work-group ids are dealt
    // round-robin over the 8 XCDs; every XCD gets a contiguous range of items, so that the query
    // tiles of one head, which all read its k panel, meet in one L2 (31.6 -> 12.7 MB fetched).
    int item = blockIdx.x;
    if (p.xcd_chunk > 0) item = (item & 7) * p.xcd_chunk + (item >> 3);
    int ti, bh, hh, b;
    if (WHOLE) {
        bh = p.d_tiles_i.div(item);
        ti = item - bh * p.tiles_i;
        b = p.d_h.div(bh);
        hh = bh - b * p.H;
    } else {
        ti = item % p.tiles_i;
        bh = item / p.tiles_i;
        hh = bh % p.H;
        b = bh / p.H;
    }
    const int i0 = ti * kRowsQ;

    const float* __restrict__ qb = p.q + b * p.qs_b + hh * p.qs_h;
    const float* __restrict__ kb = p.k + b * p.ks_b + hh * p.ks_h;

    // The reduction runs in chunks of 64 columns of d (the panel in LDS is 64 wide, so three
    // work-groups fit a CU for any D); the next chunk waits in registers while this one is
    // multiplied.  Staging unit u of thread tid: unit index tid + 256*u of the
    // (rows_q + rows_k) x (chunk/4) panel, walked without a division per unit.
    const int dc = p.D < kChunk ? p.D : kChunk;
    const int dq = dc >> 2;
    const int row_step = 256 / dq, col_step = 256 - row_step * dq;
    constexpr int rows_all = kRowsQ + kRowsK;
    int srow = tid / dq, scol = tid - srow * dq;
    f32x4 rg[UT];
    const float* rowp[UT];
    int lds_off[UT], ucol[UT];
    // WHOLE: 16 units per row, 16 rows per pass of the work-group; units 0 .. UQ-1 are q rows,
    // the rest k rows
    constexpr int UQ = kRowsQ / 16;
    uint32_t voff[UT];
    const __amdgpu_buffer_rsrc_t qrsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float*>(qb), 0, WHOLE ? 4 * ((p.S - 1) * (int)p.qs_s + p.D) : 0, 0x00020000);
    const __amdgpu_buffer_rsrc_t krsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float*>(kb), 0, WHOLE ? 4 * ((p.S - 1) * (int)p.ks_s + p.D) : 0, 0x00020000);
    if (WHOLE) {
        static_assert(!WHOLE || UT == (kRowsQ + kRowsK) / 16, "whole form: 16 units per row");
        const int r16 = tid >> 4, c16 = (tid & 15) * 4;
#pragma unroll
        for (int u = 0; u < UT; ++u) {
            const int row = r16 + 16 * u;                          // row of the panel: q rows, then k rows
            voff[u] = u < UQ ? 4u * (uint32_t)((i0 + row) * (int)p.qs_s + c16)
                             : 4u * (uint32_t)((row - kRowsQ) * (int)p.ks_s + c16);
            lds_off[u] = row * ld + c16;
        }
    } else {
#pragma unroll
        for (int u = 0; u < UT; ++u) {
            const int row = srow < rows_all ? srow : rows_all - 1;      // surplus units repeat the last row
            const bool isq = row < kRowsQ;
            // rows past S re-read row S-1; what they produce is masked or never stored
            int gr = isq ? i0 + row : row - kRowsQ;
            gr = gr < p.S ? gr : p.S - 1;
            rowp[u] = isq ? qb + gr * p.qs_s : kb + gr * p.ks_s;
            ucol[u] = 4 * scol;
            lds_off[u] = row * ld + 4 * scol;
            srow += row_step;
            scol += col_step;
            if (scol >= dq) { scol -= dq; ++srow; }
        }
    }
    auto load_chunk = [&](int d0) {
        if (WHOLE) {
#pragma unroll
            for (int u = 0; u < UT; ++u)
                rg[u] = __builtin_bit_cast(
                    f32x4, __builtin_amdgcn_raw_buffer_load_b128(u < UQ ? qrsrc : krsrc, (int)voff[u], 4 * d0, 0));
        } else {
#pragma unroll
            for (int u = 0; u < UT; ++u) {
                // columns past D (last chunk of a D that is not a multiple of 64) repeat the last four;
                // they land in LDS columns the MFMA loop does not read
                const int col = d0 + ucol[u] < p.D ? d0 + ucol[u] : p.D - 4;
                rg[u] = ldg4(rowp[u] + col);
            }
        }
    };
    auto store_chunk = [&]() {
#pragma unroll
        for (int u = 0; u < UT; ++u) *reinterpret_cast<f32x4*>(&panel[lds_off[u]]) = rg[u];
    };
    load_chunk(0);
    store_chunk();
    __syncthreads();

    // one accumulator: consecutive MFMAs on one accumulator do not stall on this hardware
    f32x16 mm;
#pragma unroll
    for (int r = 0; r < 16; ++r) mm[r] = 0.f;
    const float* arow = ks + (32 * wave + r32) * ld + 4 * h2;
    const float* brow = qs + (32 * qblk + r32) * ld + 4 * h2;
    for (int d0 = 0; d0 < p.D; d0 += kChunk) {
        const bool more = d0 + kChunk < p.D;             // uniform
        if (more) load_chunk(d0 + kChunk);
        __builtin_amdgcn_sched_barrier(0);               // keep the loads ahead of the MFMAs
        const int width = WHOLE ? kChunk : (p.D - d0 < kChunk ? p.D - d0 : kChunk);
#pragma unroll
        for (int d = 0; d < width; d += 8) {             // D is a multiple of 8
            const f32x4 a = *reinterpret_cast<const f32x4*>(arow + d);
            const f32x4 bq = *reinterpret_cast<const f32x4*>(brow + d);
#pragma unroll
            for (int e = 0; e < 4; ++e) mm = mfma32(a[e], bq[e], mm);
        }
        if (more) {
            __syncthreads();                             // every wave is done with this chunk
            store_chunk();
            __syncthreads();
        }
    }
    // the softmax works on ordinary registers (the matrix accumulator stays where the MFMAs left it)
    float acc[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = mm[r];

    // register r of lane (h2, r32): key 32*wave + 8*(r/4) + 4*h2 + r%4, query i0 + 32*qblk + r32
    const int key0 = 32 * wave + 4 * h2;
    if (SOFTMAX) {
        float mx = -INFINITY;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const bool in = WHOLE || key0 + 8 * (r / 4) + (r % 4) < p.S;
            acc[r] = in ? acc[r] : -INFINITY;
            mx = fmaxf(mx, acc[r]);
        }
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        if (h2 == 0) red[0][qblk][wave][r32] = mx;
        __syncthreads();
        // key 0 is always inside, so the maximum over the key blocks is finite
        mx = red[0][qblk][0][r32];
#pragma unroll
        for (int w = 1; w < KB; ++w) mx = fmaxf(mx, red[0][qblk][w][r32]);
        float sum = 0.f;
        // exp(s - mx) = 2^(s * log2(e) - mx * log2(e)): one multiply-add and one exponential per score
        constexpr float kLog2e = 1.44269504088896340736f;
        const float nmx = -mx * kLog2e;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            acc[r] = __builtin_amdgcn_exp2f(fmaf(acc[r], kLog2e, nmx));     // 2^(-inf) = 0 for masked keys
            sum += acc[r];
        }
        sum += __shfl_xor(sum, 32);
        if (h2 == 0) red[1][qblk][wave][r32] = sum;
        __syncthreads();
        sum = red[1][qblk][0][r32];
#pragma unroll
        for (int w = 1; w < KB; ++w) sum += red[1][qblk][w][r32];
        const float inv = 1.0f / sum;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] *= inv;
    } else {
        __syncthreads();                                 // every wave is done reading the k panel
    }

    // transpose through LDS: P[query][key], over the k panel (the launch sizes LDS for both)
    float* const ps = ks;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        f32x4 v;
        v[0] = acc[4 * g]; v[1] = acc[4 * g + 1]; v[2] = acc[4 * g + 2]; v[3] = acc[4 * g + 3];
        *reinterpret_cast<f32x4*>(&ps[(32 * qblk + r32) * kLdP + key0 + 8 * g]) = v;
    }
    __syncthreads();
    // 8*KB lanes cover one row of 32*KB probabilities with 16 bytes each; a store instruction
    // writes 8/KB whole rows, every wave 8*QBK rows in four instructions
    float* __restrict__ ob = p.out + b * p.os_b + hh * p.os_h;
    constexpr int LPR = 8 * KB, RPI = 64 / LPR;
    const int col = 4 * (lane % LPR);
    if (WHOLE && vec_store) {
        // buffer stores: the lane's row inside an instruction and its column in a register, the
        // instruction's first row in the scalar offset
        const int os_i = (int)p.os_i;
        const __amdgpu_buffer_rsrc_t orsrc =
            __builtin_amdgcn_make_buffer_rsrc(ob, 0, 4 * ((p.S - 1) * os_i + p.S), 0x00020000);
        const int voffo = 4 * ((lane / LPR) * os_i + col);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int rl = 8 * QBK * wv + RPI * i;            // uniform over the wave
            const f32x4 v = *reinterpret_cast<const f32x4*>(&ps[(rl + lane / LPR) * kLdP + col]);
            __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v), orsrc, voffo, 4 * (i0 + rl) * os_i, kBufferNonTemporal);
        }
        return;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int rl = 8 * QBK * wv + RPI * i + lane / LPR;
        const int row = i0 + rl;
        const f32x4 v = *reinterpret_cast<const f32x4*>(&ps[rl * kLdP + col]);
        if (WHOLE || row < p.S) {
            float* orow = ob + row * p.os_i;
            if (vec_store && (WHOLE || col + 3 < p.S)) {
                stg4_nt(orow + col, v);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (col + e < p.S) orow[col + e] = v[e];
            }
        }
    }
}

}  // namespace tbg
}  // namespace anr
