// fp32 GEMM on the MFMA units of gfx950: the GMM operator (C = A.B, Sec. 4.1 of
// arXiv 2006.06762) and the batch matmul of the TBS subgraph (Sec. 7.2) in its
// A.B^T form.
//
// Work-group tile BM x BN, 256 threads = 4 waves in a 2 x 2 grid; every wave
// owns a (BM/2) x (BN/2) block of C as 32x32 MFMA accumulators.  Operand tiles
// go HBM/L2 -> registers -> LDS (double buffered, one barrier per K step), and
// LDS -> registers with 16-byte reads: the 32x32x2 MFMA takes, from lane l,
// A[l%32][k] for one k chosen by l/32, and the order in which the k values of a
// tile are fed is free as long as A and B agree, so each half-wave reads four
// consecutive k of "its" row with one ds_read_b128 and spends them on four MFMAs.
#include "anr_device.h"
#include "anr_kernels.h"
#include "gemm_pipe_kernel.h"

namespace anr {
namespace {

template <int BM, int BN, int BK, bool NT, bool VEC>
__global__ __launch_bounds__(256) void gemm_kernel(const GemmArgs p)
{
    constexpr int WM = BM / 2, WN = BN / 2;
    constexpr int MB = WM / 32, NB = WN / 32;
    constexpr int LDA_S = BK + 4;
    constexpr int LDB_S = NT ? (BK + 4) : (BN + 4);
    constexpr int A_TILE = BM * LDA_S;
    constexpr int B_TILE = NT ? BN * LDB_S : BK * LDB_S;
    constexpr int KQ = BK / 4;                 // float4 per tile row of A (and of B when NT)
    constexpr int NQ = BN / 4;                 // float4 per tile row of B when NN
    constexpr int NA = BM * KQ / 256;
    constexpr int NBU = (NT ? BN * KQ : BK * NQ) / 256;
    static_assert(NA >= 1 && NBU >= 1, "tile too small for 256 threads");

    __shared__ __attribute__((aligned(16))) float As[2][A_TILE];
    __shared__ __attribute__((aligned(16))) float Bs[2][B_TILE];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int r32 = lane & 31, h = lane >> 5;
    const int wm0 = (wave >> 1) * WM, wn0 = (wave & 1) * WN;
    const int bm0 = blockIdx.y * BM, bn0 = blockIdx.x * BN;
    const int zo = blockIdx.z / p.batch_inner, zi = blockIdx.z % p.batch_inner;
    const float* __restrict__ A = p.A + zo * p.sAo + zi * p.sAi;
    const float* __restrict__ B = p.B + zo * p.sBo + zi * p.sBi;
    float* __restrict__ C = p.C + zo * p.sCo + zi * p.sCi;
    const int M = p.M, N = p.N, K = p.K;

    f32x4 ra[NA], rb[NBU];

    // tile rows are matrix rows, k contiguous (A always; B when NT)
    auto load_rows = [&](const float* __restrict__ base, int64_t ld, int row0, int rows_total,
                         int kt, auto& reg) {
        constexpr int count = sizeof(reg) / sizeof(f32x4);
#pragma unroll
        for (int i = 0; i < count; ++i) {
            const int u = tid + i * 256;
            const int row = u / KQ, kq = u % KQ;
            const int gr = row0 + row, gk = kt * BK + kq * 4;
            f32x4 v = zero4();
            if (VEC) {
                // branch-free: out-of-range units re-read a valid address and are zeroed by a
                // select (a load under a divergent branch would serialise the loads of a tile)
                const bool in = gr < rows_total && gk < K;
                const float* src = base + (int64_t)(in ? gr : 0) * ld + (in ? gk : 0);
                const f32x4 t = ldg4(src);
                v = in ? t : v;
            } else if (gr < rows_total) {
                const float* src = base + (int64_t)gr * ld + gk;
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    if (gk + c < K) v[c] = src[c];
            }
            reg[i] = v;
        }
    };
    auto store_rows = [&](float* tile, int ld_s, const auto& reg) {
        constexpr int count = sizeof(reg) / sizeof(f32x4);
#pragma unroll
        for (int i = 0; i < count; ++i) {
            const int u = tid + i * 256;
            const int row = u / KQ, kq = u % KQ;
            *reinterpret_cast<f32x4*>(&tile[row * ld_s + kq * 4]) = reg[i];
        }
    };
    auto load_b_nn = [&](int kt) {
#pragma unroll
        for (int i = 0; i < NBU; ++i) {
            const int u = tid + i * 256;
            const int k = u / NQ, nq = u % NQ;
            const int gk = kt * BK + k, gn = bn0 + nq * 4;
            f32x4 v = zero4();
            if (VEC) {
                const bool in = gk < K && gn < N;
                const float* src = B + (int64_t)(in ? gk : 0) * p.ldb + (in ? gn : 0);
                const f32x4 t = ldg4(src);
                v = in ? t : v;
            } else if (gk < K) {
                const float* src = B + (int64_t)gk * p.ldb + gn;
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    if (gn + c < N) v[c] = src[c];
            }
            rb[i] = v;
        }
    };
    auto store_b_nn = [&](float* tile) {
#pragma unroll
        for (int i = 0; i < NBU; ++i) {
            const int u = tid + i * 256;
            const int k = u / NQ, nq = u % NQ;
            *reinterpret_cast<f32x4*>(&tile[k * LDB_S + nq * 4]) = rb[i];
        }
    };
    auto load_tiles = [&](int kt) {
        load_rows(A, p.lda, bm0, M, kt, ra);
        if (NT) load_rows(B, p.ldb, bn0, N, kt, rb);
        else load_b_nn(kt);
    };
    auto store_tiles = [&](int buf) {
        store_rows(As[buf], LDA_S, ra);
        if (NT) store_rows(Bs[buf], LDB_S, rb);
        else store_b_nn(Bs[buf]);
    };

    f32x16 acc[MB][NB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mb][nb][r] = 0.f;

    const int nk = (K + BK - 1) / BK;
    load_tiles(0);
    store_tiles(0);
    __syncthreads();

    for (int kt = 0; kt < nk; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < nk) load_tiles(kt + 1);
        // keep the loads ahead of the MFMAs: the scheduler would sink them to their first use
        // (the LDS stores after the loop) and their latency would not overlap the tile's MFMAs
        __builtin_amdgcn_sched_barrier(0);

        const float* as = As[buf];
        const float* bs = Bs[buf];
#pragma unroll
        for (int kk = 0; kk < BK / 8; ++kk) {
            f32x4 a[MB];
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
                a[mb] = *reinterpret_cast<const f32x4*>(&as[(wm0 + mb * 32 + r32) * LDA_S + kk * 8 + 4 * h]);
            if (NT) {
                f32x4 b[NB];
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
                    b[nb] = *reinterpret_cast<const f32x4*>(&bs[(wn0 + nb * 32 + r32) * LDB_S + kk * 8 + 4 * h]);
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                        for (int nb = 0; nb < NB; ++nb)
                            acc[mb][nb] = mfma32(a[mb][j], b[nb][j], acc[mb][nb]);
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float* brow = &bs[(kk * 8 + 4 * h + j) * LDB_S + wn0 + NB * r32];
                    float b[NB];
                    if (NB == 2) {
                        const f32x2 t = *reinterpret_cast<const f32x2*>(brow);
                        b[0] = t[0];
                        b[NB - 1] = t[1];
                    } else {
#pragma unroll
                        for (int nb = 0; nb < NB; ++nb) b[nb] = brow[nb];
                    }
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                        for (int nb = 0; nb < NB; ++nb)
                            acc[mb][nb] = mfma32(a[mb][j], b[nb], acc[mb][nb]);
                }
            }
        }

        if (kt + 1 < nk) store_tiles(buf ^ 1);
        __syncthreads();
    }

    // Epilogue.  Register r of a 32x32 accumulator is row 8*(r/4) + 4*h + r%4, column r32
    // of the block; when NN, block nb holds the columns NB*r32 + nb of the wave's strip.
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int row = bm0 + wm0 + mb * 32 + 8 * (r / 4) + 4 * h + (r % 4);
            if (row >= M) continue;
            float* crow = C + (int64_t)row * p.ldc;
            if (NT) {
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    const int col = bn0 + wn0 + nb * 32 + r32;
                    if (col < N) crow[col] = acc[mb][nb][r];
                }
            } else {
                const int col = bn0 + wn0 + NB * r32;
                if (VEC && NB == 2) {
                    if (col < N) {
                        f32x2 v = {acc[mb][0][r], acc[mb][NB - 1][r]};
                        *reinterpret_cast<f32x2*>(crow + col) = v;
                    }
                } else {
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb)
                        if (col + nb < N) crow[col + nb] = acc[mb][nb][r];
                }
            }
        }
    }
}

// Row softmax in place (TBS): one wave per row of length n <= 1024.
__global__ __launch_bounds__(256) void softmax_rows_kernel(float* out, int64_t rows, int n,
                                                           int rows_per_mat, int mats_inner,
                                                           int64_t s_o, int64_t s_i, int64_t ld)
{
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const int64_t mat = row / rows_per_mat;
    const int i = (int)(row % rows_per_mat);
    float* v = out + (mat / mats_inner) * s_o + (mat % mats_inner) * s_i + (int64_t)i * ld;
    float x[16];
    float mx = -INFINITY;
#pragma unroll
    for (int t = 0; t < 16; ++t) {
        const int j = lane + t * 64;
        x[t] = j < n ? v[j] : -INFINITY;
        mx = fmaxf(mx, x[t]);
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
    float sum = 0.f;
#pragma unroll
    for (int t = 0; t < 16; ++t) {
        const int j = lane + t * 64;
        x[t] = j < n ? expf(x[t] - mx) : 0.f;
        sum += x[t];
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) sum += __shfl_xor(sum, o);
    const float inv = 1.0f / sum;
#pragma unroll
    for (int t = 0; t < 16; ++t) {
        const int j = lane + t * 64;
        if (j < n) v[j] = x[t] * inv;
    }
}


// ---------------------------------------------------------------------------------------
// Small problems (few output tiles, long K), e.g. the 512^3 GMM of the benchmark: 268 MFLOP
// are 64 MFMAs per SIMD if and only if all 1024 SIMDs take part, so a work-group owns one
// 32 x 32 tile of C and its NW waves split K, NST stages of 32 each (K = 128, 256, 512 run 4, 8,
// 16 waves with one stage each).  The waves share no operand; each stages its own slices of A
// (32 rows x 32 NST) and B (32 NST x 32) through a private region of LDS purely to turn fully
// coalesced 16-byte global loads (whole 128-byte lines, eight per instruction) into the
// per-lane operand order of the MFMA: issuing the operand loads straight from global memory
// costs 2.8 us of address-unit time for this shape, the staged form a third of that.  All loads
// of a wave are in flight before its first MFMA.  The partial tiles meet in LDS once; every
// wave then sums and stores 16 / NW accumulator registers.  Work-group ids are mapped to tiles
// so that the 32 work-groups that land on one XCD (ids are dealt round-robin over the 8 XCDs)
// form a compact block of C and share their panels of A and B in that XCD's L2.
// The kernel is a chain of latencies (start-up and first access ~1 us, load issue, one memory
// round trip, LDS staging, MFMAs, reduction, store), not a throughput problem: with four waves
// of four stages each (512^3) the phases took 1.6 + 2.9 + 0.35 + 0.45 us; sixteen waves of one
// stage put four waves on every SIMD, so one wave's staging overlaps another's MFMAs and each
// wave issues 8 loads instead of 32: 6.5 -> 5.8 us cold.  Weaving the later stages' loads
// between the MFMAs of the four-stage form had changed nothing.  Also measured and dropped: A
// brought to LDS by direct-to-LDS loads (unit q of row r on slot q ^ (r % 8), so the rows can sit
// 128 bytes apart without bank conflicts) and the B operand of every k-step loaded straight into
// its register (for a fixed k the 32 lanes of a half-wave read one whole line of B): no LDS store
// and no strided LDS read is left, yet 6.0 against 5.6 us cold -- sixteen 4-byte loads per lane
// are sixteen more trips through the address unit than the four 16-byte loads they replace.

constexpr int kKsLd = 36;                       // LDS row stride (floats) of a 32-wide stage
constexpr int kKsStage = 2 * 32 * kKsLd;        // floats per stage: A block then B block

template <int NST, int NW>
__global__ __launch_bounds__(64 * NW) void gemm_tile32_ksplit_kernel(const GemmArgs p, int tiles_m, int tiles_n,
                                                                     int xcd_map)
{
    static_assert(16 % NW == 0, "a wave finishes 16 / NW accumulator registers");
    extern __shared__ __attribute__((aligned(16))) float lds[];   // [NW waves][NST][kKsStage]

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int r32 = lane & 31, h = lane >> 5;

    int tm, tn;
    const int w = blockIdx.x;
    if (xcd_map) {
        const int xcd = w & 7, slot = w >> 3;
        const int rows_per = tiles_m / 4, cols_per = tiles_n / 2;
        tm = (xcd >> 1) * rows_per + slot / cols_per;
        tn = (xcd & 1) * cols_per + slot % cols_per;
    } else {
        tm = w / tiles_n;
        tn = w % tiles_n;
    }
    const float* __restrict__ A = p.A + blockIdx.z * p.sAo;
    const float* __restrict__ B = p.B + blockIdx.z * p.sBo;
    float* __restrict__ C = p.C + blockIdx.z * p.sCo;

    // staging unit of a lane: row lane/8 (+8 per t), 16 bytes at column 4*(lane%8)
    const int srow = lane >> 3, sq = (lane & 7) * 4;
    const int kbase = wave * (NST * 32);
    const float* __restrict__ ap = A + (int64_t)(tm * 32 + srow) * p.lda + kbase + sq;
    const float* __restrict__ bp = B + (int64_t)(kbase + srow) * p.ldb + tn * 32 + sq;
    float* const wl = lds + wave * (NST * kKsStage);

    f32x4 ra[NST][4], rb[NST][4];
#pragma unroll
    for (int s = 0; s < NST; ++s) {
#pragma unroll
        for (int t = 0; t < 4; ++t) ra[s][t] = ldg4(ap + (int64_t)(8 * t) * p.lda + s * 32);
#pragma unroll
        for (int t = 0; t < 4; ++t) rb[s][t] = ldg4(bp + (int64_t)(s * 32 + 8 * t) * p.ldb);
    }
    // keep every load above the first use (the scheduler would otherwise sink each load to
    // its use to save registers, and the wave would see one memory latency per stage)
    __builtin_amdgcn_sched_barrier(0);

    f32x16 acc, acc2;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = acc2[r] = 0.f;
#pragma unroll
    for (int s = 0; s < NST; ++s) {
        float* st = wl + s * kKsStage;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            *reinterpret_cast<f32x4*>(&st[(srow + 8 * t) * kKsLd + sq]) = ra[s][t];
            *reinterpret_cast<f32x4*>(&st[32 * kKsLd + (srow + 8 * t) * kKsLd + sq]) = rb[s][t];
        }
        // the staging region is private to the wave: its LDS accesses execute in order, so the
        // reads below see the writes above without a work-group barrier (which would tie every
        // wave to the slowest wave's loads, stage by stage); the fence only stops the compiler
        // from moving the reads up
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            const f32x4 av = *reinterpret_cast<const f32x4*>(&st[r32 * kKsLd + kk * 8 + 4 * h]);
            float bv[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) bv[e] = st[32 * kKsLd + (kk * 8 + 4 * h + e) * kKsLd + r32];
            acc = mfma32(av[0], bv[0], acc);
            acc2 = mfma32(av[1], bv[1], acc2);
            acc = mfma32(av[2], bv[2], acc);
            acc2 = mfma32(av[3], bv[3], acc2);
        }
    }

    __syncthreads();            // every wave is done with its staging region: reuse it
    float* red = lds;
#pragma unroll
    for (int r = 0; r < 16; ++r) red[(wave * 16 + r) * 64 + lane] = acc[r] + acc2[r];
    __syncthreads();
    // wave w finishes accumulator registers (16 / NW) w ...: register r is row 8 (r / 4) + 4 h + r % 4
#pragma unroll
    for (int q = 0; q < 16 / NW; ++q) {
        const int r = wave * (16 / NW) + q;
        float v = 0.f;
#pragma unroll
        for (int o = 0; o < NW; ++o) v += red[(o * 16 + r) * 64 + lane];
        C[(int64_t)(tm * 32 + 8 * (r / 4) + 4 * h + (r % 4)) * p.ldc + tn * 32 + r32] = v;
    }
}

template <int NST, int NW>
hipError_t launch_ksplit(const GemmArgs& a, hipStream_t stream)
{
    const int tiles_m = a.M / 32, tiles_n = a.N / 32;
    const size_t lds_bytes = sizeof(float) * NW * NST * kKsStage;
    auto kern = gemm_tile32_ksplit_kernel<NST, NW>;
    if (lds_bytes > 64 * 1024) {
        static LdsLimit granted;
        hipError_t e = raise_lds_limit(reinterpret_cast<const void*>(kern), lds_bytes, granted);
        if (e != hipSuccess) return e;
    }
    const int xcd_map = (tiles_m % 4 == 0) && (tiles_n % 2 == 0);
    return launch_kernel(kern, dim3(tiles_m * tiles_n, 1, a.batch), dim3(64 * NW), lds_bytes, stream, a, tiles_m,
                         tiles_n, xcd_map);
}

template <int BM, int BN, int BK, bool NT, bool VEC>
hipError_t launch_variant(const GemmArgs& a, hipStream_t stream)
{
    dim3 grid((a.N + BN - 1) / BN, (a.M + BM - 1) / BM, a.batch);
    return launch_kernel(gemm_kernel<BM, BN, BK, NT, VEC>, grid, dim3(256), 0, stream, a);
}


template <int BM, int BN, bool NT, int NWG = 1>
hipError_t launch_pipe(const GemmArgs& a, hipStream_t stream)
{
    const int tiles_m = (a.M + BM - 1) / BM, tiles_n = (a.N + BN - 1) / BN;
    const size_t lds_bytes = NWG * gpipe::Tiles<BM, BN, NT>::lds_bytes;
    auto kern = gpipe::gemm_pipe_kernel<BM, BN, NT, NWG>;
    if (lds_bytes > 48 * 1024) {
        static LdsLimit granted;
        hipError_t e = raise_lds_limit(reinterpret_cast<const void*>(kern), lds_bytes, granted);
        if (e != hipSuccess) return e;
    }
    return launch_kernel(kern, dim3((unsigned)(tiles_m * tiles_n), 1, a.batch), dim3(256 * NWG), lds_bytes, stream, a,
                         tiles_m, tiles_n);
}

// Tile for the pipelined kernel: the largest that still puts two work-groups on every CU (they
// fill each other's barrier and staging bubbles: 82 % MFMA utilisation against 55 % for a lone
// work-group); large tiles also pull fewer operand bytes per FLOP into the CU.
template <bool NT>
hipError_t launch_pipe_any(const GemmArgs& a, hipStream_t stream)
{
    auto tiles = [&](int bm, int bn) {
        return (int64_t)((a.M + bm - 1) / bm) * ((a.N + bn - 1) / bn) * a.batch;
    };
    if (tiles(128, 128) >= 512) return launch_pipe<128, 128, NT>(a, stream);
    if (tiles(128, 64) >= 512) return launch_pipe<128, 64, NT>(a, stream);
    // at most one 64 x 64 tile per CU and a long reduction: groups of waves share the chunk chain
    // (1024^3: 28.6 us with one group)
    const int nchunks = (a.K + gpipe::KC - 1) / gpipe::KC;
    if (tiles(64, 64) <= 256 && nchunks >= 32) return launch_pipe<64, 64, NT, 4>(a, stream);
    if (tiles(64, 64) <= 256 && nchunks >= 8) return launch_pipe<64, 64, NT, 2>(a, stream);
    return launch_pipe<64, 64, NT>(a, stream);
}

}  // namespace

hipError_t launch_gemm(const GemmArgs& a, hipStream_t stream)
{
    const bool strides4 = (a.sAo % 4 == 0) && (a.sAi % 4 == 0) && (a.sBo % 4 == 0) &&
                          (a.sBi % 4 == 0) && (a.sCo % 4 == 0) && (a.sCi % 4 == 0);
    bool vec = is_aligned16(a.A) && is_aligned16(a.B) && is_aligned16(a.C) && strides4 &&
               (a.K % 4 == 0) && (a.lda % 4 == 0) && (a.ldb % 4 == 0) && (a.ldc % 4 == 0);
    if (!a.b_is_nk) vec = vec && (a.N % 4 == 0);

    const int64_t tiles128 = (int64_t)((a.M + 127) / 128) * ((a.N + 127) / 128) * a.batch;
    const bool big = tiles128 >= 192;   // enough 128x128 tiles to occupy most of the 256 CUs

    // few tiles and a long reduction: one 32x32 tile per work-group, K split over its waves
    const int64_t tiles32 = (int64_t)(a.M / 32) * (a.N / 32) * a.batch;
    if (!a.b_is_nk && !a.softmax_rows && (a.M % 32 == 0) && (a.N % 32 == 0) && tiles32 <= 1024 &&
        a.batch_inner == 1 && is_aligned16(a.A) && is_aligned16(a.B) && (a.lda % 4 == 0) && (a.ldb % 4 == 0) &&
        (a.sAo % 4 == 0) && (a.sBo % 4 == 0) && a.batch <= 65535) {
        if (a.K == 128) return launch_ksplit<1, 4>(a, stream);
        if (a.K == 256) return launch_ksplit<1, 8>(a, stream);
        if (a.K == 512) return launch_ksplit<1, 16>(a, stream);
    }

    hipError_t err;
    // 32-bit byte offsets inside one matrix, grid limits
    const int64_t a_ext = (int64_t)(a.M - 1) * a.lda + a.K;
    const int64_t b_ext = a.b_is_nk ? (int64_t)(a.N - 1) * a.ldb + a.K : (int64_t)(a.K - 1) * a.ldb + a.N;
    const bool pipe = vec && a_ext < ((int64_t)1 << 29) && b_ext < ((int64_t)1 << 29) && a.batch <= 65535 &&
                      (int64_t)((a.M + 63) / 64) * ((a.N + 63) / 64) < ((int64_t)1 << 31);
    if (pipe && !a.b_is_nk) {
        err = launch_pipe_any<false>(a, stream);
    } else if (a.b_is_nk) {
        if (big) err = vec ? launch_variant<128, 128, 16, true, true>(a, stream)
                           : launch_variant<128, 128, 16, true, false>(a, stream);
        else     err = vec ? launch_variant<64, 64, 16, true, true>(a, stream)
                           : launch_variant<64, 64, 16, true, false>(a, stream);
    } else {
        if (big) err = vec ? launch_variant<128, 128, 16, false, true>(a, stream)
                           : launch_variant<128, 128, 16, false, false>(a, stream);
        else     err = vec ? launch_variant<64, 64, 16, false, true>(a, stream)
                           : launch_variant<64, 64, 16, false, false>(a, stream);
    }
    if (err != hipSuccess) return err;

    if (a.softmax_rows) err = launch_softmax_rows(a, stream);
    return err;
}

hipError_t launch_softmax_rows(const GemmArgs& a, hipStream_t stream)
{
    const int64_t rows = (int64_t)a.batch * a.M;
    return launch_kernel(softmax_rows_kernel, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, stream,
                         a.C, rows, a.N, a.M, a.batch_inner, a.sCo, a.sCi, a.ldc);
}

}  // namespace anr
