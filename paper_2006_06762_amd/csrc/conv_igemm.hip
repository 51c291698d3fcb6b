// C2D and the ConvLayer subgraph (Sec. 7.1, Sec. 7.2 and Appendix C of
// arXiv 2006.06762) as an implicit GEMM on the fp32 MFMA units of gfx950.
//
// GEMM view: rows m = flattened output pixels (n, oh, ow), columns = output
// channels, reduction = (c, r, s).  A work-group owns BM consecutive pixels x BN
// channels and walks the input channels in chunks of CK.
//
// What is staged in LDS is NOT an im2col matrix but the raw input patch the
// tile needs: for every channel of the chunk, the input rows from the first to
// the last one any of the tile's pixels touches, each row with its left/right
// zero padding.  Rows are addressed in "virtual image" coordinates (all images
// stacked, each with its zero rows above and below), so a tile may straddle
// image boundaries without special cases.  Every tap (r, s) then reads the
// same patch at a different constant offset, so an input element crosses
// HBM/L2 -> LDS once per tile instead of R*S times.  Rows and columns that are
// padding are zeroed once, before the first chunk, and never written again.
//
// MFMA: v_mfma_f32_16x16x4_f32.  Lane l feeds pixel (l%16) of a 16-pixel block
// for the A operand and channel (l%16) of a 16-channel block for B; its quarter
// q = l/16 picks which of the four k values of the instruction it supplies.  A
// quarter walks "its" CPG channels of the chunk, tap by tap, so the A address
// of a lane is one per-lane base plus an offset that is uniform over the wave,
// and the B (weight) values of a lane are consecutive floats of the natural
// OIHW order: weights are copied to LDS unpermuted.
//
// The batch-norm scale/shift and ReLU of ConvLayer run on the accumulators in
// the epilogue (Table 1, rule 4: fuse element-wise consumers into the tiled
// node); results are written straight from registers, 16 bytes per lane.
#include "anr_device.h"
#include "conv_internal.h"

namespace anr {
namespace {

struct IgemmGeom {
    int Mtot;       // N*OH*OW
    int HV;         // virtual image height: (OH-1)*stride_h + R
    int VR;         // virtual rows staged per tile (max over tiles)
    int RSL;        // LDS row stride, floats
    int P;          // LDS channel-plane stride, floats
    int XC;         // LDS column of input column 0 (multiple of 4)
    int W4;         // W / 4
    int n_units;    // CK * VR * W4 16-byte staging units per chunk
    int vec_store;  // 4 consecutive pixels of a lane are 16 contiguous, aligned bytes of y
    int ohow;       // OH*OW
};

constexpr int kMaxUnits = 6;

template <int WM_BLK, int WN_BLK, int WAVES_M, int WAVES_N, int R_, int S_, int CPG>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N)
void conv_igemm_kernel(const ConvArgs p, const IgemmGeom g)
{
    constexpr int NT = 64 * WAVES_M * WAVES_N;
    constexpr int BM = 16 * WM_BLK * WAVES_M, BN = 16 * WN_BLK * WAVES_N;
    constexpr int RS9 = R_ * S_;
    constexpr int CK = 4 * CPG;           // channels per chunk
    constexpr int KC = CK * RS9;          // reduction length per chunk
    constexpr int WS = KC + 2;            // LDS stride of one output channel's weights
    constexpr int STEPS = CPG * RS9;      // MFMA k-steps per chunk
    constexpr int WQ = KC / 4;
    constexpr int WU = (BN * WQ + NT - 1) / NT;
    static_assert(KC % 4 == 0, "chunk must be a whole number of float4");

    extern __shared__ __attribute__((aligned(16))) float smem[];
    const int patch_sz = CK * g.P;
    float* const patch = smem;                       // [2][patch_sz]
    float* const wts = smem + 2 * patch_sz;          // [2][BN*WS]

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int i16 = lane & 15, q = lane >> 4;
    const int wave_m = wave / WAVES_N, wave_n = wave % WAVES_N;
    const int m0 = blockIdx.x * BM, co0 = blockIdx.y * BN;

    const int g0 = m0 / p.OW;
    const int v0 = (g0 / p.OH) * g.HV + (g0 % p.OH) * p.stride_h;

    // ---- staging descriptors: which 16 bytes of x go where in the patch (fixed over chunks)
    int goff[kMaxUnits], loff[kMaxUnits];
#pragma unroll
    for (int i = 0; i < kMaxUnits; ++i) {
        const int u = tid + i * NT;
        goff[i] = -1;
        loff[i] = 0;
        if (u < g.n_units) {
            const int per_c = g.VR * g.W4;
            const int ci = u / per_c, rem = u - ci * per_c;
            const int vr = rem / g.W4, j4 = rem - vr * g.W4;
            const int v = v0 + vr;
            const int n = v / g.HV, ih = v - n * g.HV - p.pad_h;
            if (n < p.N && ih >= 0 && ih < p.H) {
                goff[i] = (int)(n * p.xs[0] + ci * p.xs[1] + ih * p.xs[2]) + 4 * j4;
                loff[i] = ci * g.P + vr * g.RSL + g.XC + 4 * j4;
            }
        }
    }

    // ---- per-lane operand bases
    int abase[WM_BLK];
#pragma unroll
    for (int mb = 0; mb < WM_BLK; ++mb) {
        int m = m0 + (wave_m * WM_BLK + mb) * 16 + i16;
        m = m < g.Mtot ? m : g.Mtot - 1;
        const int gr = m / p.OW, ow = m - gr * p.OW;
        const int n = gr / p.OH, oh = gr - n * p.OH;
        const int vrel = n * g.HV + oh * p.stride_h - v0;
        abase[mb] = q * CPG * g.P + vrel * g.RSL + (g.XC - p.pad_w) + ow * p.stride_w;
    }
    int bbase[WN_BLK];
#pragma unroll
    for (int nb = 0; nb < WN_BLK; ++nb)
        bbase[nb] = ((wave_n * WN_BLK + nb) * 16 + i16) * WS + q * CPG * RS9;

    f32x4 acc[WM_BLK][WN_BLK];
#pragma unroll
    for (int mb = 0; mb < WM_BLK; ++mb)
#pragma unroll
        for (int nb = 0; nb < WN_BLK; ++nb) acc[mb][nb] = zero4();

    f32x4 rx[kMaxUnits], rw[WU];
    const int64_t w_row = (int64_t)p.C * RS9;

    auto load_chunk = [&](int cc) {
        const float* __restrict__ xb = p.x + (int64_t)cc * CK * p.xs[1];
#pragma unroll
        for (int i = 0; i < kMaxUnits; ++i)
            if (goff[i] >= 0) rx[i] = ldg4(xb + goff[i]);
        const float* __restrict__ wb = p.w + (int64_t)cc * KC;
#pragma unroll
        for (int i = 0; i < WU; ++i) {
            const int u = tid + i * NT;
            const int co = u / WQ, kq = u - co * WQ;
            rw[i] = zero4();
            if (u < BN * WQ && co0 + co < p.K) rw[i] = ldg4(wb + (co0 + co) * w_row + 4 * kq);
        }
    };
    auto store_chunk = [&](int buf) {
        float* pt = patch + buf * patch_sz;
#pragma unroll
        for (int i = 0; i < kMaxUnits; ++i)
            if (goff[i] >= 0) *reinterpret_cast<f32x4*>(pt + loff[i]) = rx[i];
        float* wt = wts + buf * (BN * WS);
#pragma unroll
        for (int i = 0; i < WU; ++i) {
            const int u = tid + i * NT;
            const int co = u / WQ, kq = u - co * WQ;
            if (u < BN * WQ) {
                f32x2 lo = {rw[i][0], rw[i][1]}, hi = {rw[i][2], rw[i][3]};
                f32x2* dst = reinterpret_cast<f32x2*>(wt + co * WS + 4 * kq);
                dst[0] = lo;
                dst[1] = hi;
            }
        }
    };

    load_chunk(0);
    for (int idx = tid; idx < (2 * patch_sz) / 4; idx += NT)
        reinterpret_cast<f32x4*>(patch)[idx] = zero4();
    __syncthreads();
    store_chunk(0);
    __syncthreads();

    const int nchunks = p.C / CK;
    for (int cc = 0; cc < nchunks; ++cc) {
        const int buf = cc & 1;
        if (cc + 1 < nchunks) load_chunk(cc + 1);

        const float* __restrict__ pa = patch + buf * patch_sz;
        const float* __restrict__ pb = wts + buf * (BN * WS);
#pragma unroll
        for (int t = 0; t < STEPS; ++t) {
            const int cl = t / RS9, tap = t % RS9;
            const int offA = cl * g.P + (tap / S_) * g.RSL + (tap % S_);
            float a[WM_BLK], b[WN_BLK];
#pragma unroll
            for (int mb = 0; mb < WM_BLK; ++mb) a[mb] = pa[abase[mb] + offA];
#pragma unroll
            for (int nb = 0; nb < WN_BLK; ++nb) b[nb] = pb[bbase[nb] + t];
#pragma unroll
            for (int mb = 0; mb < WM_BLK; ++mb)
#pragma unroll
                for (int nb = 0; nb < WN_BLK; ++nb)
                    acc[mb][nb] = mfma16(a[mb], b[nb], acc[mb][nb]);
        }

        if (cc + 1 < nchunks) store_chunk(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue: accumulator register r of lane (q, i16) is pixel 4q+r, channel i16 of its block
#pragma unroll
    for (int nb = 0; nb < WN_BLK; ++nb) {
        const int co = co0 + (wave_n * WN_BLK + nb) * 16 + i16;
        if (co >= p.K) continue;
        float scale = 1.f, shift = 0.f;
        if (p.gamma) {
            scale = p.gamma[co] / sqrtf(p.var[co] + p.eps);
            shift = p.beta[co] - p.mean[co] * scale;
        }
#pragma unroll
        for (int mb = 0; mb < WM_BLK; ++mb) {
            const int mq = m0 + (wave_m * WM_BLK + mb) * 16 + 4 * q;
            f32x4 v = acc[mb][nb];
            if (p.gamma) {
#pragma unroll
                for (int r = 0; r < 4; ++r) v[r] = fmaxf(fmaf(v[r], scale, shift), 0.f);
            }
            if (g.vec_store) {
                if (mq < g.Mtot) {
                    const int n = mq / g.ohow, pix = mq - n * g.ohow;
                    stg4(p.y + n * p.ys[0] + co * p.ys[1] + pix, v);
                }
            } else {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int m = mq + r;
                    if (m < g.Mtot) {
                        const int gr = m / p.OW, ow = m - gr * p.OW;
                        const int n = gr / p.OH, oh = gr - n * p.OH;
                        p.y[n * p.ys[0] + co * p.ys[1] + oh * p.ys[2] + ow] = v[r];
                    }
                }
            }
        }
    }
}

// Largest number of virtual rows any M-tile of BM pixels needs.
int max_virtual_rows(const ConvArgs& a, int BM, int HV)
{
    const int64_t Mtot = (int64_t)a.N * a.OH * a.OW;
    int vr = 0;
    for (int64_t m0 = 0; m0 < Mtot; m0 += BM) {
        const int64_t m1 = (m0 + BM < Mtot ? m0 + BM : Mtot) - 1;
        const int64_t g0 = m0 / a.OW, g1 = m1 / a.OW;
        const int64_t va = (g0 / a.OH) * HV + (g0 % a.OH) * a.stride_h;
        const int64_t vb = (g1 / a.OH) * HV + (g1 % a.OH) * a.stride_h;
        const int need = (int)(vb - va) + a.R;
        if (need > vr) vr = need;
    }
    return vr;
}

template <int WM_BLK, int WN_BLK, int WAVES_M, int WAVES_N, int R_, int S_, int CPG>
struct Variant {
    static constexpr int NT = 64 * WAVES_M * WAVES_N;
    static constexpr int BM = 16 * WM_BLK * WAVES_M, BN = 16 * WN_BLK * WAVES_N;
    static constexpr int CK = 4 * CPG;
    static constexpr int WS = CK * R_ * S_ + 2;

    // Fills the geometry; false if this variant cannot run the problem.
    static bool plan(const ConvArgs& a, IgemmGeom* g, size_t* lds_bytes)
    {
        if (a.C % CK != 0) return false;
        g->Mtot = a.N * a.OH * a.OW;
        g->ohow = a.OH * a.OW;
        g->HV = (a.OH - 1) * a.stride_h + a.R;
        g->VR = max_virtual_rows(a, BM, g->HV);
        g->XC = (a.pad_w + 3) / 4 * 4;
        const int wv = (a.OW - 1) * a.stride_w + a.S;           // virtual row width
        const int need_cols = g->XC - a.pad_w + (wv > a.W + a.pad_w ? wv : a.W + a.pad_w);
        g->RSL = (need_cols + 3) / 4 * 4;
        int P = g->VR * g->RSL;
        // quarters of a wave read planes CPG*P apart: keep them 16 banks apart
        for (int it = 0; it < 8 && (CPG * P) % 32 != 16; ++it) P += 4;
        g->P = P;
        g->W4 = a.W / 4;
        g->n_units = CK * g->VR * g->W4;
        if (g->n_units > kMaxUnits * NT) return false;
        g->vec_store = (g->ohow % 4 == 0) && a.ys[2] == a.OW && (a.ys[0] % 4 == 0) &&
                       (a.ys[1] % 4 == 0) && is_aligned16(a.y);
        *lds_bytes = sizeof(float) * 2 * ((size_t)CK * P + (size_t)BN * WS);
        return *lds_bytes <= 160 * 1024;
    }

    static hipError_t launch(const ConvArgs& a, const IgemmGeom& g, size_t lds_bytes, hipStream_t stream)
    {
        auto kern = conv_igemm_kernel<WM_BLK, WN_BLK, WAVES_M, WAVES_N, R_, S_, CPG>;
        if (lds_bytes > 64 * 1024) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
            if (e != hipSuccess) return e;
        }
        dim3 grid((g.Mtot + BM - 1) / BM, (a.K + BN - 1) / BN);
        return launch_kernel(kern, grid, dim3(NT), lds_bytes, stream, a, g);
    }

    // Relative cost: rounds of work-groups over the 256 CUs times the tile volume.
    static double cost(const ConvArgs& a)
    {
        const int64_t Mtot = (int64_t)a.N * a.OH * a.OW;
        const int64_t wgs = ((Mtot + BM - 1) / BM) * ((a.K + BN - 1) / BN);
        const int64_t rounds = (wgs + 255) / 256;
        return (double)rounds * BM * BN;
    }
};

using V224x64 = Variant<7, 2, 2, 2, 3, 3, 2>;
using V112x64 = Variant<7, 1, 1, 4, 3, 3, 2>;
using V128x64 = Variant<4, 2, 2, 2, 3, 3, 2>;
using V64x64 = Variant<2, 2, 2, 2, 3, 3, 2>;

template <class V>
void consider(const ConvArgs& a, double* best_cost, int* best, int id, IgemmGeom* g, size_t* lds)
{
    IgemmGeom gg;
    size_t l = 0;
    if (!V::plan(a, &gg, &l)) return;
    const double c = V::cost(a);
    if (*best < 0 || c < *best_cost) {
        *best_cost = c;
        *best = id;
        *g = gg;
        *lds = l;
    }
}

}  // namespace

hipError_t launch_conv2d_igemm(const ConvArgs& a, hipStream_t stream, bool* taken)
{
    *taken = false;
    const int64_t x_extent = (int64_t)(a.N - 1) * a.xs[0] + (int64_t)(a.C - 1) * a.xs[1] +
                             (int64_t)(a.H - 1) * a.xs[2] + a.W;
    const bool ok = a.R == 3 && a.S == 3 && (a.W % 4 == 0) && (a.C % 8 == 0) && is_aligned16(a.x) &&
                    is_aligned16(a.w) && (a.xs[0] % 4 == 0) && (a.xs[1] % 4 == 0) &&
                    (a.xs[2] % 4 == 0) && x_extent < (int64_t)1 << 31 &&
                    (int64_t)a.N * a.OH * a.OW < (int64_t)1 << 31;
    if (!ok) return hipSuccess;

    double best_cost = 0.0;
    int best = -1;
    IgemmGeom g;
    size_t lds = 0;
    consider<V224x64>(a, &best_cost, &best, 0, &g, &lds);
    consider<V112x64>(a, &best_cost, &best, 1, &g, &lds);
    consider<V128x64>(a, &best_cost, &best, 2, &g, &lds);
    consider<V64x64>(a, &best_cost, &best, 3, &g, &lds);
    if (best < 0) return hipSuccess;
    *taken = true;
    switch (best) {
        case 0: return V224x64::launch(a, g, lds, stream);
        case 1: return V112x64::launch(a, g, lds, stream);
        case 2: return V128x64::launch(a, g, lds, stream);
        default: return V64x64::launch(a, g, lds, stream);
    }
}

hipError_t launch_conv2d(const ConvArgs& a, hipStream_t stream)
{
    bool taken = false;
    hipError_t err = launch_conv2d_igemm(a, stream, &taken);
    if (taken || err != hipSuccess) return err;
    return launch_conv2d_direct(a, stream);
}

}  // namespace anr
