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

// divisors of the row kernels: row chunks per plane group, lanes per row, channels
struct RowDivs {
    FastDiv row_chunks, lanes_per_row, channels;
};

template <int ROWS, int WPB = 4>
__global__ __launch_bounds__(64 * WPB) void dwconv3x3_kernel(const ConvArgs p, int lanes_per_row,
                                                        int planes_per_wave, int64_t planes,
                                                        int row_chunks, RowDivs dv)
{
    // wave, plane and channel indices by multiply-shift (the launch keeps them below 2^31): the
    // 64-bit divisions they replace were some 300 vector-ALU instructions ahead of the first load
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)blockIdx.x * WPB + (int)(threadIdx.x >> 6));
    const int pgroup = dv.row_chunks.div(wave);
    const int oh0 = (wave - pgroup * row_chunks) * ROWS;

    const int pl = dv.lanes_per_row.div(lane), ch = lane - pl * lanes_per_row;
    const int64_t plane = (int64_t)pgroup * planes_per_wave + pl;
    const bool active = (pl < planes_per_wave) && (plane < planes);
    const int n = active ? dv.channels.div((int)plane) : 0;
    const int c = active ? (int)plane - n * p.C : 0;
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
                                                          int row_chunks, RowDivs dv)
{
    constexpr int IN = 2 * ROWS + 1;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)blockIdx.x * WPB + (int)(threadIdx.x >> 6));
    const int pgroup = dv.row_chunks.div(wave);
    const int oh0 = (wave - pgroup * row_chunks) * ROWS;

    const int pl = dv.lanes_per_row.div(lane), ch = lane - pl * lanes_per_row;
    const int64_t plane = (int64_t)pgroup * planes_per_wave + pl;
    const bool active = (pl < planes_per_wave) && (plane < planes);
    const int n = active ? dv.channels.div((int)plane) : 0;
    const int c = active ? (int)plane - n * p.C : 0;
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

// Stride 1, 3x3, pad 1 on dense NCHW tensors, as a pure stream.  An item is a run of RC output
// rows of one plane; its input rows (RC + 2, clipped at the plane's edges) are ONE contiguous
// range of x and its output rows one contiguous range of y.  A wave owns an item: it pulls the
// input range into its private slice of LDS with direct-to-LDS loads (consecutive lanes fetch
// consecutive 16-byte units, so every request covers whole cache lines, and the data never
// passes through registers), then each lane computes output units from LDS (one 16-byte read
// per input row plus the two neighbouring columns) and stores them, again with consecutive
// lanes on consecutive units.  Loads and stores are non-temporal: x is read once and y written
// once, and lines that linger in L2 are written back when the kernel ends, which a measured
// 26 MB copy pays with 6.8 instead of 5.3 us.  No work-group barrier: a wave's slice of LDS is
// its own.
//
// Per-wave timestamps showed the arithmetic, not the traffic, to be what such a kernel adds to a
// copy: its waves get their data within the same microsecond and then share the vector ALUs.
// So a round of the wave covers whole rows (RPR = floor(64 / (W/4)) of them, LPR = RPR * W/4
// lanes): a lane keeps its column for all rounds, so whether it sits at the plane's left or right
// edge is decided once and costs one select per edge and round; a zero row in LDS stands in for
// the row above and below the plane; and with the width known at compile time every LDS and
// global address of a round is the lane's base plus an instruction immediate: 38 multiply-adds
// and two selects per round and next to nothing else.  (Tried: the neighbouring columns by DPP wave shift instead of
// 4-byte LDS reads, which fall on 16 banks: 6.9 against 6.3 us, the shifts are vector-ALU work;
// edge taps under a branch or as predicated reads: 6.7 us; two to eight items per wave with the
// loads of all of them in flight: 6.7 to 12.8 us, a wave's chain is what counts; starting the
// waves' loads in staggered groups so that stores of one group overlap loads of the next: slower
// at every delay.)
struct StreamGeom {
    int W4;               // W / 4
    int RPR, LPR;         // rows and lanes per round
    int RC;               // output rows per item
    int chunks;           // items per plane = ceil(H / RC)
    int hw;               // H * W
    int slice;            // floats of LDS per wave, slack included (a multiple of 4)
    int items;            // planes * chunks
    FastDiv d_chunks, d_w4, d_c;
};

// NI: rounds that cover an item's input rows (its output rows are fewer); W4_T: W / 4, or 0 for any width
template <int W4_T, int NI>
__global__ __launch_bounds__(256) void dwconv3x3_stream_kernel(const ConvArgs p, const StreamGeom g)
{
    extern __shared__ __attribute__((aligned(16))) float slds[];
    const int W4 = W4_T ? W4_T : g.W4, W = 4 * W4;
    const int RPR = W4_T ? 64 / W4_T : g.RPR, LPR = RPR * W4;
    const int lane = threadIdx.x & 63;
    const int wv = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int item = __builtin_amdgcn_readfirstlane((int)blockIdx.x * 4 + wv);
    if (item >= g.items) return;                                   // whole wave
    // four floats of slack ahead of the slice: the read left of its first unit stays inside LDS
    float* const lx = slds + 4 + wv * g.slice;
    const int plane = g.d_chunks.div(item);
    const int r0 = (item - plane * g.chunks) * g.RC;               // first output row
    const int r1 = r0 + g.RC < p.H ? r0 + g.RC : p.H;              // one past the last
    const int in0 = r0 > 0 ? r0 - 1 : 0;                           // first input row staged
    const int in1 = r1 < p.H ? r1 + 1 : p.H;
    const int c = plane - g.d_c.div(plane) * p.C;

    // ---- LDS row j of the slice is input row r0 - 1 + j.  Rows in0 .. in1-1 are (in1 - in0) * W4
    //      consecutive units of x and land on consecutive units of the slice, LPR per instruction
    //      (lanes past a round or past the end sit the instruction out).  A row above or below the
    //      plane is zero-filled by the wave itself, so the taps need no test for it.
    const float* __restrict__ src = p.x + (int64_t)plane * g.hw + in0 * W + 4 * lane;
    const int n_in = (in1 - in0) * W4;
    float* const land = lx + (in0 - (r0 - 1)) * W;                  // W floats further when r0 == 0
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        if (lane < LPR && lane + LPR * i < n_in)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src + 4 * LPR * i),
                                             (__attribute__((address_space(3))) void*)(land + 4 * LPR * i), 16, 0, 2);
    }
    if (r0 == 0 && lane < W4) *reinterpret_cast<f32x4*>(lx + 4 * lane) = zero4();
    if (r1 == p.H && lane < W4) *reinterpret_cast<f32x4*>(lx + (r1 - r0 + 1) * W + 4 * lane) = zero4();

    // the lane's column never changes, so whether it has a neighbour to its left and right is
    // decided once
    const int ch = lane - g.d_w4.div(lane) * W4;
    const bool has_l = ch > 0, has_r = ch < W4 - 1;
    float wt[9];
#pragma unroll
    for (int i = 0; i < 9; ++i) wt[i] = p.w[c * 9 + i];
    // The compiler does not order LDS reads after direct-to-LDS loads by itself: wait for the
    // loads here, and keep every later memory access behind the wait.
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");

    // ---- output rows r0 .. r1-1, RPR per round: the unit of lane l in round i is unit l + LPR * i
    //      of the item, and its tap rows are that unit of slice rows j, j + 1, j + 2.  The columns
    //      left and right of a unit are read from LDS as they lie (inside a row the neighbouring
    //      unit; at the plane's edge the end of another row or the slack around the slice).  The
    //      first and last output of a unit are summed without those taps first; the lanes that have
    //      the neighbour then take the sum with them, the others the sum without: one select per
    //      edge and round, and a tap across the edge is never multiplied at all.
    float* __restrict__ dst = p.y + (int64_t)plane * g.hw + r0 * W + 4 * lane;
    const int n_out = (r1 - r0) * W4;
    const float* const t0 = lx + 4 * lane;
    // All rounds are computed before the first store is issued: the compiler makes every LDS read
    // that follows a store wait for that store (it cannot tell the store from the direct-to-LDS
    // loads), which would put a trip to L2 between one round and the next.
    f32x4 res[NI];
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        if (lane < LPR && lane + LPR * i < n_out) {
            f32x4 acc;
            float al, ar;
#pragma unroll
            for (int r = 0; r < 3; ++r) {
                const float* row = t0 + 4 * LPR * i + r * W;
                const f32x4 m = *reinterpret_cast<const f32x4*>(row);
                const float l = row[-1], rr = row[4];
                const float w0 = wt[3 * r], w1 = wt[3 * r + 1], w2 = wt[3 * r + 2];
                if (r == 0) {
                    acc[0] = w1 * m[0];
                    acc[1] = w0 * m[0];
                    acc[2] = w0 * m[1];
                    acc[3] = w0 * m[2];
                    al = w0 * l;
                    ar = w2 * rr;
                } else {
                    acc[0] = fmaf(w1, m[0], acc[0]);
                    acc[1] = fmaf(w0, m[0], acc[1]);
                    acc[2] = fmaf(w0, m[1], acc[2]);
                    acc[3] = fmaf(w0, m[2], acc[3]);
                    al = fmaf(w0, l, al);
                    ar = fmaf(w2, rr, ar);
                }
                acc[0] = fmaf(w2, m[1], acc[0]);
                acc[1] = fmaf(w1, m[1], acc[1]);
                acc[2] = fmaf(w1, m[2], acc[2]);
                acc[3] = fmaf(w1, m[3], acc[3]);
                acc[1] = fmaf(w2, m[2], acc[1]);
                acc[2] = fmaf(w2, m[3], acc[2]);
            }
            acc[0] += has_l ? al : 0.f;
            acc[3] += has_r ? ar : 0.f;
            res[i] = acc;
        }
    }
#pragma unroll
    for (int i = 0; i < NI; ++i)
        if (lane < LPR && lane + LPR * i < n_out)
            stg4_nt(dst + 4 * LPR * i, res[i]);
}

// Small planes (14 x 14 and 7 x 7 maps of the MobileNet shape list, any kernel, stride, padding
// and dilation) of dense NCHW tensors: a work-group takes G consecutive planes, which are one
// contiguous range of x and of y.  The range is copied to LDS with coalesced 16-byte loads, the
// outputs are computed from LDS into LDS and leave as coalesced 16-byte stores.  With one thread per output reading x through the vector caches,
// 7x7x1024 at batch 16 took 9.8 us for 6.4 MB; a plane's nine-fold tap reuse belongs in LDS.
struct SmallPlanes {
    int G;              // planes per work-group (a multiple of 4: ranges start 16-byte aligned)
    int hw, ohw;        // H*W, OH*OW
    int rs;             // R*S
    int64_t planes;     // N*C
    FastDiv d_ohw, d_ow, d_c;
};

template <int R_, int S_>     // kernel size, or 0, 0 for any
__global__ __launch_bounds__(256) void dwconv_small_planes_kernel(const ConvArgs p, const SmallPlanes g)
{
    extern __shared__ __attribute__((aligned(16))) float dlds[];   // x[G*hw], y[G*ohw], w[G*rs]
    float* const lx = dlds;
    float* const ly = dlds + ((g.G * g.hw + 3) & ~3);
    float* const lw = ly + ((g.G * g.ohw + 3) & ~3);

    const int tid = threadIdx.x;
    const int64_t plane0 = (int64_t)blockIdx.x * g.G;
    const int nplanes = g.planes - plane0 < g.G ? (int)(g.planes - plane0) : g.G;

    // ---- planes plane0 .. plane0 + nplanes - 1: nplanes * hw contiguous floats of x
    {
        const float* __restrict__ src = p.x + plane0 * g.hw;
        const int count = nplanes * g.hw;
        for (int i = 4 * tid; i < count; i += 4 * 256) {
            if (i + 3 < count) {
                *reinterpret_cast<f32x4*>(lx + i) = ldg4(src + i);
            } else {
                for (int e = i; e < count; ++e) lx[e] = src[e];
            }
        }
        for (int i = tid; i < nplanes * g.rs; i += 256) {
            const int pl = i / g.rs, t = i - pl * g.rs;
            const int64_t plane = plane0 + pl;
            const int c = (int)(plane - (int64_t)g.d_c.div((int)plane) * p.C);
            lw[i] = p.w[(int64_t)c * g.rs + t];
        }
    }
    __syncthreads();

    // ---- a thread computes outputs tid, tid + 256, ...; with the kernel size known at compile time
    //      the taps of an output are unrolled, so its LDS reads are in flight together (one output
    //      row per thread with run-time loops waited for each of its 63 reads in turn: 3 us)
    {
        const int count = nplanes * g.ohw;
        for (int o = tid; o < count; o += 256) {
            const int pl = g.d_ohw.div(o), pix = o - pl * g.ohw;
            const int oh = g.d_ow.div(pix), ow = pix - oh * p.OW;
            const float* xin = lx + pl * g.hw;
            const float* wt = lw + pl * g.rs;
            const int ih0 = oh * p.stride_h - p.pad_h, iw0 = ow * p.stride_w - p.pad_w;
            float acc = 0.f;
            if (R_ > 0) {
#pragma unroll
                for (int r = 0; r < R_; ++r)
#pragma unroll
                    for (int s = 0; s < S_; ++s) {
                        const int ih = ih0 + r * p.dil_h, iw = iw0 + s * p.dil_w;
                        const bool ok = ((unsigned)ih < (unsigned)p.H) & ((unsigned)iw < (unsigned)p.W);
                        const float v = xin[ok ? ih * p.W + iw : 0];
                        acc = fmaf(ok ? v : 0.f, wt[r * S_ + s], acc);
                    }
            } else {
                for (int r = 0; r < p.R; ++r)
                    for (int s = 0; s < p.S; ++s) {
                        const int ih = ih0 + r * p.dil_h, iw = iw0 + s * p.dil_w;
                        if (((unsigned)ih < (unsigned)p.H) & ((unsigned)iw < (unsigned)p.W))
                            acc = fmaf(xin[ih * p.W + iw], wt[r * p.S + s], acc);
                    }
            }
            ly[o] = acc;
        }
    }
    __syncthreads();

    // ---- nplanes * ohw contiguous floats of y
    {
        float* __restrict__ dst = p.y + plane0 * g.ohw;
        const int count = nplanes * g.ohw;
        for (int i = 4 * tid; i < count; i += 4 * 256) {
            if (i + 3 < count) {
                stg4(dst + i, *reinterpret_cast<const f32x4*>(ly + i));
            } else {
                for (int e = i; e < count; ++e) dst[e] = ly[e];
            }
        }
    }
}

}  // namespace dw
}  // namespace anr
