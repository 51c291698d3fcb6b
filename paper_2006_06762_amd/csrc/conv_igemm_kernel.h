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
// MFMA: v_mfma_f32_32x32x2_f32 (measured on MI355X: it sustains 99 % of the
// 157.3 TFLOP/s fp32 matrix peak from one wave per SIMD, the 16x16x4 form only
// 78-85 %).  Lane l feeds pixel (l%32) of a 32-pixel block for the A operand
// and channel (l%32) of a 32-channel block for B; its half h = l/32 picks which
// of the two k values of the instruction it supplies.  A half-wave walks "its"
// CPH channels of the chunk, tap by tap, so the A address of a lane is one
// per-lane base plus an offset that is uniform over the wave, and the B
// (weight) values of a lane are consecutive floats of the natural OIHW order:
// weights are copied to LDS unpermuted.
//
// Waves: WAVES_M x WAVES_N wave tiles of (32*WM_BLK) x (32*WN_BLK), times
// KSPLIT waves per tile that split the k-steps of every chunk among them (the
// tile shapes that divide the benchmark problems evenly over 256 CUs have an
// odd number of 32-pixel blocks, so the waves of a work-group share a tile
// along k instead of cutting it).  After the last chunk the partial
// accumulators are reduce-scattered through LDS: every 32x32 block has an owner
// wave that sums the others' partials and runs the epilogue for that block, so
// the reduction takes one barrier and the stores are spread over all waves.
//
// Inside a chunk the operands of step t+1 are read from LDS before the MFMAs
// of step t are issued (register double buffering).  Staging of the next chunk
// is woven into the MFMA stream one instruction at a time: an MFMA occupies the
// matrix pipe for 64 cycles but the wave only 4 to issue it, so one global load
// goes out behind each of the first MFMAs of a chunk and one LDS store behind
// each of the last ones, and neither costs matrix time.  Loads and stores are
// branch-free (spare staging slots duplicate a real unit, padding rows store
// zeros): a load inside a divergent branch makes the compiler drain all
// outstanding loads first, which serialises a chunk's memory latency.
// One barrier per chunk: at its end with two staging buffers (run-time LDS
// strides), a k-step before its end with the ring of three buffers that the
// instantiations for fixed layer geometries use (described at the loop).
//
// Set-up order: the loads of the first chunk are issued as soon as their
// offsets exist; operand addresses, accumulators and the zeroing of the padding
// follow while they are in flight.
//
// The batch-norm scale/shift and ReLU of ConvLayer run on the summed partial
// tiles in the epilogue (Table 1, rule 4: fuse element-wise consumers into the
// tiled node); where four consecutive pixels are 16 aligned bytes of y, the
// k-split reduction doubles as a transposition and results leave in 128-byte
// runs, otherwise straight from the accumulator layout.
#pragma once
#include <type_traits>

#include "anr_device.h"
#include "conv_internal.h"

namespace anr {
namespace igemm {

struct Geom {
    int Mtot;       // N*OH*OW
    int HV;         // virtual image height: (OH-1)*stride_h + R
    int VR;         // virtual rows staged per tile (max over tiles)
    int RSL;        // LDS row stride, floats
    int P;          // LDS channel-plane stride, floats
    int XC;         // LDS column of input column 0 (multiple of 4)
    int W4;         // W / 4
    int n_units;    // CK * VR * W4 16-byte staging units per chunk
    int st_ci, st_vr, st_j4;   // the work-group's thread count as (channels, rows, quads) of staging units
    int row_groups; // > 0: a thread stages one (row, quad) of channels cg, cg + row_groups, ... (cg < row_groups)
    int slots;      // staging slots a thread needs under the mapping in use
    int vec_store;  // 4 consecutive pixels of a lane are 16 contiguous, aligned bytes of y
    int ohow;       // OH*OW
    FastDiv d_ow, d_oh, d_hv, d_w4, d_perc, d_ohow, d_units;   // divisors OW, OH, HV, W4, VR*W4, OH*OW, n_units
    // work-group id -> tile: ids are dealt round-robin over the 8 XCDs, so id % 8 picks a
    // rectangle of (tiles_m / xcd_m) x (tiles_n / xcd_n) tiles that one XCD's L2 serves
    int tiles_m, tiles_n, xcd_m, xcd_n;
    int sub_m, sub_n, xcd_n_shift;   // tiles_m / xcd_m, tiles_n / xcd_n, log2(xcd_n)
    uint32_t x_bytes, w_bytes;   // extents of the x view and of w, for the buffer descriptors
    uint32_t wpack_bytes;        // extent of the packed weights: tiles_n * chunks * BN * (KC + 4) floats
    FastDiv d_sub_n;            // divisor tiles_n / xcd_n
    FastDiv d_tiles_m;
};


constexpr int kMaxUnits = 8;

// PACKED: the weights come from a pack made by conv_pack_patch_kernel, in which the LDS image of
// every (channel tile, chunk) is one contiguous run: staging them is a straight copy in 16-byte
// units, and the batch-norm scale and shift are read, not computed.
template <int WM_BLK, int WN_BLK, int WAVES_M, int WAVES_N, int KSPLIT, int R_, int S_, int CPH, int XU,
          int RSL_T, int P_T, bool PACKED, int NBUF>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N * KSPLIT)
void conv_igemm_kernel(const ConvArgs p, const Geom g)
{
    constexpr int NT = 64 * WAVES_M * WAVES_N * KSPLIT;
    constexpr int BM = 32 * WM_BLK * WAVES_M, BN = 32 * WN_BLK * WAVES_N;
    constexpr int RS9 = R_ * S_;
    constexpr int CK = 2 * CPH;           // channels per chunk
    constexpr int KC = CK * RS9;          // reduction length per chunk
    // LDS stride of one output channel's weights: a multiple of four floats, so that a staging unit
    // is ONE 16-byte LDS store (with KC + 2, two 8-byte ones: conflict-free operand reads, but 0.5-1.3 us
    // slower per benchmark layer -- the operand reads of 32 consecutive rows now fall on 16 banks,
    // which costs nothing measurable)
    constexpr int WS = KC + 4;
    constexpr int STEPS = CPH * RS9;      // MFMA k-steps per chunk (all waves of a tile together)
    constexpr int SPW = STEPS / KSPLIT;   // k-steps per chunk of one wave
    constexpr int WQ = KC / 4;
    constexpr int PU = BN * WS / 4;       // 16-byte units of a packed chunk image
    static_assert((BN * WS) % 4 == 0, "a chunk image is a whole number of 16-byte units");
    constexpr int WU = ((PACKED ? PU : BN * WQ) + NT - 1) / NT;
    constexpr int NBLK = WM_BLK * WN_BLK; // MFMAs per k-step of one wave
    constexpr int SLOTS = SPW * NBLK;     // MFMAs per chunk of one wave = issue slots for staging
    constexpr int NSIDE = XU + WU;        // staging units per thread and chunk
    constexpr int STORE0 = SLOTS - NSIDE; // the last NSIDE slots carry the LDS stores
    static_assert(KC % 4 == 0, "chunk must be a whole number of float4");
    static_assert(CPH % KSPLIT == 0, "waves split a half-wave's channels evenly");
    static_assert(2 * NSIDE <= SLOTS, "not enough MFMAs in a chunk to hide the staging behind");

    // LDS geometry: compile-time for the instantiations made for one problem shape (every LDS
    // address in the main loop is then a per-lane register plus an instruction immediate, and
    // the loop holds no vector ALU instruction at all: on this hardware each VALU or VMEM
    // instruction between two MFMAs delays the second by 5-13 cycles, LDS and scalar ones do not)
    const int RSL = RSL_T ? RSL_T : g.RSL;
    const int P = P_T ? P_T : g.P;
    const int patch_sz = CK * P;                     // floats per patch buffer
    constexpr int WTS_SZ = BN * WS;                  // floats per weight buffer

    static_assert(NBUF == 2 || NBUF == 3, "two staging buffers, or a ring of three");
    extern __shared__ __attribute__((aligned(16))) float smem[];
    // layout: patch[NBUF][patch_sz], then wts[NBUF][WTS_SZ]
    char* const lds = reinterpret_cast<char*>(smem);

    const int tid = threadIdx.x;
    touch_kernel_arguments<sizeof(ConvArgs) + sizeof(Geom)>();
    const int lane = tid & 63, wave = tid >> 6;
    const int r32 = lane & 31, h = lane >> 5;
    const int tile_wave = wave % (WAVES_M * WAVES_N), ks = wave / (WAVES_M * WAVES_N);
    const int wave_m = tile_wave / WAVES_N, wave_n = tile_wave % WAVES_N;
    int tile_m, tile_n;
    {
        const int w = blockIdx.x;
        if (g.xcd_n) {        // the tile grid splits eight ways (xcd_n is a power of two)
            const int xcd = w & 7, slot = w >> 3;
            const int lm = g.d_sub_n.div(slot);
            tile_m = (xcd >> g.xcd_n_shift) * g.sub_m + lm;
            tile_n = (xcd & (g.xcd_n - 1)) * g.sub_n + (slot - lm * g.sub_n);
        } else {
            tile_n = g.d_tiles_m.div(w);
            tile_m = w - tile_n * g.tiles_m;
        }
    }
    const int m0 = tile_m * BM, co0 = tile_n * BN;

    const int g0 = g.d_ow.div(m0);
    const int n_first = g.d_oh.div(g0);
    const int v0 = n_first * g.HV + (g0 - n_first * p.OH) * p.stride_h;

    // ---- staging: which 16 bytes of x and w go where in LDS (fixed over chunks), and the loads of
    //      the first chunk, each issued as soon as its offset is known: everything else the
    //      kernel sets up (operand addresses, accumulators, zeroed padding) then runs while they
    //      are in flight.
    //      Every slot of every thread loads something, so that the main loop has no branch
    //      around a load: slots past the end of the patch duplicate an earlier unit (same data
    //      to the same place), units whose row is padding load offset 0 and skip the store
    //      (their rows were zeroed before the first chunk).  Offsets are in bytes, relative to
    //      the first channel of a chunk.
    // Buffer loads: the descriptor (base, extent) sits in scalar registers for the whole kernel, the
    // lane supplies a 32-bit byte offset and the chunk a scalar one, so a load in the main loop
    // needs no vector ALU work for its address.
    const __amdgpu_buffer_rsrc_t xrsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(p.x), 0, (int)g.x_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t wrsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float*>(PACKED ? p.wpack : p.w), 0, (int)(PACKED ? g.wpack_bytes : g.w_bytes), 0x00020000);
    f32x4 rx[XU], rw[WU];
    // weight staging: unit u is 16 bytes of output channel co0 + u / WQ; slots past the tile
    // duplicate earlier units, channels past K re-read the last valid channel (their products
    // land in accumulator columns that are never stored)
    uint32_t woff[WU], wlds[WU];
    const int nchunks = p.C / CK;
#pragma unroll
    for (int i = 0; i < WU; ++i) {
        if (PACKED) {
            // unit u of the chunk image goes to unit u of the LDS buffer
            const int u = (tid + i * NT) % PU;
            woff[i] = 4u * (uint32_t)(tile_n * nchunks * (BN * WS) + 4 * u);
            wlds[i] = 4u * (uint32_t)(NBUF * patch_sz + 4 * u);
        } else {
            const int u = (tid + i * NT) % (BN * WQ);
            const int co = u / WQ, kq = u - co * WQ;
            const int gco = co0 + co < p.K ? co0 + co : p.K - 1;
            woff[i] = 4u * (uint32_t)(gco * (p.C * RS9) + 4 * kq);
            wlds[i] = 4u * (uint32_t)(NBUF * patch_sz + co * WS + 4 * kq);
        }
        rw[i] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(wrsrc, (int)woff[i], 0, 0));
    }
    // x staging.  A unit is (channel ci of the chunk, virtual row vr of the patch, quad j4 of the
    // row).  Where a channel's units fit the work-group (row_groups > 0), a thread keeps ONE (vr, j4)
    // and its slots walk the channels ci = cg, cg + row_groups, ...: image, input row and validity
    // are worked out once per thread and a slot costs an add and a select.  Otherwise unit u = tid +
    // i * NT: the first slot is decomposed by division, the others follow by adding the
    // decomposition of NT with carries.  A slot whose unit lies past the patch repeats the thread's
    // first one.
    uint32_t xoff[XU], xlds[XU];
    bool xvalid[XU];
    if (g.row_groups) {
        int cg = g.d_perc.div(tid);
        const int ru = tid - cg * (g.VR * g.W4);
        cg = cg < g.row_groups ? cg : 0;       // surplus threads repeat units of the first group
        const int vr = g.d_w4.div(ru), j4 = ru - vr * g.W4;
        const int v = v0 + vr;
        const int n = g.d_hv.div(v), ih = v - n * g.HV - p.pad_h;
        const bool valid = n < p.N && ih >= 0 && ih < p.H;
        const uint32_t offc = 4u * (uint32_t)(n * p.xs[0] + cg * p.xs[1] + ih * p.xs[2] + 4 * j4);
        const uint32_t ldsc = 4u * (uint32_t)(cg * P + vr * RSL + g.XC + 4 * j4);
        const uint32_t step_off = 4u * (uint32_t)(g.row_groups * p.xs[1]), step_lds = 4u * (uint32_t)(g.row_groups * P);
#pragma unroll
        for (int i = 0; i < XU; ++i) {
            const bool in = cg + i * g.row_groups < CK;
            xvalid[i] = valid;
            xoff[i] = valid ? (in ? offc + (uint32_t)i * step_off : offc) : 0u;
            xlds[i] = in ? ldsc + (uint32_t)i * step_lds : ldsc;
            rx[i] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(xrsrc, (int)xoff[i], 0, 0));
        }
    } else {
        int ci = 0, vr = 0, j4 = 0, ci0 = 0, vr0 = 0, j40 = 0;
#pragma unroll
        for (int i = 0; i < XU; ++i) {
            if (i == 0) {
                int u = tid;
                u -= g.d_units.div(u) * g.n_units;
                ci = g.d_perc.div(u);
                const int rem = u - ci * (g.VR * g.W4);
                vr = g.d_w4.div(rem);
                j4 = rem - vr * g.W4;
                ci0 = ci, vr0 = vr, j40 = j4;
            } else {
                j4 += g.st_j4;
                int carry = j4 >= g.W4;
                j4 -= carry ? g.W4 : 0;
                vr += g.st_vr + carry;
                carry = vr >= g.VR;
                vr -= carry ? g.VR : 0;
                ci += g.st_ci + carry;
            }
            const bool past = ci >= CK;
            const int eci = past ? ci0 : ci, evr = past ? vr0 : vr, ej4 = past ? j40 : j4;
            const int v = v0 + evr;
            const int n = g.d_hv.div(v), ih = v - n * g.HV - p.pad_h;
            xvalid[i] = n < p.N && ih >= 0 && ih < p.H;
            xoff[i] = xvalid[i] ? 4u * (uint32_t)(n * p.xs[0] + eci * p.xs[1] + ih * p.xs[2] + 4 * ej4) : 0u;
            xlds[i] = 4u * (uint32_t)(eci * P + evr * RSL + g.XC + 4 * ej4);
            rx[i] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(xrsrc, (int)xoff[i], 0, 0));
        }
    }
    __builtin_amdgcn_sched_barrier(0);     // the loads stay here: the compiler would sink them to their first use

    // ---- per-lane operand addresses in LDS, bytes (the wave's share of the k-steps is folded in)
    uint32_t abase[WM_BLK];
#pragma unroll
    for (int mb = 0; mb < WM_BLK; ++mb) {
        int m = m0 + (wave_m * WM_BLK + mb) * 32 + r32;
        m = m < g.Mtot ? m : g.Mtot - 1;
        const int gr = g.d_ow.div(m), ow = m - gr * p.OW;
        const int n = g.d_oh.div(gr), oh = gr - n * p.OH;
        const int vrel = n * g.HV + oh * p.stride_h - v0;
        abase[mb] = 4u * (uint32_t)((h * CPH + ks * (CPH / KSPLIT)) * P + vrel * RSL + (g.XC - p.pad_w) +
                                    ow * p.stride_w);
    }
    uint32_t bbase[WN_BLK];
#pragma unroll
    for (int nb = 0; nb < WN_BLK; ++nb)
        bbase[nb] = 4u * (uint32_t)(NBUF * patch_sz + ((wave_n * WN_BLK + nb) * 32 + r32) * WS + h * CPH * RS9 +
                                    ks * SPW);

    f32x16 acc[WM_BLK][WN_BLK];
#pragma unroll
    for (int mb = 0; mb < WM_BLK; ++mb)
#pragma unroll
        for (int nb = 0; nb < WN_BLK; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mb][nb][r] = 0.f;

    // staging unit j of a later chunk: global -> registers
    auto side_load = [&](int j, uint32_t xchunk_b, uint32_t wchunk_b) {
        if (j < XU)
            rx[j] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(xrsrc, (int)xoff[j], (int)xchunk_b, 0));
        else
            rw[j - XU] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(wrsrc, (int)woff[j - XU], (int)wchunk_b, 0));
    };
    // staging unit j: registers -> LDS, xbuf_b / wbuf_b = byte offset of the target buffer
    auto side_store = [&](int j, int xbuf_b, int wbuf_b) {
        if (j < XU) {
            if (xvalid[j]) *reinterpret_cast<f32x4*>(lds + xlds[j] + xbuf_b) = rx[j];
        } else {
            const f32x4 v = rw[j - XU];
            *reinterpret_cast<f32x4*>(lds + wlds[j - XU] + wbuf_b) = v;
        }
    };

    for (int idx = tid; idx < (NBUF * patch_sz) / 4; idx += NT)
        reinterpret_cast<f32x4*>(smem)[idx] = zero4();
    __syncthreads();
#pragma unroll
    for (int j = 0; j < NSIDE; ++j) side_store(j, 0, 0);

    if constexpr (NBUF == 3) {
        // Ring of three staging buffers.  Chunk c is multiplied from buffer c % 3; meanwhile, in
        // the first half of the chunk, the data of chunk c + 1 (requested during chunk c - 1) goes
        // to buffer (c + 1) % 3, then comes the chunk's one barrier, then the requests for chunk
        // c + 2.  A wave that has passed the barrier of chunk c knows that every wave has stored
        // chunk c + 1 and is beyond chunk c - 1, so it may read buffer (c + 1) % 3 as soon as it is
        // done with chunk c and overwrite buffer (c + 2) % 3 in the first half of chunk c + 1.  With
        // two buffers the barrier has to stand at the end of a chunk, where every wave then waits
        // with nothing queued on its matrix pipe for the first operands of the next chunk to come
        // from LDS (about 260 cycles per chunk); here the barrier stands between two MFMAs whose
        // operands are already in registers, and the first operands of the next chunk are read
        // during the last k-step of this one.
        // slots of a chunk: stores [ST0, LD0), requests for chunk c + 2 [LD0, LD0 + NSIDE), the
        // barrier after slot BAR: GAP MFMAs behind the last store, so the stores have landed when the
        // wave waits for them, and before the last k-step, which reads the next chunk's operands
        constexpr int GAP = NSIDE > 8 ? 8 : 4;    // measured: 8 pays with eleven stores to drain (stride 2: 69.7 -> 68.8 us), not with six or eight
        constexpr int BAR = SLOTS - NBLK - 1;
        constexpr int LD0 = BAR + 1 - GAP, ST0 = LD0 - NSIDE;
        static_assert(ST0 >= 0 && LD0 + NSIDE <= SLOTS, "a chunk has too few MFMAs for this schedule");
        {
            const int c1 = nchunks > 1 ? 1 : 0;
            const uint32_t xb = 4u * (uint32_t)c1 * (uint32_t)(CK * p.xs[1]);
            const uint32_t wb = 4u * (uint32_t)c1 * (uint32_t)(PACKED ? BN * WS : KC);
#pragma unroll
            for (int j = 0; j < NSIDE; ++j) side_load(j, xb, wb);     // chunk 1, stored during chunk 0
        }
        __syncthreads();
        float a_cur[WM_BLK], b_cur[WN_BLK], a_nxt[WM_BLK], b_nxt[WN_BLK];
        // the third buffer may lie beyond the 64 KB an LDS instruction's immediate offset reaches:
        // it gets address registers of its own rather than an addition per read
        uint32_t abase2[WM_BLK];
#pragma unroll
        for (int mb = 0; mb < WM_BLK; ++mb) abase2[mb] = abase[mb] + 4u * (uint32_t)(2 * patch_sz);
        auto read_step = [&](int t, int buf, float* a, float* b) {
            const int cl = t / RS9, tap = t % RS9;
            const int offA = 4 * (cl * P + (tap / S_) * RSL + (tap % S_)) + (buf == 1 ? 4 * patch_sz : 0);
#pragma unroll
            for (int mb = 0; mb < WM_BLK; ++mb)
                a[mb] = *reinterpret_cast<const float*>(lds + (buf == 2 ? abase2[mb] : abase[mb]) + offA);
#pragma unroll
            for (int nb = 0; nb < WN_BLK; ++nb)
                b[nb] = *reinterpret_cast<const float*>(lds + bbase[nb] + 4 * t + 4 * buf * WTS_SZ);
        };
        read_step(0, 0, a_cur, b_cur);
        auto chunk = [&](int cc, auto buf_c) {
            constexpr int buf = decltype(buf_c)::value, nbuf = (buf + 1) % 3;
            // chunks past the last one are the last one again: loaded and stored, never read
            const int c2 = cc + 2 < nchunks ? cc + 2 : nchunks - 1;
            const uint32_t xb = 4u * (uint32_t)c2 * (uint32_t)(CK * p.xs[1]);
            const uint32_t wb = 4u * (uint32_t)c2 * (uint32_t)(PACKED ? BN * WS : KC);
#pragma unroll
            for (int t = 0; t < SPW; ++t) {
                if (t + 1 < SPW)
                    read_step(t + 1, buf, a_nxt, b_nxt);
                else
                    read_step(0, nbuf, a_nxt, b_nxt);          // first operands of the next chunk
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int mb = 0; mb < WM_BLK; ++mb)
#pragma unroll
                    for (int nb = 0; nb < WN_BLK; ++nb) {
                        acc[mb][nb] = mfma32(a_cur[mb], b_cur[nb], acc[mb][nb]);
                        const int slot = (t * WM_BLK + mb) * WN_BLK + nb;
                        if (slot >= ST0 && slot < LD0) side_store(slot - ST0, 4 * nbuf * patch_sz, 4 * nbuf * WTS_SZ);
                        if (slot >= LD0 && slot < LD0 + NSIDE) side_load(slot - LD0, xb, wb);
                        if (slot == BAR) __syncthreads();
                        __builtin_amdgcn_sched_barrier(0);
                    }
#pragma unroll
                for (int mb = 0; mb < WM_BLK; ++mb) a_cur[mb] = a_nxt[mb];
#pragma unroll
                for (int nb = 0; nb < WN_BLK; ++nb) b_cur[nb] = b_nxt[nb];
            }
        };
        for (int cc = 0; cc < nchunks; cc += 3) {
            chunk(cc, std::integral_constant<int, 0>{});
            if (cc + 1 < nchunks) chunk(cc + 1, std::integral_constant<int, 1>{});
            if (cc + 2 < nchunks) chunk(cc + 2, std::integral_constant<int, 2>{});
        }
        __syncthreads();        // the partial sums below go where the staging buffers are
    } else {
        __syncthreads();

        // One chunk: MFMAs on LDS buffer `buf`, staging of chunk cc+1 into the other buffer.
        auto chunk = [&](int cc, auto buf_c) {
            constexpr int buf = decltype(buf_c)::value;
            // the chunk after the last one is the last one again: loaded and stored, never read
            const int cn = cc + 1 < nchunks ? cc + 1 : cc;
            const uint32_t xb = 4u * (uint32_t)cn * (uint32_t)(CK * p.xs[1]);     // byte offset of the chunk
            const uint32_t wb = 4u * (uint32_t)cn * (uint32_t)(PACKED ? BN * WS : KC);
            const int rd_a = 4 * buf * patch_sz, rd_b = 4 * buf * WTS_SZ;
            const int st_a = 4 * (buf ^ 1) * patch_sz, st_b = 4 * (buf ^ 1) * WTS_SZ;

            float a_cur[WM_BLK], b_cur[WN_BLK], a_nxt[WM_BLK], b_nxt[WN_BLK];
            auto read_step = [&](int t, float* a, float* b) {
                const int cl = t / RS9, tap = t % RS9;
                const int offA = 4 * (cl * P + (tap / S_) * RSL + (tap % S_)) + rd_a;
#pragma unroll
                for (int mb = 0; mb < WM_BLK; ++mb) a[mb] = *reinterpret_cast<const float*>(lds + abase[mb] + offA);
#pragma unroll
                for (int nb = 0; nb < WN_BLK; ++nb)
                    b[nb] = *reinterpret_cast<const float*>(lds + bbase[nb] + 4 * t + rd_b);
            };
            read_step(0, a_cur, b_cur);
#pragma unroll
            for (int t = 0; t < SPW; ++t) {
                // reads of step t+1 are issued before the MFMAs of step t: their latency hides
                // behind those MFMAs instead of stalling the next ones
                if (t + 1 < SPW) read_step(t + 1, a_nxt, b_nxt);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int mb = 0; mb < WM_BLK; ++mb)
#pragma unroll
                    for (int nb = 0; nb < WN_BLK; ++nb) {
                        acc[mb][nb] = mfma32(a_cur[mb], b_cur[nb], acc[mb][nb]);
                        const int slot = (t * WM_BLK + mb) * WN_BLK + nb;
                        if (slot < NSIDE) side_load(slot, xb, wb);
                        if (slot >= STORE0) side_store(slot - STORE0, st_a, st_b);
                        __builtin_amdgcn_sched_barrier(0);
                    }
#pragma unroll
                for (int mb = 0; mb < WM_BLK; ++mb) a_cur[mb] = a_nxt[mb];
#pragma unroll
                for (int nb = 0; nb < WN_BLK; ++nb) b_cur[nb] = b_nxt[nb];
            }
            __syncthreads();
        };
        for (int cc = 0; cc < nchunks; cc += 2) {
            chunk(cc, std::integral_constant<int, 0>{});
            if (cc + 1 < nchunks) chunk(cc + 1, std::integral_constant<int, 1>{});
        }
    }

    // ---- Outputs whose quads of four pixels are 16 aligned bytes of y (every tuned shape): the
    //      k-split reduction and the transposition for the stores are one trip through LDS.  In the
    //      accumulator layout a lane is a channel, so storing from it writes 64 separate 16-byte
    //      pieces per instruction.  Instead every wave leaves all its partial blocks in LDS, quad q
    //      (pixels 4q .. 4q+3) of channel c on unit q*32 + (c ^ q) of the block (the XOR keeps both
    //      sides free of bank conflicts); the block's owner then reads with lane = (channel c8 of
    //      eight, quad q), adding the KSPLIT partials in a fixed order, so that eight consecutive
    //      lanes hold 32 consecutive pixels of a channel and a store instruction writes eight whole
    //      128-byte runs, non-temporally (y is not read again).  Cold launches of the 56x56x64 layer:
    //      39.2 us storing from the accumulator layout, 37.9 us with the runs, 36.5 us with the runs
    //      stored non-temporally (the 16-byte pieces stored non-temporally: 43.7 us).
    if (g.vec_store) {
        const int c8 = lane >> 3, q = lane & 7;
        // batch-norm constants of the lane's four channels per channel block, requested before the
        // partials go to LDS so that they arrive behind that and the barrier
        float scale[WN_BLK][4], shift[WN_BLK][4];
        if (p.gamma) {
#pragma unroll
            for (int nb = 0; nb < WN_BLK; ++nb)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    int co = co0 + (wave_n * WN_BLK + nb) * 32 + 8 * j + c8;
                    co = co < p.K ? co : p.K - 1;
                    if (p.scale_shift) {         // folded ahead of time (pre-packed call)
                        scale[nb][j] = p.scale_shift[co];
                        shift[nb][j] = p.scale_shift[p.K + co];
                    } else {
                        scale[nb][j] = p.gamma[co] / sqrtf(p.var[co] + p.eps);
                        shift[nb][j] = p.beta[co] - p.mean[co] * scale[nb][j];
                    }
                }
        }
        f32x4* red = reinterpret_cast<f32x4*>(smem);
#pragma unroll
        for (int b = 0; b < NBLK; ++b) {
            const f32x16& c = acc[b / WN_BLK][b % WN_BLK];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int qa = 2 * v + h;      // the quad these four accumulator registers are
                f32x4 t = {c[4 * v], c[4 * v + 1], c[4 * v + 2], c[4 * v + 3]};
                red[((tile_wave * NBLK + b) * KSPLIT + ks) * 256 + qa * 32 + (r32 ^ qa)] = t;
            }
        }
        __syncthreads();
        // an owned block: all its partial quads are requested from LDS before the first is used (one
        // latency per block, not one per channel), then summed, scaled and stored
        auto finish_block = [&](int b, auto with_bn) {
            const int mb = b / WN_BLK, nb = b % WN_BLK;
            const int mq = m0 + (wave_m * WM_BLK + mb) * 32 + 4 * q;
            const int mc = mq < g.Mtot ? mq : 0;
            const int n = g.d_ohow.div(mc), pix = mc - n * g.ohow;
            float* const yq = p.y + n * p.ys[0] + pix;
            const f32x4* blk = red + (tile_wave * NBLK + b) * KSPLIT * 256 + q * 32;
            f32x4 part[4][KSPLIT];
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int src = 0; src < KSPLIT; ++src) part[j][src] = blk[src * 256 + ((8 * j + c8) ^ q)];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                f32x4 v = part[j][0];
#pragma unroll
                for (int src = 1; src < KSPLIT; ++src)
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] += part[j][src][e];
                if (decltype(with_bn)::value) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = fmaxf(fmaf(v[e], scale[nb][j], shift[nb][j]), 0.f);
                }
                const int co = co0 + (wave_n * WN_BLK + nb) * 32 + 8 * j + c8;
                if (mq < g.Mtot && co < p.K) stg4_nt(yq + co * p.ys[1], v);
            }
        };
#pragma unroll
        for (int b = 0; b < NBLK; ++b) {
            if (ks != b % KSPLIT) continue;
            if (p.gamma)
                finish_block(b, std::true_type{});
            else
                finish_block(b, std::false_type{});
        }
        return;
    }

    // ---- reduce-scatter of the k-split partial accumulators: block b belongs to wave ks == b % KSPLIT
    //      of its tile; the others leave their partials in LDS (the staging buffers are free now)
    if (KSPLIT > 1) {
        f32x4* red = reinterpret_cast<f32x4*>(smem);
#pragma unroll
        for (int b = 0; b < NBLK; ++b) {
            const int owner = b % KSPLIT;
            if (ks != owner) {
                const int src = (ks - owner - 1 + KSPLIT) % KSPLIT;
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const f32x16& c = acc[b / WN_BLK][b % WN_BLK];
                    f32x4 t = {c[4 * v], c[4 * v + 1], c[4 * v + 2], c[4 * v + 3]};
                    red[((((tile_wave * NBLK + b) * (KSPLIT - 1)) + src) * 4 + v) * 64 + lane] = t;
                }
            }
        }
        __syncthreads();
#pragma unroll
        for (int b = 0; b < NBLK; ++b) {
            if (ks == b % KSPLIT) {
#pragma unroll
                for (int src = 0; src < KSPLIT - 1; ++src)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const f32x4 t = red[((((tile_wave * NBLK + b) * (KSPLIT - 1)) + src) * 4 + v) * 64 + lane];
#pragma unroll
                        for (int e = 0; e < 4; ++e) acc[b / WN_BLK][b % WN_BLK][4 * v + e] += t[e];
                    }
            }
        }
    }

    // ---- epilogue, per owned block: accumulator register r of lane (h, r32) is pixel
    //      8*(r/4) + 4*h + r%4, channel r32 of the 32x32 block: four consecutive pixels per quad
#pragma unroll
    for (int b = 0; b < NBLK; ++b) {
        const int mb = b / WN_BLK, nb = b % WN_BLK;
        if (ks != b % KSPLIT) continue;
        const int co = co0 + (wave_n * WN_BLK + nb) * 32 + r32;
        if (co >= p.K) continue;
        float scale = 1.f, shift = 0.f;
        if (p.gamma && p.scale_shift) {         // folded ahead of time (pre-packed call)
            scale = p.scale_shift[co];
            shift = p.scale_shift[p.K + co];
        } else if (p.gamma) {
            scale = p.gamma[co] / sqrtf(p.var[co] + p.eps);
            shift = p.beta[co] - p.mean[co] * scale;
        }
#pragma unroll
        for (int v4 = 0; v4 < 4; ++v4) {
            const int mq = m0 + (wave_m * WM_BLK + mb) * 32 + 8 * v4 + 4 * h;
            f32x4 v = {acc[mb][nb][4 * v4], acc[mb][nb][4 * v4 + 1], acc[mb][nb][4 * v4 + 2],
                       acc[mb][nb][4 * v4 + 3]};
            if (p.gamma) {
#pragma unroll
                for (int r = 0; r < 4; ++r) v[r] = fmaxf(fmaf(v[r], scale, shift), 0.f);
            }
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
    }
}

// Largest number of virtual rows any M-tile of BM pixels needs.  What a whole tile needs
// depends only on where in an image it starts, m0 mod OH*OW, and that repeats after
// OH*OW / gcd(BM, OH*OW) tiles; the clipped last tile needs no more than a whole one at the
// same start.  So one period is scanned, not every tile of a large batch.
inline int max_virtual_rows(const ConvArgs& a, int BM, int HV)
{
    const int64_t Mtot = (int64_t)a.N * a.OH * a.OW;
    const int64_t ohow = (int64_t)a.OH * a.OW;
    int64_t x = BM, y = ohow;
    while (y) { const int64_t t = x % y; x = y; y = t; }
    const int64_t period = ohow / x;                      // tiles until the start offset repeats
    const int64_t tiles = (Mtot + BM - 1) / BM;
    const int64_t scan = tiles < period ? tiles : period;
    int vr = 0;
    for (int64_t t = 0; t < scan; ++t) {
        const int64_t m0 = t * BM;
        const int64_t m1 = (m0 + BM < Mtot ? m0 + BM : Mtot) - 1;
        const int64_t g0 = m0 / a.OW, g1 = m1 / a.OW;
        const int64_t va = (g0 / a.OH) * HV + (g0 % a.OH) * a.stride_h;
        const int64_t vb = (g1 / a.OH) * HV + (g1 % a.OH) * a.stride_h;
        const int need = (int)(vb - va) + a.R;
        if (need > vr) vr = need;
    }
    return vr;
}

template <int WM_BLK, int WN_BLK, int WAVES_M, int WAVES_N, int KSPLIT, int R_, int S_, int CPH>
struct Variant {
    static constexpr int NT = 64 * WAVES_M * WAVES_N * KSPLIT;
    static constexpr int BM = 32 * WM_BLK * WAVES_M, BN = 32 * WN_BLK * WAVES_N;
    static constexpr int CK = 2 * CPH;
    static constexpr int WS = CK * R_ * S_ + 4;
    // staging units per thread the main loop can hide: half of a wave's MFMAs per chunk carry one
    static constexpr int WU = (BN * (CK * R_ * S_ / 4) + NT - 1) / NT;
    static constexpr int SLOTS = (CPH * R_ * S_ / KSPLIT) * WM_BLK * WN_BLK;
    static constexpr int kMaxXU = (SLOTS / 2 - WU) < kMaxUnits ? (SLOTS / 2 - WU) : kMaxUnits;

    // Floats of the packed weights: per channel tile and chunk one LDS image of BN rows of KC + 4.
    static int64_t packed_floats(const ConvArgs& a)
    {
        return (int64_t)((a.K + BN - 1) / BN) * (a.C / CK) * BN * WS;
    }

    // Fills the geometry; false if this variant cannot run the problem.
    static bool plan(const ConvArgs& a, Geom* g, size_t* lds_bytes)
    {
        if (a.R != R_ || a.S != S_ || a.C % CK != 0) return false;
        g->Mtot = a.N * a.OH * a.OW;
        g->ohow = a.OH * a.OW;
        g->HV = (a.OH - 1) * a.stride_h + a.R;
        g->VR = max_virtual_rows(a, BM, g->HV);
        g->XC = (a.pad_w + 3) / 4 * 4;
        const int wv = (a.OW - 1) * a.stride_w + a.S;           // virtual row width
        const int need_cols = g->XC - a.pad_w + (wv > a.W + a.pad_w ? wv : a.W + a.pad_w);
        g->RSL = (need_cols + 3) / 4 * 4;
        g->P = g->VR * g->RSL;
        g->W4 = a.W / 4;
        g->n_units = CK * g->VR * g->W4;
        {
            const int per_c = g->VR * g->W4, rest = NT % per_c;
            g->st_ci = NT / per_c;
            g->st_vr = rest / g->W4;
            g->st_j4 = rest % g->W4;
            // one (row, quad) per thread where that needs no more slots than dealing the units out singly
            g->slots = (g->n_units + NT - 1) / NT;
            g->row_groups = 0;
            if (per_c <= NT) {
                const int groups = NT / per_c < CK ? NT / per_c : CK;
                const int slots = (CK + groups - 1) / groups;
                if (slots <= g->slots) {
                    g->row_groups = groups;
                    g->slots = slots;
                }
            }
        }
        if (kMaxXU < 1 || g->n_units > kMaxXU * NT) return false;
        // virtual row numbers must stay below 2^31 for the fast division
        if ((int64_t)a.N * g->HV + g->VR >= ((int64_t)1 << 31)) return false;
        g->vec_store = (g->ohow % 4 == 0) && a.ys[2] == a.OW && (a.ys[0] % 4 == 0) &&
                       (a.ys[1] % 4 == 0) && is_aligned16(a.y);
        g->d_ow = make_fastdiv(a.OW);
        g->d_oh = make_fastdiv(a.OH);
        g->d_hv = make_fastdiv(g->HV);
        g->d_w4 = make_fastdiv(g->W4);
        g->d_perc = make_fastdiv(g->VR * g->W4);
        g->d_ohow = make_fastdiv(g->ohow);
        g->d_units = make_fastdiv(g->n_units);
        g->x_bytes = (uint32_t)(4 * ((int64_t)(a.N - 1) * a.xs[0] + (int64_t)(a.C - 1) * a.xs[1] +
                                     (int64_t)(a.H - 1) * a.xs[2] + a.W));
        g->w_bytes = (uint32_t)(4 * (int64_t)a.K * a.C * a.R * a.S);
        g->wpack_bytes = (uint32_t)(4 * packed_floats(a));
        // XCD-aware tile mapping: split the tile grid 8 ways (xcd_m x xcd_n) so that the bytes one
        // XCD has to pull through its L2 (its share of x plus its share of w) are smallest
        g->tiles_m = (g->Mtot + BM - 1) / BM;
        g->tiles_n = (a.K + BN - 1) / BN;
        if ((int64_t)g->tiles_m * g->tiles_n >= ((int64_t)1 << 31)) return false;
        g->xcd_m = g->xcd_n = 0;
        {
            const double xb = (double)a.N * a.C * a.H * a.W, wb = (double)a.K * a.C * a.R * a.S;
            double best = 0.0;
            for (int xm = 1; xm <= 8; xm *= 2) {
                const int xn = 8 / xm;
                if (g->tiles_m % xm != 0 || g->tiles_n % xn != 0) continue;
                const double bytes = xb / xm + wb / xn;
                if (g->xcd_m == 0 || bytes < best) {
                    best = bytes;
                    g->xcd_m = xm;
                    g->xcd_n = xn;
                }
            }
        }
        g->sub_m = g->xcd_m ? g->tiles_m / g->xcd_m : 0;
        g->sub_n = g->xcd_n ? g->tiles_n / g->xcd_n : 0;
        g->xcd_n_shift = 0;
        while (g->xcd_n && (1 << g->xcd_n_shift) < g->xcd_n) ++g->xcd_n_shift;
        g->d_sub_n = make_fastdiv(g->xcd_n ? g->sub_n : 1);
        g->d_tiles_m = make_fastdiv(g->tiles_m);
        *lds_bytes = lds_bytes_for(*g, 2);
        return *lds_bytes <= 160 * 1024;
    }

    // LDS of a work-group with `nbuf` staging buffers
    static size_t lds_bytes_for(const Geom& g, int nbuf)
    {
        size_t floats = nbuf * ((size_t)CK * g.P + (size_t)BN * WS);
        // the k-split reduction reuses the staging memory: every wave's partial blocks
        const size_t red = (size_t)KSPLIT * WAVES_M * WAVES_N * WM_BLK * WN_BLK * 64 * 16;
        if (red > floats) floats = red;
        return sizeof(float) * floats;
    }

    template <int XU, int RSL_T, int P_T, int NBUF = 2>
    static hipError_t launch_inst(const ConvArgs& a, const Geom& g, size_t lds_bytes, hipStream_t stream)
    {
        return a.wpack ? launch_as<XU, RSL_T, P_T, true, NBUF>(a, g, lds_bytes, stream)
                       : launch_as<XU, RSL_T, P_T, false, NBUF>(a, g, lds_bytes, stream);
    }

    template <int XU, int RSL_T, int P_T, bool PACKED, int NBUF>
    static hipError_t launch_as(const ConvArgs& a, const Geom& g, size_t lds_bytes, hipStream_t stream)
    {
        auto kern = conv_igemm_kernel<WM_BLK, WN_BLK, WAVES_M, WAVES_N, KSPLIT, R_, S_, CPH, XU, RSL_T, P_T, PACKED, NBUF>;
        if (lds_bytes > 64 * 1024) {
            static LdsLimit granted;
            hipError_t e = raise_lds_limit(reinterpret_cast<const void*>(kern), lds_bytes, granted);
            if (e != hipSuccess) return e;
        }
        dim3 grid((unsigned)(g.tiles_m * g.tiles_n));
        return launch_kernel(kern, grid, dim3(NT), lds_bytes, stream, a, g);
    }

    static int units_per_thread(const Geom& g) { return g.slots; }

    // Instantiation with the LDS geometry (row stride, plane stride) and the number of staging
    // units per thread fixed at compile time; the caller has checked that g matches.  These run
    // the ring of three staging buffers (every shape they are made for leaves room for it).
    template <int XU, int RSL_T, int P_T, int NBUF = 2>
    static hipError_t launch_fixed(const ConvArgs& a, const Geom& g, size_t lds_bytes, hipStream_t stream)
    {
        static_assert(NBUF * sizeof(float) * ((size_t)CK * P_T + (size_t)BN * WS) <= 160 * 1024, "LDS");
        return launch_inst<XU, RSL_T, P_T, NBUF>(a, g, NBUF == 2 ? lds_bytes : lds_bytes_for(g, NBUF), stream);
    }

    // Any geometry: LDS strides are run-time values (address arithmetic stays in the loop).
    static hipError_t launch(const ConvArgs& a, const Geom& g, size_t lds_bytes, hipStream_t stream)
    {
        const int per_thread = units_per_thread(g);
        if constexpr (kMaxXU >= 2) {
            if (per_thread <= 2) return launch_inst<2, 0, 0>(a, g, lds_bytes, stream);
        }
        if constexpr (kMaxXU >= 4) {
            if (per_thread <= 4) return launch_inst<4, 0, 0>(a, g, lds_bytes, stream);
        }
        if constexpr (kMaxXU >= 6) {
            if (per_thread <= 6) return launch_inst<6, 0, 0>(a, g, lds_bytes, stream);
        }
        if constexpr (kMaxXU >= 1) return launch_inst<kMaxXU, 0, 0>(a, g, lds_bytes, stream);
        return hipErrorInvalidValue;     // unreachable: plan() rejects variants with kMaxXU < 1
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

}  // namespace igemm
}  // namespace anr
