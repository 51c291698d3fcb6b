// Tile and split-K selection and launch of the general implicit-GEMM convolution (kernels
// and their description in conv_gather_kernel.h).
#include <algorithm>
#include "conv_gather_kernel.h"

namespace anr {
namespace {

using namespace gconv;

struct Tile {
    int bm, bn;
    double chunk_us;    // CU time per chunk and work-group when the CU is saturated with work-groups
    double lone_us;     // time per chunk of a work-group that has its CU to itself
    int occupancy;      // work-groups one CU holds (LDS, registers)
};
constexpr Tile kTiles[] = {{128, 128, 3.2, 2.8, 2}, {128, 64, 1.6, 1.9, 3}, {64, 64, 0.8, 1.1, 4}};
constexpr int kCUs = 256;
constexpr double kLaunchUs = 2.0;            // launch plus prologue and epilogue
constexpr double kWsBytesPerUs = 3.0e6;      // workspace traffic, bytes per microsecond

bool make_plan(const ConvArgs& a, Plan* g, bool allow_taps = true)
{
    const int64_t x_extent = (int64_t)(a.N - 1) * a.xs[0] + (int64_t)(a.C - 1) * a.xs[1] +
                             (int64_t)(a.H - 1) * a.xs[2] + a.W;
    const int64_t w_extent = (int64_t)a.K * (a.C / a.groups) * a.R * a.S;
    const int64_t Mtot = (int64_t)a.N * a.OH * a.OW;
    // byte offsets must stay below the out-of-range marker of the buffer loads (2^31)
    if (x_extent >= ((int64_t)1 << 29) || w_extent >= ((int64_t)1 << 29) || Mtot >= ((int64_t)1 << 30))
        return false;
    // the tap table packs row and column displacements into 16 bits each, and a displacement
    // of kNoRow must leave every image
    if (a.H + a.pad_h >= kMaxExtent || a.W + a.pad_w >= kMaxExtent || (a.R - 1) * (int64_t)a.dil_h >= kMaxExtent ||
        (a.S - 1) * (int64_t)a.dil_w >= kMaxExtent)
        return false;
    g->Mtot = (int)Mtot;
    g->ohow = a.OH * a.OW;
    g->RS = a.R * a.S;
    g->Cg = a.C / a.groups;
    g->Kg = a.K / a.groups;
    g->groups = a.groups;
    g->pack_cg = g->pack_kg = 0;
    g->d_pack_kg = make_fastdiv(1);
    // 1 x 1 kernels of small groups: 64 / Kg groups share a column tile (conv_taps_kernel, PACK)
    if (allow_taps && is_aligned16(a.w) && a.R == 1 && a.S == 1 && a.groups > 1 && g->Kg < 64 && 64 % g->Kg == 0 &&
        g->Cg % 4 == 0 && (g->Kg <= 16 || g->Cg % 32 != 0)) {
        const int pack = 64 / g->Kg;
        if (a.groups % pack == 0 && (pack * g->Cg) % 32 == 0) {
            g->pack_cg = g->Cg;
            g->pack_kg = g->Kg;
            g->d_pack_kg = make_fastdiv(g->Kg);
            g->groups = a.groups / pack;
            g->Cg *= pack;
            g->Kg = 64;
        }
    }
    g->Ktot = g->Cg * g->RS;
    g->d_kg = make_fastdiv(g->Kg);
    // 3 x 3 and 1 x 1 kernels whose channels fill whole chunks take the form with compile-time taps
    g->taps = 0;
    g->kc = KC;
    // 7 x 7 and 5 x 5: one channel per chunk, its 49 (25) taps padded to 52 (28)
    if (allow_taps && a.R == 7 && a.S == 7) { g->taps = 49; g->kc = 52; }
    if (allow_taps && a.R == 5 && a.S == 5) { g->taps = 25; g->kc = 28; }
    if (allow_taps && is_aligned16(a.w)) {
        if (a.R == 3 && a.S == 3 && g->Cg % 4 == 0) { g->taps = 9; g->kc = 36; }
        if (a.R == 1 && a.S == 1 && g->Cg % 32 == 0) { g->taps = 1; g->kc = 32; }
    }
    g->nchunks = g->taps >= 25 ? g->Cg : (g->Ktot + g->kc - 1) / g->kc;
    g->w_vec = (g->Ktot % 4 == 0) && is_aligned16(a.w);
    g->vec_store = (g->ohow % 4 == 0) && a.ys[2] == a.OW && (a.ys[0] % 4 == 0) && (a.ys[1] % 4 == 0) &&
                   is_aligned16(a.y);
    g->x_bytes = (uint32_t)(4 * x_extent);
    g->w_bytes = (uint32_t)(4 * w_extent);
    g->d_ow = make_fastdiv(a.OW);
    g->d_oh = make_fastdiv(a.OH);
    g->d_rs = make_fastdiv(g->RS);
    g->d_s = make_fastdiv(a.S);
    g->d_ohow = make_fastdiv(g->ohow);

    return true;
}

// Fixes the tile and the split of the reduction (ks is lowered until no split is empty).
void set_tile(const ConvArgs& a, Plan* g, int bm, int bn, int ks)
{
    g->bm = bm;
    g->bn = bn;
    g->tiles_m = (g->Mtot + bm - 1) / bm;
    g->tiles_ng = (g->Kg + bn - 1) / bn;
    g->tiles_n = g->groups * g->tiles_ng;
    g->d_tiles_ng = make_fastdiv(g->tiles_ng);
    if (ks < 1) ks = 1;
    if (ks > g->nchunks) ks = g->nchunks;
    g->chunks_per_split = (g->nchunks + ks - 1) / ks;
    g->ksplit = (g->nchunks + g->chunks_per_split - 1) / g->chunks_per_split;
    g->Mpad = g->tiles_m * bm;
    g->Kpad = g->tiles_n * bn;
    g->d_tiles_m = make_fastdiv(g->tiles_m);
    g->d_tiles = make_fastdiv(g->tiles_m * g->tiles_n);
    // conv_taps_kernel: with at most one work-group per CU and a long chain of chunks, two or four
    // groups of waves share the chain (measured: 196 work-groups x 16 chunks 18.3 -> 16.9 us, x 32
    // chunks 27.7 -> 24.3 us; with more work-groups per CU or short chains the larger work-groups
    // only cost occupancy)
    g->nwg = 1;
    if ((g->taps == 9 || g->taps == 1) && g->pack_cg == 0 && (int64_t)g->tiles_m * g->tiles_n * g->ksplit <= kCUs) {
        if (g->chunks_per_split >= 32) g->nwg = 4;
        else if (g->chunks_per_split >= 8) g->nwg = 2;
    }
    // tiles stored in runs of 64 pixels per channel (1 x 1 layers, 56 x 56 and 28 x 28 maps at batch 16:
    // 3-4 % faster than one 16-byte piece per lane and channel; the 7 x 7 stem at batch 16, which writes
    // 51 MB: 7 %; partial tiles of a split reduction, whose workspace is padded and aligned: 1-2 %)
    g->tstore = (g->taps != 0 || (bm == 64 && bn == 64)) && g->nwg == 1 && (g->ksplit > 1 || g->vec_store);
    g->rblocks = (g->Mpad / 4 * reduce_lanes(g->ksplit) + 255) / 256;
    g->d_rblocks = make_fastdiv(g->rblocks);
}

// Estimated run time in microseconds of tile t with the reduction split ks ways.  Two bounds:
// the work of the busiest CU when it is saturated (work-groups are dealt evenly over the CUs
// and those on one CU share its matrix pipes), and the serial chain of chunks of one
// work-group, which only concurrency across work-groups hides.  Constants are fits to
// measurements on the shape lists of Appendix C.
double estimate_us(const Plan& g, const ConvArgs& a, const Tile& t, int ks)
{
    const int64_t tiles = (int64_t)((g.Mtot + t.bm - 1) / t.bm) * g.groups * ((g.Kg + t.bn - 1) / t.bn);
    const int cps = (g.nchunks + ks - 1) / ks;
    const int ks_eff = (g.nchunks + cps - 1) / cps;
    const int64_t wgs = tiles * ks_eff;
    const double per_cu = (double)((wgs + kCUs - 1) / kCUs);
    const double mfma_us = per_cu * cps * t.chunk_us;
    const double resident = per_cu < t.occupancy ? per_cu : t.occupancy;
    const double latency_us = (per_cu / resident) * (cps + 2) * t.lone_us;
    double us = kLaunchUs + (mfma_us > latency_us ? mfma_us : latency_us);
    if (ks_eff > 1) {
        // second launch; partial tiles written and read back
        const double ws_bytes = 4.0 * ks_eff * tiles * t.bm * t.bn;
        us += kLaunchUs + 2.0 * ws_bytes / kWsBytesPerUs;
    }
    return us;
}

// The same estimate for conv_taps_kernel, which runs 64 x 64 tiles only (the larger tiles were
// slower on every layer shape of a sweep over ResNet-style 3 x 3 and 1 x 1 layers at batch 1, 4
// and 16).  A work-group's chain is a prologue plus its chunks; a chunk takes kLoneUs when the
// work-group has the CU to itself and kChunkUs per resident work-group once they saturate it.
double estimate_taps_us(const Plan& g, const ConvArgs& a, int ks)
{
    constexpr double kPrologueUs = 0.9, kLoneUs = 0.78, kChunkUs = 0.65;   // per chunk of 36
    constexpr double kMainUs = 2.6, kReduceUs = 4.5, kWsRate = 4.85e6;     // launches; workspace bytes per us
    const int64_t tiles = (int64_t)((g.Mtot + 63) / 64) * g.groups * ((g.Kg + 63) / 64);
    const int cps = (g.nchunks + ks - 1) / ks;
    const int ks_eff = (g.nchunks + cps - 1) / cps;
    const int64_t wgs = tiles * ks_eff;
    const double per_cu = (double)((wgs + kCUs - 1) / kCUs);
    const double resident = per_cu < 4.0 ? per_cu : 4.0;
    const double per_chunk = resident * kChunkUs > kLoneUs ? resident * kChunkUs : kLoneUs;
    double us = kMainUs + (per_cu / resident) * (kPrologueUs + cps * (g.kc / 36.0) * per_chunk);
    if (ks_eff > 1) us += kReduceUs + 2.0 * 4.0 * ks_eff * tiles * 4096.0 / kWsRate;
    return us;
}

// The reduction is split over work-groups only when x and w are 16-byte aligned (null pointers,
// i.e. planning without buffers, count as aligned): the workspace a descriptor needs is then the
// need of that one plan, whatever pointers a call brings.
bool choose_tile(const ConvArgs& a, Plan* g)
{
    double best = 0.0;
    bool have = false;
    int bm = 0, bn = 0, bks = 1;
    const bool may_split = is_aligned16(a.x) && is_aligned16(a.w);
    if (g->taps) {
        const int64_t tiles = (int64_t)((g->Mtot + 63) / 64) * g->groups * ((g->Kg + 63) / 64);
        if (tiles >= ((int64_t)1 << 24)) return false;
        const int most = (tiles >= 2 * kCUs || !may_split) ? 1 : g->nchunks;
        int last_cps = 0;
        for (int ks = 1; ks <= most; ++ks) {
            const int cps = (g->nchunks + ks - 1) / ks;
            if (cps == last_cps) continue;
            last_cps = cps;
            if (ks > 1 && 4.0 * ks * tiles * 4096.0 > 256e6) break;   // keep the workspace modest
            const double us = estimate_taps_us(*g, a, ks);
            if (!have || us < best) {
                have = true;
                best = us;
                bks = ks;
            }
        }
        set_tile(a, g, 64, 64, bks);
        return true;
    }
    for (const Tile& t : kTiles) {
        const int64_t tiles = (int64_t)((g->Mtot + t.bm - 1) / t.bm) * g->groups * ((g->Kg + t.bn - 1) / t.bn);
        if (tiles >= ((int64_t)1 << 24)) continue;
        const int most = (tiles >= 2 * kCUs || !may_split) ? 1 : g->nchunks;      // enough tiles: no split
        int last_cps = 0;
        for (int ks = 1; ks <= most; ++ks) {
            const int cps = (g->nchunks + ks - 1) / ks;
            if (cps == last_cps) continue;                        // same split as the previous ks
            last_cps = cps;
            if (ks > 1 && 4.0 * ks * tiles * t.bm * t.bn > 256e6) break;     // keep the workspace modest (none without a split)
            const double us = estimate_us(*g, a, t, ks);
            if (!have || us < best) {
                have = true;
                best = us;
                bm = t.bm;
                bn = t.bn;
                bks = ks;
            }
        }
    }
    if (!have) return false;
    set_tile(a, g, bm, bn, bks);
    return true;
}

size_t plan_workspace(const Plan& g)
{
    return g.ksplit > 1 ? sizeof(float) * (size_t)g.ksplit * g.Kpad * g.Mpad : 0;
}

template <int BM, int BN, bool MASK>
hipError_t launch_tile_as(const ConvArgs& a, const Plan& g, hipStream_t stream)
{
    const size_t lds_bytes = sizeof(float) * 2 * (size_t)(BM + BN) * WS;
    auto kern = conv_gather_kernel<BM, BN, MASK>;
    if (lds_bytes > 48 * 1024) {
        static LdsLimit granted;
        hipError_t e = raise_lds_limit(reinterpret_cast<const void*>(kern), lds_bytes, granted);
        if (e != hipSuccess) return e;
    }
    const unsigned grid = (unsigned)(g.tiles_m * g.tiles_n * g.ksplit);
    return launch_kernel(kern, dim3(grid), dim3(256), lds_bytes, stream, a, g);
}

template <int BM, int BN, int R_, int S_, int NWG, bool PACK = false>
hipError_t launch_tile_taps(const ConvArgs& a, const Plan& g, hipStream_t stream)
{
    const size_t lds_bytes = sizeof(float) * NWG * 2 * (size_t)(BM + BN) * (g.kc + 2);
    auto kern = conv_taps_kernel<BM, BN, R_, S_, NWG, PACK>;
    if (lds_bytes > 48 * 1024) {
        static LdsLimit granted;
        hipError_t e = raise_lds_limit(reinterpret_cast<const void*>(kern), lds_bytes, granted);
        if (e != hipSuccess) return e;
    }
    const unsigned grid = (unsigned)(g.tiles_m * g.tiles_n * g.ksplit);
    return launch_kernel(kern, dim3(grid), dim3(256 * NWG), lds_bytes, stream, a, g);
}

template <int R_, int S_>
hipError_t launch_taps_groups(const ConvArgs& a, const Plan& g, hipStream_t stream)
{
    if (g.nwg == 4) return launch_tile_taps<64, 64, R_, S_, 4>(a, g, stream);
    if (g.nwg == 2) return launch_tile_taps<64, 64, R_, S_, 2>(a, g, stream);
    return launch_tile_taps<64, 64, R_, S_, 1>(a, g, stream);
}

template <int BM, int BN>
hipError_t launch_tile(const ConvArgs& a, const Plan& g, hipStream_t stream)
{
    // up to 31 taps fit the per-pixel mask of the cheaper gather
    return g.RS <= 31 ? launch_tile_as<BM, BN, true>(a, g, stream) : launch_tile_as<BM, BN, false>(a, g, stream);
}

}  // namespace

hipError_t launch_gather_plan(const ConvArgs& a, const Plan& g, hipStream_t stream);

size_t conv2d_gather_workspace_bytes(const ConvArgs& a)
{
    Plan g;
    return make_plan(a, &g) && choose_tile(a, &g) ? plan_workspace(g) : 0;
}

bool describe_conv2d_gather(const ConvArgs& a, ConvRoute* r)
{
    Plan g;
    if (!(make_plan(a, &g) && choose_tile(a, &g))) return false;
    r->kernel = g.taps >= 25 ? 3 : (g.taps ? 2 : 4);
    r->tile_m = g.bm;
    r->tile_n = g.bn;
    r->ksplit = g.ksplit;
    r->wave_groups = g.nwg;
    r->work_groups = g.tiles_m * g.tiles_n * g.ksplit;
    r->workspace_bytes = plan_workspace(g);
    return true;
}

hipError_t launch_conv2d_gather(const ConvArgs& a, hipStream_t stream, bool* taken, int* ws_fault)
{
    Plan g;
    *ws_fault = 0;
    *taken = make_plan(a, &g) && choose_tile(a, &g);
    if (!*taken) return hipSuccess;
    const size_t need = plan_workspace(g);
    if (need > 0) {
        if (a.ws == nullptr || a.ws_bytes < need) *ws_fault = 1;
        else if (!is_aligned16(a.ws)) *ws_fault = 2;
        if (*ws_fault) return hipSuccess;
    }
    return launch_gather_plan(a, g, stream);
}

hipError_t launch_gather_plan(const ConvArgs& a, const Plan& g, hipStream_t stream)
{
    const size_t need = plan_workspace(g);
    if (need > 0 && (a.ws == nullptr || a.ws_bytes < need || !is_aligned16(a.ws))) return hipErrorInvalidValue;
    hipError_t err;
    if (g.taps) {
        if (g.bm != 64 || g.bn != 64) return hipErrorInvalidValue;
        if (g.taps >= 25) {
            // staging tiles, or the transposed output tile of the epilogue if that is larger
            const size_t lds_bytes = sizeof(float) * std::max<size_t>((size_t)(64 + 64) * (g.kc + 2), kRunTileFloats);
            const unsigned grid = (unsigned)(g.tiles_m * g.tiles_n * g.ksplit);
            err = g.taps == 49 ? launch_kernel(conv_bigtaps_kernel<7, 7>, dim3(grid), dim3(256), lds_bytes, stream, a, g)
                               : launch_kernel(conv_bigtaps_kernel<5, 5>, dim3(grid), dim3(256), lds_bytes, stream, a, g);
        } else {
            err = g.taps == 9     ? launch_taps_groups<3, 3>(a, g, stream)
                  : g.pack_cg > 0 ? launch_tile_taps<64, 64, 1, 1, 1, true>(a, g, stream)
                                  : launch_taps_groups<1, 1>(a, g, stream);
        }
    } else if (g.bm == 128 && g.bn == 128) err = launch_tile<128, 128>(a, g, stream);
    else if (g.bm == 128) err = launch_tile<128, 64>(a, g, stream);
    else err = launch_tile<64, 64>(a, g, stream);
    if (err != hipSuccess || g.ksplit == 1) return err;
    const dim3 rgrid((unsigned)((int64_t)a.K * g.rblocks));
    switch (reduce_lanes(g.ksplit)) {
        case 8: return launch_kernel(conv_splitk_reduce_kernel<8>, rgrid, dim3(256), 0, stream, a, g);
        case 4: return launch_kernel(conv_splitk_reduce_kernel<4>, rgrid, dim3(256), 0, stream, a, g);
        case 2: return launch_kernel(conv_splitk_reduce_kernel<2>, rgrid, dim3(256), 0, stream, a, g);
        default: return launch_kernel(conv_splitk_reduce_kernel<1>, rgrid, dim3(256), 0, stream, a, g);
    }
}

}  // namespace anr
