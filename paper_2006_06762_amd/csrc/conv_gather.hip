// Tile and split-K selection and launch of the general implicit-GEMM convolution (kernels
// and their description in conv_gather_kernel.h).
#include "conv_gather_kernel.h"

namespace anr {
namespace {

using namespace gconv;

struct Tile {
    int bm, bn;
    double eff;     // MFMA issue efficiency relative to the largest tile (fewer loads per MFMA)
};
constexpr Tile kTiles[] = {{128, 128, 1.0}, {128, 64, 0.8}, {64, 64, 0.6}};
constexpr int kCUs = 256;

bool make_plan(const ConvArgs& a, Plan* g)
{
    const int64_t x_extent = (int64_t)(a.N - 1) * a.xs[0] + (int64_t)(a.C - 1) * a.xs[1] +
                             (int64_t)(a.H - 1) * a.xs[2] + a.W;
    const int64_t w_extent = (int64_t)a.K * a.C * a.R * a.S;
    const int64_t Mtot = (int64_t)a.N * a.OH * a.OW;
    // byte offsets must stay below the out-of-range marker of the buffer loads (2^31)
    if (x_extent >= ((int64_t)1 << 29) || w_extent >= ((int64_t)1 << 29) || Mtot >= ((int64_t)1 << 30))
        return false;
    g->Mtot = (int)Mtot;
    g->ohow = a.OH * a.OW;
    g->RS = a.R * a.S;
    g->Ktot = a.C * g->RS;
    g->nchunks = (g->Ktot + KC - 1) / KC;
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

    // tile and split: fewest rounds of work-groups over the CUs, weighted by the tile's efficiency
    double best = 0.0;
    bool have = false;
    for (const Tile& t : kTiles) {
        const int64_t tm = (Mtot + t.bm - 1) / t.bm, tn = (a.K + t.bn - 1) / t.bn;
        const int64_t tiles = tm * tn;
        if (tiles >= ((int64_t)1 << 24)) continue;
        int ks = 1;
        if (tiles < 192) {
            const int want = (int)((320 + tiles - 1) / tiles);          // aim at ~320 work-groups
            const int most = g->nchunks / 2 > 1 ? g->nchunks / 2 : 1;     // at least two chunks per split
            ks = want < most ? want : most;
        }
        const int cps = (g->nchunks + ks - 1) / ks;
        ks = (g->nchunks + cps - 1) / cps;                               // no empty split
        const int64_t wgs = tiles * ks;
        const double rounds = (double)((wgs + kCUs - 1) / kCUs);
        double cost = rounds * cps * (double)t.bm * t.bn / t.eff;
        if (ks > 1) cost += 3.0 * 128 * 128;                             // second launch and the partial tiles
        if (!have || cost < best) {
            have = true;
            best = cost;
            g->bm = t.bm;
            g->bn = t.bn;
            g->tiles_m = (int)tm;
            g->tiles_n = (int)tn;
            g->ksplit = ks;
            g->chunks_per_split = cps;
        }
    }
    if (!have) return false;
    g->Mpad = g->tiles_m * g->bm;
    g->Kpad = g->tiles_n * g->bn;
    g->d_tiles_m = make_fastdiv(g->tiles_m);
    g->d_tiles = make_fastdiv(g->tiles_m * g->tiles_n);
    return true;
}

size_t plan_workspace(const Plan& g)
{
    return g.ksplit > 1 ? sizeof(float) * (size_t)g.ksplit * g.Kpad * g.Mpad : 0;
}

template <int BM, int BN>
hipError_t launch_tile(const ConvArgs& a, const Plan& g, hipStream_t stream)
{
    const size_t lds_bytes = sizeof(float) * 2 * (size_t)(BM + BN) * WS;
    auto kern = conv_gather_kernel<BM, BN>;
    if (lds_bytes > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return e;
    }
    const unsigned grid = (unsigned)(g.tiles_m * g.tiles_n * g.ksplit);
    return launch_kernel(kern, dim3(grid), dim3(256), lds_bytes, stream, a, g);
}

}  // namespace

size_t conv2d_gather_workspace_bytes(const ConvArgs& a)
{
    Plan g;
    return make_plan(a, &g) ? plan_workspace(g) : 0;
}

hipError_t launch_conv2d_gather(const ConvArgs& a, hipStream_t stream, bool* taken)
{
    Plan g;
    *taken = make_plan(a, &g);
    if (!*taken) return hipSuccess;
    const size_t need = plan_workspace(g);
    if (need > 0 && (a.ws == nullptr || a.ws_bytes < need || !is_aligned16(a.ws))) return hipErrorInvalidValue;
    hipError_t err;
    if (g.bm == 128 && g.bn == 128) err = launch_tile<128, 128>(a, g, stream);
    else if (g.bm == 128) err = launch_tile<128, 64>(a, g, stream);
    else err = launch_tile<64, 64>(a, g, stream);
    if (err != hipSuccess || g.ksplit == 1) return err;
    const int64_t threads = (int64_t)a.K * (g.Mpad / 4);
    return launch_kernel(conv_splitk_reduce_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, stream,
                         a, g);
}

}  // namespace anr
