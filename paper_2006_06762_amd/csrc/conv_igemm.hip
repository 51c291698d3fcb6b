// Variant table and shape-driven selection for the implicit-GEMM convolution
// (kernel and its description in conv_igemm_kernel.h).
#include "conv_igemm_kernel.h"

namespace anr {
namespace {

using namespace igemm;

//                       WM WN  wM wN ks  R  S CPH   (tile = 32*WM*wM pixels x 32*WN*wN channels)
using V224x64 = Variant<7, 1, 1, 2, 2, 3, 3, 4>;   // 4 waves: two 7x1-block tiles, 2-way k split
using V224x32 = Variant<7, 1, 1, 1, 4, 3, 3, 4>;   // 4 waves share one 7x1-block tile along k
using V128x64 = Variant<2, 2, 2, 1, 2, 3, 3, 4>;   // 4 waves, 2x2 blocks each, 2-way k split
using V64x64 = Variant<2, 2, 1, 1, 4, 3, 3, 4>;    // 4 waves share one 2x2-block tile along k

template <class V>
void consider(const ConvArgs& a, double* best_cost, int* best, int id, Geom* g, size_t* lds)
{
    Geom gg;
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

// Instantiations whose LDS geometry is a compile-time constant, one per (tile variant, LDS
// row stride, LDS plane stride): the shapes of the ResNet-style 3x3 layers this library is
// tuned on.  Anything else runs the same kernel with run-time strides.
template <class V, int XU, int RSL_T, int P_T, int NBUF>
bool try_fixed(const ConvArgs& a, const Geom& g, size_t lds, hipStream_t stream, hipError_t* err)
{
    if (g.RSL != RSL_T || g.P != P_T || V::units_per_thread(g) > XU) return false;
    *err = V::template launch_fixed<XU, RSL_T, P_T, NBUF>(a, g, lds, stream);
    return true;
}


// Picks the variant for `a`: its index, geometry and LDS size; -1 when no variant runs it.
int select_variant(const ConvArgs& a, Geom* g, size_t* lds)
{
    const int64_t x_extent = (int64_t)(a.N - 1) * a.xs[0] + (int64_t)(a.C - 1) * a.xs[1] +
                             (int64_t)(a.H - 1) * a.xs[2] + a.W;
    const int64_t w_extent = (int64_t)a.K * a.C * a.R * a.S;
    // 32-bit byte offsets inside x and w, 31-bit pixel and virtual-row indices
    // 3 x 3 only: pointwise layers were measured through this kernel as well (chunks of 32
    // channels) and ran level with or behind conv_taps_kernel on every ResNet-style shape
    const bool k3 = a.R == 3 && a.S == 3 && (a.C % 8 == 0);
    const bool ok = k3 && a.dil_h == 1 && a.dil_w == 1 && a.groups == 1 && (a.W % 4 == 0) && is_aligned16(a.x) &&
                    is_aligned16(a.w) && (a.xs[0] % 4 == 0) && (a.xs[1] % 4 == 0) &&
                    (a.xs[2] % 4 == 0) && x_extent < (int64_t)1 << 30 && w_extent < (int64_t)1 << 30 &&
                    (int64_t)a.N * a.OH * a.OW < (int64_t)1 << 30;
    if (!ok) return -1;

    double best_cost = 0.0;
    int best = -1;
    consider<V224x64>(a, &best_cost, &best, 0, g, lds);
    consider<V224x32>(a, &best_cost, &best, 1, g, lds);
    consider<V128x64>(a, &best_cost, &best, 2, g, lds);
    consider<V64x64>(a, &best_cost, &best, 3, g, lds);
    return best;
}

// The tuned kernel has no split of the reduction across work-groups: with few output tiles
// (batch 1) most CUs would idle, and the general kernel with split-K is faster.
constexpr int kMinTunedWorkGroups = 112;

struct IgemmPlan {
    int variant;     // 0 V224x64, 1 V224x32, 2 V128x64, 3 V64x64; -1: the kernel does not take the call
    Geom g;
    size_t lds;
};

// The one planning pass of a call: variant, geometry and LDS size, with the descriptor's route
// applied (1: whenever a variant runs the shape; 2: never; 0: with enough output tiles).  Depends
// on the descriptor and on the alignment of x and w only (null pointers count as aligned), so a
// pack made for a descriptor fits every later call with it.
void plan_igemm(const ConvArgs& a, IgemmPlan* p)
{
    p->variant = -1;
    if (a.route == 2) return;
    const int best = select_variant(a, &p->g, &p->lds);
    if (best < 0) return;
    if (a.route != 1 && (int64_t)p->g.tiles_m * p->g.tiles_n < kMinTunedWorkGroups) return;
    p->variant = best;
}

hipError_t launch_igemm_plan(const ConvArgs& a, const IgemmPlan& p, hipStream_t stream)
{
    const Geom& g = p.g;
    const size_t lds = p.lds;
    hipError_t err = hipSuccess;
    switch (p.variant) {
        case 0:
            if (try_fixed<V224x64, 3, 64, 384, 3>(a, g, lds, stream, &err)) return err;     // 56x56 maps, stride 1
            return V224x64::launch(a, g, lds, stream);
        case 1:
            if (try_fixed<V224x32, 3, 36, 432, 3>(a, g, lds, stream, &err)) return err;     // 28x28 maps, stride 1
            if (try_fixed<V224x32, 8, 32, 1088, 3>(a, g, lds, stream, &err)) return err;    // 28x28 maps, stride 2
            return V224x32::launch(a, g, lds, stream);
        case 2: return V128x64::launch(a, g, lds, stream);
        default: return V64x64::launch(a, g, lds, stream);
    }
}

// Floats of the packed weights of plan p, and its channel tile and chunk (output channels x input channels).
int64_t packed_floats(const ConvArgs& a, const IgemmPlan& p, int* bn, int* ck)
{
    switch (p.variant) {
        case 0: *bn = V224x64::BN; *ck = V224x64::CK; return V224x64::packed_floats(a);
        case 1: *bn = V224x32::BN; *ck = V224x32::CK; return V224x32::packed_floats(a);
        case 2: *bn = V128x64::BN; *ck = V128x64::CK; return V128x64::packed_floats(a);
        case 3: *bn = V64x64::BN; *ck = V64x64::CK; return V64x64::packed_floats(a);
        default: *bn = *ck = 0; return 0;
    }
}

// Writes the pack's weights part in the patch kernel's order: for channel tile t and chunk q the
// LDS image of the tile's BN channels, KC = CK * 9 weights each in OIHW order followed by the four
// floats of padding of an LDS row; channels past K are zero.  One thread per float.
__global__ __launch_bounds__(256) void conv_pack_patch_kernel(const float* __restrict__ w, float* __restrict__ out,
                                                              int K, int C, int bn, int ck, int64_t total)
{
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int kc = ck * 9, ws = kc + 4, nchunks = C / ck;
    const int j = (int)(idx % ws);
    int64_t t = idx / ws;
    const int col = (int)(t % bn);
    t /= bn;
    const int chunk = (int)(t % nchunks);
    const int tile = (int)(t / nchunks);
    const int co = tile * bn + col;
    out[idx] = (j < kc && co < K) ? w[((int64_t)co * C + (int64_t)chunk * ck) * 9 + j] : 0.f;
}

// Plain copy (plans other than the patch kernel keep OIHW order).
__global__ __launch_bounds__(256) void conv_pack_copy_kernel(const float* __restrict__ w, float* __restrict__ out, int64_t total)
{
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx < total) out[idx] = w[idx];
}

// Folded batch norm, the same fp32 arithmetic as the kernels' own epilogue: scale, then shift.
__global__ __launch_bounds__(256) void conv_pack_bn_kernel(const float* __restrict__ gamma, const float* __restrict__ beta,
                                                           const float* __restrict__ mean, const float* __restrict__ var,
                                                           float eps, float* __restrict__ out, int K)
{
    const int k = blockIdx.x * 256 + threadIdx.x;
    if (k >= K) return;
    const float scale = gamma[k] / sqrtf(var[k] + eps);
    out[k] = scale;
    out[K + k] = beta[k] - mean[k] * scale;
}

}  // namespace

bool conv2d_igemm_takes(const ConvArgs& a)
{
    IgemmPlan p;
    plan_igemm(a, &p);
    return p.variant >= 0;
}

bool describe_conv2d_igemm(const ConvArgs& a, ConvRoute* r)
{
    IgemmPlan p;
    plan_igemm(a, &p);
    if (p.variant < 0) return false;
    static const int kTileM[5] = {224, 224, 128, 64, 224}, kTileN[5] = {64, 32, 64, 64, 32};
    r->kernel = 1;
    r->tile_m = kTileM[p.variant];
    r->tile_n = kTileN[p.variant];
    r->ksplit = 1;
    r->wave_groups = 1;
    r->work_groups = p.g.tiles_m * p.g.tiles_n;
    r->workspace_bytes = 0;
    return true;
}

void describe_conv2d(const ConvArgs& a, ConvRoute* r)
{
    if (describe_conv2d_igemm(a, r) || describe_conv2d_pointwise(a, r) || describe_conv2d_gather(a, r)) return;
    *r = ConvRoute{5, 0, 0, 1, 1, 0, 0};
}

hipError_t launch_conv2d_igemm(const ConvArgs& a, hipStream_t stream, bool* taken)
{
    IgemmPlan p;
    plan_igemm(a, &p);
    *taken = p.variant >= 0;
    return *taken ? launch_igemm_plan(a, p, stream) : hipSuccess;
}

size_t conv2d_workspace_bytes(const ConvArgs& a)
{
    if (conv2d_igemm_takes(a)) return 0;
    ConvRoute r;
    if (describe_conv2d_pointwise(a, &r)) return 0;
    return conv2d_gather_workspace_bytes(a);
}

ConvPackLayout conv2d_pack_layout(const ConvArgs& a)
{
    ConvPackLayout l{};
    l.ss_floats = ((size_t)2 * a.K + 63) / 64 * 64;
    // the plan for aligned pointers, whatever a.x and a.w hold at pack time
    ConvArgs b = a;
    b.x = nullptr;
    b.w = nullptr;
    b.wpack = nullptr;
    IgemmPlan p;
    plan_igemm(b, &p);
    int bn = 0, ck = 0;
    const int64_t pf = packed_floats(b, p, &bn, &ck);
    l.patch_layout = p.variant >= 0 && pf < ((int64_t)1 << 30);
    l.w_floats = l.patch_layout ? (size_t)pf : (size_t)a.K * (a.C / a.groups) * a.R * a.S;
    return l;
}

hipError_t launch_conv2d_pack(const ConvArgs& a, float* pack, hipStream_t stream)
{
    const ConvPackLayout l = conv2d_pack_layout(a);
    if (a.gamma) {
        hipError_t e = launch_kernel(conv_pack_bn_kernel, dim3((unsigned)((a.K + 255) / 256)), dim3(256), 0, stream, a.gamma,
                                     a.beta, a.mean, a.var, a.eps, pack, a.K);
        if (e != hipSuccess) return e;
    }
    float* wout = pack + l.ss_floats;
    const int64_t total = (int64_t)l.w_floats;
    const dim3 grid((unsigned)((total + 255) / 256));
    if (!l.patch_layout) return launch_kernel(conv_pack_copy_kernel, grid, dim3(256), 0, stream, a.w, wout, total);
    ConvArgs b = a;
    b.x = nullptr;
    b.w = nullptr;
    IgemmPlan p;
    plan_igemm(b, &p);
    int bn = 0, ck = 0;
    packed_floats(b, p, &bn, &ck);
    return launch_kernel(conv_pack_patch_kernel, grid, dim3(256), 0, stream, a.w, wout, a.K, a.C, bn, ck, total);
}

hipError_t launch_conv2d(const ConvArgs& a, hipStream_t stream, int* ws_fault)
{
    *ws_fault = 0;
    bool taken = false;
    hipError_t err = launch_conv2d_igemm(a, stream, &taken);
    if (taken || err != hipSuccess) return err;
    err = launch_conv2d_pointwise(a, stream, &taken);
    if (taken || err != hipSuccess) return err;
    err = launch_conv2d_gather(a, stream, &taken, ws_fault);
    if (taken || err != hipSuccess) return err;
    return launch_conv2d_direct(a, stream);
}

}  // namespace anr
