// C-ABI layer: argument validation (host only, before any launch), descriptor
// normalisation and dispatch to the kernel launchers.  See include/anr.h for
// the contract of every entry point.
#include "anr.h"

#include <cmath>

#include "anr_kernels.h"
#include "conv_internal.h"

namespace {

constexpr int kVersion = 300;   // 0.3.0

// HIP status of the most recent failed launch made by this thread (diagnostics only).
thread_local int g_last_hip_error = 0;

anr_status launch_status(hipError_t e)
{
    if (e == hipSuccess) return ANR_OK;
    g_last_hip_error = (int)e;
    return ANR_ERR_LAUNCH;
}

bool all_zero(const int64_t s[4]) { return s[0] == 0 && s[1] == 0 && s[2] == 0 && s[3] == 0; }

struct ConvGeom {
    int OH, OW;
    int64_t xs[4], ys[4];
};

// Checks a convolution descriptor; `depthwise` additionally requires K == C.
anr_status check_conv(const anr_conv_desc* d, bool depthwise, ConvGeom* g)
{
    if (!d) return ANR_ERR_NULL;
    if (d->N < 1 || d->C < 1 || d->H < 1 || d->W < 1 || d->K < 1 || d->R < 1 || d->S < 1)
        return ANR_ERR_INVALID_ARG;
    if (d->stride_h < 1 || d->stride_w < 1 || d->pad_h < 0 || d->pad_w < 0) return ANR_ERR_INVALID_ARG;
    if (d->dil_h < 1 || d->dil_w < 1) return ANR_ERR_INVALID_ARG;
    if (depthwise && d->K != d->C) return ANR_ERR_INVALID_ARG;
    if (d->groups < 0) return ANR_ERR_INVALID_ARG;
    if (d->route != ANR_CONV_ROUTE_AUTO && d->route != ANR_CONV_ROUTE_PATCH && d->route != ANR_CONV_ROUTE_GENERAL)
        return ANR_ERR_INVALID_ARG;
    if (!depthwise && d->groups > 1 && (d->C % d->groups != 0 || d->K % d->groups != 0)) return ANR_ERR_INVALID_ARG;
    if (d->layout != ANR_LAYOUT_NCHW) return ANR_ERR_UNSUPPORTED;
    const int64_t eh = (int64_t)d->H + 2 * (int64_t)d->pad_h - (int64_t)d->dil_h * (d->R - 1) - 1;
    const int64_t ew = (int64_t)d->W + 2 * (int64_t)d->pad_w - (int64_t)d->dil_w * (d->S - 1) - 1;
    if (eh < 0 || ew < 0) return ANR_ERR_INVALID_ARG;
    g->OH = (int)(eh / d->stride_h) + 1;
    g->OW = (int)(ew / d->stride_w) + 1;

    const int64_t xdims[4] = {d->N, d->C, d->H, d->W};
    const int64_t ydims[4] = {d->N, d->K, g->OH, g->OW};
    for (int t = 0; t < 2; ++t) {
        const int64_t* in = t ? d->y_stride : d->x_stride;
        const int64_t* dims = t ? ydims : xdims;
        int64_t* out = t ? g->ys : g->xs;
        if (all_zero(in)) {
            out[3] = 1;
            out[2] = dims[3];
            out[1] = dims[2] * dims[3];
            out[0] = dims[1] * dims[2] * dims[3];
            continue;
        }
        for (int i = 0; i < 4; ++i)
            if (in[i] < 1) return ANR_ERR_INVALID_ARG;
        if (in[3] != 1) return ANR_ERR_UNSUPPORTED;
        // nested, non-self-overlapping view: w inside h inside c inside n
        if (in[2] < dims[3] || in[1] < (dims[2] - 1) * in[2] + dims[3] ||
            in[0] < (dims[1] - 1) * in[1] + (dims[2] - 1) * in[2] + dims[3])
            return ANR_ERR_INVALID_ARG;
        for (int i = 0; i < 4; ++i) out[i] = in[i];
    }
    // element counts must fit the kernels' 32-bit pixel indices
    const int64_t out_elems = (int64_t)d->N * d->K * g->OH * g->OW;
    if (out_elems >= ((int64_t)1 << 40)) return ANR_ERR_UNSUPPORTED;
    if ((int64_t)d->N * g->OH * g->OW >= ((int64_t)1 << 31)) return ANR_ERR_UNSUPPORTED;
    if ((int64_t)d->C * d->R * d->S >= ((int64_t)1 << 31)) return ANR_ERR_UNSUPPORTED;
    return ANR_OK;
}

anr::ConvArgs make_conv_args(const anr_conv_desc* d, const ConvGeom& g, const float* x, const float* w,
                             float* y)
{
    anr::ConvArgs a{};
    a.x = x;
    a.w = w;
    a.y = y;
    a.N = d->N; a.C = d->C; a.H = d->H; a.W = d->W; a.K = d->K; a.R = d->R; a.S = d->S;
    a.stride_h = d->stride_h; a.stride_w = d->stride_w; a.pad_h = d->pad_h; a.pad_w = d->pad_w;
    a.dil_h = d->dil_h; a.dil_w = d->dil_w;
    a.groups = d->groups > 1 ? d->groups : 1;
    a.route = d->route;
    a.OH = g.OH; a.OW = g.OW;
    for (int i = 0; i < 4; ++i) { a.xs[i] = g.xs[i]; a.ys[i] = g.ys[i]; }
    a.gamma = a.beta = a.mean = a.var = nullptr;
    a.eps = 0.f;
    a.wpack = nullptr;
    a.scale_shift = nullptr;
    a.ws = nullptr;
    a.ws_bytes = 0;
    return a;
}

// Hands the caller's workspace to the launcher, which plans the call once and reports whether
// the plan's need is met (nothing is enqueued when it is not).
anr_status run_conv2d(anr::ConvArgs* a, void* ws, size_t ws_bytes, void* hip_stream)
{
    a->ws = static_cast<float*>(ws);
    a->ws_bytes = ws ? ws_bytes : 0;
    int ws_fault = 0;
    const hipError_t e = anr::launch_conv2d(*a, static_cast<hipStream_t>(hip_stream), &ws_fault);
    if (ws_fault == 1) return ANR_ERR_WORKSPACE;
    if (ws_fault == 2) return ANR_ERR_INVALID_ARG;
    return launch_status(e);
}

anr_status check_gemm(const anr_gemm_desc* d)
{
    if (!d) return ANR_ERR_NULL;
    if (d->M < 1 || d->N < 1 || d->K < 1 || d->batch < 1) return ANR_ERR_INVALID_ARG;
    if (d->lda < d->K || d->ldb < d->N || d->ldc < d->N) return ANR_ERR_INVALID_ARG;
    if (d->strideA < 0 || d->strideB < 0 || d->strideC < 0) return ANR_ERR_INVALID_ARG;
    // extents the kernels' 32-bit tile arithmetic takes (and small enough that the products
    // below and in the launchers cannot overflow 64 bits)
    const int64_t lim = (int64_t)1 << 30;
    if (d->M >= lim || d->N >= lim || d->K >= lim) return ANR_ERR_UNSUPPORTED;
    if (d->lda >= 2 * lim || d->ldb >= 2 * lim || d->ldc >= 2 * lim) return ANR_ERR_UNSUPPORTED;
    if (d->batch > 1 && d->strideC < (d->M - 1) * d->ldc + d->N) return ANR_ERR_INVALID_ARG;
    if (d->batch > 65535) return ANR_ERR_UNSUPPORTED;              // grid z limit
    if ((d->M + 63) / 64 > 65535) return ANR_ERR_UNSUPPORTED;       // grid y limit
    return ANR_OK;
}

struct TbgGeom {
    int64_t qs[4], ks[4], os[4];
};

anr_status check_tbg(const anr_tbg_desc* d, bool softmax, TbgGeom* g)
{
    if (!d) return ANR_ERR_NULL;
    if (d->B < 1 || d->S < 1 || d->H < 1 || d->D < 1) return ANR_ERR_INVALID_ARG;
    const int64_t in_dims[4] = {d->B, d->S, d->H, d->D};
    const int64_t out_dims[4] = {d->B, d->H, d->S, d->S};
    const int64_t* ins[3] = {d->q_stride, d->k_stride, d->o_stride};
    int64_t* outs[3] = {g->qs, g->ks, g->os};
    for (int t = 0; t < 3; ++t) {
        const int64_t* dims = t == 2 ? out_dims : in_dims;
        if (all_zero(ins[t])) {
            outs[t][3] = 1;
            outs[t][2] = dims[3];
            outs[t][1] = dims[2] * dims[3];
            outs[t][0] = dims[1] * dims[2] * dims[3];
            continue;
        }
        for (int i = 0; i < 4; ++i)
            if (ins[t][i] < 1) return ANR_ERR_INVALID_ARG;
        if (ins[t][3] != 1) return ANR_ERR_UNSUPPORTED;
        for (int i = 0; i < 4; ++i) outs[t][i] = ins[t][i];
    }
    // the output view must not overlap itself: rows inside matrices inside heads inside batches
    const int64_t S = d->S;
    if (g->os[2] < S) return ANR_ERR_INVALID_ARG;
    if (g->os[2] >= ((int64_t)1 << 40) || g->os[1] >= ((int64_t)1 << 50)) return ANR_ERR_UNSUPPORTED;
    if (g->os[1] < (S - 1) * g->os[2] + S) return ANR_ERR_INVALID_ARG;
    if (g->os[0] < (d->H - 1) * g->os[1] + (S - 1) * g->os[2] + S) return ANR_ERR_INVALID_ARG;
    if ((int64_t)d->B * d->H > 65535) return ANR_ERR_UNSUPPORTED;
    if (softmax && d->S > 1024) return ANR_ERR_UNSUPPORTED;
    return ANR_OK;
}

anr_status run_tbg(const anr_tbg_desc* d, const float* q, const float* k, float* out, bool softmax,
                   void* hip_stream)
{
    TbgGeom g;
    anr_status st = check_tbg(d, softmax, &g);
    if (st != ANR_OK) return st;
    if (!q || !k || !out) return ANR_ERR_NULL;
    anr::GemmArgs a{};
    a.A = q; a.B = k; a.C = out;
    a.M = d->S; a.N = d->S; a.K = d->D;
    a.lda = g.qs[1]; a.ldb = g.ks[1]; a.ldc = g.os[2];
    a.batch = d->B * d->H; a.batch_inner = d->H;
    a.sAo = g.qs[0]; a.sAi = g.qs[2];
    a.sBo = g.ks[0]; a.sBi = g.ks[2];
    a.sCo = g.os[0]; a.sCi = g.os[1];
    a.b_is_nk = true;
    a.softmax_rows = softmax;
    return launch_status(anr::launch_tbg(a, static_cast<hipStream_t>(hip_stream)));
}

anr_status check_nrm(const anr_nrm_desc* d, anr::NrmArgs* a)
{
    if (!d) return ANR_ERR_NULL;
    if (d->N < 1 || d->M < 1 || d->batch < 1 || d->ld < d->M || d->stride < 0) return ANR_ERR_INVALID_ARG;
    if (d->batch > 65535) return ANR_ERR_UNSUPPORTED;
    if (d->N >= ((int64_t)1 << 31) || d->M >= ((int64_t)1 << 31) || d->ld >= ((int64_t)1 << 32))
        return ANR_ERR_UNSUPPORTED;
    // matrices of a batch must not overlap (stride 0: the same matrix every time)
    if (d->batch > 1 && d->stride != 0 && d->stride < (d->N - 1) * d->ld + d->M) return ANR_ERR_INVALID_ARG;
    a->N = d->N; a->M = d->M; a->ld = d->ld; a->stride = d->stride;
    a->batch = (int)d->batch;
    return ANR_OK;
}

}  // namespace

extern "C" {

anr_status anr_gemm(const anr_gemm_desc* d, const float* A, const float* B, float* C, void* ws,
                    size_t ws_bytes, void* hip_stream)
{
    (void)ws; (void)ws_bytes;
    anr_status st = check_gemm(d);
    if (st != ANR_OK) return st;
    if (!A || !B || !C) return ANR_ERR_NULL;
    anr::GemmArgs a{};
    a.A = A; a.B = B; a.C = C;
    a.M = (int)d->M; a.N = (int)d->N; a.K = (int)d->K;
    a.lda = d->lda; a.ldb = d->ldb; a.ldc = d->ldc;
    a.batch = (int)d->batch; a.batch_inner = 1;
    a.sAo = d->strideA; a.sBo = d->strideB; a.sCo = d->strideC;
    a.sAi = a.sBi = a.sCi = 0;
    a.b_is_nk = false;
    a.softmax_rows = false;
    return launch_status(anr::launch_gemm(a, static_cast<hipStream_t>(hip_stream)));
}

anr_status anr_conv2d(const anr_conv_desc* d, const float* x, const float* w, float* y, void* ws,
                      size_t ws_bytes, void* hip_stream)
{
    ConvGeom g;
    anr_status st = check_conv(d, false, &g);
    if (st != ANR_OK) return st;
    if (!x || !w || !y) return ANR_ERR_NULL;
    anr::ConvArgs a = make_conv_args(d, g, x, w, y);
    return run_conv2d(&a, ws, ws_bytes, hip_stream);
}

anr_status anr_conv2d_noalloc(const anr_conv_desc* d, const float* x, const float* w, float* y, void* hip_stream)
{
    ConvGeom g;
    anr_status st = check_conv(d, false, &g);
    if (st != ANR_OK) return st;
    if (!x || !w || !y) return ANR_ERR_NULL;
    anr::ConvArgs a = make_conv_args(d, g, x, w, y);
    // plans that need no workspace never touch the array (nor the runtime, to look it up)
    if (anr::conv2d_workspace_bytes(a) == 0) return run_conv2d(&a, nullptr, 0, hip_stream);
    void* scratch = nullptr;
    size_t scratch_bytes = 0;
    const hipError_t e = anr::static_scratch(&scratch, &scratch_bytes);
    if (e != hipSuccess) return launch_status(e);
    return run_conv2d(&a, scratch, scratch_bytes, hip_stream);
}

anr_status anr_conv2d_packed_size(const anr_conv_desc* d, size_t* bytes)
{
    if (!bytes) return ANR_ERR_NULL;
    ConvGeom g;
    const anr_status st = check_conv(d, false, &g);
    if (st != ANR_OK) return st;
    const anr::ConvArgs a = make_conv_args(d, g, nullptr, nullptr, nullptr);
    const anr::ConvPackLayout l = anr::conv2d_pack_layout(a);
    *bytes = sizeof(float) * (l.ss_floats + l.w_floats);
    return ANR_OK;
}

anr_status anr_conv2d_pack_weights(const anr_conv_desc* d, const float* w, const float* gamma, const float* beta,
                                   const float* mean, const float* var, float eps, void* packed, size_t packed_bytes,
                                   void* hip_stream)
{
    ConvGeom g;
    anr_status st = check_conv(d, false, &g);
    if (st != ANR_OK) return st;
    if (!w || !packed) return ANR_ERR_NULL;
    // batch-norm vectors: all four or none
    const int given = (gamma != nullptr) + (beta != nullptr) + (mean != nullptr) + (var != nullptr);
    if (given != 0 && given != 4) return ANR_ERR_NULL;
    if (given == 4 && !std::isfinite(eps)) return ANR_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(packed) & 255) return ANR_ERR_INVALID_ARG;
    anr::ConvArgs a = make_conv_args(d, g, nullptr, w, nullptr);
    const anr::ConvPackLayout l = anr::conv2d_pack_layout(a);
    if (packed_bytes < sizeof(float) * (l.ss_floats + l.w_floats)) return ANR_ERR_WORKSPACE;
    a.gamma = gamma; a.beta = beta; a.mean = mean; a.var = var; a.eps = eps;
    return launch_status(anr::launch_conv2d_pack(a, static_cast<float*>(packed), static_cast<hipStream_t>(hip_stream)));
}

namespace {
anr_status run_packed(const anr_conv_desc* d, const float* x, const void* packed, float* y, bool fused, void* ws,
                      size_t ws_bytes, void* hip_stream)
{
    ConvGeom g;
    const anr_status st = check_conv(d, false, &g);
    if (st != ANR_OK) return st;
    if (!x || !packed || !y) return ANR_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(packed) & 255) return ANR_ERR_INVALID_ARG;
    anr::ConvArgs a = make_conv_args(d, g, x, nullptr, y);
    const anr::ConvPackLayout l = anr::conv2d_pack_layout(a);
    const float* pack = static_cast<const float*>(packed);
    if (l.patch_layout) {
        a.wpack = pack + l.ss_floats;
        // the pack presumes the plan for 16-byte aligned x: a view that kernel cannot read cannot use it
        if (!anr::conv2d_igemm_takes(a)) return ANR_ERR_INVALID_ARG;
    } else {
        a.w = pack + l.ss_floats;
    }
    if (fused) {
        a.gamma = pack;            // marker: fused epilogue, constants from scale_shift
        a.scale_shift = pack;
    }
    return run_conv2d(&a, ws, ws_bytes, hip_stream);
}
}  // namespace

anr_status anr_conv2d_packed(const anr_conv_desc* d, const float* x, const void* packed, float* y, void* ws,
                             size_t ws_bytes, void* hip_stream)
{
    return run_packed(d, x, packed, y, false, ws, ws_bytes, hip_stream);
}

anr_status anr_conv_bn_relu_packed(const anr_conv_desc* d, const float* x, const void* packed, float* y, void* ws,
                                   size_t ws_bytes, void* hip_stream)
{
    return run_packed(d, x, packed, y, true, ws, ws_bytes, hip_stream);
}

anr_status anr_conv_bn_relu(const anr_conv_desc* d, const float* x, const float* w, const float* gamma,
                            const float* beta, const float* mean, const float* var, float eps, float* y,
                            void* ws, size_t ws_bytes, void* hip_stream)
{
    ConvGeom g;
    anr_status st = check_conv(d, false, &g);
    if (st != ANR_OK) return st;
    if (!std::isfinite(eps)) return ANR_ERR_INVALID_ARG;
    if (!x || !w || !y || !gamma || !beta || !mean || !var) return ANR_ERR_NULL;
    anr::ConvArgs a = make_conv_args(d, g, x, w, y);
    a.gamma = gamma; a.beta = beta; a.mean = mean; a.var = var; a.eps = eps;
    return run_conv2d(&a, ws, ws_bytes, hip_stream);
}

anr_status anr_dwconv(const anr_conv_desc* d, const float* x, const float* w, float* y, void* ws,
                      size_t ws_bytes, void* hip_stream)
{
    (void)ws; (void)ws_bytes;
    ConvGeom g;
    anr_status st = check_conv(d, true, &g);
    if (st != ANR_OK) return st;
    if (!x || !w || !y) return ANR_ERR_NULL;
    const anr::ConvArgs a = make_conv_args(d, g, x, w, y);
    return launch_status(anr::launch_dwconv(a, static_cast<hipStream_t>(hip_stream)));
}

anr_status anr_tbg(const anr_tbg_desc* d, const float* q, const float* k, float* out, void* ws,
                   size_t ws_bytes, void* hip_stream)
{
    (void)ws; (void)ws_bytes;
    return run_tbg(d, q, k, out, false, hip_stream);
}

anr_status anr_tbs(const anr_tbg_desc* d, const float* q, const float* k, float* out, void* ws,
                   size_t ws_bytes, void* hip_stream)
{
    (void)ws; (void)ws_bytes;
    return run_tbg(d, q, k, out, true, hip_stream);
}

anr_status anr_nrm(const anr_nrm_desc* d, const float* x, float* out, void* ws, size_t ws_bytes,
                   void* hip_stream)
{
    anr::NrmArgs a{};
    anr_status st = check_nrm(d, &a);
    if (st != ANR_OK) return st;
    if (!x || !out) return ANR_ERR_NULL;
    a.x = x;
    a.out = out;
    const size_t need = anr::nrm_workspace_bytes(a);
    if (need > 0) {
        if (!ws || ws_bytes < need) return ANR_ERR_WORKSPACE;
        if (reinterpret_cast<uintptr_t>(ws) & 3) return ANR_ERR_INVALID_ARG;
        a.ws = static_cast<float*>(ws);
        a.ws_bytes = ws_bytes;
    }
    return launch_status(anr::launch_nrm(a, static_cast<hipStream_t>(hip_stream)));
}

anr_status anr_workspace_size(int op, const void* desc, size_t* bytes)
{
    if (!desc || !bytes) return ANR_ERR_NULL;
    anr_status st;
    ConvGeom cg;
    TbgGeom tg;
    anr::NrmArgs na{};
    switch (op) {
        case ANR_OP_GEMM: st = check_gemm(static_cast<const anr_gemm_desc*>(desc)); break;
        case ANR_OP_CONV2D:
        case ANR_OP_CONV_BN_RELU: st = check_conv(static_cast<const anr_conv_desc*>(desc), false, &cg); break;
        case ANR_OP_DWCONV: st = check_conv(static_cast<const anr_conv_desc*>(desc), true, &cg); break;
        case ANR_OP_TBG: st = check_tbg(static_cast<const anr_tbg_desc*>(desc), false, &tg); break;
        case ANR_OP_TBS: st = check_tbg(static_cast<const anr_tbg_desc*>(desc), true, &tg); break;
        case ANR_OP_NRM: st = check_nrm(static_cast<const anr_nrm_desc*>(desc), &na); break;
        default: return ANR_ERR_INVALID_ARG;
    }
    if (st != ANR_OK) return st;
    *bytes = 0;
    if (op == ANR_OP_NRM) *bytes = anr::nrm_workspace_bytes(na);
    if (op == ANR_OP_CONV2D || op == ANR_OP_CONV_BN_RELU) {
        // the need of the plan for 16-byte aligned pointers (what anr_conv2d_route reports); plans
        // for less aligned pointers never split the reduction and need none
        const anr::ConvArgs a = make_conv_args(static_cast<const anr_conv_desc*>(desc), cg, nullptr, nullptr, nullptr);
        *bytes = anr::conv2d_workspace_bytes(a);
    }
    return ANR_OK;
}

anr_status anr_conv2d_route(const anr_conv_desc* d, anr_conv_route* route)
{
    if (!route) return ANR_ERR_NULL;
    ConvGeom cg;
    const anr_status st = check_conv(d, false, &cg);
    if (st != ANR_OK) return st;
    const anr::ConvArgs a = make_conv_args(d, cg, nullptr, nullptr, nullptr);
    anr::ConvRoute r{};
    anr::describe_conv2d(a, &r);
    route->kernel = r.kernel;
    route->tile_m = r.tile_m;
    route->tile_n = r.tile_n;
    route->ksplit = r.ksplit;
    route->wave_groups = r.wave_groups;
    route->work_groups = r.work_groups;
    route->workspace_bytes = r.workspace_bytes;
    return ANR_OK;
}

const char* anr_status_string(anr_status status)
{
    switch (status) {
        case ANR_OK: return "ok";
        case ANR_ERR_NULL: return "a required pointer is NULL";
        case ANR_ERR_INVALID_ARG: return "invalid argument";
        case ANR_ERR_UNSUPPORTED: return "valid but unsupported configuration";
        case ANR_ERR_WORKSPACE: return "workspace too small";
        case ANR_ERR_LAUNCH: return "kernel launch failed";
    }
    return "unknown status";
}

int anr_version(void) { return kVersion; }

int anr_last_hip_error(void) { return g_last_hip_error; }

const char* anr_last_hip_error_string(void)
{
    return hipGetErrorString(static_cast<hipError_t>(g_last_hip_error));
}

}  // extern "C"
