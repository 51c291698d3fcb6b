// Shape-agnostic convolution kernels: one thread per output element, plain
// loops over (c, r, s).  They serve every geometry the fast kernels do not
// take (odd widths, unaligned views, large kernels, strides other than the
// tuned ones) and compute the operator definitions of Sec. 7.1 / Appendix C
// (C2D, DEP) and Sec. 7.2 (ConvLayer epilogue) directly.
#include "anr_device.h"
#include "anr_kernels.h"
#include "conv_internal.h"

namespace anr {
namespace {

__global__ __launch_bounds__(256) void conv2d_direct_kernel(const ConvArgs p, int64_t total)
{
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int ow = (int)(idx % p.OW);
    int64_t t = idx / p.OW;
    const int oh = (int)(t % p.OH);
    t /= p.OH;
    const int k = (int)(t % p.K);
    const int n = (int)(t / p.K);

    // output channel k belongs to group k / (K/groups) and sees that group's C/groups channels
    const int cg = p.C / p.groups, grp = k / (p.K / p.groups);
    const float* __restrict__ xn = p.x + n * p.xs[0] + (int64_t)grp * cg * p.xs[1];
    const float* __restrict__ wk = p.w + (int64_t)k * cg * p.R * p.S;
    const int ih0 = oh * p.stride_h - p.pad_h, iw0 = ow * p.stride_w - p.pad_w;
    float acc = 0.f;
    for (int c = 0; c < cg; ++c) {
        const float* __restrict__ xc = xn + c * p.xs[1];
        const float* __restrict__ wc = wk + (int64_t)c * p.R * p.S;
        for (int r = 0; r < p.R; ++r) {
            const int ih = ih0 + r * p.dil_h;
            if (ih < 0 || ih >= p.H) continue;
            for (int s = 0; s < p.S; ++s) {
                const int iw = iw0 + s * p.dil_w;
                if (iw < 0 || iw >= p.W) continue;
                acc = fmaf(xc[ih * p.xs[2] + iw], wc[r * p.S + s], acc);
            }
        }
    }
    if (p.gamma) {
        const float scale = p.scale_shift ? p.scale_shift[k] : p.gamma[k] / sqrtf(p.var[k] + p.eps);
        const float shift = p.scale_shift ? p.scale_shift[p.K + k] : p.beta[k] - p.mean[k] * scale;
        acc = fmaxf(fmaf(acc, scale, shift), 0.f);
    }
    p.y[n * p.ys[0] + k * p.ys[1] + oh * p.ys[2] + ow] = acc;
}

__global__ __launch_bounds__(256) void dwconv_direct_kernel(const ConvArgs p, int64_t total)
{
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int ow = (int)(idx % p.OW);
    int64_t t = idx / p.OW;
    const int oh = (int)(t % p.OH);
    t /= p.OH;
    const int c = (int)(t % p.C);
    const int n = (int)(t / p.C);

    const float* __restrict__ xc = p.x + n * p.xs[0] + c * p.xs[1];
    const float* __restrict__ wc = p.w + (int64_t)c * p.R * p.S;
    const int ih0 = oh * p.stride_h - p.pad_h, iw0 = ow * p.stride_w - p.pad_w;
    float acc = 0.f;
    for (int r = 0; r < p.R; ++r) {
        const int ih = ih0 + r * p.dil_h;
        if (ih < 0 || ih >= p.H) continue;
        for (int s = 0; s < p.S; ++s) {
            const int iw = iw0 + s * p.dil_w;
            if (iw < 0 || iw >= p.W) continue;
            acc = fmaf(xc[ih * p.xs[2] + iw], wc[r * p.S + s], acc);
        }
    }
    p.y[n * p.ys[0] + c * p.ys[1] + oh * p.ys[2] + ow] = acc;
}

}  // namespace

hipError_t launch_conv2d_direct(const ConvArgs& a, hipStream_t stream)
{
    const int64_t total = (int64_t)a.N * a.K * a.OH * a.OW;
    return launch_kernel(conv2d_direct_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream,
                         a, total);
}

hipError_t launch_dwconv_direct(const ConvArgs& a, hipStream_t stream)
{
    const int64_t total = (int64_t)a.N * a.C * a.OH * a.OW;
    return launch_kernel(dwconv_direct_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream,
                         a, total);
}

}  // namespace anr
