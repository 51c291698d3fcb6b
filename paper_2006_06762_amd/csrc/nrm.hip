// NRM (Sec. 7.1 / Appendix C of arXiv 2006.06762; named in Sec. 4.1 as the operator with
// parallelism only in its reduction dimensions): out[b] = sqrt(sum_{i,j} x[b,i,j]^2) for
// each N x M matrix of a batch.
//
// Pure streaming: 4 bytes read per 2 FLOP, bound by HBM.  The parallelism the operator lacks
// in space is taken from the reduction (rule 6 of Table 1, "rfactor"): every matrix is cut
// into `parts` contiguous slices, one work-group each, so that ~2000 work-groups stream at
// once however small the batch; a thread keeps eight 16-byte loads in flight and four
// independent partial sums.  Partial sums are combined in a fixed order (lanes by shuffle,
// waves through LDS, slices by a second small kernel reading the workspace), so the result
// does not depend on scheduling: no float atomics.
#include "anr_device.h"
#include "anr_kernels.h"

namespace anr {
namespace {

constexpr int kNT = 256;

__device__ __forceinline__ float block_sum(float v, float* red)
{
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) red[wave] = v;
    __syncthreads();
    return (red[0] + red[1]) + (red[2] + red[3]);
}

// One work-group reduces elements [part * per_part, (part + 1) * per_part) of the flattened
// matrix (per_part is a multiple of 4 * kNT when VEC).  Writes sqrt of the sum when the
// matrix has a single part, else the partial sum to ws[b * parts + part].
template <bool VEC>
__global__ __launch_bounds__(kNT) void nrm_partial_kernel(const NrmArgs p, int64_t per_part, int parts)
{
    __shared__ float red[4];
    const int part = blockIdx.x, b = blockIdx.y;
    const int64_t total = p.N * p.M;
    const int64_t begin = (int64_t)part * per_part;
    const int64_t end = begin + per_part < total ? begin + per_part : total;
    const float* __restrict__ x = p.x + b * p.stride;
    float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
    if (VEC) {
        // packed rows: the slice is one contiguous run of 16-byte units
        const f32x4* __restrict__ x4 = reinterpret_cast<const f32x4*>(x);
        const int64_t u0 = begin / 4 + threadIdx.x, u1 = end / 4;      // total is a multiple of 4
        int64_t u = u0;
        for (; u + 7 * kNT < u1; u += 8 * kNT) {
            f32x4 v[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] = x4[u + i * kNT];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                s0 = fmaf(v[i][0], v[i][0], s0);
                s1 = fmaf(v[i][1], v[i][1], s1);
                s2 = fmaf(v[i][2], v[i][2], s2);
                s3 = fmaf(v[i][3], v[i][3], s3);
            }
        }
        for (; u < u1; u += kNT) {
            const f32x4 v = x4[u];
            s0 = fmaf(v[0], v[0], s0);
            s1 = fmaf(v[1], v[1], s1);
            s2 = fmaf(v[2], v[2], s2);
            s3 = fmaf(v[3], v[3], s3);
        }
    } else {
        // any row stride: element e of the flattened matrix is row e / M, column e % M
        for (int64_t e = begin + threadIdx.x; e < end; e += kNT) {
            const int64_t row = e / p.M, col = e - row * p.M;
            const float v = x[row * p.ld + col];
            s0 = fmaf(v, v, s0);
        }
    }
    const float sum = block_sum((s0 + s1) + (s2 + s3), red);
    if (threadIdx.x == 0) {
        if (parts == 1) p.out[b] = sqrtf(sum);
        else p.ws[(int64_t)b * parts + part] = sum;
    }
}

__global__ __launch_bounds__(kNT) void nrm_final_kernel(const NrmArgs p, int parts)
{
    __shared__ float red[4];
    const int b = blockIdx.x;
    float s = 0.f;
    for (int i = threadIdx.x; i < parts; i += kNT) s += p.ws[(int64_t)b * parts + i];
    const float sum = block_sum(s, red);
    if (threadIdx.x == 0) p.out[b] = sqrtf(sum);
}

}  // namespace

// Slices per matrix: enough work-groups to fill the chip (about 8 per CU), at least 16 K
// elements per slice.
int nrm_parts(const NrmArgs& a)
{
    const int64_t total = a.N * a.M;
    int64_t want = (2048 + a.batch - 1) / a.batch;
    const int64_t most = (total + 16383) / 16384;
    if (want > most) want = most;
    if (want < 1) want = 1;
    if (want > 65535) want = 65535;
    return (int)want;
}

size_t nrm_workspace_bytes(const NrmArgs& a)
{
    const int parts = nrm_parts(a);
    return parts > 1 ? sizeof(float) * (size_t)parts * (size_t)a.batch : 0;
}

hipError_t launch_nrm(const NrmArgs& a, hipStream_t stream)
{
    const int parts = nrm_parts(a);
    const int64_t total = a.N * a.M;
    if (parts > 1 && (a.ws == nullptr || a.ws_bytes < nrm_workspace_bytes(a))) return hipErrorInvalidValue;
    const bool vec = a.ld == a.M && (total % 4 == 0) && (a.stride % 4 == 0) && is_aligned16(a.x);
    // slice length: a whole number of passes of the work-group over 16-byte units
    int64_t per_part = (total + parts - 1) / parts;
    per_part = (per_part + 4 * kNT - 1) / (4 * kNT) * (4 * kNT);
    const dim3 grid((unsigned)parts, (unsigned)a.batch);
    hipError_t err = vec ? launch_kernel(nrm_partial_kernel<true>, grid, dim3(kNT), 0, stream, a, per_part, parts)
                         : launch_kernel(nrm_partial_kernel<false>, grid, dim3(kNT), 0, stream, a, per_part, parts);
    if (err != hipSuccess || parts == 1) return err;
    return launch_kernel(nrm_final_kernel, dim3((unsigned)a.batch), dim3(kNT), 0, stream, a, parts);
}

}  // namespace anr
