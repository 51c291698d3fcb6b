// Internal launch interface between the C-ABI layer (api.cpp) and the kernel
// translation units.  Every launcher enqueues on `stream` and returns the
// hipError_t of the launch; none of them allocates or synchronises.  The
// arguments have been validated by the caller.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

namespace anr {

template <typename T>
struct NonDeduced {
    using type = T;
};

// Launch with the status returned by the launch call itself (hipGetLastError would also
// report, and clear, errors left behind by other users of the runtime in this thread).
template <typename... KArgs>
inline hipError_t launch_kernel(void (*kern)(KArgs...), dim3 grid, dim3 block, size_t lds_bytes,
                                hipStream_t stream, typename NonDeduced<KArgs>::type... args)
{
    void* ptrs[] = {const_cast<void*>(static_cast<const void*>(&args))...};
    return hipLaunchKernel(reinterpret_cast<const void*>(kern), grid, block, ptrs, lds_bytes, stream);
}

inline bool is_aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

// Dynamic shared-memory limit already granted to one kernel, per device.  The runtime call
// that raises it costs microseconds (more than some of the kernels run), so a launcher keeps
// one of these per kernel instantiation and calls the runtime only when a launch needs more
// than any earlier one on that device.  Setting the attribute twice is harmless, so a race
// between two threads costs one redundant call and nothing else.
struct LdsLimit {
    static constexpr int kDevices = 16;
    std::atomic<int> bytes[kDevices];
};

inline hipError_t raise_lds_limit(const void* kernel, size_t bytes, LdsLimit& lim)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const bool tracked = dev >= 0 && dev < LdsLimit::kDevices;
    if (tracked && lim.bytes[dev].load(std::memory_order_acquire) >= (int)bytes) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e == hipSuccess && tracked) lim.bytes[dev].store((int)bytes, std::memory_order_release);
    return e;
}

// Batched C = A.B (B_IS_NK false: B is K x N, row stride ldb) or C = A.B^T
// (B_IS_NK true: B is N x K, row stride ldb).  Batch index z in [0, batch) is
// split as z = zo*batch_inner + zi, and operand X starts at
// X + zo*sXo + zi*sXi.
struct GemmArgs {
    const float* A;
    const float* B;
    float* C;
    int M, N, K;
    int64_t lda, ldb, ldc;
    int batch, batch_inner;
    int64_t sAo, sAi, sBo, sBi, sCo, sCi;
    bool b_is_nk;
    bool softmax_rows;   // TBS: softmax over each output row (requires N <= 1024)
};
hipError_t launch_gemm(const GemmArgs& a, hipStream_t stream);
// The TBS batch matmul (a.b_is_nk set, batch = B*H, batch_inner = H), optionally followed by the
// row softmax; picks the dedicated tile kernel when the operands allow it.
hipError_t launch_tbg(const GemmArgs& a, hipStream_t stream);
// In-place softmax over every row of the a.batch output matrices of `a` (a.N <= 1024).
hipError_t launch_softmax_rows(const GemmArgs& a, hipStream_t stream);

struct ConvArgs {
    const float* x;
    const float* w;
    float* y;
    int N, C, H, W, K, R, S;
    int stride_h, stride_w, pad_h, pad_w;
    int dil_h, dil_w;
    int groups;      // >= 1; weights are [K, C/groups, R, S] (ignored by the depthwise launchers)
    int route;       // the descriptor's anr_conv_route_choice: 0 library's choice, 1 patch kernel, 2 general
    int OH, OW;
    int64_t xs[4];   // element strides n,c,h,w (w stride is 1)
    int64_t ys[4];
    // fused epilogue (ConvLayer): nullptr gamma means plain convolution (in a pre-packed call gamma
    // is only this marker: the constants come from scale_shift)
    const float* gamma;
    const float* beta;
    const float* mean;
    const float* var;
    float eps;
    // pre-packed constants (anr_conv2d_pack_weights): the weights in the order the kernel chosen
    // for this descriptor stages them (w is then the OIHW copy inside the pack, or null when the
    // pack holds no such copy), and the folded batch-norm scale[K] then shift[K]; null: not packed
    const float* wpack;
    const float* scale_shift;
    // caller's workspace (device memory, 16-byte aligned) for the split-K partial tiles
    float* ws;
    size_t ws_bytes;
};
// Workspace the convolution of `a` needs (0 for most shapes): that of the plan for 16-byte
// aligned x and w (null pointers count as aligned); plans for less aligned pointers need none.
size_t conv2d_workspace_bytes(const ConvArgs& a);
// Plans once, checks a.ws / a.ws_bytes against the plan, launches.  *ws_fault: 0 fine, 1 the
// workspace is missing or too small, 2 it is not 16-byte aligned (nothing is enqueued then).
hipError_t launch_conv2d(const ConvArgs& a, hipStream_t stream, int* ws_fault);

// Pre-packed weights.  The pack is [scale K | shift K, padded to 64 floats][weights]; for a plan
// of the patch-staging kernel the weights are that kernel's LDS images, chunk after chunk
// (`patch_layout`), for every other plan a plain OIHW copy.
struct ConvPackLayout {
    bool patch_layout;
    size_t ss_floats;        // floats ahead of the weights
    size_t w_floats;         // floats of the weights part
};
ConvPackLayout conv2d_pack_layout(const ConvArgs& a);
// Writes the pack for `a` (a.w: OIHW weights; a.gamma ..: batch-norm vectors or null) to `pack`.
hipError_t launch_conv2d_pack(const ConvArgs& a, float* pack, hipStream_t stream);
hipError_t launch_dwconv(const ConvArgs& a, hipStream_t stream);

// The library's static scratch array (static_scratch.hip): device address of the current
// device's copy and its size.  Allocates nothing.
constexpr size_t kStaticScratchBytes = (size_t)16 << 20;
hipError_t static_scratch(void** ptr, size_t* bytes);

// out[b] = sqrt(sum of squares of the N x M matrix b); rows `ld` apart, matrices `stride` apart.
struct NrmArgs {
    const float* x;
    float* out;
    int64_t N, M, ld, stride;
    int batch;           // <= 65535
    float* ws;           // partial sums of the slices (see nrm_workspace_bytes)
    size_t ws_bytes;
};
size_t nrm_workspace_bytes(const NrmArgs& a);
hipError_t launch_nrm(const NrmArgs& a, hipStream_t stream);

}  // namespace anr
