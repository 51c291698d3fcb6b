/*
 * anr.h - C ABI of the MI355X (gfx950) fp32 operator library.
 *
 * The entry points are the dense fp32 operator programs evaluated in
 * arXiv 2006.06762 ("Ansor"): GMM, C2D and DEP of the single-operator
 * benchmark (Sec. 7.1, shapes in Appendix C) and the ConvLayer and TBS
 * subgraphs (Sec. 7.2).  All arithmetic is fp32 in, fp32 accumulate, fp32 out
 * (Sec. 7: float32 is used for all evaluations).
 *
 * Conventions common to every call
 *   - Every tensor pointer is DEVICE memory owned by the caller.  The library
 *     never allocates, frees or synchronises.  Work is enqueued on the HIP
 *     stream passed as `hip_stream` (a hipStream_t cast to void*; NULL is the
 *     default stream) and the call returns without waiting for it.
 *   - Descriptors are HOST structs, read during the call only.
 *   - Inputs are read-only; outputs are fully overwritten (no accumulate) and
 *     must not overlap any input.
 *   - Pointers must be 4-byte aligned.  16-byte aligned pointers together
 *     with row extents/strides that are multiples of 4 elements select the
 *     vectorised kernels; anything else runs a slower kernel with the same
 *     results.
 *   - `ws`/`ws_bytes` is a device workspace owned by the caller, 16-byte
 *     aligned.  anr_workspace_size() says how many bytes an operation needs
 *     for a descriptor; the figure depends on the descriptor only (it is the
 *     need of the plan for 16-byte aligned pointers, the one
 *     anr_conv2d_route reports; a call whose pointers are less aligned runs
 *     kernels that need no workspace); ws may be NULL when it is 0.  Two
 *     operations use one: the convolutions for shapes with few output tiles
 *     and a long reduction (batch 1, 7x7 maps), whose reduction is split
 *     over work-groups that leave partial tiles there, and anr_nrm for the
 *     partial sums of a matrix's slices.  Its contents on entry do not
 *     matter and are undefined on return.  A call that needs more than it
 *     is given returns ANR_ERR_WORKSPACE.  Calls that share one workspace
 *     must be ordered (same stream).
 *   - Errors are return codes.  All argument checks happen on the host before
 *     anything is launched, so an invalid call has no effect on the device.
 *   - Thread-safe and re-entrant.  The library reads no environment variable
 *     and no configuration file: what a call does follows from its arguments
 *     alone.  The only state is a thread-local copy of the last HIP launch
 *     error, kept for anr_last_hip_error(), and two idempotent per-device
 *     notes: that a kernel's shared-memory limit has been raised, and the
 *     address of the static scratch array of anr_conv2d_noalloc (whose
 *     CONTENTS are shared by all calls of that one entry point on a GPU: see
 *     there).
 */
#ifndef ANR_H
#define ANR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    ANR_OK = 0,
    ANR_ERR_NULL = 1,         /* a required pointer is NULL                        */
    ANR_ERR_INVALID_ARG = 2,  /* non-positive extent, bad stride, empty output ... */
    ANR_ERR_UNSUPPORTED = 3,  /* valid but not implemented (layout, w-stride != 1,
                                 extents beyond the kernels' index range)          */
    ANR_ERR_WORKSPACE = 4,    /* ws_bytes smaller than anr_workspace_size()        */
    ANR_ERR_LAUNCH = 5        /* the HIP runtime refused the launch                */
} anr_status;

typedef enum { ANR_LAYOUT_NCHW = 0 } anr_layout;

typedef enum {
    ANR_OP_GEMM = 0, ANR_OP_CONV2D = 1, ANR_OP_CONV_BN_RELU = 2, ANR_OP_DWCONV = 3,
    ANR_OP_TBG = 4, ANR_OP_TBS = 5, ANR_OP_NRM = 6
} anr_op;

/*
 * GMM.  C[b] = A[b] (M x K) . B[b] (K x N), b = 0 .. batch-1; all row-major.
 * Element (i,k) of A[b] is A[b*strideA + i*lda + k]; likewise B (ldb) and C
 * (ldc).  Requirements: M,N,K,batch >= 1; lda >= K; ldb >= N; ldc >= N;
 * for batch > 1, strideC >= (M-1)*ldc + N (outputs must not overlap);
 * strideA/strideB may be 0 to share an operand across the batch.
 */
typedef struct {
    int64_t M, N, K;
    int64_t lda, ldb, ldc;
    int64_t batch;
    int64_t strideA, strideB, strideC;
} anr_gemm_desc;

/*
 * Convolution geometry shared by C2D, ConvLayer, DEP and the GRP / DIL
 * variants of C2D (Sec. 7.1, Appendix C).
 *   x [N,C,H,W], y [N,K,OH,OW] with
 *   OH = floor((H + 2*pad_h - dil_h*(R-1) - 1)/stride_h) + 1 (OW alike).
 *   Cross-correlation (no kernel flip); tap (r,s) reads input row
 *   oh*stride_h - pad_h + r*dil_h; zero padding, the same amount on both
 *   sides.  K is the number of output channels; for the depthwise call K
 *   must equal C (channel multiplier 1).
 *   groups (0 means 1): input and output channels are cut into `groups`
 *   equal runs and output channel k only sees the C/groups input channels of
 *   run k / (K/groups); C and K must be multiples of it.  The depthwise call
 *   ignores the field.
 *   Weights are always packed: OIHW [K, C/groups, R, S] for conv2d /
 *   conv_bn_relu, [C,1,R,S] for dwconv.
 *   x_stride / y_stride are element strides for (n, c, h, w).  All four zero
 *   means packed NCHW.  Otherwise every stride must be >= 1 and the view must
 *   not alias itself (w-stride 1 is required by this version: anything else
 *   returns ANR_ERR_UNSUPPORTED).
 *   layout must be ANR_LAYOUT_NCHW (else ANR_ERR_UNSUPPORTED).  pad >= 0,
 *   stride >= 1, dil >= 1; pad < kernel extent is NOT required.  OH <= 0 or
 *   OW <= 0 is ANR_ERR_INVALID_ARG.
 *   route (an anr_conv_route_choice; any other value is ANR_ERR_INVALID_ARG)
 *   selects between the library's two families of convolution kernels:
 *   ANR_CONV_ROUTE_AUTO lets the library choose by shape; ANR_CONV_ROUTE_PATCH
 *   asks for the 3x3 patch-staging kernel whenever it can run the shape and
 *   pointers at all (it has no split of the reduction over work-groups, so it
 *   is slow when there are few output tiles); ANR_CONV_ROUTE_GENERAL never
 *   uses it.  Results agree to rounding whatever the route; anr_workspace_size
 *   and anr_conv2d_route follow the field.  The depthwise call ignores it.
 */
typedef enum {
    ANR_CONV_ROUTE_AUTO = 0, ANR_CONV_ROUTE_PATCH = 1, ANR_CONV_ROUTE_GENERAL = 2
} anr_conv_route_choice;

typedef struct {
    int32_t N, C, H, W;
    int32_t K, R, S;
    int32_t stride_h, stride_w;
    int32_t pad_h, pad_w;
    int32_t dil_h, dil_w;
    int32_t layout;
    int64_t x_stride[4];
    int64_t y_stride[4];
    int32_t groups;      /* 0 or 1: ordinary convolution */
    int32_t route;       /* anr_conv_route_choice; 0: the library chooses */
} anr_conv_desc;

/*
 * TBG / TBS.  q and k are indexed [b, s, h, d] (B x S x H x D), out is
 * indexed [b, h, i, j] (B x H x S x S).  Strides are in elements; all four
 * zero means packed in that index order.  The d-stride of q and k and the
 * j-stride of out must be 1 in this version.
 */
typedef struct {
    int32_t B, S, H, D;
    int64_t q_stride[4];
    int64_t k_stride[4];
    int64_t o_stride[4];
} anr_tbg_desc;

/* GMM (Sec. 4.1: C(i,j) = sum_k A[i,k] * B[k,j]; benchmark shapes in
 * Appendix C "GMM"). */
anr_status anr_gemm(const anr_gemm_desc *desc, const float *A, const float *B, float *C,
                    void *ws, size_t ws_bytes, void *hip_stream);

/* C2D (Sec. 7.1, Appendix C "C2D"): y[n,k,oh,ow] = sum_{c,r,s}
 * x[n,c,oh*stride_h-pad_h+r, ow*stride_w-pad_w+s] * w[k,c,r,s], taps outside
 * the image contributing zero. */
anr_status anr_conv2d(const anr_conv_desc *desc, const float *x, const float *w, float *y,
                      void *ws, size_t ws_bytes, void *hip_stream);

/* anr_conv2d for callers that cannot allocate device memory, and so cannot bring a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, kernels and results as anr_conv2d (bit for bit), but the
 * partial tiles of a split reduction go to a fixed array of
 * ANR_STATIC_SCRATCH_BYTES that the library holds in the memory of every GPU it is
 * loaded on, from load time until the process ends.  The call allocates and frees
 * nothing and synchronises nothing.  A descriptor whose plan needs more
 * (anr_workspace_size(ANR_OP_CONV2D, desc) > ANR_STATIC_SCRATCH_BYTES) returns
 * ANR_ERR_WORKSPACE before anything is launched; the limit covers every layer of the
 * paper's shape lists at batch 1 and 16.  All calls on one GPU share that GPU's
 * array: calls that need it and may overlap in time (different streams, different
 * threads) race on it, so keep them on one stream or order them yourself; its
 * contents need not be cleared between calls (every partial tile is written before
 * it is read).  The first call on a device that needs the array looks its address
 * up in the runtime once; make that call outside a graph capture. */
#define ANR_STATIC_SCRATCH_BYTES ((size_t)16 << 20)
anr_status anr_conv2d_noalloc(const anr_conv_desc *desc, const float *x, const float *w, float *y,
                              void *hip_stream);

/*
 * Pre-packed constants (Sec. 4.2 "Random annotation": the layouts of constant tensors
 * are rewritten ahead of time to fit the tile structure, at no run-time cost, because
 * convolution weights are constants for inference; Sec. 7.3 credits this rewrite with
 * about 40 % of the ResNet-50 result).  x and y stay in their plain NCHW layout (Sec. 7.1:
 * inputs and outputs must not be packed); only the weights, and for ConvLayer the folded
 * batch-norm constants, are rewritten, once, into a `pack` that the caller keeps.
 *
 *   anr_conv2d_packed_size   bytes of the pack for `desc` (a function of the descriptor
 *                            only, `route` included).
 *   anr_conv2d_pack_weights  writes the pack: the weights w (OIHW [K, C/groups, R, S]) in
 *                            the order in which the kernel planned for `desc` stages them
 *                            (for the 3x3 patch-staging kernel: per channel tile and chunk
 *                            of input channels one contiguous image of its LDS buffer; for
 *                            every other plan a plain copy), preceded by scale[K], shift[K]
 *                            = gamma/sqrt(var+eps), beta - mean*scale in fp32 when the four
 *                            batch-norm vectors are given (all four or none; none: that part
 *                            of the pack is left unwritten).  `packed`: device memory,
 *                            256-byte aligned, packed_bytes >= anr_conv2d_packed_size (else
 *                            ANR_ERR_WORKSPACE).  Enqueued on the stream like any call.
 *   anr_conv2d_packed        anr_conv2d with the pack in place of w: same results bit for
 *   anr_conv_bn_relu_packed  bit (the same products are summed in the same order), same
 *                            workspace rule.  The descriptor must equal the one the pack
 *                            was made for (not checked: the pack lives in device memory);
 *                            anr_conv_bn_relu_packed needs a pack made with the batch-norm
 *                            vectors.  A pack in the patch kernel's order presumes that
 *                            kernel's alignment rules for x (16-byte aligned pointer,
 *                            strides multiples of 4): a call with another x returns
 *                            ANR_ERR_INVALID_ARG.
 */
anr_status anr_conv2d_packed_size(const anr_conv_desc *desc, size_t *bytes);
anr_status anr_conv2d_pack_weights(const anr_conv_desc *desc, const float *w,
                                   const float *gamma, const float *beta,
                                   const float *mean, const float *var, float eps,
                                   void *packed, size_t packed_bytes, void *hip_stream);
anr_status anr_conv2d_packed(const anr_conv_desc *desc, const float *x, const void *packed, float *y,
                             void *ws, size_t ws_bytes, void *hip_stream);
anr_status anr_conv_bn_relu_packed(const anr_conv_desc *desc, const float *x, const void *packed, float *y,
                                   void *ws, size_t ws_bytes, void *hip_stream);

/* ConvLayer (Sec. 7.2): the convolution above, then inference batch
 * normalisation per output channel, gamma*(v-mean)/sqrt(var+eps)+beta, then
 * ReLU, in one kernel (Table 1 rule 4: element-wise consumers are fused into
 * the tiled producer).  gamma, beta, mean, var: K device floats each.
 * eps must be finite and var[k]+eps > 0 is the caller's responsibility. */
anr_status anr_conv_bn_relu(const anr_conv_desc *desc, const float *x, const float *w,
                            const float *gamma, const float *beta,
                            const float *mean, const float *var, float eps,
                            float *y, void *ws, size_t ws_bytes, void *hip_stream);

/* DEP (Sec. 7.1, Appendix C "DEP"): depthwise convolution, multiplier 1:
 * y[n,c,oh,ow] = sum_{r,s} x[n,c,ih,iw] * w[c,0,r,s]. */
anr_status anr_dwconv(const anr_conv_desc *desc, const float *x, const float *w, float *y,
                      void *ws, size_t ws_bytes, void *hip_stream);

/* TBS without the softmax (Sec. 7.2: two transposes and one batch matmul of
 * multi-head attention): out[b,h,i,j] = sum_d q[b,i,h,d] * k[b,j,h,d].  The
 * transposes [B,S,H,D] -> [B,H,S,D] are folded into the addressing; no
 * 1/sqrt(D) scaling. */
anr_status anr_tbg(const anr_tbg_desc *desc, const float *q, const float *k, float *out,
                   void *ws, size_t ws_bytes, void *hip_stream);

/* Full TBS (Sec. 7.2, Appendix C "TBS"): the scores of anr_tbg followed by a
 * softmax over j (max-subtracted): out[b,h,i,:] = softmax_j(sum_d q.k).  One
 * fused kernel when S <= 128 and D is a multiple of 8 up to 1024; otherwise the
 * anr_tbg kernel and an in-place softmax kernel on the same stream.
 * Requires S <= 1024 (else ANR_ERR_UNSUPPORTED). */
anr_status anr_tbs(const anr_tbg_desc *desc, const float *q, const float *k, float *out,
                   void *ws, size_t ws_bytes, void *hip_stream);

/*
 * NRM.  N x M row-major matrices, row stride ld >= M, matrix b at x + b*stride
 * (stride >= (N-1)*ld + M for batch > 1, or 0 to reduce one matrix `batch`
 * times); batch <= 65535.
 */
typedef struct {
    int64_t N, M, ld;
    int64_t batch, stride;
} anr_nrm_desc;

/* NRM (Sec. 7.1, Appendix C "NRM"; Sec. 4.1 names it as the operator with
 * parallelism only in its reduction): out[b] = sqrt(sum_{i,j} x[b,i,j]^2),
 * `batch` device floats.  Matrices of more than 16 K elements are reduced in
 * slices whose partial sums pass through `ws` (anr_workspace_size); the sum
 * order is fixed, so results do not vary from run to run. */
anr_status anr_nrm(const anr_nrm_desc *desc, const float *x, float *out,
                   void *ws, size_t ws_bytes, void *hip_stream);

/* Bytes of device workspace `op` (an anr_op) needs for `desc` (the matching
 * descriptor type): a function of the descriptor only, enough for any pointer
 * alignment.  Writes 0 when none is needed.  Validates the descriptor the same
 * way the operation does. */
anr_status anr_workspace_size(int op, const void *desc, size_t *bytes);

/* Which kernel anr_conv2d / anr_conv_bn_relu would run for `desc` with 16-byte aligned
 * pointers, and how (host-side planning only: nothing is launched, no GPU is needed).  For
 * callers that want to know why a layer takes the time it does, and for tests of the
 * selection logic.  tile_m x tile_n is the work-group's output tile (pixels x channels),
 * ksplit the number of work-groups that share a tile's reduction through the workspace,
 * wave_groups the groups of four waves inside a work-group that share its chunk chain. */
enum {
    ANR_CONV_KERNEL_PATCH = 1,     /* 3x3 patch-staging kernel tuned on the ResNet-style layers   */
    ANR_CONV_KERNEL_TAPS = 2,      /* 3x3 / 1x1 gather kernel with compile-time taps              */
    ANR_CONV_KERNEL_BIGTAPS = 3,   /* 5x5 / 7x7 gather kernel, one channel per chunk              */
    ANR_CONV_KERNEL_GATHER = 4,    /* any-geometry gather kernel                                  */
    ANR_CONV_KERNEL_DIRECT = 5,    /* one thread per output (extents beyond 32-bit offsets)       */
    ANR_CONV_KERNEL_POINTWISE = 6  /* streaming 1x1 kernel for layers with few channels           */
};
typedef struct {
    int32_t kernel;                /* ANR_CONV_KERNEL_*                                           */
    int32_t tile_m, tile_n;        /* 0 for ANR_CONV_KERNEL_DIRECT                                */
    int32_t ksplit;                /* 1: no split                                                 */
    int32_t wave_groups;           /* 1, 2 or 4                                                   */
    int32_t work_groups;           /* launched by the main kernel                                 */
    uint64_t workspace_bytes;      /* what this plan needs (== anr_workspace_size)                */
} anr_conv_route;
anr_status anr_conv2d_route(const anr_conv_desc *desc, anr_conv_route *route);

/* Static, NUL-terminated description of a status code. */
const char *anr_status_string(anr_status status);

/* Library version: major*10000 + minor*100 + patch. */
int anr_version(void);

/* Diagnostics for ANR_ERR_LAUNCH: the hipError_t value (and its runtime description) of
 * the most recent launch that failed in the calling thread; 0 if none has. */
int anr_last_hip_error(void);
const char *anr_last_hip_error_string(void);

#ifdef __cplusplus
}
#endif
#endif /* ANR_H */
