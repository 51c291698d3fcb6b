// Launch logic of the TBS batch matmul (kernel in tbg_kernel.h): the tile kernel when the
// operands allow 16-byte loads, the general batched GEMM otherwise.
#include "tbg_kernel.h"

namespace anr {
hipError_t launch_tbg(const GemmArgs& a, hipStream_t stream)
{
    // a describes out[z] = A[z] . B[z]^T with z = (b, h): see GemmArgs
    const bool fast = a.b_is_nk && a.M == a.N && (a.K % 4 == 0) && is_aligned16(a.A) && is_aligned16(a.B) &&
                      (a.lda % 4 == 0) && (a.ldb % 4 == 0) && (a.sAo % 4 == 0) && (a.sAi % 4 == 0) &&
                      (a.sBo % 4 == 0) && (a.sBi % 4 == 0);
    const int tiles = (a.M + tbg::kTile - 1) / tbg::kTile;
    const int64_t blocks = (int64_t)a.batch * tiles * tiles;
    if (!fast || blocks >= ((int64_t)1 << 31)) {
        GemmArgs g = a;
        return launch_gemm(g, stream);
    }
    tbg::Args t{};
    t.q = a.A; t.k = a.B; t.out = a.C;
    t.S = a.M; t.D = a.K; t.H = a.batch_inner;
    t.qs_b = a.sAo; t.qs_s = a.lda; t.qs_h = a.sAi;
    t.ks_b = a.sBo; t.ks_s = a.ldb; t.ks_h = a.sBi;
    t.os_b = a.sCo; t.os_h = a.sCi; t.os_i = a.ldc;
    t.tiles_i = tiles; t.tiles_j = tiles;
    t.xcd_chunk = (blocks % 8 == 0) ? (int)(blocks / 8) : 0;
    hipError_t err = launch_kernel(tbg::tbg_tile_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, t);
    if (err != hipSuccess || !a.softmax_rows) return err;
    return launch_softmax_rows(a, stream);
}

}  // namespace anr
