// Launch logic of the TBS batch matmul (kernel in tbg_kernel.h): the tile kernel when the
// operands allow 16-byte loads, the general batched GEMM otherwise.
#include "tbg_kernel.h"

namespace anr {
namespace {

template <int UT, int KB>
hipError_t launch_tbs_rows32(const tbg::Args& t0, int batch, int vec_store, hipStream_t stream)
{
    using T = tbg::TbsShape<KB>;
    tbg::Args t = t0;
    const int ld = (t.D < tbg::kChunk ? t.D : tbg::kChunk) + 4;     // the panel in LDS is one chunk wide
    t.tiles_i = (t.S + T::rows_q - 1) / T::rows_q;
    const int64_t items = (int64_t)batch * t.tiles_i;
    t.xcd_chunk = (items % 8 == 0) ? (int)(items / 8) : 0;
    // q rows, then the k panel, which the staged probabilities (rows_q x ldp) later overwrite
    const size_t kpanel = (size_t)T::rows_k * ld, probs = (size_t)T::rows_q * T::ldp;
    const size_t lds_bytes = sizeof(float) * ((size_t)T::rows_q * ld + (kpanel > probs ? kpanel : probs));
    t.d_tiles_i = make_fastdiv(t.tiles_i);
    t.d_h = make_fastdiv(t.H);
    // the whole form: S is exactly the keys of KB blocks and whole blocks of queries, D whole
    // chunks, 32-bit byte offsets inside one (b, h) view
    constexpr bool whole_ut = UT == (T::rows_q + T::rows_k) / 16;
    const bool whole = whole_ut && t.S == T::rows_k && (t.S % T::rows_q == 0) && (t.D % tbg::kChunk == 0) &&
                       (int64_t)(t.S - 1) * t.qs_s + t.D < ((int64_t)1 << 29) &&
                       (int64_t)(t.S - 1) * t.ks_s + t.D < ((int64_t)1 << 29) &&
                       (int64_t)(t.S - 1) * t.os_i + t.S < ((int64_t)1 << 29);
    constexpr int UTW = (T::rows_q + T::rows_k) / 16;
    auto kern = whole ? tbg::tbs_rows32_kernel<UTW, true, KB, true> : tbg::tbs_rows32_kernel<UT, true, KB, false>;
    if (lds_bytes > 48 * 1024) {
        static LdsLimit granted[2];    // one per kernel form
        hipError_t e = raise_lds_limit(reinterpret_cast<const void*>(kern), lds_bytes, granted[whole ? 1 : 0]);
        if (e != hipSuccess) return e;
    }
    return launch_kernel(kern, dim3((unsigned)items), dim3(256), lds_bytes, stream, t, ld, vec_store);
}

// UT for D <= 32 / more is (rows_q + rows_k) * (chunk/4) / 256 rounded up: 160 rows for KB = 4
// and 1, 128 rows for KB = 2; the chunk is at most 64 columns.
template <int KB>
hipError_t launch_tbs_by_d(const tbg::Args& t, int batch, int vec_store, hipStream_t stream)
{
    constexpr int rows = tbg::TbsShape<KB>::rows_q + tbg::TbsShape<KB>::rows_k;
    if (t.D <= 32) return launch_tbs_rows32<(rows * 8 + 255) / 256, KB>(t, batch, vec_store, stream);
    return launch_tbs_rows32<(rows * 16 + 255) / 256, KB>(t, batch, vec_store, stream);
}

}  // namespace

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
    if (a.softmax_rows && a.M <= tbg::kMaxKeys && a.K <= 1024 && (a.K % 8 == 0)) {
        // fused TBS: a block of query rows x all keys per work-group
        const int vec_store = is_aligned16(a.C) && (a.ldc % 4 == 0) && (a.sCo % 4 == 0) && (a.sCi % 4 == 0);
        if (a.M <= 32) return launch_tbs_by_d<1>(t, a.batch, vec_store, stream);
        if (a.M <= 64) return launch_tbs_by_d<2>(t, a.batch, vec_store, stream);
        return launch_tbs_by_d<4>(t, a.batch, vec_store, stream);
    }
    // whole tiles, whole chunks and 32-bit byte offsets inside one (b, h) view: the lean form
    const bool whole = (a.M % tbg::kTile == 0) && (a.K % tbg::kChunk == 0) &&
                       (int64_t)(a.M - 1) * a.lda + a.K < ((int64_t)1 << 29) &&
                       (int64_t)(a.N - 1) * a.ldb + a.K < ((int64_t)1 << 29) &&
                       (int64_t)(a.M - 1) * a.ldc + a.N < ((int64_t)1 << 29);
    t.d_tiles_j = make_fastdiv(t.tiles_j);
    t.d_tiles_i = make_fastdiv(t.tiles_i);
    t.d_h = make_fastdiv(t.H);
    hipError_t err = whole ? launch_kernel(tbg::tbg_tile64_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, t)
                           : launch_kernel(tbg::tbg_tile_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, t);
    if (err != hipSuccess || !a.softmax_rows) return err;
    return launch_softmax_rows(a, stream);
}

}  // namespace anr
