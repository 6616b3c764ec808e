// Dispatcher of the bf16 NT GEMM (qkv / proj / fc1 / fc2 of the SAM block).
#include "gemm_kernel.h"

namespace {

template <int BM, int BN, int EPI>
int launch_gemm(const bf16 *A, const bf16 *W, const float *bias, bf16 *C, int M, int N, int K,
                const GemmRowMap &rm, hipStream_t st)
{
    constexpr size_t lds = gemm_lds_bytes<BM, BN>();
    auto kern = gemm_bf16_nt_kernel<BM, BN, EPI>;
    // more than 64 KiB of LDS per workgroup needs the per-kernel opt-in (idempotent, host-side only)
    if (lds > 64 * 1024 &&
        hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
        return SSAM_EHIP;
    int tiles_m = ssam_div_up(M, BM), tiles_n = N / BN;
    int per_xcd = ssam_div_up((long)tiles_m * tiles_n, 8);
    hipLaunchKernelGGL(kern, dim3(per_xcd * 8), dim3(GEMM_THREADS), lds, st, A, W, bias, C, M, N, K, tiles_m, tiles_n, rm);
    SSAM_CHECK_LAUNCH();
    return SSAM_OK;
}

template <int BM, int BN>
int launch_gemm_epi(int epi, const bf16 *A, const bf16 *W, const float *bias, bf16 *C, int M, int N, int K,
                    const GemmRowMap &rm, hipStream_t st)
{
    switch (epi) {
    case SSAM_EPI_BIAS: return launch_gemm<BM, BN, SSAM_EPI_BIAS>(A, W, bias, C, M, N, K, rm, st);
    case SSAM_EPI_BIAS_GELU: return launch_gemm<BM, BN, SSAM_EPI_BIAS_GELU>(A, W, bias, C, M, N, K, rm, st);
    case SSAM_EPI_BIAS_SCATTER_ADD: return launch_gemm<BM, BN, SSAM_EPI_BIAS_SCATTER_ADD>(A, W, bias, C, M, N, K, rm, st);
    default: return SSAM_EINVAL;
    }
}

// Pick the tile by a small cost model: relative throughput of a full machine of such tiles
// (measured on MI355X on the ViT-H layer shapes: the 256x256 tile reads least LDS per flop; the
// 128x128 tile runs two workgroups per CU) times the fill of the last round of workgroups.
int pick_tile(int M, int N)
{
    struct Cand { int id, bm, bn, slots; double eff; };
    const Cand cands[3] = { { 1, 256, 256, 256, 1.00 }, { 2, 256, 128, 256, 0.78 }, { 3, 128, 128, 512, 0.80 } };
    int best = 3;
    double best_score = -1.0;
    for (const Cand &c : cands) {
        if (N % c.bn != 0) continue;
        long tiles = (long)ssam_div_up(M, c.bm) * (N / c.bn);
        long rounds = (tiles + c.slots - 1) / c.slots;
        double fill = (double)tiles / (double)(rounds * c.slots);
        double ragged = (double)M / ((double)ssam_div_up(M, c.bm) * c.bm);
        double score = c.eff * fill * ragged;
        if (score > best_score) { best_score = score; best = c.id; }
    }
    return best;
}

}  // namespace

int ssam_linear_impl(const void *A, const void *W, const float *bias, void *C, int M, int N, int K,
                     int epilogue, const GemmRowMap &rm, int tile, hipStream_t st)
{
    const bf16 *a = (const bf16 *)A, *w = (const bf16 *)W;
    bf16 *c = (bf16 *)C;
    if (tile == 0) tile = pick_tile(M, N);
    switch (tile) {
    case 1: if (N % 256) return SSAM_EUNSUPPORTED; return launch_gemm_epi<256, 256>(epilogue, a, w, bias, c, M, N, K, rm, st);
    case 2: return launch_gemm_epi<256, 128>(epilogue, a, w, bias, c, M, N, K, rm, st);
    case 3: return launch_gemm_epi<128, 128>(epilogue, a, w, bias, c, M, N, K, rm, st);
    default: return SSAM_EINVAL;
    }
}

extern "C" int ssam_linear_tiled(const void *A, const void *W, const float *bias, void *C, int M, int N, int K,
                                 int epilogue, const int32_t *row_map, int rows_per_batch, int map_batch_stride,
                                 int dst_rows_per_batch, int tile, void *stream)
{
    if (!A || !W || !bias || !C || M <= 0 || N <= 0 || K <= 0) return SSAM_EINVAL;
    if (!ssam_aligned16(A) || !ssam_aligned16(W) || !ssam_aligned16(bias) || !ssam_aligned16(C)) return SSAM_EINVAL;
    if (N % 128 != 0 || K % GEMM_BK != 0) return SSAM_EUNSUPPORTED;
    if (tile < 0 || tile > 3) return SSAM_EINVAL;
    GemmRowMap rm = { nullptr, 1, 0, 1 };
    if (epilogue == SSAM_EPI_BIAS_SCATTER_ADD) {
        if (!row_map || rows_per_batch <= 0 || map_batch_stride < 0 || dst_rows_per_batch <= 0) return SSAM_EINVAL;
        rm = { row_map, rows_per_batch, map_batch_stride, dst_rows_per_batch };
    } else if (epilogue != SSAM_EPI_BIAS && epilogue != SSAM_EPI_BIAS_GELU) {
        return SSAM_EINVAL;
    }
    return ssam_linear_impl(A, W, bias, C, M, N, K, epilogue, rm, tile, (hipStream_t)stream);
}

extern "C" int ssam_linear(const void *A, const void *W, const float *bias, void *C, int M, int N, int K,
                           int epilogue, const int32_t *row_map, int rows_per_batch, int map_batch_stride,
                           int dst_rows_per_batch, void *stream)
{
    return ssam_linear_tiled(A, W, bias, C, M, N, K, epilogue, row_map, rows_per_batch, map_batch_stride,
                             dst_rows_per_batch, 0, stream);
}
