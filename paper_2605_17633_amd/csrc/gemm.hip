// Dispatcher of the bf16 NT GEMM (qkv / proj / fc1 / fc2 of the SAM block).
#include "gemm_kernel.h"

namespace {

struct SplitWs { void *ptr; size_t bytes; };

// How a launch of `total` large tiles over `slots` concurrent workgroups is cut: `rem` left-over large
// tiles go to a second launch of `subs` smaller tiles each (0: none, when the tiles do not fill one
// round, fill the last one exactly, fill more than half of it, or give every CU a workgroup), and that launch also cuts K into
// `parts` ranges (1: no) when a workspace is there, K is long and the left-over is small.  A problem of less
// than one round is treated as all left-over when cutting K gives it at least twice the workgroups.
struct TailPlan { int rem, parts; };

TailPlan plan_tail(int total, int slots, int nk, int subs, size_t sub_tile_bytes, const SplitWs &ws)
{
    TailPlan p = { total % slots, 1 };
    if (total < slots) {
        // not even one round of large tiles (small batches): a handful of workgroups would each walk all of K
        // alone.  With a workspace the whole problem runs as the left-over form instead: smaller tiles, K cut
        // into ranges, so that about 512 workgroups share it.
        const int n_all = total * subs;
        int parts = nk / 4;
        if (n_all > 0 && parts > 512 / n_all) parts = 512 / n_all;
        if (ws.ptr && parts >= 2 && (size_t)n_all * parts * sub_tile_bytes <= ws.bytes) {
            p.rem = total;
            p.parts = parts;
            return p;
        }
        p.rem = 0;
    }
    // A last round that is more than half full stays in the main launch.  So does one that gives every CU a
    // workgroup (tiles that run two per CU: a lone workgroup has the CU to itself and finishes in about 0.6 of
    // a full round's time, sooner than the same work as a second launch of smaller tiles).
    if (p.rem > slots / 2 || p.rem >= 256) p.rem = 0;
    if (p.rem == 0) return p;
    const int n_sub = p.rem * subs;
    int parts = nk / 4;                         // at least 4 slabs per workgroup
    if (parts > 256 / n_sub) parts = 256 / n_sub;
    if (ws.ptr && parts >= 4 && (size_t)n_sub * parts * sub_tile_bytes <= ws.bytes) p.parts = parts;
    return p;
}

template <int BM, int BN, int EPI, int SUB_M, int SUB_N, int WGM = 2, int WGN = 2, bool WPACK = false, bool LNF = false>
int launch_range(const bf16 *A, const bf16 *W, const float *bias, bf16 *C, int M, int N, int K,
                 const GemmLd &ld, const GemmTileRange &tr, const GemmRowMap &rm, const GemmSplit &sp, const GemmFold &fold,
                 hipStream_t st)
{
    if (tr.tile_count <= 0) return SSAM_OK;
    constexpr size_t lds = gemm_lds_bytes<BM, BN, WGM, WGN, WPACK>();
    auto kern = gemm_bf16_nt_kernel<BM, BN, EPI, SUB_M, SUB_N, WGM, WGN, WPACK, LNF>;
    // more than 64 KiB of LDS per workgroup needs the per-kernel opt-in (idempotent, host-side only)
    if (lds > 64 * 1024 &&
        hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
        return SSAM_EHIP;
    int per_xcd = ssam_div_up((long)tr.tile_count * SUB_M * SUB_N * sp.parts, 8);
    hipLaunchKernelGGL(kern, dim3(per_xcd * 8), dim3(64 * WGM * WGN), lds, st, A, W, bias, C, M, N, K, ld, tr, rm, sp, fold);
    SSAM_CHECK_LAUNCH();
    return SSAM_OK;
}

// Whole rounds of BM x BN tiles, then the left-over tiles (when they would fill less than half a round)
// as TM x TN tiles, BM = SUB_M*TM, BN = SUB_N*TN.  slots = workgroups the chip runs at once with the large
// tile.  With a workspace, a long K and few left-over tiles, the left-over launch also cuts K (see the kernel).
template <int BM, int BN, int TM, int TN, int EPI, int WGM = 2, int WGN = 2, bool WPACK = false, bool LNF = false>
int launch_split(const bf16 *A, const bf16 *W, const float *bias, bf16 *C, int M, int N, int K,
                 const GemmLd &ld, int slots, const GemmRowMap &rm, const SplitWs &ws, const GemmFold &fold, hipStream_t st)
{
    constexpr int SUB_M = BM / TM, SUB_N = BN / TN;
    const GemmSplit whole = { nullptr, 1 };
    GemmTileRange tr = { ssam_div_up(M, BM), ssam_div_up(N, BN), 0, 0 };
    const int total = tr.tiles_m * tr.tiles_n;
    const int nk = ssam_div_up(K, GEMM_BK);
    const TailPlan plan = plan_tail(total, slots, nk, SUB_M * SUB_N, (size_t)TM * TN * sizeof(float), ws);
    const int rem = plan.rem, parts = plan.parts;
    tr.tile_count = total - rem;
    if constexpr (WGM * WGN == 4 && WPACK) if (rem != 0 && tr.tile_count != 0) {
        // four-wave large tiles: whole rounds and left-over share one launch (see the fused kernel); a K-split
        // left-over is then finished by the reduce kernel as usual
        GemmTileRange tt = tr;
        tt.tile_begin = total - rem;
        tt.tile_count = rem;
        const int n_sub = rem * SUB_M * SUB_N;
        const int n_tail = ssam_div_up(n_sub * parts, 8) * 8, n_main = ssam_div_up(tr.tile_count, 8) * 8;
        constexpr size_t lds_main = gemm_lds_bytes<BM, BN, WGM, WGN, WPACK>(), lds_tail = gemm_lds_bytes<TM, TN, 2, 2, WPACK>();
        constexpr size_t lds = lds_main > lds_tail ? lds_main : lds_tail;
        static_assert(lds <= 64 * 1024, "the fused launch stays within the default LDS limit");
        if (parts > 1) {
            const GemmSplit sp = { (float *)ws.ptr, parts };
            hipLaunchKernelGGL((gemm_bf16_nt_fused_kernel<BM, BN, EPI, WGM, WGN, TM, TN, GEMM_EPI_PARTIAL, SUB_M, SUB_N, WPACK, LNF>),
                               dim3(n_tail + n_main), dim3(256), lds, st, A, W, bias, C, M, N, K, ld, tr, tt, rm, sp, n_tail, fold);
            SSAM_CHECK_LAUNCH();
            constexpr int RPB = 256 / (TN / 8);
            hipLaunchKernelGGL((gemm_tail_reduce_kernel<TM, TN, EPI, SUB_M, SUB_N, LNF>), dim3(n_sub * (TM / RPB)), dim3(256), 0, st,
                               (const float *)ws.ptr, parts, bias, C, M, N, ld, tt, rm, fold);
        } else {
            hipLaunchKernelGGL((gemm_bf16_nt_fused_kernel<BM, BN, EPI, WGM, WGN, TM, TN, EPI, SUB_M, SUB_N, WPACK, LNF>),
                               dim3(n_tail + n_main), dim3(256), lds, st, A, W, bias, C, M, N, K, ld, tr, tt, rm, whole, n_tail, fold);
        }
        SSAM_CHECK_LAUNCH();
        return SSAM_OK;
    }
    int rc = launch_range<BM, BN, EPI, 1, 1, WGM, WGN, WPACK, LNF>(A, W, bias, C, M, N, K, ld, tr, rm, whole, fold, st);
    if (rc != SSAM_OK || rem == 0) return rc;
    tr.tile_begin = total - rem;
    tr.tile_count = rem;
    const int n_sub = rem * SUB_M * SUB_N;
    if (parts > 1) {
        const GemmSplit sp = { (float *)ws.ptr, parts };
        rc = launch_range<TM, TN, GEMM_EPI_PARTIAL, SUB_M, SUB_N, 2, 2, WPACK, LNF>(A, W, bias, C, M, N, K, ld, tr, rm, sp, fold, st);
        if (rc != SSAM_OK) return rc;
        constexpr int RPB = 256 / (TN / 8);
        hipLaunchKernelGGL((gemm_tail_reduce_kernel<TM, TN, EPI, SUB_M, SUB_N, LNF>), dim3(n_sub * (TM / RPB)), dim3(256), 0, st,
                           (const float *)ws.ptr, parts, bias, C, M, N, ld, tr, rm, fold);
        SSAM_CHECK_LAUNCH();
        return SSAM_OK;
    }
    return launch_range<TM, TN, EPI, SUB_M, SUB_N, 2, 2, WPACK, LNF>(A, W, bias, C, M, N, K, ld, tr, rm, whole, fold, st);
}

const GemmFold no_fold = { nullptr, nullptr, nullptr };

template <int EPI, bool LNF = false>
int launch_tile_packed(int tile, const bf16 *A, const bf16 *W, const float *bias, bf16 *C, int M, int N, int K,
                       const GemmLd &ld, const GemmRowMap &rm, const SplitWs &ws, hipStream_t st, const GemmFold &fold = no_fold)
{
    switch (tile) {
    case 1: return launch_split<256, 256, 128, 128, EPI, 2, 4, true, LNF>(A, W, bias, C, M, N, K, ld, 256, rm, ws, fold, st);
    case 3: return launch_split<128, 128, 64, 128, EPI, 2, 2, true, LNF>(A, W, bias, C, M, N, K, ld, 512, rm, ws, fold, st);
    case 4: return launch_split<128, 256, 128, 128, EPI, 1, 4, true, LNF>(A, W, bias, C, M, N, K, ld, 512, rm, ws, fold, st);
    default: return SSAM_EUNSUPPORTED;
    }
}

template <int EPI>
int launch_tile(int tile, const bf16 *A, const bf16 *W, const float *bias, bf16 *C, int M, int N, int K,
                const GemmLd &ld, const GemmRowMap &rm, const SplitWs &ws, hipStream_t st)
{
    switch (tile) {
    case 1: return launch_split<256, 256, 128, 128, EPI, 2, 4>(A, W, bias, C, M, N, K, ld, 256, rm, ws, no_fold, st);
    case 2: return launch_split<256, 128, 128, 128, EPI>(A, W, bias, C, M, N, K, ld, 256, rm, ws, no_fold, st);
    case 3: return launch_split<128, 128, 64, 128, EPI>(A, W, bias, C, M, N, K, ld, 512, rm, ws, no_fold, st);
    case 4: return launch_split<128, 256, 128, 128, EPI, 1, 4>(A, W, bias, C, M, N, K, ld, 512, rm, ws, no_fold, st);   // same plan as packed
    default: return SSAM_EINVAL;
    }
}

// Pick the tile by a time model in microseconds, fitted on MI355X to the ViT-H layer shapes: a round of
// workgroups costs nk * t_slab + t_epi.  The 256x256 tile (eight waves, one workgroup per CU) and the 128x256
// tile (four waves in a row, two workgroups per CU) give a wave the same 128x64 piece and move the same data
// per flop; with two independent workgroups per CU one's epilogue overlaps the other's main loop, which is worth
// 5 us a round behind the GELU epilogue and 1-2.5 us behind the others.  The 128x128 tile (two per CU) moves
// more data per flop and is for small problems.  The left-over launch costs a lone workgroup's walk over its
// K range, latency bound, plus the reduce.
int pick_tile(int M, int N, int K, int epilogue, const SplitWs &ws, bool packed)
{
    struct Cand { int id, bm, bn, tm, tn, slots; double t_slab, t_epi[4]; };   // t_epi: bias, +GELU, scatter-add, scatter
    const Cand cands[4] = { { 1, 256, 256, 128, 128, 256, 1.73, { 5.1, 13.6, 13.5, 6.0 } },
                            { 2, 256, 128, 128, 128, 256, 1.15, { 4.0, 9.0, 9.5, 4.5 } },
                            { 3, 128, 128, 64, 128, 512, 1.10, { 3.5, 6.6, 6.8, 4.0 } },
                            { 4, 128, 256, 128, 128, 512, 1.71, { 5.0, 9.0, 11.5, 5.5 } } };
    const int nk = ssam_div_up(K, GEMM_BK);
    int best = 3;
    double best_time = 1e30;
    for (const Cand &c : cands) {
        if (c.id == 2) continue;    // 256x128 is never the fastest on these shapes: kept as a forced choice only
        if (c.id == 4 && !packed) continue;   // with W in LDS a 128x256 workgroup needs 96 KB: one per CU, nothing overlaps
        const int subs = (c.bm / c.tm) * (c.bn / c.tn);
        const int total = ssam_div_up(M, c.bm) * ssam_div_up(N, c.bn);
        const TailPlan plan = plan_tail(total, c.slots, nk, subs, (size_t)c.tm * c.tn * sizeof(float), ws);
        const double round = nk * c.t_slab + c.t_epi[epilogue];
        const int in_main = total - plan.rem, last = in_main % c.slots;
        double t = (double)(in_main / c.slots) * round;
        if (last != 0) t += round * (c.slots > 256 && last * 2 <= c.slots ? 0.62 : 1.0);   // lone workgroups on their CUs
        if (plan.rem != 0) {
            const int n_sub = plan.rem * subs;
            t += plan.parts > 1 ? ssam_div_up(nk, plan.parts) * 0.9 + 11.0 : (nk * 0.75 + 5.0) * (1.0 + n_sub / 1024.0);
        }
        if (t < best_time) { best_time = t; best = c.id; }
    }
    return best;
}

}  // namespace

int ssam_linear_impl(const void *A, const void *W, const float *bias, void *C, int M, int N, int K,
                     const GemmLd &ld, bool packed, int epilogue, const GemmRowMap &rm, int tile,
                     void *split_ws, size_t split_ws_bytes, hipStream_t st)
{
    const SplitWs ws = { split_ws, split_ws_bytes };
    const bf16 *a = (const bf16 *)A, *w = (const bf16 *)W;
    bf16 *c = (bf16 *)C;
    if (tile == 0) tile = pick_tile(M, N, K, epilogue, ws, packed);
    if (packed) {
        switch (epilogue) {
        case SSAM_EPI_BIAS: return launch_tile_packed<SSAM_EPI_BIAS>(tile, a, w, bias, c, M, N, K, ld, rm, ws, st);
        case SSAM_EPI_BIAS_GELU: return launch_tile_packed<SSAM_EPI_BIAS_GELU>(tile, a, w, bias, c, M, N, K, ld, rm, ws, st);
        case SSAM_EPI_BIAS_SCATTER_ADD: return launch_tile_packed<SSAM_EPI_BIAS_SCATTER_ADD>(tile, a, w, bias, c, M, N, K, ld, rm, ws, st);
        case SSAM_EPI_BIAS_SCATTER: return launch_tile_packed<SSAM_EPI_BIAS_SCATTER>(tile, a, w, bias, c, M, N, K, ld, rm, ws, st);
        default: return SSAM_EINVAL;
        }
    }
    switch (epilogue) {
    case SSAM_EPI_BIAS: return launch_tile<SSAM_EPI_BIAS>(tile, a, w, bias, c, M, N, K, ld, rm, ws, st);
    case SSAM_EPI_BIAS_GELU: return launch_tile<SSAM_EPI_BIAS_GELU>(tile, a, w, bias, c, M, N, K, ld, rm, ws, st);
    case SSAM_EPI_BIAS_SCATTER_ADD: return launch_tile<SSAM_EPI_BIAS_SCATTER_ADD>(tile, a, w, bias, c, M, N, K, ld, rm, ws, st);
    case SSAM_EPI_BIAS_SCATTER: return launch_tile<SSAM_EPI_BIAS_SCATTER>(tile, a, w, bias, c, M, N, K, ld, rm, ws, st);
    default: return SSAM_EINVAL;
    }
}

// fc1 of the routed MLP with gather and LN2 folded in (see GemmFold): rows src[m] of A, packed folded weights,
// GELU epilogue, any M; the tile is picked as for the plain contraction of the same shape.
int ssam_linear_fold_gelu_impl(const void *A, const int32_t *src, const float *stats, const void *Wfp, const float *colsum,
                               const float *bias_f, void *C, int M, int N, int K, const GemmLd &ld,
                               void *split_ws, size_t split_ws_bytes, hipStream_t st)
{
    const SplitWs ws = { split_ws, split_ws_bytes };
    const GemmFold fold = { reinterpret_cast<const float2 *>(stats), colsum, src };
    const GemmRowMap none = { nullptr, 1, 0, 1 };
    const int tile = pick_tile(M, N, K, SSAM_EPI_BIAS_GELU, ws, true);
    return launch_tile_packed<SSAM_EPI_BIAS_GELU, true>(tile, (const bf16 *)A, (const bf16 *)Wfp, bias_f, (bf16 *)C, M, N, K, ld,
                                                        none, ws, st, fold);
}

// The contraction with the LayerNorm of its A rows folded in (see GemmFold): 128x256 tiles, packed weights,
// mapped store; M a multiple of 128 and N of 256, so there are no left-over tiles.
int ssam_linear_ln_impl(const void *A, const float *stats, const void *Wfp, const float *colsum, const float *bias_f,
                        void *C, int M, int N, int K, const GemmLd &ld, const GemmRowMap &rm, hipStream_t st)
{
    constexpr size_t lds = gemm_lds_bytes<128, 256, 1, 4, true>();
    static_assert(lds <= 64 * 1024, "default LDS limit");
    GemmTileRange tr = { M / 128, N / 256, 0, (M / 128) * (N / 256) };
    const GemmFold fold = { reinterpret_cast<const float2 *>(stats), colsum, nullptr };
    const int per_xcd = ssam_div_up(tr.tile_count, 8);
    hipLaunchKernelGGL((gemm_bf16_nt_lnf_kernel<128, 256, SSAM_EPI_BIAS_SCATTER, 1, 4>), dim3(per_xcd * 8), dim3(256), lds, st,
                       (const bf16 *)A, (const bf16 *)Wfp, bias_f, (bf16 *)C, M, N, K, ld, tr, rm, fold);
    SSAM_CHECK_LAUNCH();
    return SSAM_OK;
}

extern "C" int ssam_linear_ln(const void *x, int ldx, const float *stats, const void *Wfp, const float *colsum,
                              const float *bias_f, void *C, int ldc, int M, int N, int K,
                              const int32_t *row_map, int rows_per_batch, int map_batch_stride, int dst_rows_per_batch,
                              void *stream)
{
    if (!x || !stats || !Wfp || !colsum || !bias_f || !C || !row_map || M <= 0 || N <= 0 || K <= 0) return SSAM_EINVAL;
    if (!ssam_aligned16(x) || !ssam_aligned16(Wfp) || !ssam_aligned16(colsum) || !ssam_aligned16(bias_f) || !ssam_aligned16(C) ||
        ((uintptr_t)stats & 7))
        return SSAM_EINVAL;
    if (ldx < K || ldc < N || ldx % 8 || ldc % 8 || rows_per_batch <= 0 || map_batch_stride < 0 || dst_rows_per_batch <= 0) return SSAM_EINVAL;
    if (M % 128 != 0 || N % 256 != 0 || K % GEMM_BK != 0) return SSAM_EUNSUPPORTED;
    const GemmRowMap rm = { row_map, rows_per_batch, map_batch_stride, dst_rows_per_batch };
    return ssam_linear_ln_impl(x, stats, Wfp, colsum, bias_f, C, M, N, K, GemmLd{ ldx, K, ldc }, rm, (hipStream_t)stream);
}

extern "C" size_t ssam_linear_workspace_bytes(void) { return GEMM_SPLIT_WS_BYTES; }

__global__ void __launch_bounds__(256)
pack_weight_kernel(const bf16 *__restrict__ W, int ldw, bf16 *__restrict__ Wp, int N, int K)
{
    // one thread per 16-byte chunk of the packed matrix: chunk id = ((nb*ksteps + s)*64 + lane); lane = 16*quad + l
    // holds row 16*nb + l, k = 32*s + 8*quad .. + 7: the operand-b fragment of the 16x16x32 MFMA
    const long id = (long)blockIdx.x * 256 + threadIdx.x;
    const int ksteps = K / 32;
    if (id >= (long)(N / 16) * ksteps * 64) return;
    const int lane = (int)(id & 63), l = lane & 15, quad = lane >> 4;
    const long cell = id >> 6;
    const int ks = (int)(cell % ksteps), nb = (int)(cell / ksteps);
    reinterpret_cast<u32x4 *>(Wp)[id] = *reinterpret_cast<const u32x4 *>(W + (long)(16 * nb + l) * ldw + 32 * ks + 8 * quad);
}

extern "C" int ssam_pack_weight(const void *W, int ldw, void *Wp, int N, int K, void *stream)
{
    if (!W || !Wp || N <= 0 || K <= 0 || ldw < K || ldw % 8) return SSAM_EINVAL;
    if (!ssam_aligned16(W) || !ssam_aligned16(Wp)) return SSAM_EINVAL;
    if (N % 16 != 0 || K % 32 != 0) return SSAM_EUNSUPPORTED;
    const long chunks = (long)N * K / 8;
    hipLaunchKernelGGL(pack_weight_kernel, dim3((unsigned)ssam_div_up(chunks, 256)), dim3(256), 0, (hipStream_t)stream,
                       (const bf16 *)W, ldw, (bf16 *)Wp, N, K);
    SSAM_CHECK_LAUNCH();
    return SSAM_OK;
}

extern "C" int ssam_linear_ld(const void *A, int lda, const void *W, int ldw, int w_packed, const float *bias, void *C, int ldc,
                              int M, int N, int K, int epilogue, const int32_t *row_map, int rows_per_batch,
                              int map_batch_stride, int dst_rows_per_batch, int tile,
                              void *workspace, size_t workspace_bytes, void *stream)
{
    if (!A || !W || !bias || !C || M <= 0 || N <= 0 || K <= 0) return SSAM_EINVAL;
    if (!ssam_aligned16(A) || !ssam_aligned16(W) || !ssam_aligned16(bias) || !ssam_aligned16(C)) return SSAM_EINVAL;
    if (N % 8 != 0 || K % 8 != 0) return SSAM_EUNSUPPORTED;
    if (w_packed && (N % 128 != 0 || K % GEMM_BK != 0)) return SSAM_EUNSUPPORTED;
    if (lda < K || ldc < N || lda % 8 || ldc % 8 || (!w_packed && (ldw < K || ldw % 8))) return SSAM_EINVAL;
    if (workspace && !ssam_aligned16(workspace)) return SSAM_EINVAL;
    if (tile < 0 || tile > 4) return SSAM_EINVAL;
    if (w_packed && tile == 2) return SSAM_EUNSUPPORTED;
    GemmRowMap rm = { nullptr, 1, 0, 1 };
    if (epilogue == SSAM_EPI_BIAS_SCATTER_ADD || epilogue == SSAM_EPI_BIAS_SCATTER) {
        if (!row_map || rows_per_batch <= 0 || map_batch_stride < 0 || dst_rows_per_batch <= 0) return SSAM_EINVAL;
        rm = { row_map, rows_per_batch, map_batch_stride, dst_rows_per_batch };
    } else if (epilogue != SSAM_EPI_BIAS && epilogue != SSAM_EPI_BIAS_GELU) {
        return SSAM_EINVAL;
    }
    GemmLd ld = { lda, ldw, ldc };
    return ssam_linear_impl(A, W, bias, C, M, N, K, ld, w_packed != 0, epilogue, rm, tile, workspace, workspace ? workspace_bytes : 0,
                            (hipStream_t)stream);
}

extern "C" int ssam_linear_tiled(const void *A, const void *W, const float *bias, void *C, int M, int N, int K,
                                 int epilogue, const int32_t *row_map, int rows_per_batch, int map_batch_stride,
                                 int dst_rows_per_batch, int tile, void *stream)
{
    return ssam_linear_ld(A, K, W, K, 0, bias, C, N, M, N, K, epilogue, row_map, rows_per_batch, map_batch_stride,
                          dst_rows_per_batch, tile, nullptr, 0, stream);
}

extern "C" int ssam_linear(const void *A, const void *W, const float *bias, void *C, int M, int N, int K,
                           int epilogue, const int32_t *row_map, int rows_per_batch, int map_batch_stride,
                           int dst_rows_per_batch, void *stream)
{
    return ssam_linear_ld(A, K, W, K, 0, bias, C, N, M, N, K, epilogue, row_map, rows_per_batch, map_batch_stride,
                          dst_rows_per_batch, 0, nullptr, 0, stream);
}
