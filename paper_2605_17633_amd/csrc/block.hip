// Composition of the structured-sparse encoder block: Stripe-Sort attention half
// (Sec. 4.1, App. A.1) and Residual-Consistency MLP half (Sec. 4.2), and the
// stack of blocks that shares one keep-set (Sec. 1, Sec. 4.1 "performed once").
// Host code only: every step is a kernel of this library enqueued on the
// caller's stream; intermediate tensors live in the caller's workspace.
#include "gemm_kernel.h"

int ssam_linear_impl(const void *A, const void *W, const float *bias, void *C, int M, int N, int K,
                     const GemmLd &ld, bool packed, int epilogue, const GemmRowMap &rm, int tile,
                     void *split_ws, size_t split_ws_bytes, hipStream_t st);

int ssam_compact_slots(const int32_t *table, int table_batch_stride, int B, int Nout, int N,
                       int32_t *real_slot, int32_t *real_spatial, int32_t *slot_row, int32_t *pad_slot, hipStream_t st);
int ssam_fill_bias_rows(void *C, long ldc, const float *bias, int n_cols, const int32_t *pad_slot, int npad,
                        int rows_per_batch, int B, hipStream_t st);
int ssam_invert_table(const int32_t *table, int table_batch_stride, int B, int Nout, int N, int32_t *inv, hipStream_t st);
int ssam_linear_ln_impl(const void *A, const float *stats, const void *Wfp, const float *colsum, const float *bias_f,
                        void *C, int M, int N, int K, const GemmLd &ld, const GemmRowMap &rm, hipStream_t st);

int ssam_linear_fold_gelu_impl(const void *A, const int32_t *src, const float *stats, const void *Wfp, const float *colsum,
                               const float *bias_f, void *C, int M, int N, int K, const GemmLd &ld,
                               void *split_ws, size_t split_ws_bytes, hipStream_t st);
int ssam_ln_stats_impl(const void *x, float *stats, long rows, int D, float eps, const int32_t *idx, int idx_batch_stride,
                       int Nin, int Nout, int32_t *src, hipStream_t st);

namespace {

inline size_t align256(size_t n) { return (n + 255) & ~(size_t)255; }

struct BlockGeom {
    int S, w, nW, Nout, N, d;
};

bool block_geom(const ssam_block_cfg *c, BlockGeom &g)
{
    if (!c || c->B <= 0 || c->g <= 0 || c->D <= 0 || c->heads <= 0 || c->Dm <= 0 || c->ws < 0) return false;
    if (c->D % c->heads != 0 || c->K <= 0 || c->K > c->g * c->g) return false;
    g.N = c->g * c->g;
    g.w = c->ws > 0 ? c->ws : c->g;
    g.S = g.w * g.w;
    int nws = (c->g + g.w - 1) / g.w;
    g.nW = nws * nws;
    g.Nout = g.nW * g.S;
    g.d = c->D / c->heads;
    return true;
}

// gathered LN2 rows, hidden activations, then the K-split scratch of the fc2 contraction
size_t mlp_core_bytes(int B, int K, int D, int Dm)
{
    return align256((size_t)B * K * D * 2) + align256((size_t)B * K * Dm * 2);
}

size_t mlp_ws_bytes(int B, int K, int D, int Dm) { return mlp_core_bytes(B, K, D, Dm) + GEMM_SPLIT_WS_BYTES; }

// Tables that let the dense contractions of a windowed block skip the padding slots (see
// compact_slots_kernel): real_slot, real_spatial [B][N], slot_row [B][Nout], pad_slot [B][Nout-N].
struct PadTables {
    int32_t *real_slot, *real_spatial, *slot_row, *pad_slot;
};

size_t pad_tables_bytes(int B, const BlockGeom &g)
{
    if (g.Nout == g.N) return 0;
    return align256((size_t)B * g.N * 4) * 2 + align256((size_t)B * g.Nout * 4) + align256((size_t)B * (g.Nout - g.N) * 4);
}

PadTables carve_pad_tables(unsigned char *p, int B, const BlockGeom &g)
{
    PadTables t;
    t.real_slot = (int32_t *)p;
    p += align256((size_t)B * g.N * 4);
    t.real_spatial = (int32_t *)p;
    p += align256((size_t)B * g.N * 4);
    t.slot_row = (int32_t *)p;
    p += align256((size_t)B * g.Nout * 4);
    t.pad_slot = (int32_t *)p;
    return t;
}

// Tables of a block that depend only on its gather table, kept behind everything a block writes so that a stack
// builds them once: the padding tables (windowed blocks with padding), then slot_of [B][N], the scan-order slot of
// every token (the inverse of the gather table; the folded-LN1 qkv contraction walks the tokens in memory order
// and stores each row to its slot).
size_t block_tables_bytes(int B, const BlockGeom &g) { return pad_tables_bytes(B, g) + align256((size_t)B * g.N * 4); }

int32_t *slot_of_table(unsigned char *tables, int B, const BlockGeom &g) { return (int32_t *)(tables + pad_tables_bytes(B, g)); }

int build_block_tables(const ssam_block_cfg *cfg, const BlockGeom &g, const int32_t *gather_table, unsigned char *tables, hipStream_t st)
{
    const int per_image = cfg->content_order != 0;
    if (g.Nout != g.N) {
        const PadTables pt = carve_pad_tables(tables, cfg->B, g);
        int rc = ssam_compact_slots(gather_table, per_image ? g.Nout : 0, cfg->B, g.Nout, g.N, pt.real_slot, pt.real_spatial, pt.slot_row, pt.pad_slot, st);
        if (rc != SSAM_OK) return rc;
    }
    return ssam_invert_table(gather_table, per_image ? g.Nout : 0, per_image ? cfg->B : 1, g.Nout, g.N, slot_of_table(tables, cfg->B, g), st);
}

}  // namespace

extern "C" size_t ssam_routed_mlp_workspace_bytes(int B, int K, int D, int Dm)
{
    if (B <= 0 || K <= 0 || D <= 0 || Dm <= 0) return 0;
    return mlp_ws_bytes(B, K, D, Dm);
}

// colsum1 != NULL: gather and LN2 folded into fc1 (w1 the packed folded weight, b1 the folded bias; ln_g, ln_b unused)
static int routed_mlp_impl(void *x, const int32_t *keep_idx, const float *ln_g, const float *ln_b, float eps,
                           const void *w1, const float *b1, const void *w2, const float *b2, bool packed,
                           int B, int N, int D, int Dm, int K,
                           void *workspace, size_t workspace_bytes, void *stream, const float *colsum1 = nullptr)
{
    const bool fold = colsum1 != nullptr;
    if (!x || !keep_idx || (!fold && (!ln_g || !ln_b)) || !w1 || !b1 || !w2 || !b2 || !workspace) return SSAM_EINVAL;
    if (fold && (!packed || !ssam_aligned16(colsum1) || !ssam_aligned16(b1))) return SSAM_EINVAL;
    if (B <= 0 || N <= 0 || D <= 0 || Dm <= 0 || K <= 0 || K > N) return SSAM_EINVAL;
    if (!ssam_aligned16(workspace)) return SSAM_EINVAL;
    if (D % 8 != 0 || Dm % 8 != 0) return SSAM_EUNSUPPORTED;
    if (packed && (D % 128 != 0 || Dm % 128 != 0)) return SSAM_EUNSUPPORTED;
    if (workspace_bytes < mlp_ws_bytes(B, K, D, Dm)) return SSAM_EWORKSPACE;
    unsigned char *ws = (unsigned char *)workspace;
    void *a2 = ws;
    void *hid = ws + align256((size_t)B * K * D * 2);
    void *split = ws + mlp_core_bytes(B, K, D, Dm);
    hipStream_t st = (hipStream_t)stream;
    int rc;
    if (fold) {
        // the region of the normalised rows holds only their statistics and the rows of x they are (8 + 4 bytes a row)
        float *stats = (float *)a2;
        int32_t *src = (int32_t *)(stats + 2 * (size_t)B * K);
        rc = ssam_ln_stats_impl(x, stats, (long)B * K, D, eps, keep_idx, K, N, K, src, st);
        if (rc != SSAM_OK) return rc;
        rc = ssam_linear_fold_gelu_impl(x, src, stats, w1, colsum1, b1, hid, B * K, Dm, D, GemmLd{ D, D, Dm }, split, GEMM_SPLIT_WS_BYTES, st);
    } else {
        rc = ssam_ln_gather(x, keep_idx, K, ln_g, ln_b, eps, a2, B, N, K, D, stream);
        if (rc != SSAM_OK) return rc;
        GemmRowMap none = { nullptr, 1, 0, 1 };
        rc = ssam_linear_impl(a2, w1, b1, hid, B * K, Dm, D, GemmLd{ D, D, Dm }, packed, SSAM_EPI_BIAS_GELU, none, 0, split, GEMM_SPLIT_WS_BYTES, st);
    }
    if (rc != SSAM_OK) return rc;
    GemmRowMap scatter = { keep_idx, K, K, N };
    return ssam_linear_impl(hid, w2, b2, x, B * K, D, Dm, GemmLd{ Dm, Dm, D }, packed, SSAM_EPI_BIAS_SCATTER_ADD, scatter, 0,
                            split, GEMM_SPLIT_WS_BYTES, st);
}

extern "C" int ssam_routed_mlp(void *x, const int32_t *keep_idx, const float *ln_g, const float *ln_b, float eps,
                               const void *w1, const float *b1, const void *w2, const float *b2,
                               int B, int N, int D, int Dm, int K,
                               void *workspace, size_t workspace_bytes, void *stream)
{
    return routed_mlp_impl(x, keep_idx, ln_g, ln_b, eps, w1, b1, w2, b2, false, B, N, D, Dm, K, workspace, workspace_bytes, stream);
}

extern "C" int ssam_routed_mlp_packed(void *x, const int32_t *keep_idx, const float *ln_g, const float *ln_b, float eps,
                                      const void *w1p, const float *b1, const void *w2p, const float *b2,
                                      int B, int N, int D, int Dm, int K,
                                      void *workspace, size_t workspace_bytes, void *stream)
{
    return routed_mlp_impl(x, keep_idx, ln_g, ln_b, eps, w1p, b1, w2p, b2, true, B, N, D, Dm, K, workspace, workspace_bytes, stream);
}

extern "C" int ssam_routed_mlp_folded(void *x, const int32_t *keep_idx, float eps,
                                      const void *w1fp, const float *colsum1, const float *b1f, const void *w2p, const float *b2,
                                      int B, int N, int D, int Dm, int K,
                                      void *workspace, size_t workspace_bytes, void *stream)
{
    if (!colsum1) return SSAM_EINVAL;
    return routed_mlp_impl(x, keep_idx, nullptr, nullptr, eps, w1fp, b1f, w2p, b2, true, B, N, D, Dm, K, workspace, workspace_bytes, stream, colsum1);
}

// everything but the padding tables, which sit behind it (so that no step of either half overwrites them
// and a stack of blocks can build them once)
static size_t attn_half_bytes(const ssam_block_cfg *cfg, const BlockGeom &g)
{
    size_t rows = (size_t)cfg->B * g.Nout;
    return align256(rows * cfg->D * 2) + align256(rows * 3 * cfg->D * 2) + GEMM_SPLIT_WS_BYTES;
}

static size_t block_core_bytes(const ssam_block_cfg *cfg, const BlockGeom &g)
{
    // the two halves do not share memory: the padding slots of the qkv tensor can then keep their contents from
    // block to block (see fold_kv_bias)
    return attn_half_bytes(cfg, g) + mlp_ws_bytes(cfg->B, cfg->K, cfg->D, cfg->Dm);
}

extern "C" size_t ssam_encoder_block_workspace_bytes(const ssam_block_cfg *cfg)
{
    BlockGeom g;
    if (!block_geom(cfg, g)) return 0;
    return block_core_bytes(cfg, g) + block_tables_bytes(cfg->B, g);
}

// tables: this block's block_tables_bytes region; tables_ready: a stack has built it already
static int encoder_block_impl(void *x, const ssam_block_weights *w, const ssam_block_cfg *cfg,
                              const int32_t *gather_table, const int32_t *sigma, const int32_t *keep_idx,
                              void *workspace, size_t workspace_bytes, void **qkv_events, unsigned char *tables,
                              bool tables_ready, bool *pad_rows_zero, void *stream)
{
    BlockGeom g;
    if (!x || !w || !gather_table || !sigma || !keep_idx || !workspace || !block_geom(cfg, g)) return SSAM_EINVAL;
    if (!(cfg->r > 0.0) || cfg->r > 1.0) return SSAM_EINVAL;
    if (!ssam_aligned16(workspace) || !ssam_aligned16(x)) return SSAM_EINVAL;
    if (cfg->D % 128 != 0 || cfg->Dm % 128 != 0) return SSAM_EUNSUPPORTED;
    if (!tables) {
        if (workspace_bytes < ssam_encoder_block_workspace_bytes(cfg)) return SSAM_EWORKSPACE;
        tables = (unsigned char *)workspace + block_core_bytes(cfg, g);
    }
    const int B = cfg->B, D = cfg->D;
    const int rows = B * g.Nout;                               // slots of the scan-order layout (with padding)
    const bool padded = g.Nout != g.N;
    const int crows = B * g.N;                                 // rows the dense contractions multiply (real tokens)
    unsigned char *ws = (unsigned char *)workspace;
    void *u = ws;                                             // LN1(x) in scan order; later the attention output
    void *qkv = ws + align256((size_t)rows * D * 2);
    unsigned char *split = ws + align256((size_t)rows * D * 2) + align256((size_t)rows * 3 * D * 2);   // K-split scratch of the left-over launches
    hipStream_t st = (hipStream_t)stream;
    const int per_image = cfg->content_order != 0;             // tables carry a leading [B] dimension
    const bf16 *qp = (const bf16 *)qkv;
    const bool packed = w->packed != 0;
    GemmRowMap none = { nullptr, 1, 0, 1 };
    int rc;
    const bool fold = w->fold_ln1 != 0;
    const bool kv_shift = w->fold_kv_bias != 0;
    if (fold) {
        if (!packed || !w->qkv_colsum || !w->bqkv_folded) return SSAM_EINVAL;
        if (crows % 128 != 0 || (3 * D) % 256 != 0) return SSAM_EUNSUPPORTED;
    }
    if (kv_shift && (!fold || !w->bproj_folded)) return SSAM_EINVAL;
    const float *bproj = kv_shift ? w->bproj_folded : w->bproj;
    if (!tables_ready) {
        rc = build_block_tables(cfg, g, gather_table, tables, st);
        if (rc != SSAM_OK) return rc;
    }
    if (fold) {
        // LN1 folded into the qkv contraction: only the statistics of every token are taken here (parked at the
        // start of u, which nothing else uses before attention writes its output there); the contraction reads
        // the tokens where they lie and stores every row to its scan-order slot
        float *stats = (float *)u;
        rc = ssam_ln_stats(x, stats, crows, D, cfg->eps, stream);
        if (rc != SSAM_OK) return rc;
        if (qkv_events && qkv_events[0] && hipEventRecord((hipEvent_t)qkv_events[0], st) != hipSuccess) return SSAM_EHIP;
        GemmRowMap to_slot = { slot_of_table(tables, B, g), g.N, per_image ? g.N : 0, g.Nout };
        rc = ssam_linear_ln_impl(x, stats, w->wqkv, w->qkv_colsum, w->bqkv_folded, qkv, crows, 3 * D, D, GemmLd{ D, D, 3 * D }, to_slot, st);
        if (rc != SSAM_OK) return rc;
    }

    if (!padded) {
        if (pad_rows_zero) *pad_rows_zero = false;              // this block's qkv tensor lies over the windowed blocks' one
        if (!fold) {
            rc = ssam_ln_gather(x, gather_table, per_image ? g.Nout : 0, w->ln1_g, w->ln1_b, cfg->eps, u, B, g.N, g.Nout, D, stream);
            if (rc != SSAM_OK) return rc;
            if (qkv_events && qkv_events[0] && hipEventRecord((hipEvent_t)qkv_events[0], st) != hipSuccess) return SSAM_EHIP;
            rc = ssam_linear_impl(u, w->wqkv, w->bqkv, qkv, rows, 3 * D, D, GemmLd{ D, D, 3 * D }, packed, SSAM_EPI_BIAS, none, 0, split, GEMM_SPLIT_WS_BYTES, st);
            if (rc != SSAM_OK) return rc;
        }
        if (qkv_events && qkv_events[1] && hipEventRecord((hipEvent_t)qkv_events[1], st) != hipSuccess) return SSAM_EHIP;
        rc = ssam_sparse_attention(qp, qp + D, qp + 2 * D, 3L * D, w->rel_h, w->rel_w, sigma, per_image ? g.S : 0, u, nullptr,
                                   B * g.nW, g.S, g.w, cfg->heads, g.d, cfg->mask_block, cfg->r,
                                   1.0f / sqrtf((float)g.d), stream);
        if (rc != SSAM_OK) return rc;
        GemmRowMap back = { gather_table, g.Nout, per_image ? g.Nout : 0, g.N };
        rc = ssam_linear_impl(u, w->wproj, bproj, x, rows, D, D, GemmLd{ D, D, D }, packed, SSAM_EPI_BIAS_SCATTER_ADD, back, 0, split, GEMM_SPLIT_WS_BYTES, st);
        if (rc != SSAM_OK) return rc;
    } else {
        // Windows with padding: the padding slots are zero rows after LN1, so their qkv rows are the bias and
        // their attention outputs are dropped.  LN1 gathers the N real tokens of every image into a compact
        // [B*N][D] matrix in scan order, the qkv contraction runs on those rows and scatters them to their
        // slots, the padding slots are filled with the bias, attention writes only the real queries (compact
        // again), and the proj contraction scatters them back to spatial order.
        const PadTables pt = carve_pad_tables(tables, B, g);
        if (!fold) {
            rc = ssam_ln_gather(x, pt.real_spatial, g.N, w->ln1_g, w->ln1_b, cfg->eps, u, B, g.N, g.N, D, stream);
            if (rc != SSAM_OK) return rc;
            if (qkv_events && qkv_events[0] && hipEventRecord((hipEvent_t)qkv_events[0], st) != hipSuccess) return SSAM_EHIP;
            GemmRowMap to_slot = { pt.real_slot, g.N, g.N, g.Nout };
            rc = ssam_linear_impl(u, w->wqkv, w->bqkv, qkv, crows, 3 * D, D, GemmLd{ D, D, 3 * D }, packed, SSAM_EPI_BIAS_SCATTER, to_slot, 0, split, GEMM_SPLIT_WS_BYTES, st);
            if (rc != SSAM_OK) return rc;
        }
        // the padding slots hold the qkv of a zero row: the bias, or, with the key and value biases taken out of
        // the contraction, zeros in the columns attention reads (k, v), which then need writing only when something
        // else has used the memory since
        if (!kv_shift) {
            rc = ssam_fill_bias_rows(qkv, 3L * D, w->bqkv, 3 * D, pt.pad_slot, g.Nout - g.N, g.Nout, B, st);
            if (rc != SSAM_OK) return rc;
            if (pad_rows_zero) *pad_rows_zero = false;
        } else if (!pad_rows_zero || !*pad_rows_zero) {
            rc = ssam_fill_bias_rows(qkv, 3L * D, nullptr, 3 * D, pt.pad_slot, g.Nout - g.N, g.Nout, B, st);
            if (rc != SSAM_OK) return rc;
            if (pad_rows_zero) *pad_rows_zero = true;
        }
        if (qkv_events && qkv_events[1] && hipEventRecord((hipEvent_t)qkv_events[1], st) != hipSuccess) return SSAM_EHIP;
        rc = ssam_sparse_attention(qp, qp + D, qp + 2 * D, 3L * D, w->rel_h, w->rel_w, sigma, per_image ? g.S : 0, u, pt.slot_row,
                                   B * g.nW, g.S, g.w, cfg->heads, g.d, cfg->mask_block, cfg->r,
                                   1.0f / sqrtf((float)g.d), stream);
        if (rc != SSAM_OK) return rc;
        GemmRowMap back = { pt.real_spatial, g.N, g.N, g.N };
        rc = ssam_linear_impl(u, w->wproj, bproj, x, crows, D, D, GemmLd{ D, D, D }, packed, SSAM_EPI_BIAS_SCATTER_ADD, back, 0, split, GEMM_SPLIT_WS_BYTES, st);
        if (rc != SSAM_OK) return rc;
    }
    const size_t attn_bytes = attn_half_bytes(cfg, g);
    if (w->fold_ln2 != 0) {
        if (!packed || !w->fc1_colsum || !w->b1_folded) return SSAM_EINVAL;
        return routed_mlp_impl(x, keep_idx, nullptr, nullptr, cfg->eps, w->w1, w->b1_folded, w->w2, w->b2, true,
                               B, g.N, D, cfg->Dm, cfg->K, ws + attn_bytes, mlp_ws_bytes(B, cfg->K, D, cfg->Dm), stream, w->fc1_colsum);
    }
    return routed_mlp_impl(x, keep_idx, w->ln2_g, w->ln2_b, cfg->eps, w->w1, w->b1, w->w2, w->b2, packed,
                           B, g.N, D, cfg->Dm, cfg->K, ws + attn_bytes, mlp_ws_bytes(B, cfg->K, D, cfg->Dm), stream);
}

extern "C" int ssam_encoder_block(void *x, const ssam_block_weights *w, const ssam_block_cfg *cfg,
                                  const int32_t *gather_table, const int32_t *sigma, const int32_t *keep_idx,
                                  void *workspace, size_t workspace_bytes, void *stream)
{
    return encoder_block_impl(x, w, cfg, gather_table, sigma, keep_idx, workspace, workspace_bytes, nullptr, nullptr, false, nullptr, stream);
}

extern "C" size_t ssam_encoder_workspace_bytes(const ssam_block_cfg *cfg_local, const ssam_block_cfg *cfg_global)
{
    // what either kind of block writes, then the tables of the windowed blocks, then those of the global blocks
    BlockGeom gl, gg;
    const bool l = cfg_local && block_geom(cfg_local, gl), g = cfg_global && block_geom(cfg_global, gg);
    if ((cfg_local && !l) || (cfg_global && !g)) return 0;
    size_t core = 0, tables = 0;
    if (l) { core = block_core_bytes(cfg_local, gl); tables += block_tables_bytes(cfg_local->B, gl); }
    if (g) { size_t c = block_core_bytes(cfg_global, gg); core = c > core ? c : core; tables += block_tables_bytes(cfg_global->B, gg); }
    const ssam_block_cfg *c = cfg_local ? cfg_local : cfg_global;
    size_t s = c ? align256(ssam_score_tokens_workspace_bytes(c->B, c->g, c->g)) : 0;
    return (core > s ? core : s) + tables;
}

extern "C" int ssam_encoder_forward(void *x, const ssam_block_weights *weights, const uint8_t *is_global, int n_blocks,
                                    const ssam_block_cfg *cfg_local, const ssam_block_cfg *cfg_global,
                                    int32_t *window_table, int32_t *sigma_window,
                                    int32_t *global_table, int32_t *sigma_global,
                                    float *scores, int32_t *keep_idx,
                                    void *workspace, size_t workspace_bytes, void **qkv_events, void *stream)
{
    if (!x || !weights || !is_global || n_blocks <= 0 || !scores || !keep_idx || !workspace) return SSAM_EINVAL;
    bool any_local = false, any_global = false;
    for (int i = 0; i < n_blocks; ++i) (is_global[i] ? any_global : any_local) = true;
    if ((any_local && (!cfg_local || !window_table || !sigma_window)) ||
        (any_global && (!cfg_global || !global_table || !sigma_global)))
        return SSAM_EINVAL;
    const ssam_block_cfg *c0 = any_local ? cfg_local : cfg_global;
    if (any_local && any_global &&
        (cfg_local->B != cfg_global->B || cfg_local->g != cfg_global->g || cfg_local->D != cfg_global->D ||
         cfg_local->K != cfg_global->K))
        return SSAM_EINVAL;
    if (workspace_bytes < ssam_encoder_workspace_bytes(any_local ? cfg_local : nullptr, any_global ? cfg_global : nullptr))
        return SSAM_EWORKSPACE;
    if (any_local && any_global && (cfg_local->content_order != 0) != (cfg_global->content_order != 0)) return SSAM_EINVAL;
    int rc = ssam_score_tokens(x, scores, c0->B, c0->g, c0->g, c0->D, workspace, workspace_bytes, stream);
    if (rc != SSAM_OK) return rc;
    if (c0->content_order != 0) {                 // Sec. 4.1: the content-aware order is taken once, from these scores
        const int G = c0->stripe;
        if (G <= 0) return SSAM_EINVAL;
        if (any_local) {
            rc = ssam_build_content_tables(scores, c0->B, c0->g, cfg_local->ws, G, window_table, sigma_window, stream);
            if (rc != SSAM_OK) return rc;
        }
        if (any_global) {
            rc = ssam_build_content_tables(scores, c0->B, c0->g, cfg_global->ws, G, global_table, sigma_global, stream);
            if (rc != SSAM_OK) return rc;
        }
    }
    rc = ssam_select_tokens(scores, keep_idx, c0->B, c0->g * c0->g, c0->K, stream);
    if (rc != SSAM_OK) return rc;
    // the tables of either kind of block are the same for every block of that kind: built once, behind everything
    // the blocks write
    BlockGeom gl, gg;
    size_t core = 0;
    if (any_local) { if (!block_geom(cfg_local, gl)) return SSAM_EINVAL; core = block_core_bytes(cfg_local, gl); }
    if (any_global) {
        if (!block_geom(cfg_global, gg)) return SSAM_EINVAL;
        size_t c = block_core_bytes(cfg_global, gg);
        core = c > core ? c : core;
    }
    {
        size_t sc = align256(ssam_score_tokens_workspace_bytes(c0->B, c0->g, c0->g));
        core = core > sc ? core : sc;
    }
    unsigned char *tables_local = (unsigned char *)workspace + core;
    unsigned char *tables_global = tables_local + (any_local ? block_tables_bytes(cfg_local->B, gl) : 0);
    if (any_local) {
        rc = build_block_tables(cfg_local, gl, window_table, tables_local, (hipStream_t)stream);
        if (rc != SSAM_OK) return rc;
    }
    if (any_global) {
        rc = build_block_tables(cfg_global, gg, global_table, tables_global, (hipStream_t)stream);
        if (rc != SSAM_OK) return rc;
    }
    bool pad_rows_zero = false;                 // the padding slots of the windowed blocks' qkv tensor hold zeros
    for (int i = 0; i < n_blocks; ++i) {
        void **ev = qkv_events ? qkv_events + 2 * i : nullptr;
        rc = is_global[i]
                 ? encoder_block_impl(x, &weights[i], cfg_global, global_table, sigma_global, keep_idx, workspace, core, ev, tables_global, true, &pad_rows_zero, stream)
                 : encoder_block_impl(x, &weights[i], cfg_local, window_table, sigma_window, keep_idx, workspace, core, ev, tables_local, true, &pad_rows_zero, stream);
        if (rc != SSAM_OK) return rc;
    }
    return SSAM_OK;
}
