/*
 * ssam.h -- C ABI of the MI355X (gfx950) structured-sparse SAM ViT encoder block
 * of "SparseSAM" (arXiv 2605.17633): Stripe-Sort Attention (Sec. 4.1, App. A.1
 * Alg. 1) and the Residual-Consistency MLP (Sec. 4.2).
 *
 * Conventions (all entry points)
 *   - Return value: SSAM_OK (0) or a negative ssam_status.  Nothing throws or
 *     aborts.  A failed argument check enqueues nothing.
 *   - Ownership: the caller owns every buffer, including workspaces and index
 *     tables.  Unless a call's comment says otherwise the library allocates no
 *     device memory, keeps no global mutable state and never synchronises: it
 *     only enqueues kernels on the caller's stream.
 *   - "dev" = device (HBM) pointer, "host" = host pointer.  `stream` is a
 *     hipStream_t passed as void* (NULL = the default stream).
 *   - Tensors are dense, row-major.  Activations and Linear weights are bf16
 *     (16-bit, upper half of an IEEE fp32); LayerNorm parameters, Linear biases
 *     and token scores are fp32; indices are int32.  Device pointers must be
 *     16-byte aligned, feature widths multiples of 8.
 *   - Linear weights use the [out, in] layout (y = x W^T + b).
 *   - bf16 arithmetic: products are exact, sums are fp32, every tensor written
 *     to memory is rounded to bf16 (nearest even) once.
 */
#ifndef SSAM_H
#define SSAM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum ssam_status {
    SSAM_OK = 0,
    SSAM_EINVAL = -1,       /* null / misaligned pointer, size or density out of range */
    SSAM_EUNSUPPORTED = -2, /* a shape the kernels are not built for                   */
    SSAM_EWORKSPACE = -3,   /* workspace smaller than the matching *_workspace_bytes   */
    SSAM_EHIP = -4          /* a HIP runtime call (launch, attribute) failed           */
} ssam_status;

/* Static string for a status code. */
const char *ssam_status_string(int status);

/* ------------------------------------------------------------------------- */
/* Integer layout layer (one-time; Sec. 4.1 "precomputed once")              */
/* ------------------------------------------------------------------------- */

/* Stripe-Sort scan order of a gh x gw token grid (Fig. 2 caption; Sec. 4.1).
 * pi = Z-order (Morton) traversal: cells ranked by the bit-interleaved code in
 * which the column supplies the even bits and the row the odd bits.
 * perm = sigma = flatten(T^T), T[t][g] = pi[t*G+g]  (G = 1: perm = pi).
 * perm[p] = row-major cell index at scan position p; inv[perm[p]] = p.
 * perm, inv: host, gh*gw int32 each; inv may be NULL.
 * SSAM_EINVAL: non-positive sizes, G < 1, gh*gw not divisible by G. */
int ssam_build_perm(int gh, int gw, int G, int32_t *perm, int32_t *inv);

/* The same table computed by a HIP kernel straight into device memory
 * (perm_dev, inv_dev: dev, gh*gw int32; inv_dev may be NULL).  gh, gw <= 1024. */
int ssam_build_perm_device(int gh, int gw, int G, int32_t *perm_dev, int32_t *inv_dev, void *stream);

/* Window-major gather table (App. A.1 "window-major -> spatial perms"): the
 * g x g grid is padded to nws*ws per side, nws = ceil(g/ws), and cut into
 * ws x ws windows; inside a window tokens follow ssam_build_perm(ws, ws, G).
 * table[(wr*nws+wc)*ws*ws + p] = row*g+col of the token at scan position p of
 * window (wr,wc), or -1 for a padding cell.  table: host, nws*nws*ws*ws int32. */
int ssam_build_window_table(int g, int ws, int G, int32_t *table);

/* A-shape block mask of Alg. 1 in CSR form.  T = ceil(S/mask_block) tiles per
 * side, n_pre = floor(r*T) (double, +1e-6 guard, clamped to [0,T]); row tile i
 * lists column tiles 0..n_pre-1 and, if i >= n_pre, its diagonal tile i.
 * row_ptr: host, T+1 int32.  col_idx: host, room for T*T int32 (ascending in
 * each row).  n_pre: host, optional.  SSAM_EINVAL unless 0 < r <= 1. */
int ssam_build_block_mask(int S, int mask_block, double r, int32_t *row_ptr, int32_t *col_idx, int *n_pre);

/* Keep count of the routed MLP (Sec. 4.2): clamp(floor(rho*N + 1e-6), 1, N);
 * negative status on bad arguments. */
int ssam_keep_count(int N, double rho);

/* ------------------------------------------------------------------------- */
/* HBM-bound movers                                                          */
/* ------------------------------------------------------------------------- */

/* Row gather (Sec. 4.1: reorder tokens by the scan order):
 * y[b][p][:] = idx[p] >= 0 ? x[b][idx[p]][:] : 0.
 * x dev bf16 [B][Nin][D]; idx dev int32 [Nout], each < Nin; y dev bf16 [B][Nout][D]. */
int ssam_permute(const void *x, const int32_t *idx, void *y, int B, int Nin, int Nout, int D, void *stream);

/* Inverse scatter: x[b][idx[p]][:] = y[b][p][:] (+ residual[b][idx[p]][:] when
 * residual != NULL) for idx[p] >= 0.  idx must not repeat a row.  Rows of x no
 * idx names are left untouched.  residual may alias x. */
int ssam_unpermute(const void *y, const int32_t *idx, void *x, const void *residual,
                   int B, int Nx, int Ny, int D, void *stream);

/* Fused pre-LayerNorm + gather (block input path; also gathers the keep-set
 * for the routed MLP): y[b][p][:] = LN(x[b][idx[b*idx_batch_stride+p]][:]) with
 * biased variance, fp32 statistics; idx < 0 gives a zero row.
 * idx_batch_stride = 0 shares one table over the batch.  gamma, beta dev fp32 [D]. D <= 2048. */
int ssam_ln_gather(const void *x, const int32_t *idx, int idx_batch_stride,
                   const float *gamma, const float *beta, float eps, void *y,
                   int B, int Nin, int Nout, int D, void *stream);

/* Content-aware Stripe-Sort order (Sec. 4.1, "Gradient-Based Ordering" and
 * "Stripe-Sort Permutation"): per image and per attention group (a ws x ws
 * window of the grid padded to a multiple of ws, or the whole grid when ws = 0)
 * the group's cells are ranked by score descending (equal scores: lower cell
 * first; NaN as -inf, -0 as +0; padding cells last), pi = that ranking,
 * sigma[t'*(S/G) + t] = pi[t*G + t'].  scores dev fp32 [B][g*g] (Eq. 1).
 * Outputs, dev int32, S = w*w, nW groups per image:
 *   gather_table [B][nW*S]: scan slot -> spatial index row*g+col, -1 = padding
 *   sigma        [B*nW][S]: scan position -> cell of the group (row*w+col)
 * S % G == 0 (else SSAM_EINVAL), w <= 128 (else SSAM_EUNSUPPORTED). */
int ssam_build_content_tables(const float *scores, int B, int g, int ws, int G,
                              int32_t *gather_table, int32_t *sigma, void *stream);

/* ------------------------------------------------------------------------- */
/* Dense contraction (the block's qkv / proj / fc1 / fc2 layers)             */
/* ------------------------------------------------------------------------- */

typedef enum ssam_epilogue {
    SSAM_EPI_BIAS = 0,        /* C = A W^T + b                                         */
    SSAM_EPI_BIAS_GELU = 1,   /* C = gelu_erf(A W^T + b)                               */
    SSAM_EPI_BIAS_SCATTER_ADD = 2, /* C[dst(m)] += A W^T + b, dst from a row map (below) */
    SSAM_EPI_BIAS_SCATTER = 3     /* C[dst(m)]  = A W^T + b, same row map                */
} ssam_epilogue;

/* C = epilogue(A W^T + bias).  A dev bf16 [M][K]; W dev bf16 [N][K]; bias dev
 * fp32 [N]; C dev bf16.  N % 8 == 0 and K % 8 == 0 (else SSAM_EUNSUPPORTED;
 * multiples of 128 / 64 are the fast case: a ragged last tile column or K slab
 * is computed on clamped / zero operands and not stored).
 * SSAM_EPI_BIAS_SCATTER_ADD: row m = b*rows_per_batch + p of the product is
 * added into row b*dst_rows_per_batch + row_map[b*map_batch_stride + p] of C
 * (skipped where the map is negative); C holds the residual stream and is
 * updated in place: new = bf16(old + acc + bias).  The map must not repeat a
 * row within a batch item.  SSAM_EPI_BIAS_SCATTER stores bf16(acc + bias) into
 * the mapped row instead of adding.  Other epilogues ignore the map arguments
 * and write C [M][N]. */
int ssam_linear(const void *A, const void *W, const float *bias, void *C, int M, int N, int K,
                int epilogue, const int32_t *row_map, int rows_per_batch, int map_batch_stride,
                int dst_rows_per_batch, void *stream);

/* The same with the workgroup tile forced (tuning and tests): tile = 0 picks
 * automatically, 1 = 256x256 with 8 waves, 2 = 256x128
 * (row-major weights only), 3 = 128x128, 4 = 128x256 with 4 waves.
 * With any tile, when the tiles fill at least one round of workgroups and the
 * left-over is under half a round, the left-over tiles run as half- or
 * quarter-size tiles (in the same launch or in a second one); results do not depend on the tile choice
 * beyond fp32 summation order (which is the same: K is never split). */
int ssam_linear_tiled(const void *A, const void *W, const float *bias, void *C, int M, int N, int K,
                      int epilogue, const int32_t *row_map, int rows_per_batch, int map_batch_stride,
                      int dst_rows_per_batch, int tile, void *stream);

/* The general form: A, W and C with their own row strides lda >= K, ldw >= K,
 * ldc >= N in elements (multiples of 8, else SSAM_EINVAL; for the scatter
 * epilogue ldc is the row stride of the destination), and an optional device
 * workspace (NULL/0 for none; 16-byte aligned; ssam_linear_workspace_bytes()
 * is always enough, smaller is allowed).  With a workspace, a left-over launch
 * of few tiles (K >= 1024) is cut along K as well: partial fp32
 * tiles go to the workspace and are added in a fixed order, so results are
 * reproducible; they can differ from the no-workspace result in the last bit
 * of the fp32 sum.  The workspace is scratch: contents undefined afterwards,
 * concurrent calls need separate workspaces. */
size_t ssam_linear_workspace_bytes(void);
int ssam_linear_ld(const void *A, int lda, const void *W, int ldw, int w_packed, const float *bias, void *C, int ldc,
                   int M, int N, int K, int epilogue, const int32_t *row_map, int rows_per_batch,
                   int map_batch_stride, int dst_rows_per_batch, int tile,
                   void *workspace, size_t workspace_bytes, void *stream);

/* Weights in MFMA fragment order.  A weight matrix is static, so it can be laid
 * out once the way the matrix cores consume it: Wp[N/16][K/32][64][8] bf16 with
 *   Wp[nb][s][16*q + l][e] = W[16*nb + l][32*s + 8*q + e],   l < 16, q < 4, e < 8,
 * i.e. the 1 KB operand-B fragment (of the 16x16x32 MFMA) of every (16 output
 * channels, 32 input channels) cell is contiguous.  ssam_linear_ld with w_packed != 0 (then ldw is
 * ignored) loads such fragments straight into registers and stages only A in
 * LDS, which halves its LDS traffic; with the same tile (forced) the results are
 * bit-identical to the row-major form; the automatic choice may take another
 * tile for packed weights (the 128x256 one), and then the few left-over tiles
 * whose K range is cut can differ in fp32 summation order.  W dev bf16 [N][K] (row stride ldw), Wp dev bf16 N*K elements, N % 16 ==
 * 0 and K % 32 == 0 (else SSAM_EUNSUPPORTED; ssam_linear_ld takes packed
 * weights only for N % 128 == 0 and K % 64 == 0); W and Wp must not overlap.  Tile
 * 2 (256x128) has no packed form (SSAM_EUNSUPPORTED when forced). */
int ssam_pack_weight(const void *W, int ldw, void *Wp, int N, int K, void *stream);

/* LayerNorm folded into the Linear that follows it (SAM's pre-LN block: qkv =
 * Linear(LN1(x)), the input of Stripe-Sort attention, Sec. 4.1).  With
 * mean_m, rstd_m the statistics of row m,
 *   Linear(LN(x))[m][n] = rstd_m * (sum_k x[m][k] Wf[n][k] - mean_m * colsum[n]) + bias_f[n],
 *   Wf[n][k] = bf16(W[n][k] * gamma[k]),  colsum[n] = sum_k Wf[n][k] (of the stored
 *   values, fp32),  bias_f[n] = bias[n] + sum_k beta[k] W[n][k],
 * so the normalised rows are never written: the statistics are one read of x
 * and the contraction reads x itself.
 * ssam_ln_stats: x dev bf16 [rows][D] contiguous -> stats dev fp32 [rows][2] =
 *   { rstd, -rstd * mean } (biased variance, two-pass fp32); D % 8 == 0, D <= 2048.
 * ssam_fold_ln_weight: W dev bf16 [N][K] (row stride ldw), bias [N], gamma, beta [K]
 *   dev fp32 -> Wf dev bf16 [N][K] contiguous (give it to ssam_pack_weight), colsum,
 *   bias_f dev fp32 [N].  One-time weight preparation.
 * ssam_linear_ln: C[dst(m)][:] = the formula above for row m of x (dev bf16, row
 *   stride ldx), Wfp = ssam_pack_weight(Wf); dst(m) as for SSAM_EPI_BIAS_SCATTER
 *   (row_map required; entries outside [0, dst_rows_per_batch) skip the row).
 *   M % 128 == 0, N % 256 == 0, K % 64 == 0 (else SSAM_EUNSUPPORTED). */
int ssam_ln_stats(const void *x, float *stats, long rows, int D, float eps, void *stream);
int ssam_fold_ln_weight(const void *W, int ldw, const float *bias, const float *gamma, const float *beta,
                        void *Wf, float *colsum, float *bias_f, int N, int K, void *stream);
/* Key and value biases taken out of the qkv contraction of a block (Alg. 1: the
 * softmax runs over the keys of a query, so a term of the logit that is the same
 * for every key, q.b_k, cancels; the probabilities of a query sum to one, so
 * sum_j p_j (v_j + b_v) = sum_j p_j v_j + b_v, which the output projection turns
 * into a constant):
 *   bias_out[n] = bias_in[n] - (n >= D ? bqkv[n] : 0)          n < 3D
 *   bproj_out[j] = bproj[j] + sum_c wproj[j][c] * bqkv[2D + c]   j < D
 * bias_in: the bias the contraction would use (bqkv itself, or the bias_f of
 * ssam_fold_ln_weight); wproj dev bf16 [D][D] row-major (not packed); all other
 * arguments dev fp32.  The rows of LN1-zero padding tokens then have k = v = 0. */
int ssam_fold_kv_bias(const float *bias_in, const float *bqkv, const void *wproj, const float *bproj,
                      float *bias_out, float *bproj_out, int D, void *stream);
int ssam_linear_ln(const void *x, int ldx, const float *stats, const void *Wfp, const float *colsum,
                   const float *bias_f, void *C, int ldc, int M, int N, int K,
                   const int32_t *row_map, int rows_per_batch, int map_batch_stride, int dst_rows_per_batch,
                   void *stream);

/* ------------------------------------------------------------------------- */
/* Stripe-Sort attention (App. A.1, Alg. 1)                                  */
/* ------------------------------------------------------------------------- */

/* For every group g (a window, or a whole image for global blocks) and head:
 *   O = softmax_over_active_tiles(scale * Q K^T + B) V
 * with tokens already in scan order.  Active key tiles of query tile i:
 * {0..floor(r*T)-1} U {i}, tiles of mask_block tokens, T = ceil(S/mask_block).
 * B[p][p'] = q_p . rel_h[row(p)-row(p')+w-1] + q_p . rel_w[col(p)-col(p')+w-1]
 * (unscaled q), (row, col) = divmod(sigma[p], w): sigma maps scan position ->
 * spatial cell of the w x w grid, S = w*w.
 *   q, k, v  dev bf16; element (g, p, head, c) at ptr[(g*S+p)*row_stride + head*d + c]
 *            (a packed [groups][S][3][h][d] buffer: row_stride = 3*h*d, k = q + h*d, v = q + 2*h*d)
 *   rel_h, rel_w  dev bf16 [(2w-1)][d]
 *   sigma    dev int32: sigma_group_stride = 0: one table [S] shared by all groups (the
 *            position-only order); otherwise group g reads sigma + g*sigma_group_stride
 *            (>= S; the per-image, per-window tables of ssam_build_content_tables)
 *   out      dev bf16, rows of h*d: query p of group g is written to row g*S+p, or, with
 *            out_rows dev int32 [groups*S] != NULL, to row out_rows[g*S+p] (negative: not
 *            written; used to drop the padding queries of windows and compact the rest)
 * Built for d in {16, 32, 64, 80} (SAM uses 64 and 80), mask_block = 32 with
 * S <= 224 (windows) and mask_block = 128 with S <= 16384 (global); otherwise
 * SSAM_EUNSUPPORTED. */
int ssam_sparse_attention(const void *q, const void *k, const void *v, long row_stride,
                          const void *rel_h, const void *rel_w, const int32_t *sigma,
                          long sigma_group_stride, void *out, const int32_t *out_rows,
                          int groups, int S, int w, int h, int d, int mask_block, double r,
                          float scale, void *stream);

/* ------------------------------------------------------------------------- */
/* Residual-Consistency MLP (Sec. 4.2)                                       */
/* ------------------------------------------------------------------------- */

/* Token scores of Eq. 1: Sobel gradient magnitude (zero padding) of the map
 * summed over channels.  x dev bf16 [B][gh][gw][D]; scores dev fp32 [B][gh*gw];
 * workspace dev, >= ssam_score_tokens_workspace_bytes. */
size_t ssam_score_tokens_workspace_bytes(int B, int gh, int gw);
int ssam_score_tokens(const void *x, float *scores, int B, int gh, int gw, int D,
                      void *workspace, size_t workspace_bytes, void *stream);

/* ssam_score_tokens for callers that cannot allocate device memory or hand over a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same kernels, same result bit for bit;
 * the channel-sum map (4 bytes per token) is held in a device array that is part of the library (1 MiB on every
 * GPU the library is loaded on, until the process ends), so at most SSAM_SCORE_TOKENS_STATIC_MAX_TOKENS =
 * B*gh*gw tokens per call; more returns SSAM_EWORKSPACE and enqueues nothing.  Calls no allocator.  The first
 * call on a device looks the array's address up (a host-side query: make that call outside any capture).  All
 * calls on one GPU share the array: calls that overlap there (different streams or threads) race; calls on one
 * stream do not. */
#define SSAM_SCORE_TOKENS_STATIC_MAX_TOKENS (1 << 18)
int ssam_score_tokens_static(const void *x, float *scores, int B, int gh, int gw, int D, void *stream);

/* Keep-set: per batch item the K highest scores, ties to the lower index
 * (-0.0 == +0.0; NaN ranks as -inf), written in ascending index order.
 * scores dev fp32 [B][N]; keep_idx dev int32 [B][K]; 1 <= K <= N <= 65536. */
int ssam_select_tokens(const float *scores, int32_t *keep_idx, int B, int N, int K, void *stream);

/* x[b][i] += W2 gelu_erf(W1 LN(x[b][i]) + b1) + b2 for i in keep_idx[b][:];
 * every other row of x is never written (bit-identical).
 * x dev bf16 [B][N][D] in place; keep_idx dev int32 [B][K], distinct per b,
 * in [0,N) (contract; not checked on device).  w1 [Dm][D], w2 [D][Dm] bf16;
 * b1 [Dm], b2 [D], ln_g, ln_b [D] fp32. */
size_t ssam_routed_mlp_workspace_bytes(int B, int K, int D, int Dm);
int ssam_routed_mlp(void *x, const int32_t *keep_idx, const float *ln_g, const float *ln_b, float eps,
                    const void *w1, const float *b1, const void *w2, const float *b2,
                    int B, int N, int D, int Dm, int K,
                    void *workspace, size_t workspace_bytes, void *stream);
/* The same with w1 and w2 in MFMA fragment order (ssam_pack_weight; D and Dm
 * multiples of 128, else SSAM_EUNSUPPORTED): the form the encoder block uses
 * when ssam_block_weights.packed is set. */
int ssam_routed_mlp_packed(void *x, const int32_t *keep_idx, const float *ln_g, const float *ln_b, float eps,
                           const void *w1p, const float *b1, const void *w2p, const float *b2,
                           int B, int N, int D, int Dm, int K,
                           void *workspace, size_t workspace_bytes, void *stream);
/* The same with the gather of the kept tokens and LN2 folded into fc1 (Sec. 4.2:
 * only the kept rows are read, where they lie in the residual stream; the
 * normalised rows are never written): one pass over the kept rows takes their
 * statistics, fc1 reads those rows of x itself and finishes the LayerNorm in its
 * epilogue by the formula given with ssam_fold_ln_weight.  w1fp = packed Wf,
 * colsum1, b1f = the outputs of ssam_fold_ln_weight(w1, b1, ln_g, ln_b); w2p =
 * packed w2.  Same workspace and restrictions as ssam_routed_mlp_packed; an
 * index outside [0,N) skips its row. */
int ssam_routed_mlp_folded(void *x, const int32_t *keep_idx, float eps,
                           const void *w1fp, const float *colsum1, const float *b1f, const void *w2p, const float *b2,
                           int B, int N, int D, int Dm, int K,
                           void *workspace, size_t workspace_bytes, void *stream);

/* ------------------------------------------------------------------------- */
/* Encoder block and stack                                                   */
/* ------------------------------------------------------------------------- */

typedef struct ssam_block_weights {     /* every pointer: dev */
    const float *ln1_g, *ln1_b;         /* [D] fp32                                  */
    const void *wqkv;                   /* bf16 [3D][D], out channel = which*D+head*d+c */
    const float *bqkv;                  /* [3D] fp32                                 */
    const void *rel_h, *rel_w;          /* bf16 [(2w-1)][d], w = ws (local) or g (global) */
    const void *wproj;                  /* bf16 [D][D]                               */
    const float *bproj;                 /* [D] fp32                                  */
    const float *ln2_g, *ln2_b;         /* [D] fp32                                  */
    const void *w1;                     /* bf16 [Dm][D]                              */
    const float *b1;                    /* [Dm] fp32                                 */
    const void *w2;                     /* bf16 [D][Dm]                              */
    const float *b2;                    /* [D] fp32                                  */
    int packed;                         /* != 0: wqkv, wproj, w1, w2 are in the fragment order of ssam_pack_weight */
    int fold_ln1;                       /* != 0 (needs packed != 0): LN1 is folded into the qkv contraction, see
                                           ssam_fold_ln_weight: wqkv is the packed form of its Wf, qkv_colsum and
                                           bqkv_folded are its other outputs; bqkv stays the plain bias (the
                                           padding slots of a window are zero rows AFTER LN1) and ln1_g, ln1_b
                                           are not read.  B*g*g % 128 == 0 and 3D % 256 == 0, else
                                           SSAM_EUNSUPPORTED. */
    const float *qkv_colsum;            /* [3D] fp32 (fold_ln1 only)                 */
    const float *bqkv_folded;           /* [3D] fp32 (fold_ln1 only)                 */
    int fold_kv_bias;                   /* != 0 (needs fold_ln1 != 0): bqkv_folded and bproj_folded are the outputs
                                           of ssam_fold_kv_bias; the padding slots of a window then hold zero keys
                                           and values for every block, so a stack writes them once instead of once
                                           per block. */
    const float *bproj_folded;          /* [D] fp32 (fold_kv_bias only)              */
    int fold_ln2;                       /* != 0 (needs packed != 0): the gather of the kept tokens and LN2 are folded
                                           into fc1 (ssam_routed_mlp_folded): w1 is the packed form of the Wf that
                                           ssam_fold_ln_weight makes from w1, b1, ln2_g, ln2_b; fc1_colsum and
                                           b1_folded are its other outputs; b1, ln2_g, ln2_b are not read. */
    const float *fc1_colsum;            /* [Dm] fp32 (fold_ln2 only)                 */
    const float *b1_folded;             /* [Dm] fp32 (fold_ln2 only)                 */
} ssam_block_weights;

typedef struct ssam_block_cfg {
    int B;            /* images                                                  */
    int g;            /* token grid side (N = g*g)                               */
    int D, heads, Dm; /* width, heads (d = D/heads), MLP hidden width            */
    int ws;           /* window side; 0 = global attention over the whole grid   */
    int mask_block;   /* A-shape tile: 32 for windows, 128 for global            */
    int K;            /* kept tokens per image for the routed MLP                */
    double r;         /* attention density in (0,1]                              */
    float eps;        /* LayerNorm epsilon                                       */
    int content_order;/* 0: position-only order, tables shared by all images;
                         1: content-aware order, per-image tables (see below)    */
    int stripe;       /* G of the stripe interleave when content_order != 0 (the
                         paper's 4 x 4 mosaic: 4); ignored otherwise            */
} ssam_block_cfg;

/* One structured-sparse block, in place on x dev bf16 [B][g][g][D]:
 *   u = LN1(x) gathered into scan order (windows: zero rows for padding)
 *   qkv = u Wqkv^T + b;  o = Stripe-Sort attention;  x += scatter(o Wproj^T + b)
 *   routed MLP over keep_idx.
 * gather_table dev int32: ws > 0: ssam_build_window_table(g, ws, G) (nws*nws*ws*ws);
 *                         ws = 0: ssam_build_perm(g, g, G) (g*g).
 * sigma dev int32 [S]: ssam_build_perm(w, w, G) of one attention group.
 * With cfg->content_order != 0 both tables are the per-image outputs of
 * ssam_build_content_tables: gather_table [B][nW*S], sigma [B*nW][S].
 * keep_idx dev int32 [B][K].  workspace >= ssam_encoder_block_workspace_bytes(cfg). */
size_t ssam_encoder_block_workspace_bytes(const ssam_block_cfg *cfg);
int ssam_encoder_block(void *x, const ssam_block_weights *w, const ssam_block_cfg *cfg,
                       const int32_t *gather_table, const int32_t *sigma, const int32_t *keep_idx,
                       void *workspace, size_t workspace_bytes, void *stream);

/* A stack of blocks on one batch (Sec. 1: one static permutation set and one
 * keep-set, computed once, reused by every layer): scores (Eq. 1) and the
 * keep-set are taken from the input x, then block i runs with cfg_local or,
 * where is_global[i] != 0, cfg_global.  weights, is_global: host arrays of
 * n_blocks entries.  keep_idx dev int32 [B][K] is written and then read;
 * scores dev fp32 [B][N] likewise.  Tables as for ssam_encoder_block; with
 * content_order set in the cfgs (both or neither) the four table arguments are
 * per-image buffers that this call FILLS from the scores (Sec. 4.1: the order is
 * computed once, in the first layer) before the first block reads them.
 * workspace >= ssam_encoder_workspace_bytes(cfg_local, cfg_global).
 * qkv_events: optional instrumentation, host array of 2*n_blocks hipEvent_t
 * (NULL = none; a NULL entry = that block is not timed): events [2i] and [2i+1]
 * are recorded on the stream right before and right after block i's qkv
 * contraction, so that a benchmark can time that kernel inside its own timed
 * region.  A recorded event costs the stream a few microseconds. */
size_t ssam_encoder_workspace_bytes(const ssam_block_cfg *cfg_local, const ssam_block_cfg *cfg_global);
int ssam_encoder_forward(void *x, const ssam_block_weights *weights, const uint8_t *is_global, int n_blocks,
                         const ssam_block_cfg *cfg_local, const ssam_block_cfg *cfg_global,
                         int32_t *window_table, int32_t *sigma_window,
                         int32_t *global_table, int32_t *sigma_global,
                         float *scores, int32_t *keep_idx,
                         void *workspace, size_t workspace_bytes, void **qkv_events, void *stream);

/* ------------------------------------------------------------------------- */
/* Encoder ends (public SAM architecture around the blocks)                  */
/* ------------------------------------------------------------------------- */

/* Patch embedding + absolute position embedding: tokens[b][ty*gw+tx][:] =
 * pos[ty*gw+tx][:] + bias + sum_{c,ky,kx} w[:][c][ky][kx] img[b][c][ty*P+ky][tx*P+kx]
 * (one rounding to bf16).  img dev bf16 [B][3][H][W]; w dev bf16 [D][3*P*P]
 * (out, then in-channel, ky, kx: a convolution weight flattened); bias dev fp32
 * [D]; pos dev bf16 [(H/P)*(W/P)][D]; x dev bf16 [B][(H/P)*(W/P)][D], written.
 * P % 8 == 0, 3*P*P % 64 == 0, D % 128 == 0 (else SSAM_EUNSUPPORTED). */
size_t ssam_patch_embed_workspace_bytes(int B, int H, int W, int P);
int ssam_patch_embed(const void *img, const void *w, const float *bias, const void *pos, void *x,
                     int B, int H, int W, int P, int D, void *workspace, size_t workspace_bytes, void *stream);

/* Neck: out = LN2(conv3x3(LN1(x W1^T))) per image, LayerNorm over the C
 * channels of every token, no convolution biases, zero padding.  x dev bf16
 * [B][g*g][D]; w1 dev bf16 [C][D]; w2 dev bf16 [C][9*C] with the input index
 * ordered (ky, kx, c), i.e. a [C][C][3][3] convolution weight permuted to
 * [out][ky][kx][in]; ln*_g, ln*_b dev fp32 [C]; out dev bf16 [B][g*g][C]
 * (token-major; SAM's channel-first tensor transposed).  C % 128 == 0 and
 * D % 64 == 0 (else SSAM_EUNSUPPORTED). */
size_t ssam_neck_workspace_bytes(int B, int g, int D, int C);
int ssam_neck(const void *x, const void *w1, const float *ln1_g, const float *ln1_b,
              const void *w2, const float *ln2_g, const float *ln2_b, float eps, void *out,
              int B, int g, int D, int C, void *workspace, size_t workspace_bytes, void *stream);

/* ------------------------------------------------------------------------- */
/* Instrumentation for the benchmark's measured peaks (not part of the method) */
/* ------------------------------------------------------------------------- */

/* A loop of independent bf16 MFMAs on register operands (no memory traffic): `workgroups` workgroups of four
 * waves, `iters` iterations of 8 x (32x32x16) (shape 0) or 16 x (16x16x32) (shape 1) MFMAs per wave; the caller
 * times the launch.  ssam_probe_mfma_flops gives the flops of one launch.  sink dev fp32 [workgroups*256], written.
 * SSAM_EINVAL on a bad shape, count or pointer. */
double ssam_probe_mfma_flops(int workgroups, int iters);
int ssam_probe_mfma(int shape, int workgroups, int iters, float *sink, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* SSAM_H */
