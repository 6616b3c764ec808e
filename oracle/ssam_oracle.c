/*
 * ssam_oracle.c -- TEST INFRASTRUCTURE, not a product path.
 *
 * Plain, slow, single-source CPU reference for the structured-sparse SAM ViT
 * encoder block of "SparseSAM" (arXiv 2605.17633): Stripe-Sort Attention
 * (Sec. 4.1, App. A.1 / Alg. 1) and the Residual-Consistency MLP (Sec. 4.2).
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may call it.
 * It shares no code, header, table or constant with the HIP library.
 *
 * Conventions
 *   - every pointer is a host pointer; tensors are dense row-major
 *   - floating-point inputs and outputs are float (the callers hand in values
 *     already rounded to bf16); inside a routine every intermediate is double
 *     and nothing is rounded to bf16 anywhere; the only roundings are to
 *     float where a routine's interface is float (2^-24 relative)
 *   - no tiling, no online softmax, no physical permutation: attention works
 *     in spatial order and the sparsity mask is applied through sigma^-1, so
 *     density 1.0 is literally dense SAM attention
 *   - OpenMP parallelises outer loops only (tokens, queries, rows)
 *   - returns 0 on success, a negative value on a bad argument
 *
 * Pins (tests/test_oracle_*.py): Z-order against a recursive quadrant walk and
 * the closed form on 2^k grids; sigma against the phase-view closed form;
 * mask tile counts; attention against library softmax attention at r = 1 and
 * brute force on tiny inputs; Sobel against library correlation and the ramp
 * closed form; top-k against a full sort; MLP against a library MLP at rho = 1;
 * the block at r = rho = 1 against a library-built dense SAM block; the
 * content-aware order against a hand-derived example, a library sort with the
 * paper's transpose, its rank structure, and two properties of the block that
 * uses it (order irrelevant at r = 1; scores decreasing along the Z-order
 * reproduce the position-only block); the encoder ends (patch embedding,
 * neck) against library convolution and layer norm and closed-form cases.
 * The paper prints no worked numeric example of the block: whole-block values
 * at r < 1 are "parity unpinned" by the paper itself and rest on the pins of
 * the parts.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_EINVAL (-1)
#define ORACLE_ENOMEM (-2)

/* ------------------------------------------------------------------------ */
/* Z-order (Morton) traversal, Fig. 2 caption; bit convention: the column   */
/* index supplies the even bits, the row index the odd bits, so a 2x2       */
/* "Z-group" is visited (0,0),(0,1),(1,0),(1,1).                            */
/* ------------------------------------------------------------------------ */
static uint64_t z_code(uint32_t row, uint32_t col)
{
    uint64_t code = 0;
    for (int b = 0; b < 32; ++b) {
        code |= (uint64_t)((col >> b) & 1u) << (2 * b);
        code |= (uint64_t)((row >> b) & 1u) << (2 * b + 1);
    }
    return code;
}

typedef struct { uint64_t code; int32_t cell; } coded_cell;

static int cmp_coded_cell(const void *a, const void *b)
{
    const coded_cell *x = (const coded_cell *)a, *y = (const coded_cell *)b;
    if (x->code < y->code) return -1;
    if (x->code > y->code) return 1;
    return 0;
}

/* pi[p] = row-major index (row*gw+col) of the p-th cell of the gh x gw grid
 * along the Z curve.  Non power-of-two grids: cells are ranked by code. */
int oracle_morton_order(int gh, int gw, int32_t *pi)
{
    if (gh <= 0 || gw <= 0 || !pi) return ORACLE_EINVAL;
    int n = gh * gw;
    coded_cell *cells = (coded_cell *)malloc((size_t)n * sizeof(coded_cell));
    if (!cells) return ORACLE_ENOMEM;
    for (int row = 0; row < gh; ++row)
        for (int col = 0; col < gw; ++col) {
            cells[row * gw + col].code = z_code((uint32_t)row, (uint32_t)col);
            cells[row * gw + col].cell = row * gw + col;
        }
    qsort(cells, (size_t)n, sizeof(coded_cell), cmp_coded_cell);
    for (int p = 0; p < n; ++p) pi[p] = cells[p].cell;
    free(cells);
    return 0;
}

/* Stripe-Sort permutation (Sec. 4.1): view pi as T[t][g] = pi[t*G+g] with
 * N/G rows and G columns; sigma = flatten(T^T), i.e.
 * sigma[g*(N/G)+t] = pi[t*G+g].  sigma_inv[sigma[p]] = p. */
int oracle_stripe_sort(const int32_t *pi, int n, int G, int32_t *sigma, int32_t *sigma_inv)
{
    if (!pi || !sigma || n <= 0 || G <= 0 || n % G != 0) return ORACLE_EINVAL;
    int rows = n / G;
    for (int t = 0; t < rows; ++t)
        for (int g = 0; g < G; ++g)
            sigma[g * rows + t] = pi[t * G + g];
    if (sigma_inv)
        for (int p = 0; p < n; ++p) sigma_inv[sigma[p]] = p;
    return 0;
}

/* sigma for a w x w grid: Z-order followed by the stripe interleave. */
static int grid_sigma(int w, int G, int32_t *sigma, int32_t *sigma_inv)
{
    int n = w * w;
    int32_t *pi = (int32_t *)malloc((size_t)n * sizeof(int32_t));
    if (!pi) return ORACLE_ENOMEM;
    int rc = oracle_morton_order(w, w, pi);
    if (rc == 0) rc = oracle_stripe_sort(pi, n, G, sigma, sigma_inv);
    free(pi);
    return rc;
}

/* Content-aware order of one attention group (Sec. 4.1, "Gradient-Based
 * Ordering" + "Stripe-Sort Permutation"): pi = the group's cells sorted by
 * score M descending (equal scores: lower cell index first; NaN counts as
 * -inf), sigma = stripe_G(pi).  Cells that are window padding are passed with
 * score -INFINITY and therefore rank last. */
typedef struct { float m; int32_t cell; } ranked_cell;

static int cmp_ranked_cell(const void *a, const void *b)
{
    const ranked_cell *x = (const ranked_cell *)a, *y = (const ranked_cell *)b;
    if (x->m > y->m) return -1;
    if (x->m < y->m) return 1;
    return (x->cell > y->cell) - (x->cell < y->cell);
}

int oracle_content_order(const float *scores, int n, int G, int32_t *sigma, int32_t *sigma_inv)
{
    if (!scores || !sigma || n <= 0 || G <= 0 || n % G != 0) return ORACLE_EINVAL;
    ranked_cell *rc = (ranked_cell *)malloc((size_t)n * sizeof(ranked_cell));
    int32_t *pi = (int32_t *)malloc((size_t)n * sizeof(int32_t));
    if (!rc || !pi) { free(rc); free(pi); return ORACLE_ENOMEM; }
    for (int i = 0; i < n; ++i) {
        float m = scores[i];
        if (m != m) m = -INFINITY;
        if (m == 0.0f) m = 0.0f;                  /* -0.0 ranks as +0.0 */
        rc[i].m = m; rc[i].cell = i;
    }
    qsort(rc, (size_t)n, sizeof(ranked_cell), cmp_ranked_cell);
    for (int i = 0; i < n; ++i) pi[i] = rc[i].cell;
    int r = oracle_stripe_sort(pi, n, G, sigma, sigma_inv);
    free(rc); free(pi);
    return r;
}

/* Window-major gather table (App. A.1, "window-major -> spatial perms"; SAM's
 * window partition pads the g x g grid up to a multiple of ws).
 * table[(wr*nws+wc)*ws*ws + p] = spatial index row*g+col of the token that
 * sits at permuted position p of window (wr,wc), or -1 where that cell is
 * padding.  Inside a window the order is sigma of the ws x ws grid. */
int oracle_window_table(int g, int ws, int G, int32_t *table)
{
    if (g <= 0 || ws <= 0 || !table) return ORACLE_EINVAL;
    int nws = (g + ws - 1) / ws, S = ws * ws;
    int32_t *sigma = (int32_t *)malloc((size_t)S * sizeof(int32_t));
    if (!sigma) return ORACLE_ENOMEM;
    int rc = grid_sigma(ws, G, sigma, NULL);
    if (rc) { free(sigma); return rc; }
    for (int wr = 0; wr < nws; ++wr)
        for (int wc = 0; wc < nws; ++wc)
            for (int p = 0; p < S; ++p) {
                int lr = sigma[p] / ws, lc = sigma[p] % ws;
                int row = wr * ws + lr, col = wc * ws + lc;
                table[(wr * nws + wc) * S + p] = (row < g && col < g) ? row * g + col : -1;
            }
    free(sigma);
    return 0;
}

/* Number of dense prefix tiles floor(r*T) of Alg. 1, evaluated in double with
 * a 1e-6 guard against r*T landing just under an integer. */
static int prefix_tiles(int T, double r)
{
    int n_pre = (int)floor(r * (double)T + 1e-6);
    if (n_pre < 0) n_pre = 0;
    if (n_pre > T) n_pre = T;
    return n_pre;
}

/* A-shape block mask (Alg. 1): T = ceil(S/Bm) tiles per side; row tile i sees
 * column tiles {0..floor(r*T)-1} and its own diagonal tile i.
 * mask[i*T+j] = 1 where visible. */
int oracle_block_mask(int S, int Bm, double r, uint8_t *mask, int *n_pre_out)
{
    if (S <= 0 || Bm <= 0 || !(r > 0.0) || r > 1.0 || !mask) return ORACLE_EINVAL;
    int T = (S + Bm - 1) / Bm;
    int n_pre = prefix_tiles(T, r);
    for (int i = 0; i < T; ++i)
        for (int j = 0; j < T; ++j)
            mask[i * T + j] = (uint8_t)((j < n_pre) || (j == i));
    if (n_pre_out) *n_pre_out = n_pre;
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Stripe-Sort attention for ONE group of S = w*w tokens (a window or the    */
/* whole grid), all h heads, in SPATIAL order (Alg. 1 with the permutation   */
/* applied to the mask instead of to the data).                              */
/*   q,k,v   [h][S][d]     rel_h, rel_w [(2w-1)][d]     out [h][S][d]        */
/* logit(s,s') = tau*q_s.k_s' + B^H[s,row(s')] + B^W[s,col(s')], tau=1/sqrt d*/
/* B^H[s,p] = q_s . rel_h[row(s)-p+w-1], B^W likewise with columns; the bias */
/* uses the unscaled query (Alg. 1 divides the bias by tau before the        */
/* tau-scaled exponent, which cancels).                                      */
/* Key s' is visible to query s iff tile(sigma^-1 s') < floor(r*T) or        */
/* tile(sigma^-1 s') == tile(sigma^-1 s), tile(p) = p div Bm.                */
/* Softmax is the two-pass definition over the visible keys only.            */
/* sinv[s] = sigma^-1(s): the position of spatial token s in the scan order.  */
/* ------------------------------------------------------------------------ */
int oracle_attention_ordered(const float *q, const float *k, const float *v,
                             const float *rel_h, const float *rel_w,
                             int h, int w, int d, const int32_t *sinv, int Bm, double r, float *out)
{
    if (!q || !k || !v || !rel_h || !rel_w || !out || !sinv) return ORACLE_EINVAL;
    if (h <= 0 || w <= 0 || d <= 0 || Bm <= 0 || !(r > 0.0) || r > 1.0) return ORACLE_EINVAL;
    int S = w * w;
    int T = (S + Bm - 1) / Bm;
    int n_pre = prefix_tiles(T, r);
    const double tau = 1.0 / sqrt((double)d);
    int failed = 0;

#pragma omp parallel for collapse(2) schedule(dynamic, 8)
    for (int head = 0; head < h; ++head)
        for (int s = 0; s < S; ++s) {
            double *logit = (double *)malloc((size_t)S * sizeof(double));
            double *bh = (double *)malloc((size_t)w * sizeof(double));
            double *bw = (double *)malloc((size_t)w * sizeof(double));
            double *acc = (double *)malloc((size_t)d * sizeof(double));
            if (!logit || !bh || !bw || !acc) {
                failed = 1; free(logit); free(bh); free(bw); free(acc); continue;
            }
            const float *qs = q + ((size_t)head * S + s) * d;
            int srow = s / w, scol = s % w;
            for (int p = 0; p < w; ++p) {
                const float *rh = rel_h + (size_t)(srow - p + w - 1) * d;
                const float *rw = rel_w + (size_t)(scol - p + w - 1) * d;
                double sh = 0.0, sw = 0.0;
                for (int c = 0; c < d; ++c) { sh += (double)qs[c] * rh[c]; sw += (double)qs[c] * rw[c]; }
                bh[p] = sh; bw[p] = sw;
            }
            int my_tile = sinv[s] / Bm;
            double mx = -INFINITY;
            for (int t = 0; t < S; ++t) {
                int key_tile = sinv[t] / Bm;
                if (!(key_tile < n_pre || key_tile == my_tile)) { logit[t] = -INFINITY; continue; }
                const float *kt = k + ((size_t)head * S + t) * d;
                double dot = 0.0;
                for (int c = 0; c < d; ++c) dot += (double)qs[c] * kt[c];
                logit[t] = tau * dot + bh[t / w] + bw[t % w];
                if (logit[t] > mx) mx = logit[t];
            }
            double denom = 0.0;
            for (int t = 0; t < S; ++t)
                if (logit[t] != -INFINITY) { logit[t] = exp(logit[t] - mx); denom += logit[t]; }
                else logit[t] = 0.0;
            for (int c = 0; c < d; ++c) acc[c] = 0.0;
            for (int t = 0; t < S; ++t) {
                if (logit[t] == 0.0) continue;
                const float *vt = v + ((size_t)head * S + t) * d;
                double pr = logit[t] / denom;
                for (int c = 0; c < d; ++c) acc[c] += pr * vt[c];
            }
            float *o = out + ((size_t)head * S + s) * d;
            for (int c = 0; c < d; ++c) o[c] = (float)acc[c];
            free(logit); free(bh); free(bw); free(acc);
        }
    return failed ? ORACLE_ENOMEM : 0;
}

/* The same with the paper's position-only order: sigma = stripe_G(Z-order) of
 * the w x w grid (G = 1 leaves the plain Z-order). */
int oracle_attention(const float *q, const float *k, const float *v,
                     const float *rel_h, const float *rel_w,
                     int h, int w, int d, int G, int Bm, double r, float *out)
{
    if (w <= 0) return ORACLE_EINVAL;
    int S = w * w;
    int32_t *sigma = (int32_t *)malloc((size_t)S * sizeof(int32_t));
    int32_t *sinv = (int32_t *)malloc((size_t)S * sizeof(int32_t));
    if (!sigma || !sinv) { free(sigma); free(sinv); return ORACLE_ENOMEM; }
    int rc = grid_sigma(w, G, sigma, sinv);
    if (rc == 0) rc = oracle_attention_ordered(q, k, v, rel_h, rel_w, h, w, d, sinv, Bm, r, out);
    free(sigma); free(sinv);
    return rc;
}

/* ------------------------------------------------------------------------ */
/* Token scores, Eq. 1: Sobel gradient magnitude of the channel-summed map.  */
/* The 3x3 filter is linear, so filtering each channel and summing over the  */
/* D channels equals filtering the channel sum; the sum is taken first and   */
/* squared afterwards.  Zero padding at the border.                          */
/*   x [gh][gw][D]  ->  M [gh][gw]                                           */
/* ------------------------------------------------------------------------ */
int oracle_score_tokens(const float *x, int gh, int gw, int D, float *M)
{
    if (!x || !M || gh <= 0 || gw <= 0 || D <= 0) return ORACLE_EINVAL;
    static const int SX[3][3] = { { -1, 0, 1 }, { -2, 0, 2 }, { -1, 0, 1 } };
    double *c = (double *)malloc((size_t)gh * gw * sizeof(double));
    if (!c) return ORACLE_ENOMEM;
    for (int i = 0; i < gh * gw; ++i) {
        double s = 0.0;
        for (int ch = 0; ch < D; ++ch) s += (double)x[(size_t)i * D + ch];
        c[i] = s;
    }
    for (int i = 0; i < gh; ++i)
        for (int j = 0; j < gw; ++j) {
            double gx = 0.0, gy = 0.0;
            for (int a = 0; a < 3; ++a)
                for (int b = 0; b < 3; ++b) {
                    int ii = i + a - 1, jj = j + b - 1;
                    if (ii < 0 || ii >= gh || jj < 0 || jj >= gw) continue;
                    gx += SX[a][b] * c[ii * gw + jj];   /* horizontal derivative */
                    gy += SX[b][a] * c[ii * gw + jj];   /* S_y = S_x transposed  */
                }
            M[i * gw + j] = (float)sqrt(gx * gx + gy * gy);
        }
    free(c);
    return 0;
}

/* Keep count of the Residual-Consistency MLP: K = floor(rho*N) (1e-6 guard),
 * at least 1 and at most N. */
int oracle_keep_count(int n, double rho)
{
    if (n <= 0 || !(rho > 0.0) || rho > 1.0) return ORACLE_EINVAL;
    int K = (int)floor(rho * (double)n + 1e-6);
    if (K < 1) K = 1;
    if (K > n) K = n;
    return K;
}

typedef struct { float score; int32_t idx; } scored_token;

/* score descending, then index ascending; -0.0 equals +0.0; NaN ranks last */
static int cmp_scored_token(const void *a, const void *b)
{
    const scored_token *x = (const scored_token *)a, *y = (const scored_token *)b;
    if (x->score > y->score) return -1;
    if (x->score < y->score) return 1;
    return (x->idx > y->idx) - (x->idx < y->idx);
}

static int cmp_int32(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/* Keep-set (Sec. 4.2): the K highest-scoring of n tokens, ties to the lower
 * index, returned in ascending index order.  Comparisons are made on the
 * fp32 scores as given. */
int oracle_select_tokens(const float *scores, int n, int K, int32_t *keep)
{
    if (!scores || !keep || n <= 0 || K <= 0 || K > n) return ORACLE_EINVAL;
    scored_token *t = (scored_token *)malloc((size_t)n * sizeof(scored_token));
    if (!t) return ORACLE_ENOMEM;
    for (int i = 0; i < n; ++i) {
        t[i].score = isnan(scores[i]) ? -INFINITY : scores[i];
        t[i].idx = i;
    }
    qsort(t, (size_t)n, sizeof(scored_token), cmp_scored_token);
    for (int i = 0; i < K; ++i) keep[i] = t[i].idx;
    qsort(keep, (size_t)K, sizeof(int32_t), cmp_int32);
    free(t);
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Dense building blocks of the SAM block (standard definitions).            */
/* ------------------------------------------------------------------------ */
static void layer_norm_row(const double *x, const float *gamma, const float *beta,
                           double eps, int D, double *y)
{
    double mean = 0.0, var = 0.0;
    for (int c = 0; c < D; ++c) mean += x[c];
    mean /= D;
    for (int c = 0; c < D; ++c) var += (x[c] - mean) * (x[c] - mean);
    var /= D;                                 /* biased variance */
    double inv = 1.0 / sqrt(var + eps);
    for (int c = 0; c < D; ++c) y[c] = (x[c] - mean) * inv * gamma[c] + beta[c];
}

/* y[n] = sum_k x[k]*W[n][k] + b[n]   (W in [out][in] layout) */
static void linear_row(const double *x, const float *W, const float *b, int in, int outn, double *y)
{
    for (int n = 0; n < outn; ++n) {
        const float *wr = W + (size_t)n * in;
        double s = 0.0;
#pragma omp simd reduction(+ : s)
        for (int kk = 0; kk < in; ++kk) s += x[kk] * (double)wr[kk];
        y[n] = s + (b ? (double)b[n] : 0.0);
    }
}

static double gelu_erf(double t) { return 0.5 * t * (1.0 + erf(t * 0.70710678118654752440)); }

/* ------------------------------------------------------------------------ */
/* Residual-Consistency MLP (Sec. 4.2): for i in the keep-set                */
/*   x_i <- x_i + W2 gelu(W1 LN(x_i) + b1) + b2 ; every other row is left     */
/* untouched (bit-identical).                                                */
/*   x [n][D] in place; keep [K] distinct indices in [0,n)                   */
/* ------------------------------------------------------------------------ */
int oracle_routed_mlp(float *x, int n, int D, int Dm, const int32_t *keep, int K,
                      const float *ln_g, const float *ln_b, double eps,
                      const float *w1, const float *b1, const float *w2, const float *b2)
{
    if (!x || !keep || !ln_g || !ln_b || !w1 || !w2 || n <= 0 || D <= 0 || Dm <= 0 || K < 0 || K > n)
        return ORACLE_EINVAL;
    for (int j = 0; j < K; ++j) if (keep[j] < 0 || keep[j] >= n) return ORACLE_EINVAL;
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 4)
    for (int j = 0; j < K; ++j) {
        double *row = (double *)malloc((size_t)(2 * D + Dm) * sizeof(double));
        if (!row) { failed = 1; continue; }
        double *u = row + D, *hid = row + 2 * D;
        float *xi = x + (size_t)keep[j] * D;
        for (int c = 0; c < D; ++c) row[c] = (double)xi[c];
        layer_norm_row(row, ln_g, ln_b, eps, D, u);
        linear_row(u, w1, b1, D, Dm, hid);
        for (int m = 0; m < Dm; ++m) hid[m] = gelu_erf(hid[m]);
        linear_row(hid, w2, b2, Dm, D, u);
        for (int c = 0; c < D; ++c) xi[c] = (float)(row[c] + u[c]);
        free(row);
    }
    return failed ? ORACLE_ENOMEM : 0;
}

/* ------------------------------------------------------------------------ */
/* One structured-sparse encoder block on one image.                         */
/*   x [g][g][D] in place.  ws > 0: SAM window attention (LN1, zero-pad the  */
/*   normalised map up to a multiple of ws, ws x ws windows, pad tokens take */
/*   part as ordinary keys/queries and their outputs are dropped); ws == 0:  */
/*   global attention over the whole grid.  Then x += proj(attn), then the   */
/*   routed MLP over the keep-set.  qkv output channel = which*D + head*d + c*/
/* ------------------------------------------------------------------------ */
int oracle_encoder_block(float *x, int g, int D, int h, int Dm, int ws, int G, int Bm,
                         double r, const int32_t *keep, int K, double eps, const float *order_scores,
                         const float *ln1_g, const float *ln1_b,
                         const float *wqkv, const float *bqkv,
                         const float *rel_h, const float *rel_w,
                         const float *wproj, const float *bproj,
                         const float *ln2_g, const float *ln2_b,
                         const float *w1, const float *b1, const float *w2, const float *b2)
{
    if (!x || g <= 0 || D <= 0 || h <= 0 || D % h != 0 || ws < 0) return ORACLE_EINVAL;
    const int d = D / h, n = g * g;
    const int w = ws > 0 ? ws : g;                 /* side of one attention group */
    const int nws = (g + w - 1) / w, gp = nws * w; /* padded grid side            */
    const int S = w * w;
    int rc = 0;

    /* LN1 of every token, then zero padding */
    double *u = (double *)calloc((size_t)gp * gp * D, sizeof(double));
    if (!u) return ORACLE_ENOMEM;
#pragma omp parallel for schedule(static)
    for (int t = 0; t < n; ++t) {
        double *row = (double *)malloc((size_t)D * sizeof(double));
        for (int c = 0; c < D; ++c) row[c] = (double)x[(size_t)t * D + c];
        layer_norm_row(row, ln1_g, ln1_b, eps, D, u + ((size_t)(t / g) * gp + (t % g)) * D);
        free(row);
    }

    float *qh = (float *)malloc((size_t)3 * h * S * d * sizeof(float));
    float *oh = (float *)malloc((size_t)h * S * d * sizeof(float));
    double *qkv = (double *)malloc((size_t)S * 3 * D * sizeof(double));
    if (!qh || !oh || !qkv) { free(u); free(qh); free(oh); free(qkv); return ORACLE_ENOMEM; }
    float *kh = qh + (size_t)h * S * d, *vh = kh + (size_t)h * S * d;

    for (int wr = 0; wr < nws && rc == 0; ++wr)
        for (int wc = 0; wc < nws && rc == 0; ++wc) {
            /* qkv projection of the window's tokens (local spatial order) */
#pragma omp parallel for schedule(static)
            for (int s = 0; s < S; ++s) {
                const double *us = u + ((size_t)(wr * w + s / w) * gp + (wc * w + s % w)) * D;
                linear_row(us, wqkv, bqkv, D, 3 * D, qkv + (size_t)s * 3 * D);
            }
            /* The attention routine takes float operands: keep full double
             * precision is not possible through that interface, so round to
             * float here (2^-24 relative, far below the comparison tolerance). */
            for (int s = 0; s < S; ++s)
                for (int head = 0; head < h; ++head)
                    for (int c = 0; c < d; ++c) {
                        size_t dst = ((size_t)head * S + s) * d + c;
                        qh[dst] = (float)qkv[(size_t)s * 3 * D + 0 * D + head * d + c];
                        kh[dst] = (float)qkv[(size_t)s * 3 * D + 1 * D + head * d + c];
                        vh[dst] = (float)qkv[(size_t)s * 3 * D + 2 * D + head * d + c];
                    }
            if (order_scores) {
                /* content-aware order of this group: its cells ranked by the image's score map */
                float *ms = (float *)malloc((size_t)S * sizeof(float));
                int32_t *sg = (int32_t *)malloc((size_t)S * sizeof(int32_t));
                int32_t *si = (int32_t *)malloc((size_t)S * sizeof(int32_t));
                if (!ms || !sg || !si) { free(ms); free(sg); free(si); rc = ORACLE_ENOMEM; break; }
                for (int s = 0; s < S; ++s) {
                    int row = wr * w + s / w, col = wc * w + s % w;
                    ms[s] = (row < g && col < g) ? order_scores[(size_t)row * g + col] : -INFINITY;
                }
                rc = oracle_content_order(ms, S, G, sg, si);
                if (rc == 0) rc = oracle_attention_ordered(qh, kh, vh, rel_h, rel_w, h, w, d, si, Bm, r, oh);
                free(ms); free(sg); free(si);
            } else {
                rc = oracle_attention(qh, kh, vh, rel_h, rel_w, h, w, d, G, Bm, r, oh);
            }
            if (rc) break;
            /* concat heads, output projection, residual; padded cells dropped */
#pragma omp parallel for schedule(static)
            for (int s = 0; s < S; ++s) {
                int row = wr * w + s / w, col = wc * w + s % w;
                if (row >= g || col >= g) continue;
                double *cat = (double *)malloc((size_t)2 * D * sizeof(double));
                double *po = cat + D;
                for (int head = 0; head < h; ++head)
                    for (int c = 0; c < d; ++c)
                        cat[head * d + c] = (double)oh[((size_t)head * S + s) * d + c];
                linear_row(cat, wproj, bproj, D, D, po);
                float *xt = x + ((size_t)row * g + col) * D;
                for (int c = 0; c < D; ++c) xt[c] = (float)((double)xt[c] + po[c]);
                free(cat);
            }
        }
    free(u); free(qh); free(oh); free(qkv);
    if (rc) return rc;
    return oracle_routed_mlp(x, n, D, Dm, keep, K, ln2_g, ln2_b, eps, w1, b1, w2, b2);
}

/* ------------------------------------------------------------------------ */
/* Encoder ends of the SAM ViT image encoder.  The paper's method lives in   */
/* the blocks and it measures the whole encoder; it does not describe the    */
/* ends, which follow the public SAM architecture: a patch embedding (one    */
/* P x P, stride-P convolution = one linear map per patch) plus an absolute  */
/* position embedding in front, and a "neck" behind (1x1 convolution without */
/* bias, LayerNorm over channels, 3x3 convolution without bias and with zero */
/* padding, LayerNorm over channels).  Plain definitions, double inside.     */
/*   img [3][H][W]; w [D][3][P][P] (out, in, ky, kx); pos [gh*gw][D];        */
/*   x [gh*gw][D], gh = H/P, gw = W/P.                                       */
/* ------------------------------------------------------------------------ */
int oracle_patch_embed(const float *img, int H, int W, int P, const float *w, const float *b,
                       const float *pos, int D, float *x)
{
    if (!img || !w || !b || !pos || !x || H <= 0 || W <= 0 || P <= 0 || D <= 0 || H % P || W % P) return ORACLE_EINVAL;
    const int gh = H / P, gw = W / P;
#pragma omp parallel for collapse(2) schedule(static)
    for (int ty = 0; ty < gh; ++ty)
        for (int tx = 0; tx < gw; ++tx) {
            const size_t t = (size_t)ty * gw + tx;
            for (int o = 0; o < D; ++o) {
                double acc = (double)b[o] + (double)pos[t * D + o];
                for (int c = 0; c < 3; ++c)
                    for (int ky = 0; ky < P; ++ky)
                        for (int kx = 0; kx < P; ++kx)
                            acc += (double)w[(((size_t)o * 3 + c) * P + ky) * P + kx] *
                                   (double)img[((size_t)c * H + ty * P + ky) * W + tx * P + kx];
                x[t * D + o] = (float)acc;
            }
        }
    return 0;
}

/*   x [g*g][D] token-major; w1 [C][D]; w2 [C][C][3][3] (out, in, ky, kx);   */
/*   out [g*g][C] token-major (the channel-first tensor of SAM, transposed). */
int oracle_neck(const float *x, int g, int D, int C, const float *w1, const float *ln1_g, const float *ln1_b,
                const float *w2, const float *ln2_g, const float *ln2_b, double eps, float *out)
{
    if (!x || !w1 || !ln1_g || !ln1_b || !w2 || !ln2_g || !ln2_b || !out || g <= 0 || D <= 0 || C <= 0) return ORACLE_EINVAL;
    const int n = g * g;
    double *y = (double *)malloc((size_t)n * C * sizeof(double));
    if (!y) return ORACLE_ENOMEM;
#pragma omp parallel for schedule(static)
    for (int t = 0; t < n; ++t) {
        double *row = (double *)malloc((size_t)C * sizeof(double));
        for (int o = 0; o < C; ++o) {
            double acc = 0.0;
            for (int c = 0; c < D; ++c) acc += (double)x[(size_t)t * D + c] * (double)w1[(size_t)o * D + c];
            row[o] = acc;
        }
        layer_norm_row(row, ln1_g, ln1_b, eps, C, y + (size_t)t * C);
        free(row);
    }
#pragma omp parallel for schedule(static)
    for (int t = 0; t < n; ++t) {
        const int ty = t / g, tx = t % g;
        double *row = (double *)malloc((size_t)2 * C * sizeof(double));
        for (int o = 0; o < C; ++o) {
            double acc = 0.0;
            for (int ky = 0; ky < 3; ++ky)
                for (int kx = 0; kx < 3; ++kx) {
                    const int sy = ty + ky - 1, sx = tx + kx - 1;
                    if (sy < 0 || sy >= g || sx < 0 || sx >= g) continue;      /* zero padding */
                    const double *src = y + ((size_t)sy * g + sx) * C;
                    for (int c = 0; c < C; ++c)
                        acc += src[c] * (double)w2[(((size_t)o * C + c) * 3 + ky) * 3 + kx];
                }
            row[o] = acc;
        }
        layer_norm_row(row, ln2_g, ln2_b, eps, C, row + C);
        for (int o = 0; o < C; ++o) out[(size_t)t * C + o] = (float)row[C + o];
        free(row);
    }
    free(y);
    return 0;
}
