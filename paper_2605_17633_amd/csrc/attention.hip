// Stripe-Sort attention (App. A.1, Alg. 1) for gfx950: block-sparse, flash-style
// attention over the static A-shape tile mask, with SAM's decomposed 2-D
// relative-position bias fused in.  Tokens arrive in scan order; sigma maps a
// scan position to its spatial cell for the bias lookup.
//
// Formulation.  Scores are computed transposed, S^T = K Q^T, on the 32x32x16 bf16
// MFMA: the Q fragments (operand b) stay in registers for the whole problem, K
// rows come from LDS (operand a).  In the result layout every lane owns ONE
// query (column l & 31) and 16 of the 32 keys of a block, so the softmax row
// statistics are per-lane scalars: the row maximum needs a single exchange with
// lane l^32, the row sum none until the end.  exp(S^T) converted to bf16 is
// already in the operand-b layout of the second product O^T = V^T P^T.  Its
// operand-a fragments (8 keys of one feature column per lane, in the key order
// the result layout dictates: contraction slot e of half-wave hf of MFMA t <->
// key 16t + 8(e/4) + 4hf + (e&3)) come from the row-major V rows in LDS through
// the transposing LDS read of gfx950 (ds_read_b64_tr_b16: a 16-lane group reads
// 4 rows x 16 columns and every lane receives one column), so V is staged
// exactly like K and never transposed in memory.
// Key blocks are processed in chunks of two (64 keys; the register budget of two
// waves per SIMD): all score MFMAs of the chunk first, one max / one rescale of
// the running output per chunk, then all P V MFMAs.
// Bias: per wave, U = Q R^T is formed once with the MFMA for both tables and kept
// in LDS as fp16, pre-multiplied by log2 e; the inner loop adds two table
// look-ups per score through per-key byte offsets.  Global kernel: scattered into
// entry-major rows B^H[key_row][q], B^W[key_col][q]; window kernel: stored as the
// MFMA tile comes out, U[q][m], a key being entry q_row - key_row + w - 1.
// Memory requests are spread over a problem's / a tile's phases (see the prefetch
// macros): a wave whose loads do not fit the CU's request queues waits instead of
// computing, and a wait placed behind a branch or on a value that is used at once
// drains every load and store in flight.
//
// Two launch shapes:
//   window kernel: persistent workgroups looping over (window, head) problems, one
//                  wave per 32-query tile (= mask tile of 32), the window's whole K
//                  and V in LDS, the next problem's K and V prefetched into registers
//                  and its Q straight into LDS, in three pieces, the rel-pos tables
//                  resident in LDS;
//   global kernel: one workgroup per (128-query mask tile, image, head), 4 waves, two
//                  workgroups per CU, active 128-key tiles streamed through LDS with
//                  register prefetch (K and V requested at different points).
#include "common.h"

namespace {

constexpr float LOG2E = 1.4426950408889634f;

struct AttnParams {
    const bf16 *q, *k, *v;
    long row_stride;
    const bf16 *rel_h, *rel_w;
    const int32_t *sigma;
    long sigma_stride;      // elements between the sigma tables of consecutive groups; 0 = one shared table
    bf16 *out;
    const int32_t *out_rows;   // NULL: query p of group g goes to output row g*S+p; else to out_rows[g*S+p] (-1: dropped)
    int S, w, h, n_pre;
    float scale_log2e;
};

template <int D>
struct AttnCfg {
    static constexpr int KS = D / 16;            // k-steps of the score product
    static constexpr int DT = (D + 31) / 32;     // 32-row tiles of O^T
    static constexpr int KSTR = D + 8;           // row stride in LDS (elements): odd in 16-byte units
    static constexpr int CH = D / 8;             // 16-byte chunks per row
    // D = 16 mod 32: the last 32-row tile of O^T has 16 rows to spare and the LDS rows of V have 8 columns of
    // padding; with ones in that padding those rows come out of the P V product as the sum of the probabilities,
    // which the softmax then does not have to add up on the vector unit
    static constexpr bool ONES = D % 32 == 16;
};

// fill the padding columns of `rows` LDS rows of V with 1.0 (they are never written afterwards: tile stores cover
// the D real columns only)
template <int D>
__device__ __forceinline__ void set_ones_columns(bf16 *Vs, int rows, int tid, int nthreads)
{
    if constexpr (AttnCfg<D>::ONES) {
        const u32x4 ones = { 0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u };
        for (int p = tid; p < rows; p += nthreads) *reinterpret_cast<u32x4 *>(Vs + p * AttnCfg<D>::KSTR + D) = ones;
    }
}

// Per-wave softmax/output state for 32 queries (one per lane pair l, l^32).
template <int D>
struct WaveState {
    f32x16 o[AttnCfg<D>::DT];
    float m, l;
};

template <int D>
__device__ __forceinline__ void init_state(WaveState<D> &st)
{
#pragma unroll
    for (int dt = 0; dt < AttnCfg<D>::DT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) st.o[dt][r] = 0.f;
    st.m = -INFINITY;
    st.l = 0.f;
}

// Bias table of the wave's 32 queries in the global kernel, query-major, fp16 (see GlbTab), divided by the softmax
// scale so that (score + row entry + column entry) * scale * log2e is the logit in log2 units:
//   tq[q*tstr + (p&1)*hw + (p>>1)]            = q . rel_h[row(q)-p+w-1] / scale      (p = key row)
//   tq[q*tstr + 2*hw + (p&1)*hw + (p>>1)]     = q . rel_w[col(q)-p+w-1] / scale      (p = key column)
// hw = ceil(w/2): even and odd rows (columns) are stored apart, so that rows two apart are neighbours: the 32-key
// blocks of the position-only Stripe-Sort order are 4 x 8 patches of stride 2 (see attn_scores_patch), whose 4 row
// and 8 column entries are then contiguous.  tstr = 4*hw + 4: the 8 bytes of padding put the 32 lanes of a look-up
// (one entry, 32 queries) on distinct banks.  tq_lane: this lane's query row.  rel tables: rows of `rstr` elements.
__host__ __device__ inline int glb_tstr(int w) { return 4 * ((w + 1) >> 1) + 4; }

template <int D, typename TabT>
__device__ __forceinline__ void build_bias_rows(const bf16x8 *qf, const bf16 *rel_h, const bf16 *rel_w, int rstr,
                                                int w, int qrow, int qcol, TabT *tq_lane, float inv_scale)
{
    constexpr int KS = AttnCfg<D>::KS;
    const int lane = threadIdx.x & 63, l32 = lane & 31, half = lane >> 5;
    const int nrel = 2 * w - 1, hw = (w + 1) >> 1;
    // operand a of slab mt: rows mt*32 + l32 of both tables; rows past the table re-read its last row (their
    // products are never stored), so every load is unconditional and a slab's 2*KS loads are in flight together
    bf16x8 cur[2][KS], nxt[2][KS];
    auto load_slab = [&](bf16x8 (&a)[2][KS], int mt) {
        const int mrow = min(mt * 32 + l32, nrel - 1);
#pragma unroll
        for (int tab = 0; tab < 2; ++tab)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                a[tab][ks] = *reinterpret_cast<const bf16x8 *>((tab ? rel_w : rel_h) + (long)mrow * rstr + ks * 16 + half * 8);
    };
    load_slab(cur, 0);
    for (int mt = 0; mt * 32 < nrel; ++mt) {
        // requested before this slab's products, used after them; past the last slab it re-reads the last row:
        // an unconditional request keeps the wait below counted (a branch here would force a full drain)
        load_slab(nxt, mt + 1);
#pragma unroll
        for (int tab = 0; tab < 2; ++tab) {
            f32x16 u;
#pragma unroll
            for (int r = 0; r < 16; ++r) u[r] = 0.f;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) u = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cur[tab][ks], qf[ks], u, 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");          // MFMA passes done before u is read under predicates
            __builtin_amdgcn_sched_barrier(0);
            TabT *dst = tq_lane + (tab ? 2 * hw : 0);
            const int qpos = tab ? qcol : qrow;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                int m = mt * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
                int p = qpos + (w - 1) - m;
                if (p >= 0 && p < w && m < nrel) dst[(p & 1) * hw + (p >> 1)] = (TabT)(u[r] * inv_scale);
            }
        }
#pragma unroll
        for (int tab = 0; tab < 2; ++tab)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) cur[tab][ks] = nxt[tab][ks];
    }
}

// Window form of the bias tables.  A window has 2w-1 <= 32 relative positions, so rel x Q^T is one MFMA tile
// per table and is stored the way it leaves the matrix core, query-major and without predicates:
//   tq[q*WIN_TSTR + m]                 = log2e * q . rel_h[m]
//   tq[(32 + q)*WIN_TSTR + m]          = log2e * q . rel_w[m]        (m = 0..31; rows past 2w-2 of rel are zero)
// A key in row kr, column kc is then entry qrow - kr + w - 1 of the first and qcol - kc + w - 1 of the second
// row of the lane's query.  Entries are fp16 (see GlbTab); the row stride keeps the 8-byte stores aligned.
typedef _Float16 WinTab;
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
constexpr int WIN_TSTR = 36;
template <int D>
__device__ __forceinline__ void build_bias_rows_window(const bf16x8 *qf, const bf16 *rel_h, const bf16 *rel_w, int rstr, WinTab *tq)
{
    const int lane = threadIdx.x & 63, l32 = lane & 31, half = lane >> 5;
#pragma unroll
    for (int tab = 0; tab < 2; ++tab) {
        const bf16 *rel = (tab ? rel_w : rel_h) + l32 * rstr + half * 8;
        f32x16 u;
#pragma unroll
        for (int r = 0; r < 16; ++r) u[r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < AttnCfg<D>::KS; ++ks)
            u = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8 *>(rel + ks * 16), qf[ks], u, 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");          // MFMA passes done before u is read (as in build_bias_rows)
        __builtin_amdgcn_sched_barrier(0);
        WinTab *dst = tq + (tab * 32 + l32) * WIN_TSTR + 4 * half;    // u[4g + e] is rel row 8g + 4*half + e of query l32
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            f16x4 hv = { (_Float16)(u[4 * g] * LOG2E), (_Float16)(u[4 * g + 1] * LOG2E),
                         (_Float16)(u[4 * g + 2] * LOG2E), (_Float16)(u[4 * g + 3] * LOG2E) };
            *reinterpret_cast<f16x4 *>(dst + 8 * g) = hv;
        }
    }
}

// A chunk of nb (1..NB, wave-uniform) 32-key blocks against the wave's 32 queries.
//   Ks, Vs: LDS, row-major rows ([keys][KSTR]); blk[b]: index of the chunk's b-th block in them
//   krc:    LDS, per key two byte offsets into the bias tables, indexed like Ks: low half for the row part,
//           high half for the column part (global kernel: within the query's table row, see build_bias_rows;
//           window tables: the key's share of the entry index, see key_bias_offsets_window)
//   key0[b]: scan position of the block's first key (for the S bound; RAGGED = the chunk crosses S)
//   tq_h, tq_w: where this lane's query starts in the row-part and column-part bias tables; a key's two
//           bias terms are read at tq_h + (low half of krc) and tq_w + (high half of krc), in bytes
//   FULL:   the chunk has all NB blocks (nb is not looked at: no per-block branches, no dummy scores)
//   MIXADD: the column part of the bias is added by one mixed-precision fma (fp16 operand widened inside the
//           instruction) instead of convert + add
//   RAW:    the tables hold bias / scale and the scores stay unscaled: logit = (s + bh + bw) * scale_log2e
//           (global kernel); otherwise the tables hold bias * log2e and logit = s * scale_log2e + bh + bw
constexpr float ATTN_LAG = 8.f;

// Second half of a chunk step, the same for every way of forming the scores: s holds the chunk's logits (RAW: before
// the multiplication by scale_log2e), mx their maximum over this lane's keys, in the same units.
template <int D, int NB, bool FULL, bool RAW>
__device__ __forceinline__ void attn_softmax_pv(WaveState<D> &st, f32x16 (&s)[NB], float mx, const bf16 *Vs,
                                                const int (&blk)[NB], int nb_, float scale_log2e)
{
    using C = AttnCfg<D>;
    const int nb = FULL ? NB : nb_;
    const int lane = threadIdx.x & 63, half = lane >> 5;
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    if constexpr (RAW) mx *= scale_log2e;
    // st.m is the exponent reference of the running sums, not the running maximum: it moves only when a chunk's
    // maximum exceeds it by more than 2^ATTN_LAG, so probabilities stay below 2^ATTN_LAG (all of a query's terms
    // carry the same power of two, which the final division removes) and the rescaling of the 32 x D accumulator
    // is skipped by the whole wave in most chunks.  First chunk: st.m = -inf, every lane moves, alpha = 0.
    const bool move = mx > st.m + ATTN_LAG;
    if (__builtin_amdgcn_ballot_w64(move) != 0) {
        const float mnew = move ? mx : st.m;
        const float alpha = __builtin_amdgcn_exp2f(st.m - mnew);
        st.m = mnew;
        if constexpr (!C::ONES) st.l *= alpha;
#pragma unroll
        for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) st.o[dt][r] *= alpha;
    }
    const float mref = st.m;
    float psum = 0.f;
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        if (b < nb) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                s[b][r] = __builtin_amdgcn_exp2f(RAW ? fmaf(s[b][r], scale_log2e, -mref) : s[b][r] - mref);
                if constexpr (!C::ONES) psum += s[b][r];
            }
        }
    }
    if constexpr (!C::ONES) st.l += psum;
    // transposing read: lane li of a 16-lane group points at row (li >> 2), column chunk (li & 3) of a
    // 4-key x 16-feature block and receives the 4 keys of feature column li
    const int li = lane & 15, fblk = (lane >> 4) & 1;
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        if (b < nb) {
            const bf16 *vblk = Vs + blk[b] * 32 * C::KSTR + (4 * half + (li >> 2)) * C::KSTR;
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                bf16x8 p;
#pragma unroll
                for (int e = 0; e < 8; ++e) p[e] = (bf16)s[b][8 * t + e];
#pragma unroll
                for (int dt = 0; dt < C::DT; ++dt) {
                    int col = dt * 32 + 16 * fblk + 4 * (li & 3);
                    // feature columns past D re-read the last ones and their outputs are dropped; with ONES they are
                    // the ones columns D .. D+7, and their outputs are the sums of the probabilities
                    constexpr int CMAX = C::ONES ? D + 4 : D - 4;
                    col = col <= CMAX ? col : CMAX;
                    const bf16 *v0p = vblk + 16 * t * C::KSTR + col;
                    bf16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((__attribute__((address_space(3))) bf16x4 *)(v0p));
                    bf16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((__attribute__((address_space(3))) bf16x4 *)(v0p + 8 * C::KSTR));
                    bf16x8 a = { v0[0], v0[1], v0[2], v0[3], v1[0], v1[1], v1[2], v1[3] };
                    st.o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, p, st.o[dt], 0, 0, 0);
                }
            }
        }
    }
}

template <int D, int NB, bool RAGGED, bool FULL, typename TabT, bool MIXADD = false, bool RAW = false>
__device__ __forceinline__ void attn_chunk_step(WaveState<D> &st, const bf16x8 *qf, const bf16 *Ks, const bf16 *Vs,
                                                const uint32_t *krc, const int (&blk)[NB], const int (&key0)[NB], int nb_,
                                                int S, float scale_log2e, const TabT *tq_h, const TabT *tq_w)
{
    using C = AttnCfg<D>;
    const int nb = FULL ? NB : nb_;
    const int lane = threadIdx.x & 63, l32 = lane & 31, half = lane >> 5;
    f32x16 s[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        if (b < nb) {
            const bf16 *kblk = Ks + blk[b] * 32 * C::KSTR + l32 * C::KSTR + half * 8;
            const f32x16 zero = { 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f };
#pragma unroll
            for (int ks = 0; ks < C::KS; ++ks) {
                bf16x8 a = *reinterpret_cast<const bf16x8 *>(kblk + ks * 16);
                s[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[ks], ks == 0 ? zero : s[b], 0, 0, 0);
            }
        }
    }
    // the score MFMAs sit behind wave-uniform branches (b < nb): wait their passes out before the reads
    // (the compiler's hazard handling is only relied upon within straight-line code; see the GEMM epilogue)
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
    float mx = -INFINITY;                    // the chunk's own maximum
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        if (b < nb) {
            const unsigned char *tqh = reinterpret_cast<const unsigned char *>(tq_h);
            const unsigned char *tqw = reinterpret_cast<const unsigned char *>(tq_w);
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                if (RAGGED && key0[b] + 8 * g >= S) {      // all eight keys of this register group lie past S (wave-uniform)
#pragma unroll
                    for (int e = 0; e < 4; ++e) s[b][4 * g + e] = -INFINITY;
                    continue;
                }
                const u32x4 rc = *reinterpret_cast<const u32x4 *>(krc + blk[b] * 32 + 8 * g + 4 * half);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int r = 4 * g + e;
                    const uint32_t c = rc[e];
                    const float bh = (float)*reinterpret_cast<const TabT *>(tqh + (c & 0xffffu));
                    float val;
                    if constexpr (MIXADD) {
                        static_assert(sizeof(TabT) == 2, "bias tables are fp16");
                        const uint32_t bw16 = *reinterpret_cast<const uint16_t *>(tqw + (c >> 16));
                        val = RAW ? s[b][r] + bh : s[b][r] * scale_log2e + bh;   // the compiler forms this mixed op by itself
                        asm("v_fma_mix_f32 %0, %1, 1.0, %2 op_sel_hi:[1,0,0]" : "=v"(val) : "v"(bw16), "v"(val));
                    } else {
                        const float bw = (float)*reinterpret_cast<const TabT *>(tqw + (c >> 16));
                        val = RAW ? s[b][r] + bh + bw : s[b][r] * scale_log2e + bh + bw;
                    }
                    if (RAGGED) val = (key0[b] + 8 * g + 4 * half + e < S) ? val : -INFINITY;
                    s[b][r] = val;
                    mx = fmaxf(mx, val);
                }
            }
        }
    }
    attn_softmax_pv<D, NB, FULL, RAW>(st, s, mx, Vs, blk, nb_, scale_log2e);
}

// Scores of a chunk whose 32-key blocks are 4 x 8 patches of stride 2 in the grid: key k of a block (bits c0 r1'.. in
// scan order: bit 0 and bits 2, 4 count columns, bits 1 and 3 rows, i.e. a Z-order walk) sits 2*rr(k) rows and 2*cc(k)
// columns from the block's first key.  That is how the position-only Stripe-Sort order (Sec. 4.1: Z-order, then the
// stripe interleave with G = 4, which collects the cells of one row and column parity) lays out a power-of-two grid.
// The decomposed bias of such a block is a product: B[k][q] = sum_f E[k][f] T[f][q] with E the 0/1 matrix that
// picks a key's row entry (f = rr) and column entry (f = 4 + cc) and T the 4 row and 8 column entries of every
// query, which are contiguous in the query's table row (build_bias_rows).  So the bias is ONE more MFMA (fp16
// operands, the same fp32 accumulator, issued first) and the vector unit does no look-ups and no additions.
//   efrag:  the lane's part of E (operand a; the same for every block)
//   blkoff: LDS, per block of the tile the table offsets of its first key (as in krc)
//   tq_lane: this lane's query row of the table
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
template <int D, int NB>
__device__ __forceinline__ void attn_chunk_step_patch(WaveState<D> &st, const bf16x8 *qf, const bf16 *Ks, const bf16 *Vs,
                                                      const uint32_t *blkoff, const int (&blk)[NB], const f16x8 &efrag,
                                                      const unsigned char *tq_lane, float scale_log2e)
{
    using C = AttnCfg<D>;
    const int lane = threadIdx.x & 63, l32 = lane & 31, half = lane >> 5;
    f32x16 s[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        // operand b of the bias product: f = 8*half + e; f 0..3 the block's rows, 4..11 its columns, 12..15 meet zeros
        // of E (whatever finite values the second read of the upper half-wave returns)
        const uint32_t bo = blkoff[blk[b]];
        const f16x4 t1 = *reinterpret_cast<const f16x4 *>(tq_lane + (half ? (bo >> 16) + 8 : (bo & 0xffffu)));
        const f16x4 t2 = *reinterpret_cast<const f16x4 *>(tq_lane + (bo >> 16));
        const f16x8 tf = { t1[0], t1[1], t1[2], t1[3], t2[0], t2[1], t2[2], t2[3] };
        const f32x16 zero = { 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f };
        s[b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(efrag, tf, zero, 0, 0, 0);
        const bf16 *kblk = Ks + blk[b] * 32 * C::KSTR + l32 * C::KSTR + half * 8;
#pragma unroll
        for (int ks = 0; ks < C::KS; ++ks) {
            bf16x8 a = *reinterpret_cast<const bf16x8 *>(kblk + ks * 16);
            s[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[ks], s[b], 0, 0, 0);
        }
    }
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
    float mx = -INFINITY;
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[b][r]);
    attn_softmax_pv<D, NB, true, true>(st, s, mx, Vs, blk, NB, scale_log2e);
}

// row and column steps (in units of 2 cells) of key k of a patch block from the block's first key
__device__ __forceinline__ int patch_rr(int k) { return ((k >> 1) & 1) | ((k >> 2) & 2); }
__device__ __forceinline__ int patch_cc(int k) { return (k & 1) | ((k >> 1) & 2) | ((k >> 2) & 4); }

template <int D, int NB, typename TabT>
__device__ __forceinline__ void attn_chunk(WaveState<D> &st, const bf16x8 *qf, const bf16 *Ks, const bf16 *Vs,
                                           const uint32_t *krc, const int (&blk)[NB], const int (&key0)[NB], int nb,
                                           bool ragged, int S, float scale_log2e, const TabT *tq_h, const TabT *tq_w)
{
    if (nb == NB) {
        if (ragged) attn_chunk_step<D, NB, true, true, TabT, true>(st, qf, Ks, Vs, krc, blk, key0, nb, S, scale_log2e, tq_h, tq_w);
        else attn_chunk_step<D, NB, false, true, TabT, true>(st, qf, Ks, Vs, krc, blk, key0, nb, S, scale_log2e, tq_h, tq_w);
    } else {
        if (ragged) attn_chunk_step<D, NB, true, false, TabT, true>(st, qf, Ks, Vs, krc, blk, key0, nb, S, scale_log2e, tq_h, tq_w);
        else attn_chunk_step<D, NB, false, false, TabT, true>(st, qf, Ks, Vs, krc, blk, key0, nb, S, scale_log2e, tq_h, tq_w);
    }
}

template <int D>
__device__ __forceinline__ void load_q_frags(bf16x8 *qf, const bf16 *qrow)
{
    const int half = (threadIdx.x & 63) >> 5;
#pragma unroll
    for (int ks = 0; ks < AttnCfg<D>::KS; ++ks)
        qf[ks] = *reinterpret_cast<const bf16x8 *>(qrow + ks * 16 + half * 8);
}

// Normalise the wave's 32 x D output tile and write it out.  The accumulators hold O^T (lane = query,
// registers = 4-feature groups); the tile goes through a per-wave LDS staging area ([32][STR] bf16) so
// that the global stores are 16 bytes per lane and cover whole rows.  `stage` may overlay LDS that only
// this wave used (its bias rows).  out_head: the output tensor at this head's columns; my_row: the output
// row of this lane's query (l & 31), negative = not stored (past S, or dropped by the row map).
template <int D, int STR = AttnCfg<D>::KSTR>
__device__ __forceinline__ void finish_and_store(WaveState<D> &st, bf16 *stage, bf16 *out_head, long out_stride, long my_row)
{
    using C = AttnCfg<D>;        // STR: row stride of the staging area in elements
    const int lane = threadIdx.x & 63, l32 = lane & 31, half = lane >> 5;
    // the last P V MFMAs may still be in flight and this point is reached through loop-exit branches:
    // wait their passes out explicitly before the accumulators are read (see the GEMM epilogue)
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
    // ONES: row 16 + 4*half of the last tile of O^T is a ones column's output: the whole sum, in both half-waves
    const float l = C::ONES ? st.o[C::DT - 1][8] : st.l + __shfl_xor(st.l, 32, 64);
    const float inv = 1.0f / l;
#pragma unroll
    for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            int dd = dt * 32 + 8 * g + 4 * half;
            if (dd < D) {
                uint2 pk;
                pk.x = pack_bf16x2(st.o[dt][4 * g + 0] * inv, st.o[dt][4 * g + 1] * inv);
                pk.y = pack_bf16x2(st.o[dt][4 * g + 2] * inv, st.o[dt][4 * g + 3] * inv);
                *reinterpret_cast<uint2 *>(stage + l32 * STR + dd) = pk;
            }
        }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");      // LDS is in order per wave; keep the compiler from reordering
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const int row_lo = (int)my_row, row_hi = (int)(my_row >> 32);
#pragma unroll
    for (int i = 0; i < (32 * C::CH + 63) / 64; ++i) {
        int id = lane + 64 * i, row = id / C::CH, c = id % C::CH;
        row = row < 32 ? row : 31;
        const long orow = ((long)__shfl(row_hi, row, 64) << 32) | (unsigned)__shfl(row_lo, row, 64);   // lane `row` holds query `row`
        if (id < 32 * C::CH && orow >= 0) {
            u32x4 v = *reinterpret_cast<const u32x4 *>(stage + row * STR + c * 8);
            *reinterpret_cast<u32x4 *>(out_head + orow * out_stride + c * 8) = v;
        }
    }
}

__device__ __forceinline__ uint32_t cell_row_col(int cell, int w)
{
    cell = min(max(cell, 0), w * w - 1);
    return (uint32_t)(cell / w) | ((uint32_t)(cell % w) << 16);
}

__device__ __forceinline__ uint32_t key_row_col(const int32_t *sigma, int p, int S, int w)
{
    return cell_row_col(sigma[p < S ? p : S - 1], w);
}

// byte offsets of a cell's two entries within a query's row of the global kernel's bias table (row part in the low
// half, column part in the high half; see build_bias_rows)
__device__ __forceinline__ uint32_t cell_bias_offsets(int cell, int w)
{
    const uint32_t rc = cell_row_col(cell, w), esz = sizeof(_Float16);
    const uint32_t hw = (uint32_t)(w + 1) >> 1, row = rc & 0xffffu, col = rc >> 16;
    return (esz * ((row & 1) * hw + (row >> 1))) | ((esz * (2 * hw + (col & 1) * hw + (col >> 1))) << 16);
}

// window kernel: byte offsets of the key's entries within a query's two table rows, less the query's own part
__device__ __forceinline__ uint32_t key_bias_offsets_window(const int32_t *sigma, int p, int S, int w)
{
    uint32_t rc = key_row_col(sigma, p, S, w);
    const uint32_t esz = sizeof(WinTab);
    return (esz * (uint32_t)(w - 1 - (int)(rc & 0xffffu))) | ((esz * (uint32_t)(w - 1 - (int)(rc >> 16))) << 16);
}

// per-wave LDS scratch of the global kernel: the bias table of its 32 queries (rows of tstr fp16), later overlaid by
// its output staging tile
template <int D>
__host__ __device__ inline int wave_scratch_bytes(int tstr)
{
    int bias = 32 * tstr * 2, stage = 32 * AttnCfg<D>::KSTR * 2;
    return ((bias > stage ? bias : stage) + 15) & ~15;
}

// ------------------------------------------------------------------ window kernel
inline int window_rel_rows(int w) { return ((2 * w - 1 + 31) / 32) * 32; }

// per-wave LDS landing area of the next problem's queries: the KS operand-b fragments of the wave's 32 queries
template <int D>
__host__ __device__ constexpr int window_q_bytes() { return AttnCfg<D>::KS * 1024; }

// LDS of a gfx950 compute unit.  A compile-time layout choice below is made for it; the launch itself checks the
// size the device reports.
constexpr long GFX950_LDS_BYTES = 160 * 1024;

// Row stride of the output staging tile: padded like the K and V rows (conflict-free 8-byte stores) when a
// 7-tile window then still fits the LDS, else the bare D (d = 80).
template <int D>
__host__ __device__ constexpr int window_stage_stride()
{
    constexpr int KSTR = AttnCfg<D>::KSTR, bias = 2 * 32 * WIN_TSTR * (int)sizeof(WinTab), stage = 32 * KSTR * 2;
    constexpr long total = 7L * window_q_bytes<D>() + 2L * 224 * KSTR * 2 + 2L * 32 * KSTR * 2 +
                           7L * (bias > stage ? bias : stage) + 224 * 4;
    return total <= GFX950_LDS_BYTES ? KSTR : D;
}

template <int D>
__host__ __device__ inline int window_scratch_bytes()
{
    int bias = 2 * 32 * WIN_TSTR * (int)sizeof(WinTab), stage = 32 * window_stage_stride<D>() * 2;
    return ((bias > stage ? bias : stage) + 15) & ~15;
}

template <int D>
size_t window_lds_bytes(int nqb, int w)
{
    int SP = nqb * 32;
    return (size_t)nqb * window_q_bytes<D>() + (size_t)2 * SP * AttnCfg<D>::KSTR * 2 +
           (size_t)2 * window_rel_rows(w) * AttnCfg<D>::KSTR * 2 + (size_t)nqb * window_scratch_bytes<D>() + (size_t)SP * 4;
}

constexpr int WIN_NB = 1;            // key blocks per softmax chunk in the window kernel: one (with two the kernel has no
                                     // registers left for the ragged-block and mixed-add savings, and is no faster)
constexpr int WIN_MAX_LOADS = 5;     // 16-byte K (and V) chunks per thread: 224 keys * 10 chunks / 448 threads

template <int D>
__global__ void __launch_bounds__(448)
attn_window_kernel(AttnParams P, int n_groups)
{
    using C = AttnCfg<D>;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int nqb = blockDim.x >> 6, SP = nqb * 32;
    const int nrel = 2 * P.w - 1, rrows = ((nrel + 31) / 32) * 32;      // nrel <= 32 (checked on the host)
    bf16 *Qs = reinterpret_cast<bf16 *>(smem);    // [nqb][KS][64 lanes][8]: query fragments, one problem ahead (first in LDS)
    bf16 *Ks = Qs + nqb * (window_q_bytes<D>() / 2);
    bf16 *Vs = Ks + SP * C::KSTR;
    bf16 *Rh = Vs + SP * C::KSTR;                 // rel-pos tables, zero-padded to rrows rows
    bf16 *Rw = Rh + rrows * C::KSTR;
    unsigned char *T = reinterpret_cast<unsigned char *>(Rw + rrows * C::KSTR);
    const int wsb = window_scratch_bytes<D>();
    uint32_t *krc = reinterpret_cast<uint32_t *>(T + nqb * wsb);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31;
    const int S = P.S;
    const int nloads = (SP * C::CH + blockDim.x - 1) / blockDim.x;     // <= WIN_MAX_LOADS (checked on the host)

    // problem-independent state: scan-order geometry and the rel-pos tables
    if (P.sigma_stride == 0)
        for (int p = tid; p < SP; p += blockDim.x) krc[p] = key_bias_offsets_window(P.sigma, p, S, P.w);
    for (int id = tid; id < 2 * rrows * C::CH; id += blockDim.x) {
        int tab = id / (rrows * C::CH), rem = id % (rrows * C::CH), row = rem / C::CH, c = rem % C::CH;
        u32x4 v = { 0, 0, 0, 0 };
        if (row < nrel) v = *reinterpret_cast<const u32x4 *>((tab ? P.rel_w : P.rel_h) + (long)row * D + c * 8);
        *reinterpret_cast<u32x4 *>((tab ? Rw : Rh) + row * C::KSTR + c * 8) = v;
    }
    set_ones_columns<D>(Vs, SP, tid, (int)blockDim.x);
    const int q0 = wave * 32, qpos = q0 + l32;
    const int qclamp = qpos < S ? qpos : S - 1;
    uint32_t qrc = key_row_col(P.sigma, qclamp, S, P.w);
    WinTab *tq = reinterpret_cast<WinTab *>(T + wave * wsb);
    const int nact = P.n_pre + (wave >= P.n_pre ? 1 : 0);

    u32x4 rk[WIN_MAX_LOADS], rv[WIN_MAX_LOADS];
    bf16x8 qf[C::KS];
    int32_t row_next = -1;
    bf16 *q_mine = Qs + wave * (window_q_bytes<D>() / 2) + lane * 8;        // this lane's slot in fragment 0
    const uint32_t q_lds = __builtin_amdgcn_readfirstlane(
        (uint32_t)(size_t)(__attribute__((address_space(3))) bf16 *)(Qs + wave * (window_q_bytes<D>() / 2)));

    // The next problem's operands are requested in three pieces (K, V here, Q below) spread over the current problem's
    // phases: a CU keeps only so many cache-line requests in flight, and a wave that issues all of its loads
    // at once sits in the issue queue behind the other waves' loads instead of computing.
#define WIN_PREFETCH(prob_, WHAT)                                                                       \
    {                                                                                                   \
        __builtin_amdgcn_sched_barrier(0);                                                              \
        const int g_ = (prob_) / P.h, hd_ = (prob_) % P.h;                                              \
        const long base_ = (long)g_ * S * P.row_stride + (long)hd_ * D;                                 \
        /* K and V of a problem are read exactly once: non-temporal loads, so that they do not displace the      \
           residual stream and the attention output that the next kernels read (0.8 % of a ViT-H step) */         \
        if ((WHAT) & 3) {                                                                               \
            _Pragma("unroll") for (int i = 0; i < WIN_MAX_LOADS; ++i)                                   \
            {                                                                                           \
                int id = tid + i * (int)blockDim.x, key = id / C::CH, c = id % C::CH;                   \
                key = key < S ? key : S - 1; /* pad keys repeat the last row: finite values, masked */  \
                if (i < nloads && ((WHAT) & 1))                                                         \
                    rk[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(P.k + base_ + (long)key * P.row_stride + c * 8)); \
                if (i < nloads && ((WHAT) & 2))                                                         \
                    rv[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(P.v + base_ + (long)key * P.row_stride + c * 8)); \
            }                                                                                           \
        }                                                                                               \
        if (((WHAT) & 1) && P.out_rows != nullptr && qpos < S) row_next = P.out_rows[(long)g_ * S + qpos]; \
        __builtin_amdgcn_sched_barrier(0);                                                              \
    }
    // The queries of a problem do not pass through registers: 16-byte loads with an LDS destination drop fragment
    // ks of the wave's 32 queries into its landing area (lane l's 16 bytes at 16*l, the layout operand b wants)
    // while the problem before it is still in its chunk loop, which has no registers to spare for them.  The
    // compiler does not see these requests; the kernel waits for them itself before it reads the landing area.
    // The wait in front makes sure the LDS reads of the current fragments have returned.
#define WIN_PREFETCH_Q(prob_)                                                                           \
    {                                                                                                   \
        __builtin_amdgcn_sched_barrier(0);                                                              \
        const int g_ = (prob_) / P.h, hd_ = (prob_) % P.h;                                              \
        const bf16 *qsrc_ = P.q + (long)g_ * S * P.row_stride + (long)hd_ * D + (long)qclamp * P.row_stride + (lane >> 5) * 8; \
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");                                              \
        _Pragma("unroll") for (int ks = 0; ks < C::KS; ++ks)                                            \
            asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off"                          \
                         :: "s"(q_lds + ks * 1024), "v"(qsrc_ + ks * 16) : "m0", "memory");             \
        __builtin_amdgcn_sched_barrier(0);                                                              \
    }

    // Problems are dealt so that the heads of one window run on one XCD (workgroup b sits on XCD b & 7):
    // a head's rows are 2*D bytes at a stride of the packed row, so neighbouring heads share cache lines,
    // and those are then fetched into one L2 instead of eight.  XCD x takes windows x, x+8, ..., heads fastest.
    const int xcd = blockIdx.x & 7, nslots = ((int)gridDim.x - xcd + 7) >> 3;
    auto local_problem = [&](int lp) { int g = xcd + 8 * (lp / P.h); return g < n_groups ? g * P.h + lp % P.h : -1; };
    int lp = blockIdx.x >> 3;
    int prob = local_problem(lp);
    if (prob >= 0) {
        WIN_PREFETCH_Q(prob)
        WIN_PREFETCH(prob, 3)
    }
    for (; prob >= 0; lp += nslots, prob = local_problem(lp)) {
        const int grp = prob / P.h, head = prob % P.h;
        long my_row = -1;                         // output row of this lane's query (a mapped row was requested a problem ahead)
        if (qpos < S) my_row = P.out_rows ? (long)row_next : (long)grp * S + qpos;
        LDS_BARRIER();                            // every wave is done with the previous problem's LDS (output stores stay in flight)
#pragma unroll
        for (int i = 0; i < WIN_MAX_LOADS; ++i) {
            int id = tid + i * (int)blockDim.x, key = id / C::CH, c = id % C::CH;
            if (i < nloads && id < SP * C::CH) {
                *reinterpret_cast<u32x4 *>(Ks + key * C::KSTR + c * 8) = rk[i];
                *reinterpret_cast<u32x4 *>(Vs + key * C::KSTR + c * 8) = rv[i];
            }
        }
        if (P.sigma_stride != 0) {                // per-group order: this window's own sigma
            const int32_t *sg = P.sigma + (long)grp * P.sigma_stride;
            for (int p = tid; p < SP; p += blockDim.x) krc[p] = key_bias_offsets_window(sg, p, S, P.w);
            qrc = key_row_col(sg, qclamp, S, P.w);
        }
        // this problem's queries were sent to LDS during the previous problem (WIN_PREFETCH_Q): wait for every
        // outstanding request of this wave (the K and V registers above have been waited for already; what else is
        // in flight is the previous problem's output stores) before reading them
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
        for (int ks = 0; ks < C::KS; ++ks) qf[ks] = *reinterpret_cast<const bf16x8 *>(q_mine + ks * 512);
        const int next = local_problem(lp + nslots);
        if (next >= 0) WIN_PREFETCH(next, 1)
        build_bias_rows_window<D>(qf, Rh, Rw, C::KSTR, tq);
        const WinTab *tq_h = tq + l32 * WIN_TSTR + (int)(qrc & 0xffffu);            // this lane's query in the two tables
        const WinTab *tq_w = tq + (32 + l32) * WIN_TSTR + (int)(qrc >> 16);
        LDS_BARRIER();
        if (next >= 0) WIN_PREFETCH(next, 2)

        WaveState<D> st;
        init_state<D>(st);
        // active key tiles of query tile `wave`: the dense prefix, then the diagonal; chunks of WIN_NB
        for (int a0 = 0; a0 < nact; a0 += WIN_NB) {
            int blk[WIN_NB], key0[WIN_NB];
#pragma unroll
            for (int b = 0; b < WIN_NB; ++b) {
                int a = a0 + b;
                blk[b] = a < P.n_pre ? a : wave;
                key0[b] = blk[b] * 32;
            }
            // only the last 32-key tile of the window can cross S
            bool ragged = false;
#pragma unroll
            for (int b = 0; b < WIN_NB; ++b) ragged |= (a0 + b < nact) && key0[b] + 32 > S;
            attn_chunk<D, WIN_NB, WinTab>(st, qf, Ks, Vs, krc, blk, key0, min(WIN_NB, nact - a0), ragged, S, P.scale_log2e, tq_h, tq_w);
            // after the second chunk (the only one, when the tile has one): early enough to cover the request's
            // latency with the last chunk and the output stores on the tiles that have three, and not in the same
            // burst as the K or the V requests
            if (a0 == (nact > WIN_NB ? WIN_NB : 0) && next >= 0) WIN_PREFETCH_Q(next)
        }
        finish_and_store<D, window_stage_stride<D>()>(st, reinterpret_cast<bf16 *>(tq), P.out + (long)head * D, (long)P.h * D, my_row);
    }
}

// ------------------------------------------------------------------ global kernel
constexpr int GLB_TILE = 128;
// key blocks per softmax chunk: the register budget of two waves per SIMD allows 2 at d = 80 and 4 up to d = 64
// (the chunk step specialised for full chunks spills in this kernel at either size)
template <int D> constexpr int glb_nb() { return D <= 64 ? 4 : 2; }
// Bias rows of the global kernel are held as fp16 (11 significant bits on log2e * q.r, below the bf16
// rounding of the probabilities that feed the second product): at w = 64 that brings a workgroup to
// 78 KB of LDS, so two workgroups share a CU and one hides the other's LDS, MFMA and barrier latency.
typedef _Float16 GlbTab;

template <int D>
size_t global_lds_bytes(int w)
{
    // K and V tile, the four waves' bias tables, per key (or per block) table offsets
    return (size_t)2 * GLB_TILE * AttnCfg<D>::KSTR * 2 + (size_t)4 * wave_scratch_bytes<D>(glb_tstr(w)) + (size_t)GLB_TILE * 4;
}

// Everything a workgroup of the global kernel does once it knows which way its scores are formed.
// PATCHED: every block of every tile this workgroup visits is a patch (attn_chunk_step_patch: bias by MFMA);
// otherwise the general path (per-key table look-ups, any order).
template <int D, bool PATCHED>
__device__ __forceinline__ void attn_global_body(const AttnParams &P, int qt, int grp, int head, float inv_scale, unsigned char *smem)
{
    using C = AttnCfg<D>;
    constexpr int LOADS = GLB_TILE * C::CH / 256;       // 16-byte chunks per thread per operand
    static_assert(GLB_TILE * C::CH % 256 == 0, "tile chunks must divide over the workgroup");
    const int tstr = glb_tstr(P.w);
    bf16 *Ks = reinterpret_cast<bf16 *>(smem);
    bf16 *Vs = Ks + GLB_TILE * C::KSTR;
    unsigned char *Tb = reinterpret_cast<unsigned char *>(Vs + GLB_TILE * C::KSTR);
    const int wsb = wave_scratch_bytes<D>(tstr);
    uint32_t *krc = reinterpret_cast<uint32_t *>(Tb + 4 * wsb);    // [128] per key (general) or [4] per block (patches)

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, half = lane >> 5;
    const int S = P.S;
    const long base = (long)grp * S * P.row_stride + (long)head * D;

    const int qpos = qt * GLB_TILE + wave * 32 + l32;
    const int qclamp = qpos < S ? qpos : S - 1;
    bf16x8 qf[C::KS];
    load_q_frags<D>(qf, P.q + base + (long)qclamp * P.row_stride);
    const int32_t *sg = P.sigma + (long)grp * P.sigma_stride;
    const uint32_t qrc = key_row_col(sg, qclamp, S, P.w);
    long my_row = -1;                             // output row of this lane's query
    if (qpos < S) {
        my_row = (long)grp * S + qpos;
        if (P.out_rows) my_row = P.out_rows[my_row];
    }
    GlbTab *tq = reinterpret_cast<GlbTab *>(Tb + wave * wsb);
    GlbTab *tq_lane = tq + l32 * tstr;            // this lane's query row of the wave's bias table

    constexpr int NB = glb_nb<D>();
    const int nact = P.n_pre + (qt >= P.n_pre ? 1 : 0);
    u32x4 rk[LOADS], rv[LOADS];
    int rcell = 0;
    // this (image, head)'s K and V: a uniform base and 32-bit byte offsets (S * row_stride * 2 < 2^31, checked on the host)
    const unsigned char *kbase = reinterpret_cast<const unsigned char *>(P.k + base);
    const unsigned char *vbase = reinterpret_cast<const unsigned char *>(P.v + base);
    const uint32_t rs2 = (uint32_t)P.row_stride * 2u;

    // operand a of the bias product of patch blocks: lane (key l32, half) holds E[l32][8*half + e]
    f16x8 efrag;
    if constexpr (PATCHED) {
        const int rr = patch_rr(l32), cc = patch_cc(l32);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int f = 8 * half + e;
            efrag[e] = (_Float16)((f < 4 ? rr == f : (f < 12 ? cc == f - 4 : false)) ? 1.f : 0.f);
        }
    }

    // WHAT: 1 = K and the keys' cells, 2 = V; the two halves are requested at different points of the
    // current tile's work so that the waves do not queue up behind each other's loads.  With patches only the
    // first key of each block is looked up.
#define ATTN_LOAD_TILE(kt_, WHAT)                                                                       \
    {                                                                                                   \
        __builtin_amdgcn_sched_barrier(0);                                                              \
        const int key0_ = (kt_) * GLB_TILE;                                                             \
        _Pragma("unroll") for (int i = 0; i < LOADS; ++i)                                               \
        {                                                                                               \
            const int id = tid + i * 256, kl = id / C::CH, c = id - kl * C::CH;                         \
            /* keys past S repeat the last row (masked in the scores); 32-bit byte offset from a uniform base */ \
            const uint32_t off_ = (uint32_t)min(key0_ + kl, S - 1) * rs2 + (uint32_t)c * 16u;           \
            if ((WHAT) & 1) rk[i] = *reinterpret_cast<const u32x4 *>(kbase + off_);                     \
            if ((WHAT) & 2) rv[i] = *reinterpret_cast<const u32x4 *>(vbase + off_);                     \
        }                                                                                               \
        if (((WHAT) & 1) && tid < (PATCHED ? GLB_TILE / 32 : GLB_TILE))                                 \
            rcell = sg[min(key0_ + (PATCHED ? 32 * tid : tid), S - 1)]; /* used at the LDS store, not before */ \
        __builtin_amdgcn_sched_barrier(0);                                                              \
    }
#define ATTN_STORE_TILE()                                                                               \
    {                                                                                                   \
        _Pragma("unroll") for (int i = 0; i < LOADS; ++i)                                               \
        {                                                                                               \
            int id = tid + i * 256, key = id / C::CH, c = id % C::CH;                                   \
            *reinterpret_cast<u32x4 *>(Ks + key * C::KSTR + c * 8) = rk[i];                             \
            *reinterpret_cast<u32x4 *>(Vs + key * C::KSTR + c * 8) = rv[i];                             \
        }                                                                                               \
        if (tid < (PATCHED ? GLB_TILE / 32 : GLB_TILE)) krc[tid] = cell_bias_offsets(rcell, P.w);      \
    }

    ATTN_LOAD_TILE(0 < P.n_pre ? 0 : qt, 3)       // in flight while the bias rows are formed
    set_ones_columns<D>(Vs, GLB_TILE, tid, 256);
    build_bias_rows<D, GlbTab>(qf, P.rel_h, P.rel_w, D, P.w, (int)(qrc & 0xffffu), (int)(qrc >> 16), tq_lane, inv_scale);

    WaveState<D> st;
    init_state<D>(st);
    for (int a = 0; a < nact; ++a) {
        const int kt = a < P.n_pre ? a : qt;
        LDS_BARRIER();                         // every wave is done with the previous tile
        ATTN_STORE_TILE()
        LDS_BARRIER();
        const int kt_next = a + 1 < P.n_pre ? a + 1 : qt;
        if (a + 1 < nact) ATTN_LOAD_TILE(kt_next, NB < GLB_TILE / 32 ? 1 : 3)     // one step per tile: nothing to put V between
        // the softmax / MFMA phase goes ahead of the other workgroup's tile traffic (loads, LDS stores, barriers)
        __builtin_amdgcn_s_setprio(1);
        if constexpr (PATCHED) {
#pragma unroll
            for (int c0 = 0; c0 < GLB_TILE / 32; c0 += NB) {
                int blk[NB];
#pragma unroll
                for (int b = 0; b < NB; ++b) blk[b] = c0 + b;
                attn_chunk_step_patch<D, NB>(st, qf, Ks, Vs, krc, blk, efrag, reinterpret_cast<const unsigned char *>(tq_lane), P.scale_log2e);
                if (NB < GLB_TILE / 32 && c0 == 0 && a + 1 < nact) ATTN_LOAD_TILE(kt_next, 2)
            }
        } else {
            const int nblk = min(GLB_TILE / 32, (S - kt * GLB_TILE + 31) / 32);     // blocks wholly past the end are skipped
#pragma unroll
            for (int c0 = 0; c0 < GLB_TILE / 32; c0 += NB) {
                if (c0 >= nblk) break;
                int blk[NB], key0[NB];
#pragma unroll
                for (int b = 0; b < NB; ++b) { blk[b] = c0 + b; key0[b] = kt * GLB_TILE + 32 * (c0 + b); }
                const int nb = min(NB, nblk - c0);
                const bool ragged = key0[NB - 1] + 32 > S;
                if (ragged)
                    attn_chunk_step<D, NB, true, false, GlbTab, true, true>(st, qf, Ks, Vs, krc, blk, key0, nb, S, P.scale_log2e, tq_lane, tq_lane);
                else
                    attn_chunk_step<D, NB, false, false, GlbTab, true, true>(st, qf, Ks, Vs, krc, blk, key0, nb, S, P.scale_log2e, tq_lane, tq_lane);
                if (NB < GLB_TILE / 32 && c0 == 0 && a + 1 < nact) ATTN_LOAD_TILE(kt_next, 2)
            }
        }
        __builtin_amdgcn_s_setprio(0);
    }
    finish_and_store<D>(st, reinterpret_cast<bf16 *>(tq), P.out + (long)head * D, (long)P.h * D, my_row);
#undef ATTN_LOAD_TILE
#undef ATTN_STORE_TILE
}

// TRY_PATCH: the instantiation for a shared position-only order on a power-of-two grid.  The workgroup first looks at
// the cells of every key it will visit: if every 32-key block is a patch (see attn_chunk_step_patch) it forms the bias
// with the matrix core, otherwise (any table is legal) it takes the general path.  !TRY_PATCH: the general path only.
template <int D, bool TRY_PATCH>
__global__ void __launch_bounds__(256, 2)
attn_global_kernel(AttnParams P, int T, int n_gh, float inv_scale)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    // the query tiles of one (image, head) run on one XCD (workgroup b sits on XCD b & 7), whose L2 then
    // serves the re-reads of that problem's K and V tiles
    const int qt = (blockIdx.x >> 3) % T, gh = ((blockIdx.x >> 3) / T) * 8 + (blockIdx.x & 7);
    if (gh >= n_gh) return;
    const int grp = gh / P.h, head = gh % P.h;
    if constexpr (TRY_PATCH) {
        // A key passes if it lies inside S, sits where the patch anchored at its block's first key puts it (inside the
        // grid), and, for a block's first key, the block's 4 row and 8 column entries start at 8- and 16-byte
        // boundaries of a table row.  256 consecutive keys a pass, the cells of a pass requested together.
        const int tid = threadIdx.x, lane = tid & 63;
        const int32_t *sg = P.sigma + (long)grp * P.sigma_stride;
        const int nact = P.n_pre + (qt >= P.n_pre ? 1 : 0);
        int *flag = reinterpret_cast<int *>(smem);
        if (tid == 0) *flag = 1;
        bool ok = true;
        constexpr int BATCH = 8;                                            // cells per thread per pass: 16 tiles a pass
        for (int a = 0; a < nact; a += 2 * BATCH) {
            int cell[BATCH], key[BATCH];
#pragma unroll
            for (int j = 0; j < BATCH; ++j) {                               // the loads of a pass are in flight together
                const int a1 = min(a + 2 * j + (tid >> 7), nact - 1);       // this thread's tile (past the end: the last one again)
                const int kt = a1 < P.n_pre ? a1 : qt;
                key[j] = kt * GLB_TILE + (tid & 127);
                cell[j] = sg[min(key[j], P.S - 1)];
            }
#pragma unroll
            for (int j = 0; j < BATCH; ++j) {
                const int c0 = __shfl(cell[j], lane & 32, 64);              // cell of the block's first key
                const int k = tid & 31, r0 = c0 / P.w, cl0 = c0 - r0 * P.w;
                bool good = key[j] < P.S && c0 >= 0 && r0 + 6 < P.w && cl0 + 14 < P.w &&
                            cell[j] == c0 + 2 * P.w * patch_rr(k) + 2 * patch_cc(k);
                if (k == 0) {
                    const uint32_t off = cell_bias_offsets(cell[j], P.w);
                    good = good && (off & 7u) == 0 && ((off >> 16) & 15u) == 0;
                }
                ok = ok && good;
            }
        }
        __syncthreads();
        if (!ok) *flag = 0;
        __syncthreads();
        const bool patched = *flag != 0;
        __syncthreads();                        // the flag's word is part of the K tile from here on
        if (patched) {
            attn_global_body<D, true>(P, qt, grp, head, inv_scale, smem);
            return;
        }
    }
    attn_global_body<D, false>(P, qt, grp, head, inv_scale, smem);
}

// CU count and LDS bytes per CU of the current device, asked once per device (host-side queries, no allocation)
struct DeviceShape { int cus; size_t lds; };
inline int device_shape(DeviceShape &out)
{
    static DeviceShape cache[64] = {};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return SSAM_EHIP;
    if (cache[dev].cus == 0) {
        int cus = 0, lds = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) return SSAM_EHIP;
        if (hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerMultiprocessor, dev) != hipSuccess || lds <= 0) return SSAM_EHIP;
        cache[dev].lds = (size_t)lds;
        cache[dev].cus = cus;                    // written last: a racing first call finds 0 and asks again
    }
    out = cache[dev];
    return SSAM_OK;
}

template <int D>
int launch_attention(const AttnParams &P, int groups, int mask_block, float inv_scale, hipStream_t st)
{
    DeviceShape ds;
    if (int rc = device_shape(ds); rc != SSAM_OK) return rc;
    if (mask_block == 32) {
        int nqb = ssam_div_up(P.S, 32);
        size_t lds = window_lds_bytes<D>(nqb, P.w);
        if (lds > ds.lds) return SSAM_EUNSUPPORTED;
        // the queries of the next problem land in LDS through loads whose LDS address is a 16-bit immediate-free M0
        // offset: their landing area is first in LDS and must end below 64 KB
        if ((size_t)nqb * window_q_bytes<D>() > 64 * 1024) return SSAM_EUNSUPPORTED;
        auto kern = attn_window_kernel<D>;
        if (lds > 64 * 1024 &&
            hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
            return SSAM_EHIP;
        if (ssam_div_up((long)nqb * 32 * AttnCfg<D>::CH, nqb * 64) > WIN_MAX_LOADS) return SSAM_EUNSUPPORTED;
        if (2 * P.w - 1 > 32) return SSAM_EUNSUPPORTED;       // the window bias tables are one 32-row MFMA tile
        int n_problems = groups * P.h;
        // persistent workgroups: as many as fit on the device's CUs at once for this LDS footprint
        int per_cu = (int)(ds.lds / lds);
        if (per_cu < 1) per_cu = 1;
        if (per_cu > 4) per_cu = 4;
        int grid = n_problems < ds.cus * per_cu ? n_problems : ds.cus * per_cu;
        hipLaunchKernelGGL(kern, dim3(grid), dim3(nqb * 64), lds, st, P, groups);
    } else {
        int T = ssam_div_up(P.S, GLB_TILE);
        size_t lds = global_lds_bytes<D>(P.w);
        if (lds > ds.lds) return SSAM_EUNSUPPORTED;
        // a shared table on a power-of-two grid of 16 x 16 or more can be the position-only order whose blocks are
        // patches; the kernel checks every tile, so any table is still handled correctly
        const bool patch = P.sigma_stride == 0 && P.w >= 16 && (P.w & (P.w - 1)) == 0;
        auto kern = patch ? attn_global_kernel<D, true> : attn_global_kernel<D, false>;
        if (lds > 64 * 1024 &&
            hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
            return SSAM_EHIP;
        hipLaunchKernelGGL(kern, dim3((unsigned)((long)T * ssam_div_up(groups * P.h, 8) * 8)), dim3(256), lds, st, P, T, groups * P.h, inv_scale);
    }
    SSAM_CHECK_LAUNCH();
    return SSAM_OK;
}

}  // namespace

extern "C" int ssam_sparse_attention(const void *q, const void *k, const void *v, long row_stride,
                                     const void *rel_h, const void *rel_w, const int32_t *sigma,
                                     long sigma_group_stride, void *out, const int32_t *out_rows,
                                     int groups, int S, int w, int h, int d, int mask_block, double r,
                                     float scale, void *stream)
{
    if (!q || !k || !v || !rel_h || !rel_w || !sigma || !out) return SSAM_EINVAL;
    if (groups <= 0 || S <= 0 || w <= 0 || h <= 0 || d <= 0 || !(r > 0.0) || r > 1.0) return SSAM_EINVAL;
    if (sigma_group_stride != 0 && sigma_group_stride < S) return SSAM_EINVAL;
    if (w * w != S || row_stride < (long)h * d || row_stride % 8 != 0) return SSAM_EINVAL;
    if (!ssam_aligned16(q) || !ssam_aligned16(k) || !ssam_aligned16(v) || !ssam_aligned16(rel_h) ||
        !ssam_aligned16(rel_w) || !ssam_aligned16(out))
        return SSAM_EINVAL;
    if (mask_block == 32) {
        if (S > 224) return SSAM_EUNSUPPORTED;
    } else if (mask_block == 128) {
        if (S > 16384 || (long)ssam_div_up(S, 128) * ((long)groups * h + 7) > 0x7fffffffL) return SSAM_EUNSUPPORTED;
        if ((long)S * row_stride * 2 > 0x7fffffffL) return SSAM_EUNSUPPORTED;      // the kernel's 32-bit byte offsets within a group
    } else {
        return SSAM_EUNSUPPORTED;
    }
    if (w > 128) return SSAM_EUNSUPPORTED;
    AttnParams P;
    P.q = (const bf16 *)q; P.k = (const bf16 *)k; P.v = (const bf16 *)v;
    P.row_stride = row_stride;
    P.rel_h = (const bf16 *)rel_h; P.rel_w = (const bf16 *)rel_w;
    P.sigma = sigma;
    P.sigma_stride = sigma_group_stride;
    P.out = (bf16 *)out;
    P.out_rows = out_rows;
    P.S = S; P.w = w; P.h = h;
    P.n_pre = ssam_prefix_tiles(ssam_div_up(S, mask_block), r);
    P.scale_log2e = scale * LOG2E;
    if (!(scale > 0.f)) return SSAM_EINVAL;      // the global kernel's bias table holds bias / scale
    const float inv_scale = 1.0f / scale;
    hipStream_t st = (hipStream_t)stream;
    switch (d) {
    case 64: return launch_attention<64>(P, groups, mask_block, inv_scale, st);
    case 80: return launch_attention<80>(P, groups, mask_block, inv_scale, st);
    case 32: return launch_attention<32>(P, groups, mask_block, inv_scale, st);
    case 16: return launch_attention<16>(P, groups, mask_block, inv_scale, st);
    default: return SSAM_EUNSUPPORTED;
    }
}
