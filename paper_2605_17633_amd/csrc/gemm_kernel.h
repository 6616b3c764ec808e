// bf16 NT GEMM for gfx950: C = epilogue(A[M][K] * W[N][K]^T + bias), fp32 accumulation on the
// 16x16x32 bf16 MFMA.  Serves the block's qkv / proj / fc1 / fc2 layers (the dense contractions
// of the SAM block; the routed MLP of Sec. 4.2 reaches it with the gathered keep-set rows as A).
//
// Workgroup = WGM x WGN waves in a grid over a BM x BN tile; each wave owns (BM/WGM) x (BN/WGN) as
// 16x16 MFMA tiles.  The 256x256 tile runs 8 waves (2x4, wave tile 128x64, under 256 VGPRs): two waves
// per SIMD, so one wave's LDS, barrier and MFMA-result latency is covered by the other; the smaller
// tiles run 4 waves and two workgroups per CU.  K is consumed in slabs of 64 (two MFMA k-steps): global ->
// registers (prefetch of the next slab) -> LDS (double buffered; 16-byte chunks XOR-swizzled so that both
// the staging writes and the ds_read_b128 fragment reads are bank-conflict free).  Fragments are
// double buffered in registers and the instruction mix is pinned with sched_group_barrier so that
// LDS reads, global loads and LDS writes sit between MFMAs instead of in front of them; the
// per-slab barrier orders LDS traffic only, so global prefetches stay in flight across it.
// MFMA layout (16x16x32): lane l feeds row (l & 15), the 8 k values of chunk (l >> 4) of the 32; result
// register r of lane l is C[4*(l>>4) + r][l & 15], rows from operand a (activations), columns from b (W).
// Why this shape and not 32x32x16, which needs half as many operand fragments per flop: the chip is power
// limited under matrix load and the shader clock settles where the power budget puts it; the 16x16x32
// instruction reads and writes its fp32 accumulators half as often per flop and draws less: the same loop
// runs at 1.74-1.87 GHz instead of 1.71-1.75 and 8-12 % faster on the block's four layer shapes.
// The epilogue stages 32-row slices of the fp32 result through LDS so that each lane finishes 8
// consecutive columns and issues 16-byte global accesses.
// Tiles are dealt so that each XCD (its own L2) works on a contiguous run of tiles, ordered in
// bands of 8 tile rows: workgroups that run together share A and W panels.
// A launch covers a range [tile_begin, tile_begin + tile_count) of "parent" tiles of (BM*SUB_M) x (BN*SUB_N)
// in that order, each cut into SUB_M x SUB_N tiles of this kernel: the dispatcher runs whole rounds of
// large tiles and hands the few left-over large tiles to a second launch of smaller ones, so that the
// last round of workgroups is short instead of a full large-tile time.  When K is long those few
// workgroups would each walk all of K alone, bound by the latency of one slab after the other, so the
// left-over launch can also cut K into `parts` ranges (epilogue GEMM_EPI_PARTIAL): every workgroup
// leaves its fp32 tile in a workspace slot of its own and gemm_tail_reduce_kernel adds the slots in a
// fixed order and applies the real epilogue (the result does not depend on timing).
#pragma once

#include "common.h"

struct GemmRowMap {
    const int32_t *map;       // NULL unless the epilogue scatters
    int rows_per_batch;
    int map_batch_stride;
    int dst_rows_per_batch;
};

constexpr int GEMM_BK = 64;
constexpr int GEMM_THREADS = 256;

template <int BM, int BN, int WGM = 2, int WGN = 2, bool WPACK = false>
constexpr size_t gemm_lds_bytes()
{
    size_t pipe = (size_t)2 * (BM + (WPACK ? 0 : BN)) * GEMM_BK * sizeof(bf16);
    size_t epi = (size_t)WGM * WGN * 32 * (BN / WGN + 4) * sizeof(float) + BM * (sizeof(int) + sizeof(float2));   // staging + scatter rows + row statistics
    return pipe > epi ? pipe : epi;
}

// element offset of 16-byte chunk c (0..7) of row `row` in a [rows][64] bf16 slab
__device__ __forceinline__ int gemm_swz(int row, int c) { return row * GEMM_BK + ((c ^ ((row >> 1) & 7)) << 3); }

#define GEMM_SGB(mask, n) __builtin_amdgcn_sched_group_barrier(mask, n, 0)

// 16 zero bytes: what a K chunk past the end of a ragged K reads instead of memory
static __device__ const uint4 gemm_zero_chunk[1] = { { 0u, 0u, 0u, 0u } };

struct GemmLd { int a, w, c; };   // row strides of A, W and C in elements (multiples of 8)

struct GemmTileRange {
    int tiles_m, tiles_n;     // parent tile grid
    int tile_begin, tile_count;   // parent tiles of this launch, in band order
};

constexpr int GEMM_EPI_PARTIAL = 8;   // internal: store the fp32 tile of one K range, no bias
constexpr int GEMM_GROUP_M = 8;
constexpr size_t GEMM_SPLIT_WS_BYTES = (size_t)32 << 20;   // workspace that lets the left-over launch cut K

// LayerNorm folded into the contraction that follows it (LNF instantiations): A holds the rows before the
// normalisation, W holds W*diag(gamma), and the epilogue finishes  rstd_m * (acc - mean_m * colsum_n) + bias_n
// with bias_n = b_n + sum_k beta_k W[n][k].  With `src` the rows are also gathered: row m of the product is row
// src[m] of A (the routed MLP's kept tokens, read where they lie in the residual stream).
struct GemmFold {
    const float2 *stats;      // [M] per row of the product: { rstd, -rstd * mean } of the A row it reads
    const float *colsum;      // [N] sum over k of the folded weight as stored (bf16 values, fp32 sum)
    const int32_t *src;       // [M] row of A per row of the product (all inside A), or NULL: row m itself
};

struct GemmSplit {
    float *partial;           // [tile_count*SUB_M*SUB_N][parts][BM][BN] fp32, NULL unless GEMM_EPI_PARTIAL
    int parts;                // K ranges per tile (1 otherwise); parts <= K/64
};

// origin of sub-tile `sub` of parent tile t (band order over the parent grid)
__device__ __forceinline__ void gemm_tile_origin(const GemmTileRange &tr, int t, int sub, int sub_m, int sub_n,
                                                 int bm, int bn, int &m0, int &n0)
{
    const int band = GEMM_GROUP_M * tr.tiles_n;
    const int first_m = (t / band) * GEMM_GROUP_M;
    const int band_rows = min(GEMM_GROUP_M, tr.tiles_m - first_m);
    const int tm = first_m + (t % band) % band_rows;
    const int tn = (t % band) / band_rows;
    m0 = (tm * sub_m + sub / sub_n) * bm;
    n0 = (tn * sub_n + sub % sub_n) * bn;
}

// The workgroup's work, as a function of its index `bid` in the launch (the kernels below pass blockIdx.x, or
// blockIdx.x less the workgroups of another kind that share the launch).
template <int BM, int BN, int EPI, int SUB_M = 1, int SUB_N = 1, int WGM = 2, int WGN = 2, bool WPACK = false, bool LNF = false>
__device__ __forceinline__ void
gemm_bf16_nt_body(const bf16 *__restrict__ A, const bf16 *__restrict__ W, const float *__restrict__ bias,
                  bf16 *C, int M, int N, int K, const GemmLd &ld, const GemmTileRange &tr, const GemmRowMap &rm,
                  const GemmSplit &sp, int bid, const GemmFold &fold = GemmFold{ nullptr, nullptr, nullptr })
{
    static_assert(!LNF || WPACK, "the folded forms exist for packed weights");
    // a K range of a folded product only gathers its rows: the normalisation is finished where the ranges are added
    constexpr bool FOLD_EPI = LNF && EPI != GEMM_EPI_PARTIAL;
    constexpr int THREADS = 64 * WGM * WGN, RSTEP = THREADS / 8;   // waves in a WGM x WGN grid; rows staged per pass
    constexpr int WM = BM / WGM, WN = BN / WGN, MT = WM / 32;       // MT: 32-row slices of the epilogue
    constexpr int MT16 = WM / 16, NT16 = WN / 16;                  // the wave's accumulator tiles (16x16)
    // A slab of 64 holds two MFMA k-steps of 32.  A k-step is issued in HP phases of AF row tiles each, so that only
    // AF operand-a fragments are live per register slot: phase p = (k-step p / HP, row tiles (p % HP)*AF ...).
    constexpr int AF = MT16 < 4 ? MT16 : 4, HP = MT16 / AF, PH = 2 * HP, NP = AF * NT16;
    constexpr int A_LOADS = BM * 8 / THREADS, B_LOADS = BN * 8 / THREADS;
    static_assert(BM % RSTEP == 0 && BN % RSTEP == 0 && RSTEP % 16 == 0, "staging passes must tile the operands");
    static_assert(WM % 32 == 0 && WN % 16 == 0 && MT16 % AF == 0, "wave tile in 16x16 MFMA tiles, epilogue in 32-row slices");
    constexpr int NL = A_LOADS + B_LOADS;
    static_assert((WPACK ? A_LOADS : NL) <= NP, "a phase has an MFMA to put every staging access behind");
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    bf16 *As = reinterpret_cast<bf16 *>(smem);                 // [2][BM*64]
    bf16 *Bs = As + 2 * BM * GEMM_BK;                          // [2][BN*64]

    // ---- tile assignment: workgroups are dealt round-robin to the 8 XCDs; XCD x takes the tiles
    // x*per_xcd .. (x+1)*per_xcd-1 of the band order
    constexpr int SUBS = SUB_M * SUB_N;
    const int parts = EPI == GEMM_EPI_PARTIAL ? sp.parts : 1;
    const int total = tr.tile_count * SUBS * parts;
    const int per_xcd = (total + 7) / 8;
    const int tl = (bid & 7) * per_xcd + (bid >> 3);
    if (tl >= total) return;
    const int kpart = tl % parts, slot = tl / parts;            // slot: sub-tile index within this launch
    int m0, n0;
    gemm_tile_origin(tr, tr.tile_begin + slot / SUBS, slot % SUBS, SUB_M, SUB_N, BM, BN, m0, n0);
    if (m0 >= M) return;                        // a sub-tile wholly below the last row

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = (wave / WGN) * WM, wn = (wave % WGN) * WN;
    const int l16 = lane & 15, quad = lane >> 4;
    const int nk = (K + GEMM_BK - 1) / GEMM_BK;          // a ragged last slab reads zeros past K (K % 8 == 0)
    const int kb = (int)((long)nk * kpart / parts), ke = (int)((long)nk * (kpart + 1) / parts);   // this workgroup's slabs

    f32x4 acc[MT16][NT16];
#pragma unroll
    for (int i = 0; i < MT16; ++i)
#pragma unroll
        for (int j = 0; j < NT16; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[i][j][r] = 0.f;

    u32x4 ra[A_LOADS], rb[B_LOADS];
    bf16x8 af[2][AF], bw[2][NT16];          // operand a: one slot per phase parity; operand b: one slot per k-step

    // staging: thread owns chunk c0 of rows r0 + RSTEP*i of both operands
    const int r0 = tid >> 3, c0 = tid & 7;
    const bf16 *ga[A_LOADS];
#pragma unroll
    for (int i = 0; i < A_LOADS; ++i) {        // rows past M repeat the last row; their results are never stored
        long arow = min(m0 + r0 + RSTEP * i, M - 1);
        if constexpr (LNF) if (fold.src) arow = fold.src[arow];
        ga[i] = A + arow * ld.a + c0 * 8;
    }
    const bf16 *gb[B_LOADS];
#pragma unroll
    for (int i = 0; i < B_LOADS; ++i)          // likewise columns past N (a ragged last tile column)
        gb[i] = W + (long)min(n0 + r0 + RSTEP * i, N - 1) * ld.w + c0 * 8;
    const bf16 *zchunk = reinterpret_cast<const bf16 *>(gemm_zero_chunk);
    const int lst = gemm_swz(r0, c0);          // + i*RSTEP*64: rows a multiple of 16 apart share the swizzle term
    // fragment reads: lane (l16, quad) takes the 16-byte chunk 4*s + quad of row l16 of a 16-row tile; the 16 lanes of
    // a quad touch 8 swizzled chunk positions x 2 row parities = all 64 banks once
    const int fa0 = (wm + l16) * GEMM_BK, fb0 = (wn + l16) * GEMM_BK;
    const int sw = l16 >> 1;

#define GEMM_LOAD_GLOBAL(kt_)                                                                         \
    {                                                                                                 \
        const bool kin_ = (kt_) * GEMM_BK + c0 * 8 < K;                                               \
        _Pragma("unroll") for (int i = 0; i < A_LOADS; ++i)                                           \
            ra[i] = *reinterpret_cast<const u32x4 *>(kin_ ? ga[i] + (kt_) * GEMM_BK : zchunk);        \
        _Pragma("unroll") for (int i = 0; i < B_LOADS; ++i)                                           \
            rb[i] = *reinterpret_cast<const u32x4 *>(kin_ ? gb[i] + (kt_) * GEMM_BK : zchunk);        \
    }
#define GEMM_STORE_LDS(buf_)                                                                          \
    {                                                                                                 \
        bf16 *as_ = As + (buf_) * BM * GEMM_BK + lst, *bs_ = Bs + (buf_) * BN * GEMM_BK + lst;        \
        _Pragma("unroll") for (int i = 0; i < A_LOADS; ++i)                                           \
            *reinterpret_cast<u32x4 *>(as_ + i * RSTEP * GEMM_BK) = ra[i];                               \
        _Pragma("unroll") for (int i = 0; i < B_LOADS; ++i)                                           \
            *reinterpret_cast<u32x4 *>(bs_ + i * RSTEP * GEMM_BK) = rb[i];                               \
    }
// operand-a fragments of phase p_ into register slot slot_
#define GEMM_LOAD_AFRAGS(buf_, p_, slot_)                                                             \
    {                                                                                                 \
        const bf16 *as_ = As + (buf_) * BM * GEMM_BK + fa0 + (((p_) % HP) * AF) * 16 * GEMM_BK        \
                          + (((((p_) / HP) * 4 + quad) ^ sw) << 3);                                   \
        _Pragma("unroll") for (int i = 0; i < AF; ++i)                                                \
            af[slot_][i] = *reinterpret_cast<const bf16x8 *>(as_ + i * 16 * GEMM_BK);                 \
    }
// operand-b fragments of k-step s_ from LDS (row-major weights)
#define GEMM_LOAD_BFRAGS(buf_, s_)                                                                    \
    {                                                                                                 \
        const bf16 *bs_ = Bs + (buf_) * BN * GEMM_BK + fb0 + ((((s_) * 4 + quad) ^ sw) << 3);         \
        _Pragma("unroll") for (int j = 0; j < NT16; ++j)                                              \
            bw[s_][j] = *reinterpret_cast<const bf16x8 *>(bs_ + j * 16 * GEMM_BK);                    \
    }
#define GEMM_MFMAS(p_, slot_)                                                                         \
    {                                                                                                 \
        _Pragma("unroll") for (int i = 0; i < AF; ++i)                                                \
            _Pragma("unroll") for (int j = 0; j < NT16; ++j)                                          \
                acc[((p_) % HP) * AF + i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(               \
                    af[slot_][i], bw[(p_) / HP][j], acc[((p_) % HP) * AF + i][j], 0, 0, 0);           \
    }

    int buf = 0;
    if (WPACK) {
        // W arrives pre-shuffled into fragment order ([N/16][K/32][64 lanes][8]): every wave loads its own
        // operand-b fragments straight into registers with 1 KB coalesced loads (the fragments of a k-step of the
        // next slab are requested as soon as this slab's k-step has issued), and only A goes through LDS.
        const int ksteps = K / 32;
        // one pointer per 16-column block of the wave; a block past N (a tile wider than what is left of a
        // width that is a multiple of 128 only) re-reads the last block of W: its results are never stored
        const bf16 *wp[NT16];
#pragma unroll
        for (int j = 0; j < NT16; ++j)
            wp[j] = W + ((long)min(((n0 + wn) >> 4) + j, (N >> 4) - 1) * ksteps) * 512 + lane * 8;
#define GEMM_LOAD_W(kt_, s_)                                                                          \
        {                                                                                             \
            _Pragma("unroll") for (int j = 0; j < NT16; ++j)                                          \
                bw[s_][j] = *reinterpret_cast<const bf16x8 *>(wp[j] + ((long)(kt_) * 2 + (s_)) * 512); \
        }
#define GEMM_LOAD_GLOBAL_A(kt_)                                                                       \
        {                                                                                             \
            _Pragma("unroll") for (int i = 0; i < A_LOADS; ++i)                                       \
                ra[i] = *reinterpret_cast<const u32x4 *>(ga[i] + (kt_) * GEMM_BK);                    \
        }
#define GEMM_STORE_LDS_A(buf_)                                                                        \
        {                                                                                             \
            bf16 *as_ = As + (buf_) * BM * GEMM_BK + lst;                                             \
            _Pragma("unroll") for (int i = 0; i < A_LOADS; ++i)                                       \
                *reinterpret_cast<u32x4 *>(as_ + i * RSTEP * GEMM_BK) = ra[i];                        \
        }
        // A is requested 1.25 slabs before it is stored: the registers ra are stored to LDS in the last phase but
        // one of a slab (data of the next slab, requested in the last phase of the previous one, so the store never
        // waits for memory and completes a phase before the barrier instead of right in front of it) and refilled
        // in the last phase with the slab after next.
        GEMM_LOAD_GLOBAL_A(kb)
        GEMM_LOAD_W(kb, 0) GEMM_LOAD_W(kb, 1)
        GEMM_STORE_LDS_A(0)
        GEMM_LOAD_GLOBAL_A(min(kb + 1, ke - 1))
        LDS_BARRIER();
        // a wave in its main loop goes before the waves of the CU's other workgroup when that one is in its
        // prologue or epilogue (priority 0): their memory instructions then fill the gaps instead of delaying MFMAs
        __builtin_amdgcn_s_setprio(1);
        for (int kt = kb; kt < ke - 1; ++kt, buf ^= 1) {
            GEMM_LOAD_AFRAGS(buf, 0, 0)
#pragma unroll
            for (int p = 0; p < PH; ++p) {
                if (p + 1 < PH) GEMM_LOAD_AFRAGS(buf, p + 1, (p + 1) & 1)
                GEMM_MFMAS(p, p & 1)
                if (p == PH - 2) GEMM_STORE_LDS_A(buf ^ 1)
                if (p == PH - 1) GEMM_LOAD_GLOBAL_A(min(kt + 2, ke - 1))
                if (p % HP == HP - 1) GEMM_LOAD_W(kt + 1, p / HP)
            }
            // issue order: the fragments of phase 0, then per phase its MFMAs with the next phase's LDS reads behind
            // the first ones, the LDS writes / the next A requests behind the first ones of the last two phases, and the
            // requests for a finished k-step's operand-b fragments behind the last ones
            GEMM_SGB(0x100, AF);
#pragma unroll
            for (int p = 0; p < PH; ++p)
#pragma unroll
                for (int i = 0; i < NP; ++i) {
                    GEMM_SGB(0x008, 1);
                    if (p + 1 < PH && i < AF) GEMM_SGB(0x100, 1);
                    if (p == PH - 2 && i < A_LOADS) GEMM_SGB(0x200, 1);
                    if (p == PH - 1 && i < A_LOADS) GEMM_SGB(0x020, 1);
                    if (p % HP == HP - 1 && i >= NP - NT16) GEMM_SGB(0x020, 1);
                }
            LDS_BARRIER();
        }
        GEMM_LOAD_AFRAGS(buf, 0, 0)
#pragma unroll
        for (int p = 0; p < PH; ++p) {
            if (p + 1 < PH) GEMM_LOAD_AFRAGS(buf, p + 1, (p + 1) & 1)
            GEMM_MFMAS(p, p & 1)
        }
        __builtin_amdgcn_s_setprio(0);
    } else {
    GEMM_LOAD_GLOBAL(kb)
    GEMM_STORE_LDS(0)
    LDS_BARRIER();
    for (int kt = kb; kt < ke - 1; ++kt, buf ^= 1) {
        GEMM_LOAD_AFRAGS(buf, 0, 0)
        GEMM_LOAD_BFRAGS(buf, 0)
#pragma unroll
        for (int p = 0; p < PH; ++p) {
            if (p == 0) GEMM_LOAD_GLOBAL(kt + 1)
            if (p + 1 < PH) {
                GEMM_LOAD_AFRAGS(buf, p + 1, (p + 1) & 1)
                if ((p + 1) % HP == 0) GEMM_LOAD_BFRAGS(buf, (p + 1) / HP)
            }
            GEMM_MFMAS(p, p & 1)
            if (p == PH - 1) GEMM_STORE_LDS(buf ^ 1)
        }
        // issue order: fragments of phase 0; then per phase its MFMAs with the next phase's LDS reads, the next
        // slab's global loads (phase 0) and LDS writes (last phase) slotted in between
        GEMM_SGB(0x100, AF + NT16);
#pragma unroll
        for (int p = 0; p < PH; ++p)
#pragma unroll
            for (int i = 0; i < NP; ++i) {
                GEMM_SGB(0x008, 1);
                if (p + 1 < PH && i < AF + ((p + 1) % HP == 0 ? NT16 : 0)) GEMM_SGB(0x100, 1);
                if (p == 0 && i < NL) GEMM_SGB(0x020, 1);
                if (p == PH - 1 && i < NL) GEMM_SGB(0x200, 1);
            }
        LDS_BARRIER();
    }
    {
        GEMM_LOAD_AFRAGS(buf, 0, 0)
        GEMM_LOAD_BFRAGS(buf, 0)
#pragma unroll
        for (int p = 0; p < PH; ++p) {
            if (p + 1 < PH) {
                GEMM_LOAD_AFRAGS(buf, p + 1, (p + 1) & 1)
                if ((p + 1) % HP == 0) GEMM_LOAD_BFRAGS(buf, (p + 1) / HP)
            }
            GEMM_MFMAS(p, p & 1)
        }
    }
    }

    // The last MFMAs are still in flight here.  Reads of their accumulator registers need up to 18 wait
    // states after a 16-pass MFMA, which the compiler inserts within straight-line code; the epilogue starts
    // with wave-divergent branches (row-map look-ups by some waves only), and one instantiation read its last
    // accumulator register too early on the waves that skip the branch.  Wait the passes out explicitly.
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);

    // ---- epilogue: 32-row slices through a per-wave fp32 LDS region
    constexpr int EPS = WN + 4;                 // floats per staged row (16-byte multiple, odd in 16-byte units)
    constexpr int LPR = WN / 8;                 // lanes per row when each lane owns 8 columns
    constexpr int RPP = 64 / LPR;               // rows per pass
    float *stage = reinterpret_cast<float *>(smem) + wave * 32 * EPS;
    const int cl = lane % LPR, rl = lane / LPR;
    const int ncol = n0 + wn + cl * 8;
    float bv[8];
    if (EPI == GEMM_EPI_PARTIAL) {
#pragma unroll
        for (int e = 0; e < 8; ++e) bv[e] = 0.f;
    } else {
        const float4 *b4 = reinterpret_cast<const float4 *>(bias + (ncol < N ? ncol : 0));
        float4 x0 = b4[0], x1 = b4[1];
        bv[0] = x0.x; bv[1] = x0.y; bv[2] = x0.z; bv[3] = x0.w;
        bv[4] = x1.x; bv[5] = x1.y; bv[6] = x1.z; bv[7] = x1.w;
    }
    const bool col_ok = ncol < N;               // N % 8 == 0: a lane's 8 columns are all inside or all outside
    constexpr int PASSES = 32 / RPP;
    float sv[FOLD_EPI ? 8 : 1];
    if constexpr (FOLD_EPI) {
        const float4 *c4 = reinterpret_cast<const float4 *>(fold.colsum + (ncol < N ? ncol : 0));
        float4 x0 = c4[0], x1 = c4[1];
        sv[0] = x0.x; sv[1] = x0.y; sv[2] = x0.z; sv[3] = x0.w;
        sv[4] = x1.x; sv[5] = x1.y; sv[6] = x1.z; sv[7] = x1.w;
    }
    // The scatter epilogue is a read-modify-write of rows of the residual stream.  Its destination rows
    // are looked up once per tile (one row per thread, parked in LDS behind the staging regions) and the
    // old values of a whole 32-row slice are requested before the slice is staged, so that the slice pays
    // one memory round trip instead of one per pass.
    int *dst_row = reinterpret_cast<int *>(reinterpret_cast<float *>(smem) + WGM * WGN * 32 * EPS);   // [BM], -1 = skip
    constexpr bool MAPPED = EPI == SSAM_EPI_BIAS_SCATTER_ADD || EPI == SSAM_EPI_BIAS_SCATTER;
    float2 *row_stats = reinterpret_cast<float2 *>(dst_row + BM);    // [BM] { rstd, -rstd*mean } (LNF), parked like dst_row
    if (MAPPED || FOLD_EPI) {
        int mine = -1;
        float2 mine_stats = { 0.f, 0.f };
        if (tid < BM && m0 + tid < M) {
            int m = m0 + tid;
            if constexpr (FOLD_EPI) mine_stats = fold.stats[m];
            if (MAPPED) {
                int b = m / rm.rows_per_batch, p = m - b * rm.rows_per_batch;
                int idx = rm.map[(long)b * rm.map_batch_stride + p];
                if (idx >= 0 && idx < rm.dst_rows_per_batch) mine = b * rm.dst_rows_per_batch + idx;
            }
        }
        __syncthreads();                        // every wave is done with the pipeline buffers
        if (tid < BM) {
            if (MAPPED) dst_row[tid] = mine;
            if constexpr (FOLD_EPI) row_stats[tid] = mine_stats;
        }
    }
    __syncthreads();                            // pipeline buffers free for staging; dst_row visible
    // The bias values must have landed before the first store pass: a pass that first touched them behind its
    // row predicate would wait with a full drain of the memory counter, which on this hardware also counts the
    // stores of the passes before it, and every pass would then wait for the previous pass's store to complete.
#pragma unroll
    for (int e = 0; e < 8; ++e) asm volatile("" : "+v"(bv[e]));
    if constexpr (FOLD_EPI) {
#pragma unroll
        for (int e = 0; e < 8; ++e) asm volatile("" : "+v"(sv[e]));
    }
    // From here on a wave touches only its own staging region: LDS operations of one wave execute in
    // order, so the slices need no workgroup barrier (which would also wait for the previous slice's
    // global stores); wavefront fences keep the compiler from reordering the LDS accesses.
    // Destination rows and old values of a 32-row slice.  The loads are unconditional (a skipped row or column
    // reads row 0 / column 0 and drops the value: loads behind a predicate would each be waited for on their own)
    // and a slice's loads are issued before the stores of the slice before it, so the wait for them (a count
    // of younger operations still allowed in flight) does not wait for those stores to complete.
    uint4 old[PASSES], old_next[PASSES];
    int drow[PASSES], drow_next[PASSES];
    auto preload_slice = [&](int i, uint4 (&o)[PASSES], int (&d)[PASSES]) {
#pragma unroll
        for (int pass = 0; pass < PASSES; ++pass) {
            d[pass] = dst_row[wm + i * 32 + pass * RPP + rl];
            if (EPI == SSAM_EPI_BIAS_SCATTER_ADD)
                o[pass] = *reinterpret_cast<const uint4 *>(C + (long)max(d[pass], 0) * ld.c + (col_ok ? ncol : 0));
        }
    };
    if (MAPPED) preload_slice(0, old, drow);
#pragma unroll
    for (int i = 0; i < MT; ++i) {
#pragma unroll
        for (int t = 0; t < 2; ++t)             // the slice's two 16-row tiles: lane (l16, quad) holds rows 4*quad + r
#pragma unroll
            for (int j = 0; j < NT16; ++j)
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    stage[(t * 16 + 4 * quad + r) * EPS + j * 16 + l16] = acc[2 * i + t][j][r];
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        if (MAPPED && i + 1 < MT) preload_slice(i + 1, old_next, drow_next);
        if (EPI == SSAM_EPI_BIAS_SCATTER_ADD) {   // this slice's old values, waited for once (see the bias values above)
#pragma unroll
            for (int pass = 0; pass < PASSES; ++pass)
                asm volatile("" : "+v"(old[pass].x), "+v"(old[pass].y), "+v"(old[pass].z), "+v"(old[pass].w));
        }
#pragma unroll
        for (int pass = 0; pass < PASSES; ++pass) {
            const int row = pass * RPP + rl;
            const int m = m0 + wm + i * 32 + row;
            if (m >= M || (EPI != GEMM_EPI_PARTIAL && !col_ok)) continue;
            const float4 *s4 = reinterpret_cast<const float4 *>(stage + row * EPS + cl * 8);
            float4 y0 = s4[0], y1 = s4[1];
            if (EPI == GEMM_EPI_PARTIAL) {
                float4 *dst = reinterpret_cast<float4 *>(sp.partial + (((long)slot * parts + kpart) * BM + (wm + i * 32 + row)) * BN + wn + cl * 8);
                dst[0] = y0;
                dst[1] = y1;
                continue;
            }
            float v[8] = { y0.x, y0.y, y0.z, y0.w, y1.x, y1.y, y1.z, y1.w };
            if constexpr (FOLD_EPI) {
                const float2 t = row_stats[wm + i * 32 + row];
#pragma unroll
                for (int e = 0; e < 8; ++e) v[e] = v[e] * t.x + (t.y * sv[e] + bv[e]);
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) v[e] += bv[e];
            }
            if (EPI == SSAM_EPI_BIAS_GELU) {
#pragma unroll
                for (int e = 0; e < 8; ++e) v[e] = gelu_erf(v[e]);
            }
            if (EPI == SSAM_EPI_BIAS_SCATTER_ADD) {
                if (drow[pass] < 0) continue;
                float o[8];
                unpack_bf16x8(old[pass], o);
#pragma unroll
                for (int e = 0; e < 8; ++e) v[e] += o[e];
                *reinterpret_cast<uint4 *>(C + (long)drow[pass] * ld.c + ncol) = pack_bf16x8(v);
            } else if (EPI == SSAM_EPI_BIAS_SCATTER) {
                // (a mapped store is the qkv tensor: written once, read once by the attention kernel that follows; the
                // non-temporal hint keeps it from displacing what the later kernels of the block want cached)
                if (drow[pass] >= 0) {
                    const uint4 pk_ = pack_bf16x8(v);
                    __builtin_nontemporal_store(__builtin_bit_cast(u32x4, pk_), reinterpret_cast<u32x4 *>(C + (long)drow[pass] * ld.c + ncol));
                }
            } else {
                *reinterpret_cast<uint4 *>(C + (long)m * ld.c + ncol) = pack_bf16x8(v);
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");      // the slice is read before the next one is staged
        if (MAPPED && i + 1 < MT) {
#pragma unroll
            for (int pass = 0; pass < PASSES; ++pass) { old[pass] = old_next[pass]; drow[pass] = drow_next[pass]; }
        }
    }
}

template <int BM, int BN, int EPI, int SUB_M = 1, int SUB_N = 1, int WGM = 2, int WGN = 2, bool WPACK = false, bool LNF = false>
__global__ void __launch_bounds__(64 * WGM * WGN, (BN == 256 && WGM * WGN == 4 && WPACK) ? 2 : 1)
gemm_bf16_nt_kernel(const bf16 *__restrict__ A, const bf16 *__restrict__ W, const float *__restrict__ bias,
                    bf16 *C, int M, int N, int K, GemmLd ld, GemmTileRange tr, GemmRowMap rm, GemmSplit sp, GemmFold fold)
{
    gemm_bf16_nt_body<BM, BN, EPI, SUB_M, SUB_N, WGM, WGN, WPACK, LNF>(A, W, bias, C, M, N, K, ld, tr, rm, sp, (int)blockIdx.x, fold);
}

// The same workgroup with the LayerNorm of its A rows folded in (see GemmFold).
template <int BM, int BN, int EPI, int WGM, int WGN>
__global__ void __launch_bounds__(64 * WGM * WGN, (BN == 256 && WGM * WGN == 4) ? 2 : 1)
gemm_bf16_nt_lnf_kernel(const bf16 *__restrict__ A, const bf16 *__restrict__ W, const float *__restrict__ bias,
                        bf16 *C, int M, int N, int K, GemmLd ld, GemmTileRange tr, GemmRowMap rm, GemmFold fold)
{
    const GemmSplit whole = { nullptr, 1 };
    gemm_bf16_nt_body<BM, BN, EPI, 1, 1, WGM, WGN, true, true>(A, W, bias, C, M, N, K, ld, tr, rm, whole, (int)blockIdx.x, fold);
}

// Whole rounds and left-over tiles in ONE launch (both kinds of workgroup have 256 threads): the first `n_tail`
// workgroups (a multiple of 8, so that the XCD of a workgroup index stays the same for both kinds) run the
// left-over sub-tiles (TEPI = the epilogue proper, or GEMM_EPI_PARTIAL with K ranges), the others the large
// tiles.  The left-over workgroups are dispatched first and finish while the first round of large tiles runs,
// instead of running as a launch of their own on a mostly idle chip.
template <int BM, int BN, int EPI, int WGM, int WGN, int TM, int TN, int TEPI, int SUB_M, int SUB_N, bool WPACK, bool LNF = false>
__global__ void __launch_bounds__(256, 2)
gemm_bf16_nt_fused_kernel(const bf16 *__restrict__ A, const bf16 *__restrict__ W, const float *__restrict__ bias,
                          bf16 *C, int M, int N, int K, GemmLd ld, GemmTileRange tr_main, GemmTileRange tr_tail,
                          GemmRowMap rm, GemmSplit sp_tail, int n_tail, GemmFold fold)
{
    static_assert(WGM * WGN == 4, "both kinds of workgroup are four waves");
    if ((int)blockIdx.x < n_tail) {
        gemm_bf16_nt_body<TM, TN, TEPI, SUB_M, SUB_N, 2, 2, WPACK, LNF>(A, W, bias, C, M, N, K, ld, tr_tail, rm, sp_tail, (int)blockIdx.x, fold);
    } else {
        const GemmSplit whole = { nullptr, 1 };
        gemm_bf16_nt_body<BM, BN, EPI, 1, 1, WGM, WGN, WPACK, LNF>(A, W, bias, C, M, N, K, ld, tr_main, rm, whole, (int)blockIdx.x - n_tail, fold);
    }
}

// Second half of a K-split left-over launch: adds the `parts` fp32 slots of every sub-tile in slot
// order, then bias (with a folded LayerNorm: its row and column terms, see GemmFold) and the epilogue proper.
// One thread finishes 8 consecutive columns of a row.
template <int BM, int BN, int EPI, int SUB_M, int SUB_N, bool LNF = false>
__global__ void __launch_bounds__(256)
gemm_tail_reduce_kernel(const float *__restrict__ partial, int parts, const float *__restrict__ bias, bf16 *C,
                        int M, int N, GemmLd ld, GemmTileRange tr, GemmRowMap rm, GemmFold fold)
{
    constexpr int LPR = BN / 8, RPB = 256 / LPR;                  // lanes per row, rows per workgroup
    constexpr int SUBS = SUB_M * SUB_N;
    const int slot = blockIdx.x / (BM / RPB);
    const int row = (blockIdx.x % (BM / RPB)) * RPB + threadIdx.x / LPR;
    const int col = (threadIdx.x % LPR) * 8;
    int m0, n0;
    gemm_tile_origin(tr, tr.tile_begin + slot / SUBS, slot % SUBS, SUB_M, SUB_N, BM, BN, m0, n0);
    const int m = m0 + row, ncol = n0 + col;
    if (m >= M || ncol >= N) return;
    float v[8];
    {
        const float4 *b4 = reinterpret_cast<const float4 *>(bias + ncol);
        float4 x0 = b4[0], x1 = b4[1];
        v[0] = x0.x; v[1] = x0.y; v[2] = x0.z; v[3] = x0.w;
        v[4] = x1.x; v[5] = x1.y; v[6] = x1.z; v[7] = x1.w;
    }
    // destination row and its old value (mapped epilogues) are requested before the partial sums are walked
    constexpr bool MAPPED = EPI == SSAM_EPI_BIAS_SCATTER_ADD || EPI == SSAM_EPI_BIAS_SCATTER;
    int idx = 0, mb = 0;
    if (MAPPED) {
        mb = m / rm.rows_per_batch;
        idx = rm.map[(long)mb * rm.map_batch_stride + (m - mb * rm.rows_per_batch)];
    }
    float acc[8] = { 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f };
    const float *src = partial + ((long)slot * parts * BM + row) * BN + col;
    // four slots' loads in flight at a time; the additions keep the slot order (the result does not depend on
    // how the loads are grouped)
    int p = 0;
    for (; p + 4 <= parts; p += 4) {
        float4 y[4][2];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float4 *s4 = reinterpret_cast<const float4 *>(src + (long)(p + u) * BM * BN);
            y[u][0] = s4[0];
            y[u][1] = s4[1];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            acc[0] += y[u][0].x; acc[1] += y[u][0].y; acc[2] += y[u][0].z; acc[3] += y[u][0].w;
            acc[4] += y[u][1].x; acc[5] += y[u][1].y; acc[6] += y[u][1].z; acc[7] += y[u][1].w;
        }
    }
    for (; p < parts; ++p) {
        const float4 *s4 = reinterpret_cast<const float4 *>(src + (long)p * BM * BN);
        float4 y0 = s4[0], y1 = s4[1];
        acc[0] += y0.x; acc[1] += y0.y; acc[2] += y0.z; acc[3] += y0.w;
        acc[4] += y1.x; acc[5] += y1.y; acc[6] += y1.z; acc[7] += y1.w;
    }
    if constexpr (LNF) {
        const float2 t = fold.stats[m];
        const float4 *c4 = reinterpret_cast<const float4 *>(fold.colsum + ncol);
        const float4 x0 = c4[0], x1 = c4[1];
        const float cs[8] = { x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w };
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = acc[e] * t.x + (t.y * cs[e] + v[e]);
    } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] += acc[e];
    }
    if (EPI == SSAM_EPI_BIAS_GELU) {
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = gelu_erf(v[e]);
    }
    if (MAPPED) {
        if (idx < 0 || idx >= rm.dst_rows_per_batch) return;
        uint4 *dst = reinterpret_cast<uint4 *>(C + ((long)mb * rm.dst_rows_per_batch + idx) * ld.c + ncol);
        if (EPI == SSAM_EPI_BIAS_SCATTER_ADD) {
            float o[8];
            unpack_bf16x8(*dst, o);
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] += o[e];
        }
        *dst = pack_bf16x8(v);
    } else {
        *reinterpret_cast<uint4 *>(C + (long)m * ld.c + ncol) = pack_bf16x8(v);
    }
}
