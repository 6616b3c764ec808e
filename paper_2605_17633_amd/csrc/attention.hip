// Stripe-Sort attention (App. A.1, Alg. 1) for gfx950: block-sparse, flash-style
// attention over the static A-shape tile mask, with SAM's decomposed 2-D
// relative-position bias fused in.  Tokens arrive in scan order; sigma maps a
// scan position to its spatial cell for the bias lookup.
//
// Formulation.  Scores are computed transposed, S^T = K Q^T, on the 32x32x16 bf16
// MFMA: the Q fragments (operand b) stay in registers for the whole kernel, K
// rows come from LDS (operand a).  In the result layout every lane owns ONE
// query (column l & 31) and 16 of the 32 keys of a block, so the softmax row
// statistics are per-lane scalars: the row maximum needs a single exchange with
// lane l^32, the row sum none until the end.  exp(S^T) converted to bf16 is
// already in the operand-b layout of the second product O^T = V^T P^T; the
// operand-a fragments are read from a transposed copy of V in LDS with the key
// order the result layout dictates (contraction slot e of half-wave hf of MFMA
// t  <->  key 16t + 8(e/4) + 4hf + (e&3)).
// Bias: per wave, U = Q R^T is formed once with the MFMA for both tables and
// scattered into per-query rows B^H[q][key_row], B^W[q][key_col] in LDS
// (pre-multiplied by log2 e); the inner loop adds two table look-ups per score.
//
// Two launch shapes:
//   window kernel: one workgroup per (window, head), one wave per 32-query tile
//                  (= mask tile of 32), the window's whole K and V^T in LDS;
//   global kernel: one workgroup per (128-query mask tile, image, head), 4 waves,
//                  active 128-key tiles streamed through LDS with register prefetch.
#include "common.h"

namespace {

constexpr float LOG2E = 1.4426950408889634f;

struct AttnParams {
    const bf16 *q, *k, *v;
    long row_stride;
    const bf16 *rel_h, *rel_w;
    const int32_t *sigma;
    bf16 *out;
    int S, w, h, n_pre;
    float scale_log2e;
};

template <int D>
struct AttnCfg {
    static constexpr int KS = D / 16;            // k-steps of the score product
    static constexpr int DT = (D + 31) / 32;     // 32-row tiles of O^T
    static constexpr int KSTR = D + 8;           // K row stride in LDS (elements): odd in 16-byte units
    static constexpr int CH = D / 8;             // 16-byte chunks per row
};

// Per-wave softmax/output state for 32 queries (one per lane pair l, l^32).
template <int D>
struct WaveState {
    f32x16 o[AttnCfg<D>::DT];
    float m, l;
};

// Bias rows for the wave's 32 queries: th[q*ts + p] = log2e * q . rel_h[row(q)-p+w-1], tw likewise.
template <int D>
__device__ __forceinline__ void build_bias_rows(const bf16x8 *qf, const bf16 *rel_h, const bf16 *rel_w,
                                                int w, int qrow, int qcol, float *th, float *tw, int ts)
{
    const int lane = threadIdx.x & 63, l32 = lane & 31, half = lane >> 5;
    const int nrel = 2 * w - 1;
    for (int mt = 0; mt * 32 < nrel; ++mt) {
#pragma unroll
        for (int tab = 0; tab < 2; ++tab) {
            const bf16 *rel = tab ? rel_w : rel_h;
            f32x16 u;
#pragma unroll
            for (int r = 0; r < 16; ++r) u[r] = 0.f;
            const int mrow = mt * 32 + l32;
#pragma unroll
            for (int ks = 0; ks < AttnCfg<D>::KS; ++ks) {
                bf16x8 a;
#pragma unroll
                for (int e = 0; e < 8; ++e) a[e] = (bf16)0.f;
                if (mrow < nrel) a = *reinterpret_cast<const bf16x8 *>(rel + (long)mrow * D + ks * 16 + half * 8);
                u = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[ks], u, 0, 0, 0);
            }
            float *dst = (tab ? tw : th) + l32 * ts;
            const int qpos = tab ? qcol : qrow;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                int m = mt * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
                int p = qpos + (w - 1) - m;
                if (p >= 0 && p < w && m < nrel) dst[p] = u[r] * LOG2E;
            }
        }
    }
}

// One 32-key block against the wave's 32 queries.
//   kblk: LDS, row-major K rows of this block ([32][KSTR])
//   vt:   LDS, V^T with `vstr` elements per feature row; vcol0 = column of the block's first key
//   krc:  LDS, per key of this block (row | col << 16) of its spatial cell
//   key0: scan position of the block's first key (for the S bound)
template <int D>
__device__ __forceinline__ void attn_block_step(WaveState<D> &st, const bf16x8 *qf, const bf16 *kblk,
                                                const bf16 *vt, int vstr, int vcol0, const uint32_t *krc,
                                                int key0, int S, float scale_log2e,
                                                const float *th, const float *tw)
{
    using C = AttnCfg<D>;
    const int lane = threadIdx.x & 63, l32 = lane & 31, half = lane >> 5;
    f32x16 s;
#pragma unroll
    for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < C::KS; ++ks) {
        bf16x8 a = *reinterpret_cast<const bf16x8 *>(kblk + l32 * C::KSTR + ks * 16 + half * 8);
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[ks], s, 0, 0, 0);
    }
    float mx = st.m;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const u32x4 rc = *reinterpret_cast<const u32x4 *>(krc + 8 * g + 4 * half);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int r = 4 * g + e;
            const int kl = 8 * g + 4 * half + e;
            const uint32_t c = rc[e];
            float val = s[r] * scale_log2e + th[c & 0xffffu] + tw[c >> 16];
            val = (key0 + kl < S) ? val : -INFINITY;
            s[r] = val;
            mx = fmaxf(mx, val);
        }
    }
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float alpha = exp2f(st.m - mx);      // first block: exp2(-inf) = 0
    st.m = mx;
    float psum = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        s[r] = exp2f(s[r] - mx);
        psum += s[r];
    }
    st.l = st.l * alpha + psum;
#pragma unroll
    for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) st.o[dt][r] *= alpha;
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        bf16x8 p;
#pragma unroll
        for (int e = 0; e < 8; ++e) p[e] = (bf16)s[8 * t + e];
#pragma unroll
        for (int dt = 0; dt < C::DT; ++dt) {
            int dd = dt * 32 + l32;
            dd = dd < D ? dd : D - 1;            // rows past D repeat the last row; their outputs are dropped
            const bf16 *vrow = vt + dd * vstr + vcol0 + 16 * t + 4 * half;
            bf16x4 v0 = *reinterpret_cast<const bf16x4 *>(vrow);
            bf16x4 v1 = *reinterpret_cast<const bf16x4 *>(vrow + 8);
            bf16x8 a = { v0[0], v0[1], v0[2], v0[3], v1[0], v1[1], v1[2], v1[3] };
            st.o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, p, st.o[dt], 0, 0, 0);
        }
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

template <int D>
__device__ __forceinline__ void finish_and_store(WaveState<D> &st, bf16 *orow, bool valid)
{
    const int half = (threadIdx.x & 63) >> 5;
    const float l = st.l + __shfl_xor(st.l, 32, 64);
    const float inv = 1.0f / l;
    if (!valid) return;
#pragma unroll
    for (int dt = 0; dt < AttnCfg<D>::DT; ++dt)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            int dd = dt * 32 + 8 * g + 4 * half;
            if (dd < D) {
                uint2 pk;
                pk.x = pack_bf16x2(st.o[dt][4 * g + 0] * inv, st.o[dt][4 * g + 1] * inv);
                pk.y = pack_bf16x2(st.o[dt][4 * g + 2] * inv, st.o[dt][4 * g + 3] * inv);
                *reinterpret_cast<uint2 *>(orow + dd) = pk;
            }
        }
}

__device__ __forceinline__ uint32_t key_row_col(const int32_t *sigma, int p, int S, int w)
{
    int cell = sigma[p < S ? p : S - 1];
    cell = min(max(cell, 0), w * w - 1);
    return (uint32_t)(cell / w) | ((uint32_t)(cell % w) << 16);
}

// ------------------------------------------------------------------ window kernel
template <int D>
size_t window_lds_bytes(int nqb, int w)
{
    int SP = nqb * 32, ts = w | 1;
    return (size_t)SP * AttnCfg<D>::KSTR * 2 + (size_t)D * (SP + 4) * 2 + (size_t)nqb * 32 * 2 * ts * 4 + (size_t)SP * 4;
}

template <int D>
__global__ void __launch_bounds__(448)
attn_window_kernel(AttnParams P)
{
    using C = AttnCfg<D>;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int nqb = blockDim.x >> 6, SP = nqb * 32, vstr = SP + 4, ts = P.w | 1;
    bf16 *Ks = reinterpret_cast<bf16 *>(smem);
    bf16 *Vt = Ks + SP * C::KSTR;
    float *T = reinterpret_cast<float *>(Vt + D * vstr);
    uint32_t *krc = reinterpret_cast<uint32_t *>(T + nqb * 32 * 2 * ts);

    const int grp = blockIdx.x / P.h, head = blockIdx.x % P.h;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31;
    const int S = P.S;
    const long base = (long)grp * S * P.row_stride + (long)head * D;

    // stage K rows and V^T (pad keys are zero so that 0-probabilities meet finite values)
    for (int id = tid; id < SP * C::CH; id += blockDim.x) {
        int key = id / C::CH, c = id % C::CH;
        u32x4 kv = { 0, 0, 0, 0 }, vv = { 0, 0, 0, 0 };
        if (key < S) {
            kv = *reinterpret_cast<const u32x4 *>(P.k + base + (long)key * P.row_stride + c * 8);
            vv = *reinterpret_cast<const u32x4 *>(P.v + base + (long)key * P.row_stride + c * 8);
        }
        *reinterpret_cast<u32x4 *>(Ks + key * C::KSTR + c * 8) = kv;
        const bf16x8 ve = __builtin_bit_cast(bf16x8, vv);
#pragma unroll
        for (int e = 0; e < 8; ++e) Vt[(c * 8 + e) * vstr + key] = ve[e];
    }
    for (int p = tid; p < SP; p += blockDim.x) krc[p] = key_row_col(P.sigma, p, S, P.w);

    const int q0 = wave * 32, qpos = q0 + l32;
    const int qclamp = qpos < S ? qpos : S - 1;
    bf16x8 qf[C::KS];
    load_q_frags<D>(qf, P.q + base + (long)qclamp * P.row_stride);
    const uint32_t qrc = key_row_col(P.sigma, qclamp, S, P.w);
    float *th = T + wave * 32 * 2 * ts, *tw = th + 32 * ts;
    build_bias_rows<D>(qf, P.rel_h, P.rel_w, P.w, (int)(qrc & 0xffffu), (int)(qrc >> 16), th, tw, ts);
    __syncthreads();

    WaveState<D> st;
#pragma unroll
    for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) st.o[dt][r] = 0.f;
    st.m = -INFINITY;
    st.l = 0.f;

    // active key tiles of query tile `wave`: the dense prefix, then the diagonal
    const int nact = P.n_pre + (wave >= P.n_pre ? 1 : 0);
    for (int a = 0; a < nact; ++a) {
        const int kb = a < P.n_pre ? a : wave;
        attn_block_step<D>(st, qf, Ks + kb * 32 * C::KSTR, Vt, vstr, kb * 32, krc + kb * 32, kb * 32, S,
                           P.scale_log2e, th + l32 * ts, tw + l32 * ts);
    }
    finish_and_store<D>(st, P.out + ((long)grp * S + qclamp) * ((long)P.h * D) + (long)head * D, qpos < S);
}

// ------------------------------------------------------------------ global kernel
constexpr int GLB_TILE = 128;

template <int D>
size_t global_lds_bytes(int w)
{
    int ts = w | 1;
    return (size_t)GLB_TILE * AttnCfg<D>::KSTR * 2 + (size_t)D * (GLB_TILE + 4) * 2 + (size_t)4 * 32 * 2 * ts * 4 +
           (size_t)GLB_TILE * 4;
}

template <int D>
__global__ void __launch_bounds__(256)
attn_global_kernel(AttnParams P, int T)
{
    using C = AttnCfg<D>;
    constexpr int LOADS = GLB_TILE * C::CH / 256;       // 16-byte chunks per thread per operand
    static_assert(GLB_TILE * C::CH % 256 == 0, "tile chunks must divide over the workgroup");
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int vstr = GLB_TILE + 4, ts = P.w | 1;
    bf16 *Ks = reinterpret_cast<bf16 *>(smem);
    bf16 *Vt = Ks + GLB_TILE * C::KSTR;
    float *Tb = reinterpret_cast<float *>(Vt + D * vstr);
    uint32_t *krc = reinterpret_cast<uint32_t *>(Tb + 4 * 32 * 2 * ts);

    const int qt = blockIdx.x % T, gh = blockIdx.x / T;
    const int grp = gh / P.h, head = gh % P.h;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31;
    const int S = P.S;
    const long base = (long)grp * S * P.row_stride + (long)head * D;

    const int qpos = qt * GLB_TILE + wave * 32 + l32;
    const int qclamp = qpos < S ? qpos : S - 1;
    bf16x8 qf[C::KS];
    load_q_frags<D>(qf, P.q + base + (long)qclamp * P.row_stride);
    const uint32_t qrc = key_row_col(P.sigma, qclamp, S, P.w);
    float *th = Tb + wave * 32 * 2 * ts, *tw = th + 32 * ts;
    build_bias_rows<D>(qf, P.rel_h, P.rel_w, P.w, (int)(qrc & 0xffffu), (int)(qrc >> 16), th, tw, ts);

    WaveState<D> st;
#pragma unroll
    for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) st.o[dt][r] = 0.f;
    st.m = -INFINITY;
    st.l = 0.f;

    const int nact = P.n_pre + (qt >= P.n_pre ? 1 : 0);
    u32x4 rk[LOADS], rv[LOADS];
    uint32_t rrc = 0;

#define ATTN_LOAD_TILE(kt_)                                                                             \
    {                                                                                                   \
        const int key0_ = (kt_) * GLB_TILE;                                                             \
        _Pragma("unroll") for (int i = 0; i < LOADS; ++i)                                               \
        {                                                                                               \
            int id = tid + i * 256, key = key0_ + id / C::CH, c = id % C::CH;                           \
            key = key < S ? key : S - 1; /* keys past S repeat the last row; masked in the scores */   \
            rk[i] = *reinterpret_cast<const u32x4 *>(P.k + base + (long)key * P.row_stride + c * 8);    \
            rv[i] = *reinterpret_cast<const u32x4 *>(P.v + base + (long)key * P.row_stride + c * 8);    \
        }                                                                                               \
        if (tid < GLB_TILE) rrc = key_row_col(P.sigma, key0_ + tid, S, P.w);                            \
    }
#define ATTN_STORE_TILE()                                                                               \
    {                                                                                                   \
        _Pragma("unroll") for (int i = 0; i < LOADS; ++i)                                               \
        {                                                                                               \
            int id = tid + i * 256, key = id / C::CH, c = id % C::CH;                                   \
            *reinterpret_cast<u32x4 *>(Ks + key * C::KSTR + c * 8) = rk[i];                             \
            const bf16x8 ve = __builtin_bit_cast(bf16x8, rv[i]);                                        \
            _Pragma("unroll") for (int e = 0; e < 8; ++e) Vt[(c * 8 + e) * vstr + key] = ve[e];         \
        }                                                                                               \
        if (tid < GLB_TILE) krc[tid] = rrc;                                                             \
    }

    ATTN_LOAD_TILE(0 < P.n_pre ? 0 : qt)
    for (int a = 0; a < nact; ++a) {
        const int kt = a < P.n_pre ? a : qt;
        __syncthreads();                       // every wave is done with the previous tile
        ATTN_STORE_TILE()
        __syncthreads();
        if (a + 1 < nact) ATTN_LOAD_TILE(a + 1 < P.n_pre ? a + 1 : qt)
#pragma unroll 1
        for (int kb = 0; kb < GLB_TILE / 32; ++kb) {
            if (kt * GLB_TILE + kb * 32 >= S) break;     // wholly past the end
            attn_block_step<D>(st, qf, Ks + kb * 32 * C::KSTR, Vt, vstr, kb * 32, krc + kb * 32,
                               kt * GLB_TILE + kb * 32, S, P.scale_log2e, th + l32 * ts, tw + l32 * ts);
        }
    }
    finish_and_store<D>(st, P.out + ((long)grp * S + qclamp) * ((long)P.h * D) + (long)head * D, qpos < S);
}

template <int D>
int launch_attention(const AttnParams &P, int groups, int mask_block, hipStream_t st)
{
    if (mask_block == 32) {
        int nqb = ssam_div_up(P.S, 32);
        size_t lds = window_lds_bytes<D>(nqb, P.w);
        if (lds > 160 * 1024) return SSAM_EUNSUPPORTED;
        auto kern = attn_window_kernel<D>;
        if (lds > 64 * 1024 &&
            hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
            return SSAM_EHIP;
        hipLaunchKernelGGL(kern, dim3(groups * P.h), dim3(nqb * 64), lds, st, P);
    } else {
        int T = ssam_div_up(P.S, GLB_TILE);
        size_t lds = global_lds_bytes<D>(P.w);
        if (lds > 160 * 1024) return SSAM_EUNSUPPORTED;
        auto kern = attn_global_kernel<D>;
        if (lds > 64 * 1024 &&
            hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
            return SSAM_EHIP;
        hipLaunchKernelGGL(kern, dim3((unsigned)((long)T * groups * P.h)), dim3(256), lds, st, P, T);
    }
    SSAM_CHECK_LAUNCH();
    return SSAM_OK;
}

}  // namespace

extern "C" int ssam_sparse_attention(const void *q, const void *k, const void *v, long row_stride,
                                     const void *rel_h, const void *rel_w, const int32_t *sigma, void *out,
                                     int groups, int S, int w, int h, int d, int mask_block, double r,
                                     float scale, void *stream)
{
    if (!q || !k || !v || !rel_h || !rel_w || !sigma || !out) return SSAM_EINVAL;
    if (groups <= 0 || S <= 0 || w <= 0 || h <= 0 || d <= 0 || !(r > 0.0) || r > 1.0) return SSAM_EINVAL;
    if (w * w != S || row_stride < (long)h * d || row_stride % 8 != 0) return SSAM_EINVAL;
    if (!ssam_aligned16(q) || !ssam_aligned16(k) || !ssam_aligned16(v) || !ssam_aligned16(rel_h) ||
        !ssam_aligned16(rel_w) || !ssam_aligned16(out))
        return SSAM_EINVAL;
    if (mask_block == 32) {
        if (S > 224) return SSAM_EUNSUPPORTED;
    } else if (mask_block == 128) {
        if (S > 16384 || (long)ssam_div_up(S, 128) * groups * h > 0x7fffffffL) return SSAM_EUNSUPPORTED;
    } else {
        return SSAM_EUNSUPPORTED;
    }
    if (w > 128) return SSAM_EUNSUPPORTED;
    AttnParams P;
    P.q = (const bf16 *)q; P.k = (const bf16 *)k; P.v = (const bf16 *)v;
    P.row_stride = row_stride;
    P.rel_h = (const bf16 *)rel_h; P.rel_w = (const bf16 *)rel_w;
    P.sigma = sigma;
    P.out = (bf16 *)out;
    P.S = S; P.w = w; P.h = h;
    P.n_pre = ssam_prefix_tiles(ssam_div_up(S, mask_block), r);
    P.scale_log2e = scale * LOG2E;
    hipStream_t st = (hipStream_t)stream;
    switch (d) {
    case 64: return launch_attention<64>(P, groups, mask_block, st);
    case 80: return launch_attention<80>(P, groups, mask_block, st);
    case 32: return launch_attention<32>(P, groups, mask_block, st);
    case 16: return launch_attention<16>(P, groups, mask_block, st);
    default: return SSAM_EUNSUPPORTED;
    }
}
