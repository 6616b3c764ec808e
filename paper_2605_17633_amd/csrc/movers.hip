// HBM-bound kernels: row gather / scatter in scan order (Sec. 4.1), fused
// LayerNorm + gather, token scores (Eq. 1) and keep-set selection (Sec. 4.2).
// Every global access is a 16-byte vector per lane along the feature axis.
#include "common.h"

namespace {

// ---------------------------------------------------------------- permute
__global__ void __launch_bounds__(256)
permute_kernel(const uint4 *__restrict__ x, const int32_t *__restrict__ idx, uint4 *__restrict__ y,
               int B, int Nin, int Nout, int chunks)
{
    long total = (long)B * Nout * chunks;
    long stride = (long)gridDim.x * blockDim.x;
    for (long i = (long)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
        int c = (int)(i % chunks);
        long row = i / chunks;
        int p = (int)(row % Nout);
        int b = (int)(row / Nout);
        int src = idx[p];
        uint4 v = make_uint4(0, 0, 0, 0);
        if (src >= 0 && src < Nin) v = x[((long)b * Nin + src) * chunks + c];
        y[i] = v;
    }
}

__global__ void __launch_bounds__(256)
unpermute_kernel(const uint4 *__restrict__ y, const int32_t *__restrict__ idx, uint4 *x,
                 const uint4 *residual, int B, int Nx, int Ny, int chunks)
{
    long total = (long)B * Ny * chunks;
    long stride = (long)gridDim.x * blockDim.x;
    for (long i = (long)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
        int c = (int)(i % chunks);
        long row = i / chunks;
        int p = (int)(row % Ny);
        int b = (int)(row / Ny);
        int dst = idx[p];
        if (dst < 0 || dst >= Nx) continue;
        long o = ((long)b * Nx + dst) * chunks + c;
        uint4 v = y[i];
        if (residual) {
            float a[8], r[8];
            unpack_bf16x8(v, a);
            unpack_bf16x8(residual[o], r);
#pragma unroll
            for (int e = 0; e < 8; ++e) a[e] += r[e];
            v = pack_bf16x8(a);
        }
        x[o] = v;
    }
}

// ---------------------------------------------------------------- LN + gather
// One wave per output row; the row lives in registers (MAXC 16-byte chunks per
// lane), two-pass statistics in fp32.
template <int MAXC>
__global__ void __launch_bounds__(256)
ln_gather_kernel(const uint4 *__restrict__ x, const int32_t *__restrict__ idx, int idx_batch_stride,
                 const float *__restrict__ gamma, const float *__restrict__ beta, float eps,
                 uint4 *__restrict__ y, int B, int Nin, int Nout, int chunks)
{
    int lane = threadIdx.x & 63;
    long row = (long)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (row >= (long)B * Nout) return;
    int p = (int)(row % Nout), b = (int)(row / Nout);
    int src = idx[(long)b * idx_batch_stride + p];
    uint4 *yrow = y + row * chunks;
    if (src < 0 || src >= Nin) {
#pragma unroll
        for (int i = 0; i < MAXC; ++i) {
            int c = lane + 64 * i;
            if (c < chunks) yrow[c] = make_uint4(0, 0, 0, 0);
        }
        return;
    }
    const uint4 *xrow = x + ((long)b * Nin + src) * chunks;
    // every load of the row is requested before the first is used, without predicates (a chunk index past the
    // row re-reads its last chunk and is masked in the arithmetic): behind `c < chunks` each load would be
    // waited for on its own, one memory round trip after the other
    uint4 raw[MAXC];
    float4 g0[MAXC], g1[MAXC], b0[MAXC], b1[MAXC];
#pragma unroll
    for (int i = 0; i < MAXC; ++i) raw[i] = xrow[min(lane + 64 * i, chunks - 1)];
#pragma unroll
    for (int i = 0; i < MAXC; ++i) {
        const int c = min(lane + 64 * i, chunks - 1);
        const float4 *g4 = reinterpret_cast<const float4 *>(gamma) + 2 * c;
        const float4 *b4 = reinterpret_cast<const float4 *>(beta) + 2 * c;
        g0[i] = g4[0]; g1[i] = g4[1]; b0[i] = b4[0]; b1[i] = b4[1];
    }
    float v[MAXC][8];
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < MAXC; ++i) {
        unpack_bf16x8(raw[i], v[i]);
        if (lane + 64 * i < chunks) {
#pragma unroll
            for (int e = 0; e < 8; ++e) s += v[i][e];
        }
    }
    int D = chunks * 8;
    float mean = wave_sum(s) / (float)D;
    float q = 0.f;
#pragma unroll
    for (int i = 0; i < MAXC; ++i) {
        if (lane + 64 * i < chunks) {
#pragma unroll
            for (int e = 0; e < 8; ++e) { float t = v[i][e] - mean; q += t * t; }
        }
    }
    float inv = rsqrtf(wave_sum(q) / (float)D + eps);
#pragma unroll
    for (int i = 0; i < MAXC; ++i) {
        int c = lane + 64 * i;
        if (c < chunks) {
            float gg[8] = { g0[i].x, g0[i].y, g0[i].z, g0[i].w, g1[i].x, g1[i].y, g1[i].z, g1[i].w };
            float bb[8] = { b0[i].x, b0[i].y, b0[i].z, b0[i].w, b1[i].x, b1[i].y, b1[i].z, b1[i].w };
            float o[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = (v[i][e] - mean) * inv * gg[e] + bb[e];
            yrow[c] = pack_bf16x8(o);
        }
    }
}

// ---------------------------------------------------------------- LN statistics only
// The statistics half of the LayerNorm above, for a contraction that has the normalisation folded in:
// one wave per row, stats[row] = { rstd, -rstd * mean } (same two-pass fp32 arithmetic as ln_gather_kernel).
// With `idx` (the kept tokens of the routed MLP, [B][idx_batch_stride] positions inside an image of Nin rows) the
// statistics are those of the gathered rows, Nout per image, and src[row] receives the row of x that was read, for
// the contraction that gathers the same rows; an index outside [0, Nin) reads the image's first row (its result is
// dropped by the scatter that follows).
template <int MAXC>
__global__ void __launch_bounds__(256)
ln_stats_kernel(const uint4 *__restrict__ x, float2 *__restrict__ stats, long rows, int chunks, float eps,
                const int32_t *__restrict__ idx, int idx_batch_stride, int Nin, int Nout, int32_t *__restrict__ src)
{
    int lane = threadIdx.x & 63;
    long row = (long)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (row >= rows) return;
    long xr = row;
    if (idx) {
        const int b = (int)(row / Nout), p = (int)(row - (long)b * Nout);
        int t = idx[(long)b * idx_batch_stride + p];
        if (t < 0 || t >= Nin) t = 0;
        xr = (long)b * Nin + t;
        if (lane == 0) src[row] = (int32_t)xr;
    }
    const uint4 *xrow = x + xr * chunks;
    uint4 raw[MAXC];
#pragma unroll
    for (int i = 0; i < MAXC; ++i) raw[i] = xrow[min(lane + 64 * i, chunks - 1)];
    float v[MAXC][8];
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < MAXC; ++i) {
        unpack_bf16x8(raw[i], v[i]);
        if (lane + 64 * i < chunks) {
#pragma unroll
            for (int e = 0; e < 8; ++e) s += v[i][e];
        }
    }
    int D = chunks * 8;
    float mean = wave_sum(s) / (float)D;
    float q = 0.f;
#pragma unroll
    for (int i = 0; i < MAXC; ++i) {
        if (lane + 64 * i < chunks) {
#pragma unroll
            for (int e = 0; e < 8; ++e) { float t = v[i][e] - mean; q += t * t; }
        }
    }
    float inv = rsqrtf(wave_sum(q) / (float)D + eps);
    if (lane == 0) stats[row] = make_float2(inv, -inv * mean);
}

// Weight side of the fold: one wave per output channel n.
//   Wf[n][k] = bf16(W[n][k] * gamma[k]);  colsum[n] = sum_k Wf[n][k] (the stored values);  bias_f[n] = bias[n] + sum_k beta[k] W[n][k]
__global__ void __launch_bounds__(256)
fold_ln_weight_kernel(const bf16 *__restrict__ W, int ldw, const float *__restrict__ bias, const float *__restrict__ gamma,
                      const float *__restrict__ beta, bf16 *__restrict__ Wf, float *__restrict__ colsum,
                      float *__restrict__ bias_f, int N, int K)
{
    int lane = threadIdx.x & 63;
    int n = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (n >= N) return;
    float cs = 0.f, bs = 0.f;
    for (int c = lane; c < K / 8; c += 64) {
        float w[8], o[8];
        unpack_bf16x8(*reinterpret_cast<const uint4 *>(W + (long)n * ldw + c * 8), w);
#pragma unroll
        for (int e = 0; e < 8; ++e) { o[e] = w[e] * gamma[c * 8 + e]; bs += beta[c * 8 + e] * w[e]; }
        uint4 packed = pack_bf16x8(o);
        *reinterpret_cast<uint4 *>(Wf + (long)n * K + c * 8) = packed;
        unpack_bf16x8(packed, o);
#pragma unroll
        for (int e = 0; e < 8; ++e) cs += o[e];
    }
    cs = wave_sum(cs);
    bs = wave_sum(bs);
    if (lane == 0) { colsum[n] = cs; bias_f[n] = bias[n] + bs; }
}

// Key and value biases taken out of the qkv contraction (softmax over keys does not see a term that is the same
// for every key, and the probabilities of a query sum to one): one wave per output channel.
//   bias_out[n] = bias_in[n] - (n >= D ? bqkv[n] : 0)   n < 3D;   bproj_out[j] = bproj[j] + sum_c wproj[j][c] bqkv[2D + c]
__global__ void __launch_bounds__(256)
fold_kv_bias_kernel(const float *__restrict__ bias_in, const float *__restrict__ bqkv, const bf16 *__restrict__ wproj,
                    const float *__restrict__ bproj, float *__restrict__ bias_out, float *__restrict__ bproj_out, int D)
{
    int lane = threadIdx.x & 63;
    int n = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (n >= 3 * D) return;
    if (lane == 0) bias_out[n] = bias_in[n] - (n >= D ? bqkv[n] : 0.f);
    if (n < D) {
        float acc = 0.f;
        for (int c = lane; c < D / 8; c += 64) {
            float w[8];
            unpack_bf16x8(*reinterpret_cast<const uint4 *>(wproj + (long)n * D + c * 8), w);
#pragma unroll
            for (int e = 0; e < 8; ++e) acc += w[e] * bqkv[2 * D + c * 8 + e];
        }
        acc = wave_sum(acc);
        if (lane == 0) bproj_out[n] = bproj[n] + acc;
    }
}

// inv[b][table[b][p]] = p for every slot p that holds a token (table entries < 0 are padding)
__global__ void __launch_bounds__(256)
invert_table_kernel(const int32_t *__restrict__ table, int table_batch_stride, int Nout, int N, int32_t *__restrict__ inv, int total)
{
    int id = blockIdx.x * 256 + threadIdx.x;
    if (id >= total) return;
    int b = id / Nout, p = id - b * Nout;
    int s = table[(long)b * table_batch_stride + p];
    if (s >= 0 && s < N) inv[(long)b * N + s] = p;
}

// ---------------------------------------------------------------- scores
// channel sum of every token: one wave per token
__global__ void __launch_bounds__(256)
channel_sum_kernel(const uint4 *__restrict__ x, float *__restrict__ csum, long tokens, int chunks)
{
    int lane = threadIdx.x & 63;
    long t = (long)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (t >= tokens) return;
    const uint4 *row = x + t * chunks;
    float s = 0.f;
    for (int c = lane; c < chunks; c += 64) {
        float f[8];
        unpack_bf16x8(row[c], f);
        s += ((f[0] + f[1]) + (f[2] + f[3])) + ((f[4] + f[5]) + (f[6] + f[7]));
    }
    s = wave_sum(s);
    if (lane == 0) csum[t] = s;
}

// Sobel magnitude with zero padding on the channel-sum map
__global__ void __launch_bounds__(256)
sobel_kernel(const float *__restrict__ csum, float *__restrict__ scores, int B, int gh, int gw)
{
    long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    long n = (long)gh * gw;
    if (i >= (long)B * n) return;
    int b = (int)(i / n), cell = (int)(i % n), row = cell / gw, col = cell % gw;
    const float *c = csum + (long)b * n;
    auto at = [&](int rr, int cc) -> float {
        return (rr < 0 || rr >= gh || cc < 0 || cc >= gw) ? 0.f : c[rr * gw + cc];
    };
    float a00 = at(row - 1, col - 1), a01 = at(row - 1, col), a02 = at(row - 1, col + 1);
    float a10 = at(row, col - 1), a12 = at(row, col + 1);
    float a20 = at(row + 1, col - 1), a21 = at(row + 1, col), a22 = at(row + 1, col + 1);
    float gx = (a02 - a00) + 2.f * (a12 - a10) + (a22 - a20);
    float gy = (a20 - a00) + 2.f * (a21 - a01) + (a22 - a02);
    scores[i] = sqrtf(gx * gx + gy * gy);
}

// ---------------------------------------------------------------- select
// Order-preserving key: larger float <=> larger unsigned.  NaN -> -inf, -0 -> +0.
__device__ __forceinline__ uint32_t score_key(float s)
{
    uint32_t u = __float_as_uint(s);
    if ((u & 0x7fffffffu) > 0x7f800000u) u = 0xff800000u;   // NaN ranks as -inf
    if (u == 0x80000000u) u = 0u;                            // -0.0 == +0.0
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

constexpr int SEL_THREADS = 1024;

// exclusive prefix sum of one flag per thread over the block; returns the
// thread's offset and (through total) the block total.  scratch: 16 ints.
__device__ __forceinline__ int block_exclusive_count(bool flag, int *scratch, int &total)
{
    int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    unsigned long long ballot = __ballot(flag);
    int before = __popcll(ballot & ((1ull << lane) - 1ull));
    if (lane == 0) scratch[wave] = __popcll(ballot);
    __syncthreads();
    int base = 0, sum = 0;
#pragma unroll
    for (int w = 0; w < SEL_THREADS / 64; ++w) {
        int c = scratch[w];
        if (w < wave) base += c;
        sum += c;
    }
    __syncthreads();
    total = sum;
    return base + before;
}

// One workgroup per image: 4 passes of an 8-bit radix select find the key of
// the K-th largest score, then one ordered compaction pass writes every index
// with a larger key plus the lowest-index ties, in ascending index order.
__global__ void __launch_bounds__(SEL_THREADS)
select_kernel(const float *__restrict__ scores, int32_t *__restrict__ keep, int N, int K)
{
    __shared__ int hist[256];
    __shared__ int scratch[SEL_THREADS / 64];
    __shared__ uint32_t sh_prefix;
    __shared__ int sh_remaining;
    const float *s = scores + (long)blockIdx.x * N;
    int32_t *out = keep + (long)blockIdx.x * K;

    uint32_t prefix = 0, prefix_mask = 0;
    int remaining = K;   // how many of the keys matching the prefix are still to be taken
    for (int shift = 24; shift >= 0; shift -= 8) {
        for (int i = threadIdx.x; i < 256; i += SEL_THREADS) hist[i] = 0;
        __syncthreads();
        for (int i = threadIdx.x; i < N; i += SEL_THREADS) {
            uint32_t key = score_key(s[i]);
            if ((key & prefix_mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1);
        }
        __syncthreads();
        if (threadIdx.x == 0) {
            int rem = remaining, bucket = 255;
            for (; bucket > 0; --bucket) {
                int c = hist[bucket];
                if (c >= rem) break;
                rem -= c;
            }
            sh_prefix = prefix | ((uint32_t)bucket << shift);
            sh_remaining = rem;
        }
        __syncthreads();
        prefix = sh_prefix;
        remaining = sh_remaining;
        prefix_mask |= 255u << shift;
        __syncthreads();
    }
    // prefix = key of the K-th largest element; `remaining` ties are taken, lowest index first
    const uint32_t threshold = prefix;
    int taken = 0, ties_seen = 0;
    for (int base = 0; base < N; base += SEL_THREADS) {
        int i = base + threadIdx.x;
        uint32_t key = (i < N) ? score_key(s[i]) : 0u;
        bool gt = (i < N) && key > threshold;
        bool eq = (i < N) && key == threshold;
        int eq_total, sel_total;
        int eq_rank = ties_seen + block_exclusive_count(eq, scratch, eq_total);
        bool sel = gt || (eq && eq_rank < remaining);
        int pos = taken + block_exclusive_count(sel, scratch, sel_total);
        if (sel && pos < K) out[pos] = i;
        ties_seen += eq_total;
        taken += sel_total;
    }
}

}  // namespace

// ---------------------------------------------------------------- entry points
static bool movers_args_ok(const void *a, const void *b, const void *c, int B, int n1, int n2, int D)
{
    return a && b && c && ssam_aligned16(a) && ssam_aligned16(c) && B > 0 && n1 > 0 && n2 > 0 && D > 0 && D % 8 == 0;
}

static int mover_grid(long total_chunks)
{
    long blocks = (total_chunks + 255) / 256;
    return (int)(blocks < 1 ? 1 : (blocks > 256L * 32 ? 256L * 32 : blocks));
}

// ---------------------------------------------------------------- padding compaction
// SAM pads the grid up to a multiple of the window; padding slots are zero rows after LN1, so their
// qkv rows equal the bias and their attention outputs are dropped.  One workgroup per image walks the
// gather table (slot -> spatial index, -1 = padding) in slot order and writes
//   real_slot[b][c]    the slot of the c-th real token (c-th row of the compact activations)
//   real_spatial[b][c] its spatial index
//   slot_row[b][s]     b*N + c for a real slot (the compact row), -1 for padding
//   pad_slot[b][i]     the i-th padding slot
// so that the dense contractions run on the N real rows only.
__global__ void __launch_bounds__(SEL_THREADS)
compact_slots_kernel(const int32_t *__restrict__ table, int table_batch_stride, int Nout, int N,
                     int32_t *__restrict__ real_slot, int32_t *__restrict__ real_spatial,
                     int32_t *__restrict__ slot_row, int32_t *__restrict__ pad_slot)
{
    __shared__ int scratch[SEL_THREADS / 64];
    const int b = blockIdx.x, npad = Nout - N;
    const int32_t *t = table + (long)b * table_batch_stride;
    int base = 0;
    for (int s0 = 0; s0 < Nout; s0 += SEL_THREADS) {
        const int s = s0 + threadIdx.x;
        const int v = s < Nout ? t[s] : -1;
        const bool real = s < Nout && v >= 0 && v < N;
        int total;
        const int c = base + block_exclusive_count(real, scratch, total);
        if (s < Nout) {
            if (real) {
                if (c < N) {
                    real_slot[(long)b * N + c] = s;
                    real_spatial[(long)b * N + c] = v;
                }
                slot_row[(long)b * Nout + s] = c < N ? b * N + c : -1;
            } else {
                const int pc = s - c;
                if (pc < npad) pad_slot[(long)b * npad + pc] = s;
                slot_row[(long)b * Nout + s] = -1;
            }
        }
        base += total;
    }
}

// rows[b*rows_per_batch + pad_slot[b][i]] = bf16(bias) (bias == nullptr: zeros): one wave per row, 16 bytes per lane
__global__ void __launch_bounds__(256)
fill_bias_rows_kernel(bf16 *__restrict__ C, long ldc, const float *__restrict__ bias, int n_cols,
                      const int32_t *__restrict__ pad_slot, int npad, int rows_per_batch, int total_rows)
{
    const int r = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (r >= total_rows) return;
    const int b = r / npad, i = r - b * npad;
    bf16 *dst = C + ((long)b * rows_per_batch + pad_slot[(long)b * npad + i]) * ldc;
    for (int c = lane * 8; c < n_cols; c += 64 * 8) {
        if (bias == nullptr) {
            *reinterpret_cast<uint4 *>(dst + c) = make_uint4(0, 0, 0, 0);
            continue;
        }
        const float4 *b4 = reinterpret_cast<const float4 *>(bias + c);
        float4 x0 = b4[0], x1 = b4[1];
        float v[8] = { x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w };
        *reinterpret_cast<uint4 *>(dst + c) = pack_bf16x8(v);
    }
}

// ---------------------------------------------------------------- content-aware order
// One workgroup per (image, window): the window's cells are ranked by (score descending, cell index
// ascending; padding cells last) with a bitonic sort of 64-bit keys in LDS, then the stripe interleave
// sigma[g*(S/G)+t] = pi[t*G+g] (Sec. 4.1) places rank t*G+g at scan position g*(S/G)+t.
// P = the power of two >= S that is sorted; entries S..P-1 carry the largest key.
__global__ void __launch_bounds__(1024)
content_tables_kernel(const float *__restrict__ scores, int g, int w, int nws, int G, int P,
                      int32_t *__restrict__ gather_table, int32_t *__restrict__ sigma)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    unsigned long long *keys = reinterpret_cast<unsigned long long *>(smem);
    const int S = w * w, nW = nws * nws;
    const int b = blockIdx.x / nW, win = blockIdx.x % nW;
    const int wr = win / nws, wc = win % nws;
    const float *sc = scores + (long)b * g * g;
    for (int i = threadIdx.x; i < P; i += blockDim.x) {
        unsigned long long key = ~0ull;
        if (i < S) {
            const int row = wr * w + i / w, col = wc * w + i % w;
            const float m = (row < g && col < g) ? sc[row * g + col] : -INFINITY;
            key = ((unsigned long long)(~score_key(m)) << 32) | (unsigned)i;
        }
        keys[i] = key;
    }
    __syncthreads();
    for (int k = 2; k <= P; k <<= 1)
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int t = threadIdx.x; t < P / 2; t += blockDim.x) {
                const int i = 2 * t - (t & (j - 1));            // index with bit j clear
                const int p = i | j;
                const unsigned long long a = keys[i], c = keys[p];
                const bool up = (i & k) == 0;
                if ((a > c) == up) { keys[i] = c; keys[p] = a; }
            }
            __syncthreads();
        }
    const int rows = S / G;
    for (int rk = threadIdx.x; rk < S; rk += blockDim.x) {
        const int cell = (int)(keys[rk] & 0xffffffffu);
        const int pos = (rk % G) * rows + rk / G;
        const int row = wr * w + cell / w, col = wc * w + cell % w;
        const long o = ((long)b * nW + win) * S + pos;
        sigma[o] = cell;
        gather_table[o] = (row < g && col < g) ? row * g + col : -1;
    }
}

extern "C" int ssam_permute(const void *x, const int32_t *idx, void *y, int B, int Nin, int Nout, int D, void *stream)
{
    if (!movers_args_ok(x, idx, y, B, Nin, Nout, D)) return SSAM_EINVAL;
    int chunks = D / 8;
    hipLaunchKernelGGL(permute_kernel, dim3(mover_grid((long)B * Nout * chunks)), dim3(256), 0, (hipStream_t)stream,
                       (const uint4 *)x, idx, (uint4 *)y, B, Nin, Nout, chunks);
    SSAM_CHECK_LAUNCH();
    return SSAM_OK;
}

extern "C" int ssam_unpermute(const void *y, const int32_t *idx, void *x, const void *residual,
                              int B, int Nx, int Ny, int D, void *stream)
{
    if (!movers_args_ok(y, idx, x, B, Nx, Ny, D)) return SSAM_EINVAL;
    if (residual && !ssam_aligned16(residual)) return SSAM_EINVAL;
    int chunks = D / 8;
    hipLaunchKernelGGL(unpermute_kernel, dim3(mover_grid((long)B * Ny * chunks)), dim3(256), 0, (hipStream_t)stream,
                       (const uint4 *)y, idx, (uint4 *)x, (const uint4 *)residual, B, Nx, Ny, chunks);
    SSAM_CHECK_LAUNCH();
    return SSAM_OK;
}

extern "C" int ssam_ln_gather(const void *x, const int32_t *idx, int idx_batch_stride,
                              const float *gamma, const float *beta, float eps, void *y,
                              int B, int Nin, int Nout, int D, void *stream)
{
    if (!movers_args_ok(x, idx, y, B, Nin, Nout, D) || !gamma || !beta || idx_batch_stride < 0) return SSAM_EINVAL;
    if (!ssam_aligned16(gamma) || !ssam_aligned16(beta)) return SSAM_EINVAL;
    if (D > 2048) return SSAM_EUNSUPPORTED;
    int chunks = D / 8;
    long rows = (long)B * Nout;
    dim3 grid(ssam_div_up(rows, 4)), block(256);
    hipStream_t st = (hipStream_t)stream;
    if (chunks <= 128)
        hipLaunchKernelGGL(ln_gather_kernel<2>, grid, block, 0, st, (const uint4 *)x, idx, idx_batch_stride,
                           gamma, beta, eps, (uint4 *)y, B, Nin, Nout, chunks);
    else if (chunks <= 192)
        hipLaunchKernelGGL(ln_gather_kernel<3>, grid, block, 0, st, (const uint4 *)x, idx, idx_batch_stride,
                           gamma, beta, eps, (uint4 *)y, B, Nin, Nout, chunks);
    else
        hipLaunchKernelGGL(ln_gather_kernel<4>, grid, block, 0, st, (const uint4 *)x, idx, idx_batch_stride,
                           gamma, beta, eps, (uint4 *)y, B, Nin, Nout, chunks);
    SSAM_CHECK_LAUNCH();
    return SSAM_OK;
}

extern "C" size_t ssam_score_tokens_workspace_bytes(int B, int gh, int gw)
{
    if (B <= 0 || gh <= 0 || gw <= 0) return 0;
    return (size_t)B * gh * gw * sizeof(float);
}

extern "C" int ssam_score_tokens(const void *x, float *scores, int B, int gh, int gw, int D,
                                 void *workspace, size_t workspace_bytes, void *stream)
{
    if (!x || !scores || !workspace || B <= 0 || gh <= 0 || gw <= 0 || D <= 0 || D % 8 != 0) return SSAM_EINVAL;
    if (!ssam_aligned16(x) || !ssam_aligned16(workspace)) return SSAM_EINVAL;
    if (workspace_bytes < ssam_score_tokens_workspace_bytes(B, gh, gw)) return SSAM_EWORKSPACE;
    long tokens = (long)B * gh * gw;
    float *csum = (float *)workspace;
    hipLaunchKernelGGL(channel_sum_kernel, dim3(ssam_div_up(tokens, 4)), dim3(256), 0, (hipStream_t)stream,
                       (const uint4 *)x, csum, tokens, D / 8);
    SSAM_CHECK_LAUNCH();
    hipLaunchKernelGGL(sobel_kernel, dim3(ssam_div_up(tokens, 256)), dim3(256), 0, (hipStream_t)stream,
                       (const float *)csum, scores, B, gh, gw);
    SSAM_CHECK_LAUNCH();
    return SSAM_OK;
}

// ---- ssam_score_tokens for callers that cannot allocate: the channel-sum map lives in a file-scope device array.
// In host code the array's name is only a stand-in; its device address is looked up once per device and kept.
static __device__ __align__(256) float scratch[SSAM_SCORE_TOKENS_STATIC_MAX_TOKENS];

namespace {
constexpr int kMaxDevices = 64;
float *scratch_ptr[kMaxDevices];        // device address of `scratch` on each GPU this process has used it on

int scratch_on_current_device(float **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SSAM_EHIP;
    float *p = __atomic_load_n(&scratch_ptr[dev], __ATOMIC_ACQUIRE);
    if (!p) {                           // first call on this device (racing first calls resolve the same address)
        void *sym = nullptr;
        if (hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch)) != hipSuccess || !sym) return SSAM_EHIP;
        p = (float *)sym;
        __atomic_store_n(&scratch_ptr[dev], p, __ATOMIC_RELEASE);
    }
    *out = p;
    return SSAM_OK;
}
}  // namespace

extern "C" int ssam_score_tokens_static(const void *x, float *scores, int B, int gh, int gw, int D, void *stream)
{
    if (!x || !scores || B <= 0 || gh <= 0 || gw <= 0 || D <= 0 || D % 8 != 0) return SSAM_EINVAL;
    if (!ssam_aligned16(x)) return SSAM_EINVAL;
    const long tokens = (long)B * gh * gw;
    if (tokens > SSAM_SCORE_TOKENS_STATIC_MAX_TOKENS) return SSAM_EWORKSPACE;
    float *csum = nullptr;
    int rc = scratch_on_current_device(&csum);
    if (rc != SSAM_OK) return rc;
    // channel_sum_kernel writes the sum of every token it is given and sobel_kernel reads only those, so nothing
    // in the array has to start at zero and what an earlier (larger) call left behind is never read
    hipLaunchKernelGGL(channel_sum_kernel, dim3(ssam_div_up(tokens, 4)), dim3(256), 0, (hipStream_t)stream,
                       (const uint4 *)x, csum, tokens, D / 8);
    SSAM_CHECK_LAUNCH();
    hipLaunchKernelGGL(sobel_kernel, dim3(ssam_div_up(tokens, 256)), dim3(256), 0, (hipStream_t)stream,
                       (const float *)csum, scores, B, gh, gw);
    SSAM_CHECK_LAUNCH();
    return SSAM_OK;
}

extern "C" int ssam_select_tokens(const float *scores, int32_t *keep_idx, int B, int N, int K, void *stream)
{
    if (!scores || !keep_idx || B <= 0 || N <= 0 || K <= 0 || K > N) return SSAM_EINVAL;
    if (N > 65536) return SSAM_EUNSUPPORTED;
    hipLaunchKernelGGL(select_kernel, dim3(B), dim3(SEL_THREADS), 0, (hipStream_t)stream, scores, keep_idx, N, K);
    SSAM_CHECK_LAUNCH();
    return SSAM_OK;
}

extern "C" int ssam_build_content_tables(const float *scores, int B, int g, int ws, int G,
                                         int32_t *gather_table, int32_t *sigma, void *stream)
{
    if (!scores || !gather_table || !sigma || B <= 0 || g <= 0 || ws < 0 || G <= 0) return SSAM_EINVAL;
    const int w = ws > 0 ? ws : g;
    if (w > 128) return SSAM_EUNSUPPORTED;
    const int S = w * w, nws = (g + w - 1) / w;
    if (S % G != 0) return SSAM_EINVAL;
    int P = 2;
    while (P < S) P <<= 1;
    const int threads = P / 2 < 1024 ? (P / 2 < 64 ? 64 : P / 2) : 1024;
    const size_t lds = (size_t)P * sizeof(unsigned long long);
    if (lds > 64 * 1024 &&
        hipFuncSetAttribute(reinterpret_cast<const void *>(content_tables_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
        return SSAM_EHIP;
    hipLaunchKernelGGL(content_tables_kernel, dim3(B * nws * nws), dim3(threads), lds, (hipStream_t)stream,
                       scores, g, w, nws, G, P, gather_table, sigma);
    SSAM_CHECK_LAUNCH();
    return SSAM_OK;
}

// internal (block composition): see compact_slots_kernel / fill_bias_rows_kernel
int ssam_compact_slots(const int32_t *table, int table_batch_stride, int B, int Nout, int N,
                       int32_t *real_slot, int32_t *real_spatial, int32_t *slot_row, int32_t *pad_slot, hipStream_t st)
{
    hipLaunchKernelGGL(compact_slots_kernel, dim3(B), dim3(SEL_THREADS), 0, st, table, table_batch_stride, Nout, N,
                       real_slot, real_spatial, slot_row, pad_slot);
    SSAM_CHECK_LAUNCH();
    return SSAM_OK;
}

int ssam_fill_bias_rows(void *C, long ldc, const float *bias, int n_cols, const int32_t *pad_slot, int npad,
                        int rows_per_batch, int B, hipStream_t st)
{
    const int total = B * npad;
    if (total <= 0) return SSAM_OK;
    hipLaunchKernelGGL(fill_bias_rows_kernel, dim3(ssam_div_up(total, 4)), dim3(256), 0, st, (bf16 *)C, ldc, bias, n_cols,
                       pad_slot, npad, rows_per_batch, total);
    SSAM_CHECK_LAUNCH();
    return SSAM_OK;
}

// statistics of rows idx[b][p] of image b (idx == NULL: of every row in order), see ln_stats_kernel
int ssam_ln_stats_impl(const void *x, float *stats, long rows, int D, float eps, const int32_t *idx, int idx_batch_stride,
                       int Nin, int Nout, int32_t *src, hipStream_t st)
{
    if (!x || !stats || rows <= 0 || D <= 0 || D % 8 != 0) return SSAM_EINVAL;
    if (!ssam_aligned16(x) || ((uintptr_t)stats & 7)) return SSAM_EINVAL;
    if (idx && (!src || Nin <= 0 || Nout <= 0 || (long)(rows / Nout) * Nin > 0x7fffffffL)) return SSAM_EINVAL;
    if (D > 2048) return SSAM_EUNSUPPORTED;
    int chunks = D / 8;
    dim3 grid((unsigned)ssam_div_up(rows, 4)), block(256);
    if (chunks <= 128)
        hipLaunchKernelGGL(ln_stats_kernel<2>, grid, block, 0, st, (const uint4 *)x, (float2 *)stats, rows, chunks, eps, idx, idx_batch_stride, Nin, Nout, src);
    else if (chunks <= 192)
        hipLaunchKernelGGL(ln_stats_kernel<3>, grid, block, 0, st, (const uint4 *)x, (float2 *)stats, rows, chunks, eps, idx, idx_batch_stride, Nin, Nout, src);
    else
        hipLaunchKernelGGL(ln_stats_kernel<4>, grid, block, 0, st, (const uint4 *)x, (float2 *)stats, rows, chunks, eps, idx, idx_batch_stride, Nin, Nout, src);
    SSAM_CHECK_LAUNCH();
    return SSAM_OK;
}

extern "C" int ssam_ln_stats(const void *x, float *stats, long rows, int D, float eps, void *stream)
{
    return ssam_ln_stats_impl(x, stats, rows, D, eps, nullptr, 0, 0, 0, nullptr, (hipStream_t)stream);
}

extern "C" int ssam_fold_ln_weight(const void *W, int ldw, const float *bias, const float *gamma, const float *beta,
                                   void *Wf, float *colsum, float *bias_f, int N, int K, void *stream)
{
    if (!W || !bias || !gamma || !beta || !Wf || !colsum || !bias_f || N <= 0 || K <= 0 || ldw < K || ldw % 8) return SSAM_EINVAL;
    if (!ssam_aligned16(W) || !ssam_aligned16(Wf)) return SSAM_EINVAL;
    if (K % 8 != 0) return SSAM_EUNSUPPORTED;
    hipLaunchKernelGGL(fold_ln_weight_kernel, dim3(ssam_div_up(N, 4)), dim3(256), 0, (hipStream_t)stream,
                       (const bf16 *)W, ldw, bias, gamma, beta, (bf16 *)Wf, colsum, bias_f, N, K);
    SSAM_CHECK_LAUNCH();
    return SSAM_OK;
}

// internal (block composition): see invert_table_kernel
int ssam_invert_table(const int32_t *table, int table_batch_stride, int B, int Nout, int N, int32_t *inv, hipStream_t st)
{
    const int total = B * Nout;
    hipLaunchKernelGGL(invert_table_kernel, dim3(ssam_div_up(total, 256)), dim3(256), 0, st, table, table_batch_stride, Nout, N, inv, total);
    SSAM_CHECK_LAUNCH();
    return SSAM_OK;
}

extern "C" int ssam_fold_kv_bias(const float *bias_in, const float *bqkv, const void *wproj, const float *bproj,
                                 float *bias_out, float *bproj_out, int D, void *stream)
{
    if (!bias_in || !bqkv || !wproj || !bproj || !bias_out || !bproj_out || D <= 0) return SSAM_EINVAL;
    if (!ssam_aligned16(wproj)) return SSAM_EINVAL;
    if (D % 8 != 0) return SSAM_EUNSUPPORTED;
    hipLaunchKernelGGL(fold_kv_bias_kernel, dim3(ssam_div_up(3 * D, 4)), dim3(256), 0, (hipStream_t)stream,
                       bias_in, bqkv, (const bf16 *)wproj, bproj, bias_out, bproj_out, D);
    SSAM_CHECK_LAUNCH();
    return SSAM_OK;
}
