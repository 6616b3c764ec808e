// Encoder ends of the SAM ViT image encoder around the structured-sparse blocks: patch embedding +
// absolute position embedding in front, the neck behind (public SAM architecture; the paper measures the
// whole encoder and changes only the blocks).  Both are dense contractions on the library's GEMM, fed by
// two small gather kernels (patch -> row, 3x3 neighbourhood -> row), so the ends add no new math kernels:
//   tokens = pos + patches W_pe^T + b        (GEMM epilogue adds into rows pre-set to pos: one rounding)
//   neck   = LN(conv3x3(LN(tokens W_1^T)))   (1x1 conv = GEMM; 3x3 conv = GEMM over gathered 9*C rows)
#include "gemm_kernel.h"

int ssam_linear_impl(const void *A, const void *W, const float *bias, void *C, int M, int N, int K,
                     const GemmLd &ld, bool packed, int epilogue, const GemmRowMap &rm, int tile,
                     void *split_ws, size_t split_ws_bytes, hipStream_t st);

namespace {

inline size_t align256(size_t n) { return (n + 255) & ~(size_t)255; }

// A[(b*gh + ty)*gw + tx][(c*P + ky)*P + kx] = img[b][c][ty*P + ky][tx*P + kx]; one thread per 8 pixels of a patch row
__global__ void __launch_bounds__(256)
patch_rows_kernel(const bf16 *__restrict__ img, bf16 *__restrict__ A, int B, int H, int W, int P)
{
    const int gh = H / P, gw = W / P, cpr = P / 8;             // 16-byte chunks per patch row
    const long total = (long)B * gh * gw * 3 * P * cpr;
    const long id = (long)blockIdx.x * 256 + threadIdx.x;
    if (id >= total) return;
    const int ch = (int)(id % cpr);
    long t = id / cpr;
    const int ky = (int)(t % P); t /= P;
    const int c = (int)(t % 3); t /= 3;
    const int tx = (int)(t % gw); t /= gw;
    const int ty = (int)(t % gh);
    const int b = (int)(t / gh);
    const u32x4 v = *reinterpret_cast<const u32x4 *>(img + (((long)b * 3 + c) * H + ty * P + ky) * W + tx * P + ch * 8);
    *reinterpret_cast<u32x4 *>(A + (((long)b * gh + ty) * gw + tx) * (3L * P * P) + ((long)c * P + ky) * P + ch * 8) = v;
}

// x[b][t][:] = pos[t][:] and map[t] = t
__global__ void __launch_bounds__(256)
broadcast_pos_kernel(const u32x4 *__restrict__ pos, u32x4 *__restrict__ x, int32_t *__restrict__ map, int B, int N, int chunks)
{
    const long id = (long)blockIdx.x * 256 + threadIdx.x;
    if (id < N) map[id] = (int32_t)id;
    if (id >= (long)B * N * chunks) return;
    x[id] = pos[id % ((long)N * chunks)];
}

// A[(b*g + ty)*g + tx][(ky*3 + kx)*C + c] = y[b][ty+ky-1][tx+kx-1][c], zero outside the grid
__global__ void __launch_bounds__(256)
conv3_rows_kernel(const u32x4 *__restrict__ y, u32x4 *__restrict__ A, int B, int g, int chunks)
{
    const long total = (long)B * g * g * 9 * chunks;
    const long id = (long)blockIdx.x * 256 + threadIdx.x;
    if (id >= total) return;
    const int ch = (int)(id % chunks);
    long t = id / chunks;
    const int tap = (int)(t % 9); t /= 9;
    const int tx = (int)(t % g); t /= g;
    const int ty = (int)(t % g);
    const int b = (int)(t / g);
    const int sy = ty + tap / 3 - 1, sx = tx + tap % 3 - 1;
    u32x4 v = { 0, 0, 0, 0 };
    if (sy >= 0 && sy < g && sx >= 0 && sx < g) v = y[(((long)b * g + sy) * g + sx) * chunks + ch];
    A[id] = v;
}

__global__ void __launch_bounds__(256)
zero_iota_kernel(float *__restrict__ zeros, int nz, int32_t *__restrict__ map, int nm)
{
    const int id = blockIdx.x * 256 + threadIdx.x;
    if (id < nz) zeros[id] = 0.f;
    if (id < nm) map[id] = id;
}

}  // namespace

extern "C" size_t ssam_patch_embed_workspace_bytes(int B, int H, int W, int P)
{
    if (B <= 0 || H <= 0 || W <= 0 || P <= 0 || H % P || W % P) return 0;
    const size_t N = (size_t)(H / P) * (W / P);
    return align256((size_t)B * N * 3 * P * P * 2) + align256(N * 4) + GEMM_SPLIT_WS_BYTES;
}

extern "C" int ssam_patch_embed(const void *img, const void *w, const float *bias, const void *pos, void *x,
                                int B, int H, int W, int P, int D, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!img || !w || !bias || !pos || !x || !workspace || B <= 0 || H <= 0 || W <= 0 || P <= 0 || D <= 0) return SSAM_EINVAL;
    if (H % P || W % P) return SSAM_EINVAL;
    if (!ssam_aligned16(img) || !ssam_aligned16(w) || !ssam_aligned16(bias) || !ssam_aligned16(pos) || !ssam_aligned16(x) ||
        !ssam_aligned16(workspace))
        return SSAM_EINVAL;
    const int Kc = 3 * P * P;
    if (P % 8 != 0 || D % 128 != 0 || Kc % GEMM_BK != 0) return SSAM_EUNSUPPORTED;
    if (workspace_bytes < ssam_patch_embed_workspace_bytes(B, H, W, P)) return SSAM_EWORKSPACE;
    const int N = (H / P) * (W / P);
    unsigned char *ws = (unsigned char *)workspace;
    bf16 *A = (bf16 *)ws;
    int32_t *map = (int32_t *)(ws + align256((size_t)B * N * Kc * 2));
    void *split = ws + align256((size_t)B * N * Kc * 2) + align256((size_t)N * 4);
    hipStream_t st = (hipStream_t)stream;
    const long chunks = (long)B * N * Kc / 8;
    hipLaunchKernelGGL(patch_rows_kernel, dim3((unsigned)ssam_div_up(chunks, 256)), dim3(256), 0, st, (const bf16 *)img, A, B, H, W, P);
    SSAM_CHECK_LAUNCH();
    const long xchunks = (long)B * N * (D / 8);
    hipLaunchKernelGGL(broadcast_pos_kernel, dim3((unsigned)ssam_div_up(xchunks > N ? xchunks : N, 256)), dim3(256), 0, st,
                       (const u32x4 *)pos, (u32x4 *)x, map, B, N, D / 8);
    SSAM_CHECK_LAUNCH();
    GemmRowMap ident = { map, N, 0, N };
    return ssam_linear_impl(A, w, bias, x, B * N, D, Kc, GemmLd{ Kc, Kc, D }, false, SSAM_EPI_BIAS_SCATTER_ADD, ident, 0,
                            split, GEMM_SPLIT_WS_BYTES, st);
}

extern "C" size_t ssam_neck_workspace_bytes(int B, int g, int D, int C)
{
    if (B <= 0 || g <= 0 || D <= 0 || C <= 0) return 0;
    const size_t rows = (size_t)B * g * g;
    // y (1x1 conv), its LayerNorm, the 9*C gathered rows, the 3x3 conv result; zero bias; identity map; K-split scratch
    return align256(rows * C * 2) * 3 + align256(rows * 9 * C * 2) + align256((size_t)C * 4) + align256((size_t)g * g * 4) +
           GEMM_SPLIT_WS_BYTES;
}

extern "C" int ssam_neck(const void *x, const void *w1, const float *ln1_g, const float *ln1_b,
                         const void *w2, const float *ln2_g, const float *ln2_b, float eps, void *out,
                         int B, int g, int D, int C, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!x || !w1 || !ln1_g || !ln1_b || !w2 || !ln2_g || !ln2_b || !out || !workspace || B <= 0 || g <= 0 || D <= 0 || C <= 0)
        return SSAM_EINVAL;
    if (!ssam_aligned16(x) || !ssam_aligned16(w1) || !ssam_aligned16(w2) || !ssam_aligned16(out) || !ssam_aligned16(workspace))
        return SSAM_EINVAL;
    if (C % 128 != 0 || D % GEMM_BK != 0) return SSAM_EUNSUPPORTED;
    if (workspace_bytes < ssam_neck_workspace_bytes(B, g, D, C)) return SSAM_EWORKSPACE;
    const int N = g * g, rows = B * N;
    unsigned char *p = (unsigned char *)workspace;
    bf16 *y1 = (bf16 *)p; p += align256((size_t)rows * C * 2);
    bf16 *y2 = (bf16 *)p; p += align256((size_t)rows * C * 2);
    bf16 *y3 = (bf16 *)p; p += align256((size_t)rows * C * 2);
    bf16 *A2 = (bf16 *)p; p += align256((size_t)rows * 9 * C * 2);
    float *zeros = (float *)p; p += align256((size_t)C * 4);
    int32_t *map = (int32_t *)p; p += align256((size_t)N * 4);
    void *split = p;
    hipStream_t st = (hipStream_t)stream;
    hipLaunchKernelGGL(zero_iota_kernel, dim3(ssam_div_up(N > C ? N : C, 256)), dim3(256), 0, st, zeros, C, map, N);
    SSAM_CHECK_LAUNCH();
    GemmRowMap none = { nullptr, 1, 0, 1 };
    int rc = ssam_linear_impl(x, w1, zeros, y1, rows, C, D, GemmLd{ D, D, C }, false, SSAM_EPI_BIAS, none, 0, split, GEMM_SPLIT_WS_BYTES, st);
    if (rc != SSAM_OK) return rc;
    rc = ssam_ln_gather(y1, map, 0, ln1_g, ln1_b, eps, y2, B, N, N, C, stream);
    if (rc != SSAM_OK) return rc;
    const long chunks = (long)rows * 9 * (C / 8);
    hipLaunchKernelGGL(conv3_rows_kernel, dim3((unsigned)ssam_div_up(chunks, 256)), dim3(256), 0, st, (const u32x4 *)y2, (u32x4 *)A2, B, g, C / 8);
    SSAM_CHECK_LAUNCH();
    rc = ssam_linear_impl(A2, w2, zeros, y3, rows, C, 9 * C, GemmLd{ 9 * C, 9 * C, C }, false, SSAM_EPI_BIAS, none, 0, split, GEMM_SPLIT_WS_BYTES, st);
    if (rc != SSAM_OK) return rc;
    return ssam_ln_gather(y3, map, 0, ln2_g, ln2_b, eps, out, B, N, N, C, stream);
}
