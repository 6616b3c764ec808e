// Integer layout layer: Z-order / stripe-sort scan tables, window-major gather
// table, A-shape block mask (Sec. 4.1; Fig. 2 caption; App. A.1 Alg. 1).
#include <algorithm>
#include <utility>
#include <vector>

#include "common.h"

namespace {

// Spread the low 16 bits of v onto the even bit positions.
inline uint32_t spread16(uint32_t v)
{
    v &= 0xffffu;
    v = (v | (v << 8)) & 0x00ff00ffu;
    v = (v | (v << 4)) & 0x0f0f0f0fu;
    v = (v | (v << 2)) & 0x33333333u;
    v = (v | (v << 1)) & 0x55555555u;
    return v;
}

// Z-order rank of every cell of a gh x gw grid (column bits even, row bits odd);
// cells of a non power-of-two grid are ranked by their code.
int z_order(int gh, int gw, std::vector<int32_t> &pi)
{
    if (gh <= 0 || gw <= 0 || gh > 32768 || gw > 32768) return SSAM_EINVAL;
    std::vector<std::pair<uint32_t, int32_t>> cells;
    cells.reserve((size_t)gh * gw);
    for (int row = 0; row < gh; ++row)
        for (int col = 0; col < gw; ++col)
            cells.emplace_back(spread16((uint32_t)col) | (spread16((uint32_t)row) << 1), row * gw + col);
    std::sort(cells.begin(), cells.end());
    pi.resize(cells.size());
    for (size_t p = 0; p < cells.size(); ++p) pi[p] = cells[p].second;
    return SSAM_OK;
}

// One thread per cell.  The Z-order rank of a cell is the number of grid cells
// with a smaller code; walking the quadtree from the top, every sibling quadrant
// that precedes the cell's own quadrant lies wholly before it, so the rank is
// the sum of those quadrants' overlaps with the grid.
__global__ void perm_kernel(int gh, int gw, int G, int levels, int32_t *perm, int32_t *inv)
{
    int cell = blockIdx.x * blockDim.x + threadIdx.x;
    int n = gh * gw;
    if (cell >= n) return;
    int row = cell / gw, col = cell % gw;
    int rank = 0;
    for (int b = levels - 1; b >= 0; --b) {
        int size = 1 << b;
        int r0 = (row >> (b + 1)) << (b + 1), c0 = (col >> (b + 1)) << (b + 1);
        int digit = (((row >> b) & 1) << 1) | ((col >> b) & 1);
        for (int q = 0; q < digit; ++q) {
            int qr = r0 + (q >> 1) * size, qc = c0 + (q & 1) * size;
            int hr = min(qr + size, gh) - qr, wc = min(qc + size, gw) - qc;
            if (hr > 0 && wc > 0) rank += hr * wc;
        }
    }
    int pos = (rank % G) * (n / G) + rank / G;   // sigma[g*(n/G)+t] = pi[t*G+g]
    perm[pos] = cell;
    if (inv) inv[cell] = pos;
}

}  // namespace

extern "C" int ssam_build_perm(int gh, int gw, int G, int32_t *perm, int32_t *inv)
{
    if (!perm || G < 1 || gh <= 0 || gw <= 0) return SSAM_EINVAL;
    long n = (long)gh * gw;
    if (n % G != 0) return SSAM_EINVAL;
    std::vector<int32_t> pi;
    int rc = z_order(gh, gw, pi);
    if (rc != SSAM_OK) return rc;
    long rows = n / G;
    for (long t = 0; t < rows; ++t)
        for (int g = 0; g < G; ++g) perm[g * rows + t] = pi[t * G + g];
    if (inv)
        for (long p = 0; p < n; ++p) inv[perm[p]] = (int32_t)p;
    return SSAM_OK;
}

extern "C" int ssam_build_perm_device(int gh, int gw, int G, int32_t *perm_dev, int32_t *inv_dev, void *stream)
{
    if (!perm_dev || G < 1 || gh <= 0 || gw <= 0 || gh > 1024 || gw > 1024) return SSAM_EINVAL;
    int n = gh * gw;
    if (n % G != 0) return SSAM_EINVAL;
    int levels = 0;
    while ((1 << levels) < std::max(gh, gw)) ++levels;
    hipLaunchKernelGGL(perm_kernel, dim3(ssam_div_up(n, 256)), dim3(256), 0, (hipStream_t)stream,
                       gh, gw, G, levels, perm_dev, inv_dev);
    SSAM_CHECK_LAUNCH();
    return SSAM_OK;
}

extern "C" int ssam_build_window_table(int g, int ws, int G, int32_t *table)
{
    if (!table || g <= 0 || ws <= 0 || G < 1) return SSAM_EINVAL;
    int S = ws * ws;
    if (S % G != 0) return SSAM_EINVAL;
    std::vector<int32_t> sigma(S);
    int rc = ssam_build_perm(ws, ws, G, sigma.data(), nullptr);
    if (rc != SSAM_OK) return rc;
    int nws = (g + ws - 1) / ws;
    for (int win = 0; win < nws * nws; ++win) {
        int row0 = (win / nws) * ws, col0 = (win % nws) * ws;
        for (int p = 0; p < S; ++p) {
            int row = row0 + sigma[p] / ws, col = col0 + sigma[p] % ws;
            table[(long)win * S + p] = (row < g && col < g) ? row * g + col : -1;
        }
    }
    return SSAM_OK;
}

extern "C" int ssam_build_block_mask(int S, int mask_block, double r, int32_t *row_ptr, int32_t *col_idx, int *n_pre)
{
    if (!row_ptr || !col_idx || S <= 0 || mask_block <= 0 || !(r > 0.0) || r > 1.0) return SSAM_EINVAL;
    int T = (S + mask_block - 1) / mask_block;
    int pre = ssam_prefix_tiles(T, r);
    int nnz = 0;
    for (int i = 0; i < T; ++i) {
        row_ptr[i] = nnz;
        for (int j = 0; j < pre; ++j) col_idx[nnz++] = j;
        if (i >= pre) col_idx[nnz++] = i;
    }
    row_ptr[T] = nnz;
    if (n_pre) *n_pre = pre;
    return SSAM_OK;
}

extern "C" int ssam_keep_count(int N, double rho)
{
    if (N <= 0 || !(rho > 0.0) || rho > 1.0) return SSAM_EINVAL;
    long K = (long)__builtin_floor(rho * (double)N + 1e-6);
    if (K < 1) K = 1;
    if (K > N) K = N;
    return (int)K;
}

extern "C" const char *ssam_status_string(int status)
{
    switch (status) {
    case SSAM_OK: return "ok";
    case SSAM_EINVAL: return "invalid argument";
    case SSAM_EUNSUPPORTED: return "unsupported shape";
    case SSAM_EWORKSPACE: return "workspace too small";
    case SSAM_EHIP: return "HIP runtime error";
    default: return "unknown status";
    }
}
