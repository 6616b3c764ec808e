// Instrumentation, not part of the method: what the matrix cores of the box in hand sustain, for the benchmark's
// "measured peaks".  A loop of independent bf16 MFMAs on register operands, no memory traffic: the rate a contraction
// could reach if operands cost nothing, at the clock the chip settles at under that load (it is power limited: the
// shader clock falls below its 2.4 GHz maximum under matrix work, and by how much depends on the instruction shape).
#include "common.h"

namespace {

template <int SHAPE>
__global__ void __launch_bounds__(256) mfma_loop_kernel(float *sink, int iters)
{
    bf16x8 a[2], b[2];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            a[j][e] = (bf16)((threadIdx.x & 7) * 0.125f + e + j);
            b[j][e] = (bf16)((threadIdx.x & 3) * 0.25f - e - j);
        }
    float s = 0.f;
    if (SHAPE == 0) {           // 8 x (32x32x16): 8 * 32768 flops per wave and iteration
        f32x16 acc[8];
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i & 1], b[i >> 2], acc[i], 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) s += acc[i][r];
    } else {                    // 16 x (16x16x32): the same flops
        f32x4 acc[16];
#pragma unroll
        for (int i = 0; i < 16; ++i)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[i][r] = 0.f;
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i & 1], b[i >> 3], acc[i], 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < 16; ++i)
#pragma unroll
            for (int r = 0; r < 4; ++r) s += acc[i][r];
    }
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

}  // namespace

extern "C" double ssam_probe_mfma_flops(int workgroups, int iters)
{
    if (workgroups <= 0 || iters <= 0) return 0.0;
    return (double)workgroups * 4.0 * (double)iters * 8.0 * 2.0 * 32.0 * 32.0 * 16.0;
}

extern "C" int ssam_probe_mfma(int shape, int workgroups, int iters, float *sink, void *stream)
{
    if (!sink || workgroups <= 0 || workgroups > 65536 || iters <= 0 || (shape != 0 && shape != 1)) return SSAM_EINVAL;
    if (shape == 0)
        hipLaunchKernelGGL(mfma_loop_kernel<0>, dim3(workgroups), dim3(256), 0, (hipStream_t)stream, sink, iters);
    else
        hipLaunchKernelGGL(mfma_loop_kernel<1>, dim3(workgroups), dim3(256), 0, (hipStream_t)stream, sink, iters);
    SSAM_CHECK_LAUNCH();
    return SSAM_OK;
}
