// Measurement aid, not a step of the method: what the matrix pipe of this part sustains with nothing else running.
// A register-only loop of independent bf16 MFMAs (no memory traffic, no LDS), 8 waves per compute unit, in the two
// instruction shapes the library uses (32x32x16 in the attention kernel, 16x16x32 in the GEMMs) and on two kinds of
// operand data: zeros, and normally distributed values as in the workloads. The part holds its power limit by
// lowering its clock, and the power of the matrix pipe grows with the bits that toggle in its operands, so the
// sustained rate on N(0,1) data is well below the published peak that zeros reach; the benchmark prints these
// figures beside the published 2.5 PFLOP/s so the roofline fractions can be read against both.
#include "common.h"

namespace dash {

__device__ __forceinline__ uint32_t probe_hash(uint32_t x) {
    x ^= x >> 16;
    x *= 0x7feb352dU;
    x ^= x >> 15;
    x *= 0x846ca68bU;
    x ^= x >> 16;
    return x;
}

// one N(0,1) draw per seed (Box-Muller on two hashed uniforms); only the distribution matters here
__device__ __forceinline__ float probe_normal(uint32_t seed) {
    const float u1 = (float)(probe_hash(seed) >> 8) * (1.0f / 16777216.0f) + 1e-7f;
    const float u2 = (float)(probe_hash(seed ^ 0x9e3779b9U) >> 8) * (1.0f / 16777216.0f);
    return sqrtf(-2.0f * __logf(u1)) * __cosf(6.2831853f * u2);
}

constexpr int kProbeThreads = 512;  // 8 waves per workgroup, one workgroup per compute unit

// WIDE: 32x32x16 (16 independent MFMAs per iteration and wave), else 16x16x32 (32 per iteration): 524288 flops
// per iteration and wave either way.
template <bool WIDE>
__global__ __launch_bounds__(kProbeThreads) void mfma_probe_kernel(int normal_data, int iters, float* __restrict__ sink) {
    bf16x8 a[4], b[4];
    const uint32_t tid = blockIdx.x * blockDim.x + threadIdx.x;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const uint32_t seed = tid * 131u + (uint32_t)(i * 8 + e);
            a[i][e] = (__bf16)(normal_data ? probe_normal(seed) : 0.f);
            b[i][e] = (__bf16)(normal_data ? probe_normal(seed + 0x51ed27u) : 0.f);
        }
    float total = 0.f;
    if (WIDE) {
        f32x16 acc[4];
#pragma unroll
        for (int c = 0; c < 4; ++c)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[c][r] = 0.f;
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(u + c) & 3], b[u], acc[c], 0, 0, 0);
        }
#pragma unroll
        for (int c = 0; c < 4; ++c)
#pragma unroll
            for (int r = 0; r < 16; ++r) total += acc[c][r];
    } else {
        f32x4 acc[8];
#pragma unroll
        for (int c = 0; c < 8; ++c)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[c][r] = 0.f;
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int c = 0; c < 8; ++c)
                    acc[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[(u + c) & 3], b[u], acc[c], 0, 0, 0);
        }
#pragma unroll
        for (int c = 0; c < 8; ++c)
#pragma unroll
            for (int r = 0; r < 4; ++r) total += acc[c][r];
    }
    sink[tid] = total;  // keeps the accumulators alive; the values are never read back
}

dash_status launch_mfma_probe(int wide, int normal_data, int iters, int workgroups, float* sink, hipStream_t s) {
    if (wide)
        hipLaunchKernelGGL(mfma_probe_kernel<true>, dim3(workgroups), dim3(kProbeThreads), 0, s, normal_data, iters, sink);
    else
        hipLaunchKernelGGL(mfma_probe_kernel<false>, dim3(workgroups), dim3(kProbeThreads), 0, s, normal_data, iters, sink);
    return launch_status();
}

}  // namespace dash
