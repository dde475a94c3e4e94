// Rotary position embedding of q and k, in place, with each token's ORIGINAL position (the compacted
// active sequence of Sec. 3.4 keeps the position ids of the backbone: Qwen2.5 / Llama-3, Sec. 4.1).
// "Rotate-half" pairing: for a head vector u, i < dh/2 and angle a = pos * theta^(-2i/dh):
//     u[i], u[i + dh/2]  <-  u[i] cos a - u[i + dh/2] sin a,   u[i] sin a + u[i + dh/2] cos a.
// Front end of a layer in a chain: it sits before the path proper, next to the q/k/v projections.
//
// HBM-bound (every q and k element is read and written once). One wave per row: the angle depends on
// (row, i) only, so each lane computes the sine and cosine of its two frequencies once - in fp64, positions
// reach 131072 and an fp32 product pos * frequency would be off by several 1e-3 rad - and reuses them
// for every head.
#include "common.h"

namespace dash {

template <int DH>
__global__ __launch_bounds__(256) void rope_qk_kernel(__bf16* __restrict__ q, __bf16* __restrict__ k,
                                                      const int32_t* __restrict__ pos, int n, int Hq, int Hkv,
                                                      double neg_log2_theta_2_over_dh) {
    constexpr int HALF = DH / 2;
    constexpr int LPH = HALF / 2;      // lanes per head: each lane owns two adjacent frequencies
    constexpr int HPI = kWave / LPH;   // heads per wave iteration
    const int row = (int)((blockIdx.x * (size_t)blockDim.x + threadIdx.x) / kWave);
    const int lane = threadIdx.x % kWave;
    if (row >= n) return;
    const int i0 = 2 * (lane % LPH), hsel = lane / LPH;
    const double p = (double)pos[row];
    float cs[2], sn[2];
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        const double inv_freq = exp2((double)(i0 + e) * neg_log2_theta_2_over_dh);  // theta^(-2i/dh)
        double a = p * inv_freq;
        a -= 6.283185307179586476925286766559 * rint(a * 0.15915494309189533576888376337251);
        double s, c;
        sincos(a, &s, &c);
        cs[e] = (float)c;
        sn[e] = (float)s;
    }
    auto rotate = [&](__bf16* base, int heads) {
        for (int h0 = 0; h0 < heads; h0 += HPI) {
            const int hd = h0 + hsel;
            if (hd >= heads) continue;
            __bf16* u = base + ((size_t)row * heads + hd) * DH + i0;
            const bf16x2 lo = *reinterpret_cast<const bf16x2*>(u);
            const bf16x2 hi = *reinterpret_cast<const bf16x2*>(u + HALF);
            bf16x2 olo, ohi;
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const float a = (float)lo[e], b = (float)hi[e];
                olo[e] = (__bf16)(a * cs[e] - b * sn[e]);
                ohi[e] = (__bf16)(a * sn[e] + b * cs[e]);
            }
            *reinterpret_cast<bf16x2*>(u) = olo;
            *reinterpret_cast<bf16x2*>(u + HALF) = ohi;
        }
    };
    rotate(q, Hq);
    rotate(k, Hkv);
}

dash_status launch_rope_qk(const dash_layer_params& p, void* q, void* k, const int32_t* active_idx, int n,
                           double theta, hipStream_t s) {
    if (n == 0) return DASH_OK;
    const double c = -log2(theta) * 2.0 / (double)p.head_dim;
    const int blocks = (int)(((size_t)n * kWave + 255) / 256);
    if (p.head_dim == 64)
        hipLaunchKernelGGL(rope_qk_kernel<64>, dim3(blocks), dim3(256), 0, s, (__bf16*)q, (__bf16*)k, active_idx, n,
                           p.n_q_heads, p.n_kv_heads, c);
    else
        hipLaunchKernelGGL(rope_qk_kernel<128>, dim3(blocks), dim3(256), 0, s, (__bf16*)q, (__bf16*)k, active_idx,
                           n, p.n_q_heads, p.n_kv_heads, c);
    return launch_status();
}

}  // namespace dash
