// Causal grouped-query attention forward over the compacted active rows (Attn of Eq. 1, before the
// output projection). Tiled online-softmax: the probability matrix is never written to HBM, which is
// the property the paper needs from its attention operator (no attention matrix is materialised).
//
// Causality is defined on ORIGINAL positions (active_idx). Because active_idx is strictly increasing,
// "position of key <= position of query" equals "rank of key <= rank of query"; whole tiles are
// skipped by rank and the elements of diagonal tiles are masked by comparing positions.
//
// Two kernels:
//   flash_fwd_mfma<DH>  bf16, MFMA 32x32x16, fp32 softmax and accumulation (the hot kernel)
//   flash_fwd_simple<T> one wave per (row, head), plain FMA; the fp32 path
#include "common.h"

namespace dash {

// ------------------------------------------------------------------------------------------------
// Plain kernel: one wave per (query row, head). Lane j scores key j of a 64-key block, then all
// lanes accumulate their own head dims.
// ------------------------------------------------------------------------------------------------
template <typename T, int DH>
__global__ __launch_bounds__(64) void flash_fwd_simple(const T* __restrict__ q, const T* __restrict__ k,
                                                       const T* __restrict__ v,
                                                       const int32_t* __restrict__ pos, T* __restrict__ o,
                                                       int n, int Hq, int Hkv, float scale, int causal) {
    constexpr int DPL = DH / kWave;  // head dims per lane
    __shared__ float qs[DH];
    const int i = blockIdx.x, h = blockIdx.y, lane = threadIdx.x;
    const int g = h / (Hq / Hkv);
    const T* qi = q + ((size_t)i * Hq + h) * DH;
    for (int c = lane; c < DH; c += kWave) qs[c] = to_float(qi[c]);
    __syncthreads();
    const int limit = causal ? i + 1 : n;
    const int pos_i = pos[i];
    float m = -INFINITY, l = 0.f;
    float acc[DPL];
#pragma unroll
    for (int c = 0; c < DPL; ++c) acc[c] = 0.f;
    for (int j0 = 0; j0 < limit; j0 += kWave) {
        const int j = j0 + lane;
        const bool valid = j < limit && (!causal || pos[j] <= pos_i);
        float s = -INFINITY;
        if (valid) {
            const T* kj = k + ((size_t)j * Hkv + g) * DH;
            float dot = 0.f;
#pragma unroll 8
            for (int c = 0; c < DH; ++c) dot = fmaf(qs[c], to_float(kj[c]), dot);
            s = dot * scale;
        }
        float mx = s;
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
        const float m_new = fmaxf(m, mx);  // finite: key j0 (rank <= i) is always visible
        const float alpha = expf(m - m_new);
        const float p = valid ? expf(s - m_new) : 0.f;
        float ps = p;
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) ps += __shfl_xor(ps, off);
        l = l * alpha + ps;
#pragma unroll
        for (int c = 0; c < DPL; ++c) acc[c] *= alpha;
        const int cnt = min(kWave, limit - j0);
        for (int jj = 0; jj < cnt; ++jj) {
            const float pj = __shfl(p, jj);
            const T* vj = v + ((size_t)(j0 + jj) * Hkv + g) * DH + lane * DPL;
#pragma unroll
            for (int c = 0; c < DPL; ++c) acc[c] = fmaf(pj, to_float(vj[c]), acc[c]);
        }
        m = m_new;
    }
    T* oi = o + ((size_t)i * Hq + h) * DH + lane * DPL;
#pragma unroll
    for (int c = 0; c < DPL; ++c) oi[c] = from_float<T>(acc[c] / l);
}

// ------------------------------------------------------------------------------------------------
// MFMA kernel.
//
// Workgroup = 4 waves = 128 query rows of one head; wave w owns rows 32w..32w+31. Keys/values come in
// tiles of 64, staged through LDS in their natural [key][dim] layout.
//
//   S^T = K Q^T   (A = K fragment from LDS, B = Q fragment held in registers for the whole kernel):
//         with the 32x32 accumulator layout each lane then holds 16 scores of ONE query per 32-key
//         block, so row max / row sum are in-lane reductions plus one exchange with lane^32.
//   O^T += V^T P^T (A = V^T fragment via LDS transpose reads, B = P^T): the accumulator registers of
//         S^T, converted to bf16, already ARE the B fragment - no shuffle, no LDS round trip.
//
// MFMA 32x32x16 operand layout (lane l, i = l%32, h = l/32): A holds row i, k-slots 8h..8h+7;
// B holds column i, k-slots 8h..8h+7; D register r holds row 8*(r/4) + 4h + r%4 of column i.
// ------------------------------------------------------------------------------------------------
constexpr int kFaBM = 128;  // query rows per workgroup
constexpr int kFaBN = 64;   // keys per tile
constexpr float kMaskedScore = -1.0e30f;

typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;

// LDS transpose read: within each group of 16 lanes, lane t supplies the address of 4 consecutive
// 16-bit elements of row t/4 (columns 4*(t%4)..+3) of a 4x16 block and receives column t of the block.
__device__ __forceinline__ s16x4 lds_read_tr16(const __bf16* p) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(p));
}

template <int DH>
__global__ __launch_bounds__(256, 2) void flash_fwd_mfma(const __bf16* __restrict__ q,
                                                         const __bf16* __restrict__ k,
                                                         const __bf16* __restrict__ v,
                                                         const int32_t* __restrict__ pos,
                                                         __bf16* __restrict__ o, int n, int Hq, int Hkv,
                                                         float scale_log2, int causal, int n_qtiles) {
    constexpr int KC = DH / 16;      // contraction chunks of Q K^T
    constexpr int DB = DH / 32;      // 32-wide output blocks of O^T
    constexpr int KSTR = DH + 8;     // LDS row stride of K (elements): 16 lanes x 16 B hit distinct banks
    constexpr int VSTR = DH + 32;    // LDS row stride of V: the 4x(2x32 B) transpose-read groups do
    constexpr int VEC_PER_ROW = DH / 8;
    constexpr int LOADS = kFaBN * VEC_PER_ROW / 256;
    __shared__ __attribute__((aligned(16))) __bf16 Ks[kFaBN * KSTR];
    __shared__ __attribute__((aligned(16))) __bf16 Vs[kFaBN * VSTR];
    __shared__ int pos_k[kFaBN];

    // heaviest (latest) query tiles first
    const int qt = n_qtiles - 1 - (int)blockIdx.x / Hq;
    const int head = (int)blockIdx.x % Hq;
    const int g = head / (Hq / Hkv);
    const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    const int j = lane % 32, h = lane / 32;
    const int q0 = qt * kFaBM + wave * 32;
    const int qrow = q0 + j;
    const int qrow_c = min(qrow, n - 1);
    const int pos_q = pos[qrow_c];

    bf16x8 Qf[KC];
    {
        const __bf16* qp = q + ((size_t)qrow_c * Hq + head) * DH + 8 * h;
#pragma unroll
        for (int kc = 0; kc < KC; ++kc) Qf[kc] = *reinterpret_cast<const bf16x8*>(qp + 16 * kc);
    }
    f32x16 Oacc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) Oacc[db][r] = 0.f;
    float m = kMaskedScore, lsum = 0.f;

    const int kv_end = causal ? min(n, qt * kFaBM + kFaBM) : n;
    const int n_tiles = (kv_end + kFaBN - 1) / kFaBN;
    const int wave_kend = causal ? min(n, q0 + 32) : n;  // keys at or beyond this rank are masked for the whole wave

    for (int t = 0; t < n_tiles; ++t) {
        const int key0 = t * kFaBN;
        __syncthreads();
#pragma unroll
        for (int it = 0; it < LOADS; ++it) {
            const int idx = it * 256 + tid;
            const int row = idx / VEC_PER_ROW, c8 = idx % VEC_PER_ROW;
            const int krow = min(key0 + row, n - 1);
            const size_t goff = ((size_t)krow * Hkv + g) * DH + c8 * 8;
            const u32x4 kv = *reinterpret_cast<const u32x4*>(k + goff);
            const u32x4 vv = *reinterpret_cast<const u32x4*>(v + goff);
            *reinterpret_cast<u32x4*>(&Ks[row * KSTR + c8 * 8]) = kv;
            *reinterpret_cast<u32x4*>(&Vs[row * VSTR + c8 * 8]) = vv;
        }
        if (tid < kFaBN) pos_k[tid] = pos[min(key0 + tid, n - 1)];
        __syncthreads();
        if (key0 >= wave_kend) continue;  // wave-uniform: nothing visible to this wave in this tile

        f32x16 S[2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
            for (int r = 0; r < 16; ++r) S[kb][r] = 0.f;
#pragma unroll
            for (int kc = 0; kc < KC; ++kc) {
                const bf16x8 Kf = *reinterpret_cast<const bf16x8*>(&Ks[(32 * kb + j) * KSTR + 16 * kc + 8 * h]);
                S[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Kf, Qf[kc], S[kb], 0, 0, 0);
            }
        }
        const bool need_mask = (causal && key0 + kFaBN - 1 > q0) || (key0 + kFaBN > n);
        if (need_mask) {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int kl = 32 * kb + 8 * (r / 4) + 4 * h + (r % 4);
                    const bool bad = (key0 + kl >= n) || (causal && pos_k[kl] > pos_q);
                    if (bad) S[kb][r] = kMaskedScore;
                }
        }
        // online softmax in the log2 domain
        float mx = S[0][0];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) mx = fmaxf(mx, S[kb][r]);
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m, mx * scale_log2);
        const float alpha = __builtin_amdgcn_exp2f(m - m_new);
        m = m_new;
        float psum = 0.f;
        bf16x8 Pf[4];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float p = __builtin_amdgcn_exp2f(fmaf(S[kb][r], scale_log2, -m_new));
                psum += p;
                Pf[2 * kb + r / 8][r % 8] = (__bf16)p;
            }
        lsum = lsum * alpha + psum;
        if (__any(alpha != 1.0f)) {
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) Oacc[db][r] *= alpha;
        }
        // O^T += V^T P^T
        const int tg = lane / 16, ti = lane % 16;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int kbase = 16 * c + 4 * (tg / 2) + ti / 4;  // key row this lane addresses
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                const int col = 32 * db + 16 * (tg % 2) + 4 * (ti % 4);
                const s16x4 lo = lds_read_tr16(&Vs[kbase * VSTR + col]);
                const s16x4 hi = lds_read_tr16(&Vs[(kbase + 8) * VSTR + col]);
                const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                const bf16x8 Vf = __builtin_bit_cast(bf16x8, both);
                Oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Vf, Pf[c], Oacc[db], 0, 0, 0);
            }
        }
    }

    lsum += __shfl_xor(lsum, 32);
    const float inv = 1.0f / lsum;
    if (qrow < n) {
        __bf16* op = o + ((size_t)qrow * Hq + head) * DH;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int rg = 0; rg < 4; ++rg) {
                bf16x4 ov;
#pragma unroll
                for (int e = 0; e < 4; ++e) ov[e] = (__bf16)(Oacc[db][4 * rg + e] * inv);
                *reinterpret_cast<bf16x4*>(op + 32 * db + 8 * rg + 4 * h) = ov;
            }
    }
}

template <typename T>
static dash_status launch_simple(const dash_layer_params& p, const T* q, const T* k, const T* v,
                                 const int32_t* pos, int n, T* o, float scale, hipStream_t s) {
    dim3 grid(n, p.n_q_heads);
    if (p.head_dim == 64)
        hipLaunchKernelGGL((flash_fwd_simple<T, 64>), grid, dim3(64), 0, s, q, k, v, pos, o, n, p.n_q_heads,
                           p.n_kv_heads, scale, p.causal);
    else
        hipLaunchKernelGGL((flash_fwd_simple<T, 128>), grid, dim3(64), 0, s, q, k, v, pos, o, n, p.n_q_heads,
                           p.n_kv_heads, scale, p.causal);
    return launch_status();
}

dash_status launch_flash_fwd(const dash_layer_params& p, const void* q, const void* k, const void* v,
                             const int32_t* active_idx, int n, void* o, hipStream_t s) {
    if (n == 0) return DASH_OK;
    const float scale = p.softmax_scale > 0.f ? p.softmax_scale : 1.0f / sqrtf((float)p.head_dim);
    if (p.dtype == DASH_F32)
        return launch_simple<float>(p, (const float*)q, (const float*)k, (const float*)v, active_idx, n,
                                    (float*)o, scale, s);
    const int n_qtiles = (n + kFaBM - 1) / kFaBM;
    const float scale_log2 = scale * 1.4426950408889634f;
    const dim3 grid((unsigned)n_qtiles * p.n_q_heads);
    if (p.head_dim == 64)
        hipLaunchKernelGGL((flash_fwd_mfma<64>), grid, dim3(256), 0, s, (const __bf16*)q, (const __bf16*)k,
                           (const __bf16*)v, active_idx, (__bf16*)o, n, p.n_q_heads, p.n_kv_heads, scale_log2,
                           p.causal, n_qtiles);
    else
        hipLaunchKernelGGL((flash_fwd_mfma<128>), grid, dim3(256), 0, s, (const __bf16*)q, (const __bf16*)k,
                           (const __bf16*)v, active_idx, (__bf16*)o, n, p.n_q_heads, p.n_kv_heads, scale_log2,
                           p.causal, n_qtiles);
    return launch_status();
}

}  // namespace dash
