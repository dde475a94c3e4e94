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

// Work-item -> (query tile, head) map. Workgroups are handed to the 8 XCDs round-robin
// (workgroup b runs on XCD b % 8) and each XCD has its own L2, so all workgroups of one XCD are given
// the same KV head (or as few as possible): its K/V tiles are then fetched into that L2 once and shared
// by the query heads of the group and by neighbouring query tiles. Heaviest (latest) query tiles first.
struct FaMap {
    int xcd_mode;      // 1: XCD-aware, 0: plain
    int xcds_per_g;    // XCDs serving one KV head (Hkv <= 8)
    int g_per_xcd;     // KV heads per XCD (Hkv >= 8)
    int items_per_g;   // n_qtiles * group size
};

__device__ __forceinline__ bool fa_map_block(const FaMap& mp, int bid, int n_qtiles, int Hq, int Hkv,
                                             int& qt, int& head) {
    const int group = Hq / Hkv;
    if (!mp.xcd_mode) {
        qt = n_qtiles - 1 - bid / Hq;
        head = bid % Hq;
        return true;
    }
    const int xcd = bid % 8, slot = bid / 8;
    int g, idx;
    if (mp.g_per_xcd == 1) {
        g = xcd / mp.xcds_per_g;
        idx = slot * mp.xcds_per_g + xcd % mp.xcds_per_g;
    } else {
        g = xcd * mp.g_per_xcd + slot % mp.g_per_xcd;
        idx = slot / mp.g_per_xcd;
    }
    if (idx >= mp.items_per_g) return false;
    qt = n_qtiles - 1 - idx / group;
    head = g * group + idx % group;
    return true;
}

template <int DH>
struct FaSmem {
    static constexpr int KSTR = DH + 8;   // LDS row stride of K (elements): 16 lanes x 16 B hit distinct banks
    static constexpr int VSTR = DH + 32;  // LDS row stride of V: the 4-row transpose-read groups do
    static constexpr int K_ELEMS = kFaBN * KSTR;
    static constexpr int V_ELEMS = kFaBN * VSTR;
    static constexpr int STAGE_ELEMS = K_ELEMS + V_ELEMS;
    static constexpr size_t BYTES = 2 * STAGE_ELEMS * sizeof(__bf16);  // two stages
};

template <int DH>
__global__ __launch_bounds__(256, 2) void flash_fwd_mfma(const __bf16* __restrict__ q,
                                                         const __bf16* __restrict__ k,
                                                         const __bf16* __restrict__ v,
                                                         const int32_t* __restrict__ pos,
                                                         __bf16* __restrict__ o, int n, int Hq, int Hkv,
                                                         float scale_log2, int causal, int n_qtiles,
                                                         FaMap mp) {
    using SM = FaSmem<DH>;
    constexpr int KC = DH / 16;  // contraction chunks of Q K^T
    constexpr int DB = DH / 32;  // 32-wide output blocks of O^T
    constexpr int KSTR = SM::KSTR, VSTR = SM::VSTR;
    constexpr int VEC_PER_ROW = DH / 8;
    constexpr int LOADS = kFaBN * VEC_PER_ROW / 256;
    extern __shared__ __attribute__((aligned(16))) unsigned char fa_smem_raw[];
    __bf16* smem = reinterpret_cast<__bf16*>(fa_smem_raw);

    int qt, head;
    if (!fa_map_block(mp, (int)blockIdx.x, n_qtiles, Hq, Hkv, qt, head)) return;  // whole workgroup exits
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

    // global -> register -> LDS staging of one K/V tile; thread t moves LOADS 16-byte vectors of each
    u32x4 kreg[LOADS], vreg[LOADS];
    const int ld_row = tid / VEC_PER_ROW, ld_c8 = tid % VEC_PER_ROW;
    constexpr int ROWS_PER_IT = 256 / VEC_PER_ROW;
    auto load_tile = [&](int key0) {
#pragma unroll
        for (int it = 0; it < LOADS; ++it) {
            const int krow = min(key0 + ld_row + ROWS_PER_IT * it, n - 1);
            const size_t goff = ((size_t)krow * Hkv + g) * DH + ld_c8 * 8;
            kreg[it] = *reinterpret_cast<const u32x4*>(k + goff);
            vreg[it] = *reinterpret_cast<const u32x4*>(v + goff);
        }
    };
    auto store_tile = [&](int stage) {
        __bf16* Ks = smem + stage * SM::STAGE_ELEMS;
        __bf16* Vs = Ks + SM::K_ELEMS;
#pragma unroll
        for (int it = 0; it < LOADS; ++it) {
            const int row = ld_row + ROWS_PER_IT * it;
            *reinterpret_cast<u32x4*>(&Ks[row * KSTR + ld_c8 * 8]) = kreg[it];
            *reinterpret_cast<u32x4*>(&Vs[row * VSTR + ld_c8 * 8]) = vreg[it];
        }
    };

    load_tile(0);
    store_tile(0);
    // The Q fragments have to be in registers before the loop: if their loads were still in flight at
    // loop entry, the first MFMAs of every tile would also wait for the next tile's loads (issued later,
    // returned in order). An empty asm that "uses" them pins the wait here.
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) asm volatile("" : "+v"(Qf[kc]));
    __syncthreads();

    const int tg = lane / 16, ti = lane % 16;
    for (int t = 0; t < n_tiles; ++t) {
        const int key0 = t * kFaBN;
        const bool has_next = t + 1 < n_tiles;
        if (has_next) load_tile(key0 + kFaBN);  // in flight while this tile is computed
        const __bf16* Ks = smem + (t & 1) * SM::STAGE_ELEMS;
        const __bf16* Vs = Ks + SM::K_ELEMS;

        if (key0 < wave_kend) {  // wave-uniform: otherwise nothing in this tile is visible to this wave
            f32x16 S[2];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
                for (int r = 0; r < 16; ++r) S[kb][r] = 0.f;
#pragma unroll
                for (int kc = 0; kc < KC; ++kc) {
                    const bf16x8 Kf =
                        *reinterpret_cast<const bf16x8*>(&Ks[(32 * kb + j) * KSTR + 16 * kc + 8 * h]);
                    S[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Kf, Qf[kc], S[kb], 0, 0, 0);
                }
            }
            const bool need_mask = (causal && key0 + kFaBN - 1 > q0) || (key0 + kFaBN > n);
            if (need_mask) {
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int key = key0 + 32 * kb + 8 * (r / 4) + 4 * h + (r % 4);
                        const bool bad = (key >= n) || (causal && pos[min(key, n - 1)] > pos_q);
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
        // the other stage was last read in iteration t-1, which every wave left through the barrier below
        if (has_next) store_tile((t + 1) & 1);
        __syncthreads();
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
    const int Hq = p.n_q_heads, Hkv = p.n_kv_heads, group = Hq / Hkv;
    FaMap mp{0, 1, 1, n_qtiles * group};
    unsigned blocks = (unsigned)n_qtiles * Hq;
    if (Hkv <= 8 && 8 % Hkv == 0) {
        mp.xcd_mode = 1;
        mp.xcds_per_g = 8 / Hkv;
        blocks = 8u * (unsigned)((mp.items_per_g + mp.xcds_per_g - 1) / mp.xcds_per_g);
    } else if (Hkv % 8 == 0) {
        mp.xcd_mode = 1;
        mp.g_per_xcd = Hkv / 8;
        blocks = 8u * (unsigned)(mp.items_per_g * mp.g_per_xcd);
    }
    const dim3 grid(blocks);
    if (p.head_dim == 64) {
        static const hipError_t attr64 = hipFuncSetAttribute(
            (const void*)flash_fwd_mfma<64>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)FaSmem<64>::BYTES);
        if (attr64 != hipSuccess) return DASH_ERR_HIP;
        hipLaunchKernelGGL((flash_fwd_mfma<64>), grid, dim3(256), FaSmem<64>::BYTES, s, (const __bf16*)q,
                           (const __bf16*)k, (const __bf16*)v, active_idx, (__bf16*)o, n, Hq, Hkv, scale_log2,
                           p.causal, n_qtiles, mp);
    } else {
        static const hipError_t attr128 = hipFuncSetAttribute(
            (const void*)flash_fwd_mfma<128>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)FaSmem<128>::BYTES);
        if (attr128 != hipSuccess) return DASH_ERR_HIP;
        hipLaunchKernelGGL((flash_fwd_mfma<128>), grid, dim3(256), FaSmem<128>::BYTES, s, (const __bf16*)q,
                           (const __bf16*)k, (const __bf16*)v, active_idx, (__bf16*)o, n, Hq, Hkv, scale_log2,
                           p.causal, n_qtiles, mp);
    }
    return launch_status();
}

}  // namespace dash
