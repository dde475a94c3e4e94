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
#include "lds_ops.h"
#include "staging_addr.h"

namespace dash {

// ------------------------------------------------------------------------------------------------
// Plain kernel: one wave per (query row, head). Lane j scores key j of a 64-key block, then all
// lanes accumulate their own head dims.
// ------------------------------------------------------------------------------------------------
template <typename T, int DH>
__global__ __launch_bounds__(64) void flash_fwd_simple(const T* __restrict__ q, const T* __restrict__ k,
                                                       const T* __restrict__ v,
                                                       const int32_t* __restrict__ pos, T* __restrict__ o,
                                                       int n, int Hq, int Hkv, float scale, int causal,
                                                       uint32_t* __restrict__ clear_words, int n_clear) {
    constexpr int DPL = DH / kWave;  // head dims per lane
    if (blockIdx.x == 0 && blockIdx.y == 0)  // scratch of the kernels that follow in the layer call
        for (int c = threadIdx.x; c < n_clear; c += kWave) clear_words[c] = 0u;
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
// Workgroup = 8 waves = 256 query rows of one head; wave w owns rows 32w..32w+31. Keys/values come in
// tiles of 64, staged through LDS in their natural [key][dim] layout (16-byte chunks swizzled).
//
//   S^T = K Q^T   (A = K fragment from LDS, B = Q fragment held in registers for the whole kernel):
//         with the 32x32 accumulator layout each lane then holds 16 scores of ONE query per 32-key
//         block, so row max / row sum are in-lane reductions plus one exchange with lane^32.
//   O^T += V^T P^T (A = V^T fragment via LDS transpose reads, B = P^T): the accumulator registers of
//         S^T, converted to bf16, already ARE the B fragment - no shuffle, no LDS round trip.
//
// A wave that runs MFMAs and softmax back to back leaves each pipe idle half the time. So the eight waves
// form two groups (waves 0-3 and 4-7; wave w and w+4 share a SIMD) that run the same loop body - an MFMA
// stretch (O += P V of the previous tile, then S = K Q^T of the next) followed by the softmax of that tile -
// but pass the one workgroup barrier of a round at different places, so that between two barriers
//     group 0 runs  MFMA stretch(t), softmax(t)        group 1 runs  softmax(t-1), MFMA stretch(t)
// and the SIMD co-executes one group's MFMAs with the other group's VALU work.
// K and V tiles go from global memory straight into LDS (no registers in between), K through two stages and
// V through three; the V fragments of a tile's first key chunk are read during the softmax phase, so the
// matrix-core phase that follows the barrier starts with MFMAs, not with an exposed LDS round trip.
//
// MFMA 32x32x16 operand layout (lane l, i = l%32, h = l/32): A holds row i, k-slots 8h..8h+7;
// B holds column i, k-slots 8h..8h+7; D register r holds row 8*(r/4) + 4h + r%4 of column i.
// ------------------------------------------------------------------------------------------------
constexpr int kFaBM = 256;  // query rows per workgroup
// keys per tile: kFaBN = 64 (staging_addr.h)
constexpr int kFaThreads = 512;
constexpr float kMaskedScore = -1.0e30f;
constexpr float kRowSumLimit = 1048576.0f;  // a lane's 32-key partial row sum above this moves the softmax reference

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

// LDS layout of one K or V stage: 64 rows of DH bf16, unpadded (the direct global->LDS loads write 1 KB of
// consecutive LDS per wave instruction, so rows cannot be padded). Bank conflicts are avoided by an XOR
// swizzle of the 16-byte chunk index inside each row, different for K and V because they are read
// differently: K by 16-byte reads of one chunk from 16 consecutive rows, V by transpose reads that touch
// 4 consecutive rows x 4 consecutive chunks per 32 lanes.
template <int DH>
struct FaSmem {
    static constexpr int CPR = DH / 8;             // 16-byte chunks per row
    static constexpr int RP = 256 / (DH * 2);      // rows per 256 bytes of LDS (one pass over all banks)
    static constexpr int STAGE_ELEMS = kFaBN * DH;
    static constexpr size_t BYTES = 5 * STAGE_ELEMS * sizeof(__bf16);  // two stages of K, three of V
    __device__ static constexpr int k_swz(int row) { return fa_k_swz(row, DH); }
    __device__ static constexpr int v_swz(int row) { return fa_v_swz(row, DH); }
};


template <int DH>
__global__ __launch_bounds__(kFaThreads, 1) void flash_fwd_mfma(const __bf16* __restrict__ q,
                                                                const __bf16* __restrict__ k,
                                                                const __bf16* __restrict__ v,
                                                                const int32_t* __restrict__ pos,
                                                                __bf16* __restrict__ o, int n, int Hq,
                                                                int Hkv, float scale_log2, int causal,
                                                                int n_qtiles, FaMap mp,
                                                                uint32_t* __restrict__ clear_words, int n_clear) {
    using SM = FaSmem<DH>;
    constexpr int KC = DH / 16;  // contraction chunks of Q K^T
    constexpr int DB = DH / 32;  // 32-wide output blocks of O^T
    extern __shared__ __attribute__((aligned(16))) unsigned char fa_smem_raw[];
    __bf16* Kst = reinterpret_cast<__bf16*>(fa_smem_raw);  // two K stages, then three V stages
    __bf16* Vst = Kst + 2 * SM::STAGE_ELEMS;
    __shared__ __attribute__((aligned(16))) int pos_blk[kFaBM];  // original positions of this workgroup's rows

    if (blockIdx.x == 0)  // scratch of the kernels that follow in the layer call: cleared here, no launch of its own
        for (int c = threadIdx.x; c < n_clear; c += kFaThreads) clear_words[c] = 0u;
    int qt, head;
    if (!fa_map_block(mp, (int)blockIdx.x, n_qtiles, Hq, Hkv, qt, head)) return;  // whole workgroup exits
    const int g = head / (Hq / Hkv);
    const int tid = threadIdx.x, lane = tid % kWave;
    // the wave index is made provably uniform: the role branches below must be scalar branches, never
    // exec-masked regions (MFMA ignores the exec mask)
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int grp = wave >> 2;
    const int j = lane % 32, h = lane / 32;
    const int tg = lane / 16, ti = lane % 16;
    const int q0 = qt * kFaBM + wave * 32;
    const int qrow = q0 + j;
    const int qrow_c = min(qrow, n - 1);
    const int pos_q = pos[qrow_c];

    bf16x8 Qf[KC];
    {
        const __bf16* qp = q + ((size_t)qrow_c * Hq + head) * DH + 8 * h;
#pragma unroll
        for (int kc = 0; kc < KC; ++kc) Qf[kc] = *reinterpret_cast<const bf16x8*>(qp + 16 * kc);
        // Q is scaled once by softmax_scale * log2(e) (rounded to bf16 again), so the MFMA result is already the
        // exponent in the log2 domain. Rounding the scaled row r = bf16(x) changes its length along x by the
        // factor <r, x> / <x, x>, which acts on every logit of the row like a change of the softmax temperature
        // and, for a fixed scale constant, has a common sign for most rows (measured: 3e-4 of systematic relative
        // error in ||delta||). The row is therefore rounded a second time from x scaled by the inverse of that
        // factor, which cancels the systematic part; what is left is the random part of one rounding.
        float xs[KC][8];
        float sxx = 0.f, srx = 0.f;
#pragma unroll
        for (int kc = 0; kc < KC; ++kc)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float x = (float)Qf[kc][e] * scale_log2;
                xs[kc][e] = x;
                sxx = fmaf(x, x, sxx);
                srx = fmaf((float)(__bf16)x, x, srx);
            }
        sxx += __shfl_xor(sxx, 32);  // lanes j and j + 32 hold the two halves of the row
        srx += __shfl_xor(srx, 32);
        const float comp = sxx > 0.f ? 2.0f - srx / sxx : 1.0f;  // 1 / (1 + a) to first order, a = srx / sxx - 1
#pragma unroll
        for (int kc = 0; kc < KC; ++kc)
#pragma unroll
            for (int e = 0; e < 8; ++e) Qf[kc][e] = (__bf16)(xs[kc][e] * comp);
    }
    f32x16 Oacc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) Oacc[db][r] = 0.f;
    f32x16 S[2];
    uint32_t Pw[4][4];  // P^T of the previous tile as packed bf16 pairs: Pw[c] is the B fragment of key chunk c
    // m is the softmax reference (log2 domain); Cneg holds -m in all 16 accumulator slots and is what every
    // score accumulation starts from, so S arrives as (score - m) and the common tile needs no subtraction.
    // It changes only when the reference moves; the empty asm keeps it a register block instead of 16
    // re-materialised moves per tile.
    float m = 0.f, lsum = 0.f;
    f32x16 Cneg;
#pragma unroll
    for (int r = 0; r < 16; ++r) Cneg[r] = 0.f;
    asm volatile("" : "+v"(Cneg));

    const int kv_end = causal ? min(n, qt * kFaBM + kFaBM) : n;
    const int n_tiles = (kv_end + kFaBN - 1) / kFaBN;
    const int wave_kend = causal ? min(n, q0 + 32) : n;  // keys at or beyond this rank are masked for the whole wave

    // Staging by direct global->LDS loads, no registers in between: the four waves of group 0 fetch the K
    // tiles, those of group 1 the V tiles. One wave instruction moves 1 KB = ROWS_PER_DMA rows; lane l
    // lands in physical chunk l % CPR of row l / CPR, so it fetches the logical chunk that the swizzle maps
    // there. The address of a load is a scalar tile base (advanced by scalar arithmetic) plus a 32-bit lane offset
    // that is the same for every whole tile (the launcher checks the tensors are below 2 GiB); only the last,
    // partly filled tile recomputes the offsets, with rows beyond the end clamped to the last row.
    constexpr int DMAS = fa_dmas(DH);                           // loads per wave and tile: 4 (DH 128) or 2 (DH 64)
    const int gw = wave & 3;                                    // wave inside its group
    const uint32_t tile_bytes = (uint32_t)fa_tile_bytes(Hkv, DH);
    uint32_t dma_voff[DMAS];   // byte offset of this lane's 16 bytes from the start of a whole tile
#pragma unroll
    for (int i = 0; i < DMAS; ++i) dma_voff[i] = fa_dma_voff(fa_dma_row(gw, i, lane, DH), lane, g, Hkv, DH, grp == 0);
    const char* dma_base = reinterpret_cast<const char*>(grp == 0 ? k : v);
    const uint32_t lds_stage0 = lds_addr(grp == 0 ? Kst : Vst) + (uint32_t)(gw * DMAS * 1024);
    int dma_tile = 0;  // tiles are fetched strictly in order: 0, 1, 2, ...
    auto dma_next_tile = [&](int stage) {
        const char* tile_base = dma_base + (size_t)dma_tile * tile_bytes;
        const int rows_left = n - dma_tile * kFaBN;  // >= 1: only tiles that hold a row are fetched
        ++dma_tile;
        if (rows_left >= kFaBN) {
#pragma unroll
            for (int i = 0; i < DMAS; ++i)
                dma_load16(tile_base, dma_voff[i], lds_stage0 + (uint32_t)(stage * SM::STAGE_ELEMS * 2 + i * 1024));
        } else {
#pragma unroll
            for (int i = 0; i < DMAS; ++i)
                dma_load16(tile_base, fa_dma_voff_tail(dma_voff[i], fa_dma_row(gw, i, lane, DH), rows_left, Hkv, DH),
                           lds_stage0 + (uint32_t)(stage * SM::STAGE_ELEMS * 2 + i * 1024));
        }
    };

    // A fragment of O^T += V^T P^T: V^T block (32 dims of block db) x (16 keys of chunk c) by transpose reads
    auto v_frag = [&](const __bf16* Vs, int c, int db) {
        const int kbase_row = 16 * c + 4 * (tg / 2) + ti / 4;  // key row this lane addresses
        const int col = 32 * db + 16 * (tg % 2) + 4 * (ti % 4);
        // rows kbase_row and kbase_row + 8 have the same swizzle (it repeats every 4 * RP <= 8 rows)
        const int scol = ((col / 8) ^ SM::v_swz(kbase_row)) * 8 + col % 8;
        const s16x4 lo = lds_read_tr16(&Vs[kbase_row * DH + scol]);
        const s16x4 hi = lds_read_tr16(&Vs[(kbase_row + 8) * DH + scol]);
        return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    };
    // The fragments of key chunk 0 are read during the softmax phase, before the barrier that opens the
    // matrix-core phase, so that phase starts with MFMAs instead of an exposed LDS round trip.
    bf16x8 Vpre[DB];
    auto prefetch_v = [&](int t) {
        const __bf16* Vs = Vst + (t % 3) * SM::STAGE_ELEMS;
#pragma unroll
        for (int db = 0; db < DB; ++db) Vpre[db] = v_frag(Vs, 0, db);
    };
    // O^T += V^T(t) P^T(t): A = V^T fragment, B = packed P
    auto pv_mfma = [&](int t) {
        const __bf16* Vs = Vst + (t % 3) * SM::STAGE_ELEMS;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const u32x4 pw = {Pw[c][0], Pw[c][1], Pw[c][2], Pw[c][3]};
            const bf16x8 Pf = __builtin_bit_cast(bf16x8, pw);
#pragma unroll
            for (int db = 0; db < DB; ++db)
                Oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(c == 0 ? Vpre[db] : v_frag(Vs, c, db), Pf,
                                                                   Oacc[db], 0, 0, 0);
        }
        // issue order: operand reads run DB MFMAs ahead, so no MFMA waits for a read issued just before it
        constexpr int NM = 4 * DB;
#pragma unroll
        for (int i = 0; i < NM - DB; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, DB, 0);
    };
    // S^T = K(t) Q^T. A fragment: key row 32 kb + j, chunk 2 kc + h; rows j and 32 + j swizzle alike, so the key
    // block only adds a constant to the element offset k_elem[kc].
    static_assert((32 / SM::RP) % SM::CPR == 0, "rows j and j + 32 must share the K swizzle");
    int k_elem[KC];
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) k_elem[kc] = j * DH + ((2 * kc + h) ^ SM::k_swz(j)) * 8;
    auto qk_mfma = [&](int t) {
        const __bf16* Ks = Kst + (t & 1) * SM::STAGE_ELEMS;
        // the two key blocks take turns, so that no MFMA accumulates into the result of the one issued just before it
        // (eight in a row on one block measured 0.6 % slower)
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) S[kb][r] = Cneg[r];
#pragma unroll
        for (int kc = 0; kc < KC; ++kc)
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                const bf16x8 Kf = *reinterpret_cast<const bf16x8*>(&Ks[k_elem[kc] + 32 * kb * DH]);
                S[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Kf, Qf[kc], S[kb], 0, 0, 0);
            }
        constexpr int NM = 2 * KC;
        __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
#pragma unroll
        for (int i = 0; i < NM - 4; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
    };
    auto tile_active = [&](int t) { return t >= 0 && t < n_tiles && t * kFaBN < wave_kend; };  // wave-uniform

    // matrix-core phase of tile t: finish the previous tile's P V, start this tile's scores
    auto mfma_phase = [&](int t) {
        // While a wave is in its matrix-core phase it gets issue priority over the wave of the other group
        // on the same SIMD: an MFMA is issued as soon as the pipe frees, VALU work fills the gaps.
        __builtin_amdgcn_s_setprio(3);
        if (tile_active(t - 1)) pv_mfma(t - 1);
        if (tile_active(t)) qk_mfma(t);
        __builtin_amdgcn_s_setprio(0);
    };
    // probabilities of the tile from S = score - m (minus `shift` when the reference has just moved), packed
    // to bf16 pairs into Pw; returns this lane's part of the row sum. fp32 adds on four chains: a bf16 dot2
    // would halve the instruction count, but it executes on the matrix pipe and (measured) serialises
    // with the other group's MFMAs.
    auto exp_pack = [&](bool shifted, float shift) {
        float ps[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 16; r += 2) {
                const float p0 = __builtin_amdgcn_exp2f(shifted ? S[kb][r] - shift : S[kb][r]);
                const float p1 = __builtin_amdgcn_exp2f(shifted ? S[kb][r + 1] - shift : S[kb][r + 1]);
                ps[(r / 2) % 4] += p0;
                ps[(r / 2 + 2) % 4] += p1;
                const bf16x2 pk = {(__bf16)p0, (__bf16)p1};
                Pw[2 * kb + r / 8][(r % 8) / 2] = __builtin_bit_cast(uint32_t, pk);
            }
        return (ps[0] + ps[1]) + (ps[2] + ps[3]);
    };
    // VALU phase of tile t: softmax numerators in the log2 domain on S, leaves packed P in Pw
    auto valu_phase = [&](int t) {
        if (!tile_active(t)) return;
        const int key0 = t * kFaBN;
        // Causal masks are only ever needed on tiles that lie inside the workgroup's own row range, whose
        // original positions sit in LDS (pos_blk); masking compares positions, not ranks.
        const bool diag = causal && key0 + kFaBN - 1 > q0;  // wave-uniform
        if (diag || key0 + kFaBN > n) {
            const int kl0 = key0 - qt * kFaBM;  // >= 0 whenever diag holds
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int rg = 0; rg < 4; ++rg) {
                    const int kl = 32 * kb + 8 * rg + 4 * h;  // four consecutive keys of this lane
                    int4 kp = make_int4(0, 0, 0, 0);
                    if (diag) kp = *reinterpret_cast<const int4*>(&pos_blk[kl0 + kl]);
                    const int kpe[4] = {kp.x, kp.y, kp.z, kp.w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const bool bad = (key0 + kl + e >= n) || (diag && kpe[e] > pos_q);
                        S[kb][4 * rg + e] = bad ? kMaskedScore : S[kb][4 * rg + e];
                    }
                }
        }
        // Probabilities are taken against a reference m that is NOT the running maximum: any reference
        // gives the same O / sum, it only has to keep exp2 in range. The common tile therefore computes
        // no row maximum at all: it exponentiates S (already relative to m) and looks at the row sums;
        // only if a sum is not a modest finite number (a score far above the reference), and always on
        // the first tile, the reference moves to the true running maximum, what was accumulated is
        // rescaled, and the tile's probabilities are redone.
        prefetch_v(t);
        float psum = exp_pack(false, 0.f);
        if (t == 0 || __any(!(psum < kRowSumLimit))) {
            float c0 = fmaxf(S[0][0], S[1][0]), c1 = fmaxf(S[0][1], S[1][1]);
            float c2 = fmaxf(S[0][2], S[1][2]), c3 = fmaxf(S[0][3], S[1][3]);
#pragma unroll
            for (int r = 4; r < 16; r += 4) {
                c0 = fmaxf(fmaxf(c0, S[0][r]), S[1][r]);  // v_max3_f32
                c1 = fmaxf(fmaxf(c1, S[0][r + 1]), S[1][r + 1]);
                c2 = fmaxf(fmaxf(c2, S[0][r + 2]), S[1][r + 2]);
                c3 = fmaxf(fmaxf(c3, S[0][r + 3]), S[1][r + 3]);
            }
            float mx = fmaxf(fmaxf(c0, c1), fmaxf(c2, c3));  // tile maximum relative to m
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            // The first tile (key 0 is visible to every row, so mx is finite) sets the reference outright,
            // nothing has been accumulated yet; later the reference only rises.
            const float shift = t == 0 ? mx : fmaxf(mx, 0.f);
            const float alpha = t == 0 ? 1.f : __builtin_amdgcn_exp2f(-shift);
            m += shift;
#pragma unroll
            for (int r = 0; r < 16; ++r) Cneg[r] = -m;
            asm volatile("" : "+v"(Cneg));
            lsum *= alpha;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) Oacc[db][r] *= alpha;
            psum = exp_pack(true, shift);
        }
        lsum += psum;
    };

    // K(0) by group 0; V(0) and V(1) by group 1, which waits for V(0) only
    dma_next_tile(0);
    if (grp == 1 && n_tiles > 1) {
        dma_next_tile(1);
        dma_wait_keep<DMAS>();
    } else {
        dma_wait();
    }
    if (tid < kFaBM) pos_blk[tid] = pos[min(qt * kFaBM + tid, n - 1)];
    // The Q fragments have to be in registers before the loop: if their loads were still in flight at
    // loop entry, the first MFMAs of every tile would also wait for the staging loads (issued later,
    // returned in order). An empty asm that "uses" them pins the wait here.
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) asm volatile("" : "+v"(Qf[kc]));
    __syncthreads();

    // Every wave passes the same number of barriers: waves whose rows cannot see a tile skip its work, not its
    // barriers. The extra round t = n_tiles only drains P V of the final tile.
    // barrier that orders LDS traffic only: the staging loads in flight must not be waited for here
    auto lds_barrier = [] {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
    };
    // One barrier per round and wave, at different places of the same loop: group 0 passes it after its softmax
    // phase, group 1 between its MFMA and softmax phases. Round r (between barriers r-1 and r) is therefore
    //     group 0: MFMA stretch of tile r (P V of tile r-1, S of tile r), then softmax of tile r
    //     group 1: softmax of tile r-1, then the MFMA stretch of tile r
    // so a SIMD sees the two roles in opposite order, and where one stretch outlasts the other the two MFMA
    // stretches may overlap instead of waiting for each other.
    //   K(r+1) is requested by group 0 in the middle of round r (after its matrix-core phase) and complete before
    //   barrier r; K(r) is read in round r only, K(r-1) was last read before barrier r-1: two stages. V(r+1) is
    //   requested by group 1 at the start of round r (V(0) and V(1) before the loop) and complete before barrier r;
    //   V(r) is read in round r (first fragments, group 0's softmax) and in round r+1 (P V of tile r, group 1's first
    //   fragments): three stages, and V(r-2) was last read before barrier r-1.
    for (int t = 0; t <= n_tiles; ++t) {
        mfma_phase(t);
        if (grp == 1) {
            dma_wait();  // V(t+1)
            lds_barrier();
            if (t + 2 < n_tiles) dma_next_tile((t + 2) % 3);  // V(t+2)
        }
        // Both groups request their tile at the START OF THEIR SOFTMAX PHASE, while the other group runs MFMAs: the
        // compute unit's one address unit takes 16 cycles per request and holds few, so a wave queues behind its
        // group's 16 requests, and ahead of a matrix-core phase that wait leaves the matrix pipe idle (K requested
        // before group 0's matrix-core phase, where it also met group 1's V requests: 3 % slower).
        if (grp == 0 && t + 1 < n_tiles) dma_next_tile((t + 1) & 1);  // K(t+1)
        valu_phase(t);
        if (grp == 0) {
            dma_wait();  // K(t+1)
            lds_barrier();
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
                                 const int32_t* pos, int n, T* o, float scale, uint32_t* clear_words, int n_clear,
                                 hipStream_t s) {
    dim3 grid(n, p.n_q_heads);
    if (p.head_dim == 64)
        hipLaunchKernelGGL((flash_fwd_simple<T, 64>), grid, dim3(64), 0, s, q, k, v, pos, o, n, p.n_q_heads,
                           p.n_kv_heads, scale, p.causal, clear_words, n_clear);
    else
        hipLaunchKernelGGL((flash_fwd_simple<T, 128>), grid, dim3(64), 0, s, q, k, v, pos, o, n, p.n_q_heads,
                           p.n_kv_heads, scale, p.causal, clear_words, n_clear);
    return launch_status();
}

// One-time launch attribute of the MFMA kernels: their dynamic LDS size.
dash_status init_flash_kernels() {
    static const hipError_t err = [] {
        hipError_t e = hipFuncSetAttribute((const void*)flash_fwd_mfma<64>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)FaSmem<64>::BYTES);
        if (e != hipSuccess) return e;
        return hipFuncSetAttribute((const void*)flash_fwd_mfma<128>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                   (int)FaSmem<128>::BYTES);
    }();
    return err == hipSuccess ? DASH_OK : DASH_ERR_HIP;
}

dash_status launch_flash_fwd(const dash_layer_params& p, const void* q, const void* k, const void* v,
                             const int32_t* active_idx, int n, void* o, uint32_t* clear_words, int n_clear,
                             hipStream_t s) {
    if (n == 0) return DASH_OK;
    const float scale = p.softmax_scale > 0.f ? p.softmax_scale : 1.0f / sqrtf((float)p.head_dim);
    if (p.dtype == DASH_F32)
        return launch_simple<float>(p, (const float*)q, (const float*)k, (const float*)v, active_idx, n,
                                    (float*)o, scale, clear_words, n_clear, s);
    // the MFMA kernel addresses K and V with 32-bit byte offsets
    if ((size_t)n * p.n_kv_heads * p.head_dim * 2 >= (size_t)1 << 31) return DASH_ERR_UNSUPPORTED;
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
    if (init_flash_kernels() != DASH_OK) return DASH_ERR_HIP;
    if (p.head_dim == 64) {
        hipLaunchKernelGGL((flash_fwd_mfma<64>), grid, dim3(kFaThreads), FaSmem<64>::BYTES, s, (const __bf16*)q,
                           (const __bf16*)k, (const __bf16*)v, active_idx, (__bf16*)o, n, Hq, Hkv, scale_log2,
                           p.causal, n_qtiles, mp, clear_words, n_clear);
    } else {
        hipLaunchKernelGGL((flash_fwd_mfma<128>), grid, dim3(kFaThreads), FaSmem<128>::BYTES, s, (const __bf16*)q,
                           (const __bf16*)k, (const __bf16*)v, active_idx, (__bf16*)o, n, Hq, Hkv, scale_log2,
                           p.causal, n_qtiles, mp, clear_words, n_clear);
    }
    return launch_status();
}

}  // namespace dash
