// Per-token delta-attention score (Eq. 2, or its relative form) and the halting decision
// (Eq. 3 TopK, or the threshold line of Fig. 8). HBM/latency-bound: a few bytes per row.
//
// Scores are finished here from per-row partial sums of squares that the projection stage took from
// its fp32 accumulators: partials [P, n, 2] = (sum delta^2, sum x^2), summed over P in a fixed order
// so the result is bit-reproducible.
#include <mutex>

#include "common.h"
#include "score_rows.h"

namespace dash {

// rule NONE / THRESHOLD: score, flag and the chunk's kept count in one pass. One workgroup per 64-row chunk.
__global__ __launch_bounds__(256) void score_threshold_kernel(
    const float* __restrict__ partials, int P, int n, int score_kind, int rule, float tau, int n_first,
    int n_last, float* __restrict__ scores, uint8_t* __restrict__ halt, int32_t* __restrict__ chunk_counts) {
    __shared__ float2 red[4][kChunkRows];
    const int row_base = blockIdx.x * kChunkRows;
    const float2 t = row_sums_256(partials, P, n, row_base, red);
    if (threadIdx.x >= kChunkRows) return;
    const int row = row_base + threadIdx.x;
    bool keep = false;
    if (row < n) {
        const float s = score_from_sums(t, score_kind);
        scores[row] = s;
        const bool h = rule == DASH_RULE_THRESHOLD && !row_protected(row, n, n_first, n_last) && s < tau;
        halt[row] = h ? 1 : 0;
        keep = !h;
    }
    const unsigned long long m = __ballot(keep);
    if (threadIdx.x == 0) chunk_counts[blockIdx.x] = __popcll(m);
}

__global__ __launch_bounds__(256) void score_only_kernel(const float* __restrict__ partials, int P, int n,
                                                         int score_kind, float* __restrict__ scores) {
    __shared__ float2 red[4][kChunkRows];
    const int row_base = blockIdx.x * kChunkRows;
    const float2 t = row_sums_256(partials, P, n, row_base, red);
    const int row = row_base + threadIdx.x;
    if (threadIdx.x < kChunkRows && row < n) scores[row] = score_from_sums(t, score_kind);
}

// Order-preserving map from fp32 to uint32 for the total order in which TopK ranks scores:
//   -inf < ... < -0.0 = +0.0 < ... < +inf < NaN   (every NaN, whatever its sign or payload, is one value).
// Eq. 3 ranks real numbers; this is the reading for the other values a float can hold: a NaN score ranks highest
// (the threshold rule keeps NaN rows as well, "score < tau" being false), the two zeros tie and are told apart
// by row like any tie.
__device__ __forceinline__ uint32_t order_key(float f) {
    if (f != f) return 0xFFFFFFFFu;
    const uint32_t b = __float_as_uint(f == 0.0f ? 0.0f : f);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

// Key under which TopK ranks a score: the order-preserving key, or its complement when the rows with the
// LOWEST scores are to be kept (the direction control of Sec. 5.4).
__device__ __forceinline__ uint32_t rank_key(float f, int keep_low) {
    const uint32_t k = order_key(f);
    return keep_low ? ~k : k;
}

struct TopkState {
    uint32_t threshold_key;  // key of the K-th largest candidate score
    int32_t tie_quota;       // how many rows with exactly that key are kept (earliest rows first)
    int32_t ties_ranked;     // 0: every row with that key is kept (no per-chunk tie counts were written)
};

constexpr int kSelectThreads = 1024;
constexpr int kSelectBins = 2048;   // histogram bins of one radix pass (11-bit digits)
constexpr int kSelectBatch = 16;    // scores a thread has in flight per load batch
// Copies of the histogram, one per lane % kHistCopies: adds of one wave instruction to the same LDS word are done one
// after the other, and scores that crowd into a few bins of the first pass (sign, exponent and two mantissa bits:
// the relative scores of one layer may span only an octave or two) make that pass several times longer. Two copies
// cost the widely spread case 5 % and take a third off the crowded ones; four cost more than they return.
constexpr int kHistCopies = 2;

struct SelectShared {
    int hist[kSelectBins][kHistCopies];  // the copies of a bin side by side: in different LDS banks
    int wave_tot[kSelectThreads / kWave];
    uint32_t prefix;
    int remaining, ties;
};

__device__ __forceinline__ void clear_hist(SelectShared& sh) {
    int* h = &sh.hist[0][0];
    for (int b = threadIdx.x; b < kHistCopies * kSelectBins; b += kSelectThreads) h[b] = 0;
}

__device__ __forceinline__ void hist_add(SelectShared& sh, uint32_t digit) {
    atomicAdd(&sh.hist[digit][threadIdx.x % kHistCopies], 1);
}

// After a pass has filled sh.hist (and a barrier): the bin that holds the remaining-th largest key, i.e. the largest
// b with (keys in bins >= b) >= remaining; updates prefix and remaining (uniform) and leaves the bin's count in
// sh.ties. Thread t owns bins 2t and 2t + 1; suffix sums over the threads of a wave by shuffles, over the waves
// through LDS. Called by all kSelectThreads threads; ends with a barrier after which sh.hist may be cleared.
__device__ __forceinline__ void select_bin(SelectShared& sh, int shift, uint32_t& prefix, int& remaining) {
    constexpr int kWaves = kSelectThreads / kWave;
    const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
    int h0 = 0, h1 = 0;
#pragma unroll
    for (int c = 0; c < kHistCopies; ++c) {
        h0 += sh.hist[2 * tid][c];
        h1 += sh.hist[2 * tid + 1][c];
    }
    int suf = h0 + h1;  // becomes the count of keys in bins >= 2 tid
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
        const int t = __shfl_down(suf, o);
        if (lane + o < kWave) suf += t;
    }
    if (lane == 0) sh.wave_tot[wave] = suf;
    __syncthreads();
#pragma unroll
    for (int w = 1; w < kWaves; ++w) {  // every total is read (independent LDS reads), the later waves' are added
        const int t = sh.wave_tot[w];
        if (w > wave) suf += t;
    }
    // exactly one bin satisfies excl < remaining <= incl (the keys under the prefix number at least `remaining`)
    const int incl1 = suf - h0, excl1 = incl1 - h1;  // bin 2 tid + 1
    const int incl0 = suf, excl0 = incl1;            // bin 2 tid
    if (excl1 < remaining && remaining <= incl1) {
        sh.prefix = prefix | ((uint32_t)(2 * tid + 1) << shift);
        sh.remaining = remaining - excl1;
        sh.ties = h1;
    } else if (excl0 < remaining && remaining <= incl0) {
        sh.prefix = prefix | ((uint32_t)(2 * tid) << shift);
        sh.remaining = remaining - excl0;
        sh.ties = h0;
    }
    __syncthreads();
    prefix = sh.prefix;
    remaining = sh.remaining;
}

__device__ __forceinline__ int pass_shift(int pass) { return pass == 0 ? 21 : (pass == 1 ? 10 : 0); }
__device__ __forceinline__ uint32_t pass_digit_mask(int pass) { return pass == 2 ? 0x3FFu : 0x7FFu; }
__device__ __forceinline__ uint32_t pass_high_mask(int pass) {
    return pass == 0 ? 0u : (0xFFFFFFFFu << (pass == 1 ? 21 : 10));
}

// TopK selection (Eq. 3): one workgroup finds the key of the k_cand-th largest score among the unprotected rows by
// three radix passes over the order-preserving keys (digits of 11, 11 and 10 bits, integer histograms in LDS: the
// order of the adds does not matter, so the result is exact and reproducible). A pass streams the scores with 16
// independent loads per thread in flight, so its time is a few memory latencies plus the adds, not a latency per
// 1024 rows. When more
// rows tie with the K-th key than may be kept, it also counts those ties per 64-row chunk, so the flag kernel can
// keep the earliest ones; with distinct scores (the usual case) that pass over the scores is skipped.
__global__ __launch_bounds__(kSelectThreads) void topk_select_kernel(
    const float* __restrict__ scores, int n, int n_first, int n_last, int k_keep, int keep_low,
    TopkState* __restrict__ st, int32_t* __restrict__ tie_counts) {
    __shared__ SelectShared sh;
    const int tid = threadIdx.x;
    const int lane = tid % kWave, wave = tid / kWave;
    const int lo = min(n_first, n), hi = max(lo, n - n_last);  // candidates are rows [lo, hi)
    const int n_cand = hi - lo;
    const int n_prot = n - n_cand;
    int k_cand = k_keep - n_prot;
    k_cand = max(0, min(k_cand, n_cand));
    if (k_cand == 0) {
        // nothing unprotected survives: no key exceeds the threshold and no tie is kept
        if (tid == 0) {
            st->threshold_key = 0xFFFFFFFFu;
            st->tie_quota = 0;
            st->ties_ranked = 0;
        }
        return;
    }
    uint32_t prefix = 0u;      // digits found so far (in place), uniform
    int remaining = k_cand;    // rank of the wanted key among the keys that share the prefix, uniform
#pragma unroll 1
    for (int pass = 0; pass < 3; ++pass) {
        const int shift = pass_shift(pass);
        const uint32_t digit_mask = pass_digit_mask(pass), hi_mask = pass_high_mask(pass);
        clear_hist(sh);
        __syncthreads();
        for (int r0 = lo; r0 < hi; r0 += kSelectThreads * kSelectBatch) {
            float v[kSelectBatch];
#pragma unroll
            for (int u = 0; u < kSelectBatch; ++u) {
                const int r = r0 + u * kSelectThreads + tid;
                v[u] = r < hi ? scores[r] : 0.f;
            }
#pragma unroll
            for (int u = 0; u < kSelectBatch; ++u) {
                const int r = r0 + u * kSelectThreads + tid;
                const uint32_t key = rank_key(v[u], keep_low);
                // plain LDS adds: with 11-bit digits the keys of a wave spread over many bins (folding the lanes that
                // share a bin into one add by ballots measured a third slower on the workloads' scores; it only pays
                // for heavily tied scores, which stay correct and 3-6 times slower)
                if (r < hi && (key & hi_mask) == prefix) hist_add(sh, (key >> shift) & digit_mask);
            }
        }
        __syncthreads();
        select_bin(sh, shift, prefix, remaining);
    }
    const uint32_t T = prefix;
    const bool rank_ties = sh.ties > remaining;  // more rows tie with the K-th key than may be kept
    if (tid == 0) {
        st->threshold_key = T;
        st->tie_quota = remaining;  // >= 1: ties (key == T) still to be kept
        st->ties_ranked = rank_ties ? 1 : 0;
    }
    if (!rank_ties) return;
    // ties per chunk, one wave per chunk, four chunks in flight per wave
    const int n_chunks = (n + kChunkRows - 1) / kChunkRows;
    constexpr int kWaves = kSelectThreads / kWave;
    for (int c0 = wave; c0 < n_chunks; c0 += 4 * kWaves) {
        float v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int row = (c0 + u * kWaves) * kChunkRows + lane;
            v[u] = row < hi ? scores[row] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int c = c0 + u * kWaves;
            const int row = c * kChunkRows + lane;
            const bool tie = row >= lo && row < hi && rank_key(v[u], keep_low) == T;
            const unsigned long long m = __ballot(tie);
            if (lane == 0 && c < n_chunks) tie_counts[c] = __popcll(m);
        }
    }
}

// TopK flags: keep protected rows, rows above the threshold key, and the first tie_quota rows equal to it.
__global__ __launch_bounds__(256) void topk_flag_kernel(const float* __restrict__ scores, int n, int n_first,
                                                        int n_last, int keep_low,
                                                        const TopkState* __restrict__ st,
                                                        const int32_t* __restrict__ tie_counts,
                                                        uint8_t* __restrict__ halt,
                                                        int32_t* __restrict__ chunk_counts) {
    __shared__ int wave_part[4];
    const int chunk = blockIdx.x;  // one workgroup per 64-row chunk; wave 0 decides
    const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
    const bool ranked = st->ties_ranked != 0;  // uniform
    int tie_base = 0;
    if (ranked) {
        int part = 0;
        for (int c = tid; c < chunk; c += 256) part += tie_counts[c];
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) part += __shfl_xor(part, o);
        if (lane == 0) wave_part[wave] = part;
        __syncthreads();
        tie_base = wave_part[0] + wave_part[1] + wave_part[2] + wave_part[3];
    }
    if (wave != 0) return;
    const uint32_t T = st->threshold_key;
    const int quota = st->tie_quota;
    const int row = chunk * kChunkRows + lane;
    bool keep = false, tie = false;
    if (row < n) {
        if (row_protected(row, n, n_first, n_last)) {
            keep = true;
        } else {
            const uint32_t key = rank_key(scores[row], keep_low);
            keep = key > T;
            tie = key == T;
        }
    }
    const unsigned long long tie_mask = __ballot(tie);
    // unranked: every tie is kept when any is (quota 0 only with the all-halt state, where no key is kept)
    if (tie) keep = ranked ? tie_base + __popcll(tie_mask & ((1ull << lane) - 1ull)) < quota : quota > 0;
    if (row < n) halt[row] = keep ? 0 : 1;
    const unsigned long long m = __ballot(keep);
    if (lane == 0) chunk_counts[chunk] = __popcll(m);
}

// TopK decision (Eq. 3) of up to 1024 * B rows in ONE launch of one workgroup: selection and flags together.
// Thread t holds the keys of rows u * 1024 + t (u < B) in registers, so the scores are read once: the three radix
// passes, the flags and the kept counts per 64-row chunk (chunk u * 16 + w is what wave w holds at step u) all work
// from those registers. Same total order, same tie rule (earliest rows first) and same outputs as the
// topk_select_kernel + topk_flag_kernel pair, which serves longer inputs. One compute unit does all of it, so the
// time is that unit's instruction throughput (about 20 vector instructions per row over the three passes and the
// flags), not memory: 16-byte loads with four flags per store, and the keys in LDS under short rolled loops,
// measured slower than this plain form.
template <int B>
__global__ __launch_bounds__(kSelectThreads) void topk_decide_small_kernel(
    const float* __restrict__ scores, int n, int n_first, int n_last, int k_keep, int keep_low,
    uint8_t* __restrict__ halt, int32_t* __restrict__ chunk_counts) {
    constexpr int kWaves = kSelectThreads / kWave;
    constexpr int kChunks = B * kWaves;
    __shared__ SelectShared sh;
    __shared__ int tie_base[kChunks];  // ties per chunk, then ties in all earlier chunks
    const int tid = threadIdx.x;
    const int lane = tid % kWave, wave = tid / kWave;
    const int lo = min(n_first, n), hi = max(lo, n - n_last);  // candidates are rows [lo, hi)
    const int n_cand = hi - lo;
    const int k_cand = max(0, min(k_keep - (n - n_cand), n_cand));
    uint32_t key[B];
    uint32_t cand = 0u;  // bit u: row u * 1024 + tid is a candidate
#pragma unroll
    for (int u = 0; u < B; ++u) {
        const int r = u * kSelectThreads + tid;
        key[u] = rank_key(r < n ? scores[r] : 0.f, keep_low);
        if (r >= lo && r < hi) cand |= 1u << u;
    }
    // nothing unprotected survives: no key exceeds the threshold and no tie is kept
    uint32_t T = 0xFFFFFFFFu;
    int quota = 0;
    bool rank_ties = false;
    if (k_cand > 0) {
        uint32_t prefix = 0u;
        int remaining = k_cand;
#pragma unroll 1
        for (int pass = 0; pass < 3; ++pass) {
            const int shift = pass_shift(pass);
            const uint32_t digit_mask = pass_digit_mask(pass), hi_mask = pass_high_mask(pass);
            clear_hist(sh);
            __syncthreads();
#pragma unroll
            for (int u = 0; u < B; ++u)
                if (((cand >> u) & 1u) && (key[u] & hi_mask) == prefix)
                    hist_add(sh, (key[u] >> shift) & digit_mask);
            __syncthreads();
            select_bin(sh, shift, prefix, remaining);
        }
        T = prefix;
        quota = remaining;               // >= 1: ties (key == T) still to be kept
        rank_ties = sh.ties > remaining; // more rows tie with the K-th key than may be kept
    }
    if (rank_ties) {
#pragma unroll
        for (int u = 0; u < B; ++u) {
            const unsigned long long m = __ballot(((cand >> u) & 1u) && key[u] == T);
            if (lane == 0) tie_base[u * kWaves + wave] = __popcll(m);
        }
        __syncthreads();
        if (wave == 0) {  // exclusive prefix over the chunks in row order: B/4 consecutive chunks per lane
            constexpr int kPer = kChunks / kWave;
            int v[kPer], tot = 0;
#pragma unroll
            for (int j = 0; j < kPer; ++j) {
                v[j] = tie_base[lane * kPer + j];
                tot += v[j];
            }
            int incl = tot;
#pragma unroll
            for (int o = 1; o < kWave; o <<= 1) {
                const int t = __shfl_up(incl, o);
                if (lane >= o) incl += t;
            }
            int run = incl - tot;
#pragma unroll
            for (int j = 0; j < kPer; ++j) {
                tie_base[lane * kPer + j] = run;
                run += v[j];
            }
        }
        __syncthreads();
    }
#pragma unroll
    for (int u = 0; u < B; ++u) {
        const int r = u * kSelectThreads + tid;
        const int chunk = u * kWaves + wave;
        const bool is_cand = (cand >> u) & 1u;
        const bool tie = is_cand && key[u] == T;
        bool keep = r < n && (!is_cand || key[u] > T);
        const unsigned long long tie_mask = __ballot(tie);
        // unranked: every tie is kept when any is (quota 0 only with the all-halt state, where no key is kept)
        if (tie)
            keep = rank_ties ? tie_base[chunk] + __popcll(tie_mask & ((1ull << lane) - 1ull)) < quota : quota > 0;
        if (r < n) halt[r] = keep ? 0 : 1;
        const unsigned long long m = __ballot(keep);
        if (lane == 0 && chunk * kChunkRows < n) chunk_counts[chunk] = __popcll(m);
    }
}

// Standalone score of Eq. 2 from a stored fp32 delta and x: one wave per row, 16-byte loads.
template <typename T>
__global__ __launch_bounds__(256) void score_rows_kernel(const float* __restrict__ delta, const T* __restrict__ x,
                                                         int n, int d, int kind, float* __restrict__ scores) {
    const int row = (blockIdx.x * blockDim.x + threadIdx.x) / kWave;
    const int lane = threadIdx.x % kWave;
    if (row >= n) return;
    const float* dr = delta + (size_t)row * d;
    const T* xr = x + (size_t)row * d;
    float sd = 0.f, sx = 0.f;
    for (int c = lane * 4; c < d; c += kWave * 4) {  // d % 4 == 0 is checked by the caller
        const float4 dv = *reinterpret_cast<const float4*>(dr + c);
        sd += dv.x * dv.x + dv.y * dv.y + dv.z * dv.z + dv.w * dv.w;
        if (kind == DASH_SCORE_REL) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float xv = to_float(xr[c + e]);
                sx += xv * xv;
            }
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        sd += __shfl_xor(sd, o);
        sx += __shfl_xor(sx, o);
    }
    if (lane == 0) {
        const float nd = sqrtf(sd);
        scores[row] = kind == DASH_SCORE_ABS ? nd : nd / fmaxf(sqrtf(sx), kNormEps);
    }
}

size_t decide_workspace_bytes() { return 256; }

// ------------------------------------------------------------------------------------------------
// Scratch of the allocation-free TopK entry point (dash_decide_topk_static): the selection state and the tie
// counts of up to kStaticTopkMaxRows rows live in this file-scope device array instead of a caller's workspace.
// Every GPU the library runs on holds its own copy at its own address until the process ends. In host code the
// array's name is only a stand-in for the symbol: the device address is asked for once per device
// (hipGetSymbolAddress with that device current) and that pointer is what the launches get.
// ------------------------------------------------------------------------------------------------
constexpr size_t kStaticTopkScratchBytes = 256 + sizeof(int32_t) * (size_t)(kStaticTopkMaxRows / kChunkRows);
static __device__ __align__(256) unsigned char topk_static_scratch[kStaticTopkScratchBytes];

constexpr int kMaxDevices = 64;
static void* g_topk_scratch_ptr[kMaxDevices];   // device address of topk_static_scratch, per device; nullptr = not asked yet
static std::mutex g_topk_scratch_mutex;

// Device address of the current device's copy of the scratch array (asked for on the first call on that device).
dash_status topk_static_scratch_ptr(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return DASH_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_topk_scratch_mutex);
    if (!g_topk_scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(topk_static_scratch)) != hipSuccess || !ptr) return DASH_ERR_HIP;
        g_topk_scratch_ptr[dev] = ptr;
    }
    *out = g_topk_scratch_ptr[dev];
    return DASH_OK;
}

// The TopK decision on n > 0 scores: up to 16384 rows in one launch that keeps the keys in registers (when the
// caller allows it: 9 us at 8192 rows, 12.6 at 16384, where the two launches take 14; at 32768 rows it would take 23
// against their 20, the flags of the longer input being spread over many workgroups), longer inputs by the selection
// kernel, which leaves its state and tie counts in ws, and the flag kernel.
static void launch_topk(const float* scores, int n, int n_first, int n_last, int k_keep, int keep_low, uint8_t* halt,
                        int32_t* chunk_counts, void* ws, bool one_launch_allowed, hipStream_t s) {
    if (one_launch_allowed && n <= 8 * kSelectThreads) {
        hipLaunchKernelGGL(topk_decide_small_kernel<8>, dim3(1), dim3(kSelectThreads), 0, s, scores, n, n_first,
                           n_last, k_keep, keep_low, halt, chunk_counts);
    } else if (one_launch_allowed && n <= 16 * kSelectThreads) {
        hipLaunchKernelGGL(topk_decide_small_kernel<16>, dim3(1), dim3(kSelectThreads), 0, s, scores, n, n_first,
                           n_last, k_keep, keep_low, halt, chunk_counts);
    } else {
        TopkState* st = reinterpret_cast<TopkState*>(ws);
        int32_t* tie_counts = reinterpret_cast<int32_t*>(reinterpret_cast<char*>(ws) + 256);
        const int n_chunks = (n + kChunkRows - 1) / kChunkRows;
        hipLaunchKernelGGL(topk_select_kernel, dim3(1), dim3(kSelectThreads), 0, s, scores, n, n_first, n_last,
                           k_keep, keep_low, st, tie_counts);
        hipLaunchKernelGGL(topk_flag_kernel, dim3(n_chunks), dim3(256), 0, s, scores, n, n_first, n_last, keep_low,
                           st, tie_counts, halt, chunk_counts);
    }
}

dash_status launch_score_decide(const dash_layer_params& p, const float* partials, int n_partials, int n,
                                float* scores, uint8_t* halt, int32_t* chunk_counts, void* ws,
                                hipStream_t s) {
    if (n == 0) return DASH_OK;
    const int blocks = (n + kChunkRows - 1) / kChunkRows;
    if (p.rule != DASH_RULE_TOPK) {
        hipLaunchKernelGGL(score_threshold_kernel, dim3(blocks), dim3(256), 0, s, partials, n_partials, n,
                           p.score_kind, p.rule, p.tau, p.keep_first_n, p.keep_last_n, scores, halt,
                           chunk_counts);
        return launch_status();
    }
    int64_t k_keep = p.k_keep;
    if (k_keep < 0) k_keep = dash_keep_count(n, p.rho, 0, 0, 0);
    if (k_keep > n) k_keep = n;
    hipLaunchKernelGGL(score_only_kernel, dim3(blocks), dim3(256), 0, s, partials, n_partials, n,
                       p.score_kind, scores);
    launch_topk(scores, n, p.keep_first_n, p.keep_last_n, (int)k_keep, 0, halt, chunk_counts, ws, true, s);
    return launch_status();
}

// TopK decision on scores the caller provides (any signal: the block-level one, random numbers for the random
// control); keep_low selects the direction control.
dash_status launch_decide_topk(const dash_layer_params& p, const float* scores, int n, int keep_low, uint8_t* halt,
                               int32_t* chunk_counts, void* ws, bool one_launch_allowed, hipStream_t s) {
    if (n == 0) return DASH_OK;
    int64_t k_keep = p.k_keep;
    if (k_keep < 0) k_keep = dash_keep_count(n, p.rho, 0, 0, 0);
    if (k_keep > n) k_keep = n;
    launch_topk(scores, n, p.keep_first_n, p.keep_last_n, (int)k_keep, keep_low ? 1 : 0, halt, chunk_counts, ws,
                one_launch_allowed, s);
    return launch_status();
}

// Block-level signal of the ablation (Sec. 5.4): Eq. 2 on the change of a row across a whole block,
// ||x_new - x_old||_2, optionally relative to ||x_old||_2. One wave per row, 16-byte loads, two reads per element.
template <typename T>
__global__ __launch_bounds__(256) void score_diff_rows_kernel(const T* __restrict__ x_new, const T* __restrict__ x_old,
                                                              int n, int d, int kind, float* __restrict__ scores) {
    constexpr int VEC = 16 / (int)sizeof(T);
    const int row = (int)((blockIdx.x * (size_t)blockDim.x + threadIdx.x) / kWave);
    const int lane = threadIdx.x % kWave;
    if (row >= n) return;
    const T* a = x_new + (size_t)row * d;
    const T* b = x_old + (size_t)row * d;
    float sd = 0.f, sx = 0.f;
    for (int c = lane * VEC; c < d; c += kWave * VEC) {  // d % VEC == 0 is checked by the caller
        T va[VEC], vb[VEC];
        *reinterpret_cast<u32x4*>(va) = *reinterpret_cast<const u32x4*>(a + c);
        *reinterpret_cast<u32x4*>(vb) = *reinterpret_cast<const u32x4*>(b + c);
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            const float o = to_float(vb[e]), df = to_float(va[e]) - o;
            sd = fmaf(df, df, sd);
            sx = fmaf(o, o, sx);
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        sd += __shfl_xor(sd, o);
        sx += __shfl_xor(sx, o);
    }
    if (lane == 0) {
        const float nd = sqrtf(sd);
        scores[row] = kind == DASH_SCORE_ABS ? nd : nd / fmaxf(sqrtf(sx), kNormEps);
    }
}

dash_status launch_score_diff_rows(const void* x_new, const void* x_old, int n, int d, int dtype, int kind,
                                   float* scores, hipStream_t s) {
    if (n == 0) return DASH_OK;
    const int blocks = (int)(((size_t)n * kWave + 255) / 256);
    if (dtype == DASH_BF16)
        hipLaunchKernelGGL(score_diff_rows_kernel<__bf16>, dim3(blocks), dim3(256), 0, s, (const __bf16*)x_new,
                           (const __bf16*)x_old, n, d, kind, scores);
    else
        hipLaunchKernelGGL(score_diff_rows_kernel<float>, dim3(blocks), dim3(256), 0, s, (const float*)x_new,
                           (const float*)x_old, n, d, kind, scores);
    return launch_status();
}

dash_status launch_score_rows(const float* delta, const void* x, int n, int d, int dtype, int kind,
                              float* scores, hipStream_t s) {
    if (n == 0) return DASH_OK;
    const int blocks = (int)(((size_t)n * kWave + 255) / 256);
    if (dtype == DASH_BF16)
        hipLaunchKernelGGL(score_rows_kernel<__bf16>, dim3(blocks), dim3(256), 0, s, delta,
                           (const __bf16*)x, n, d, kind, scores);
    else
        hipLaunchKernelGGL(score_rows_kernel<float>, dim3(blocks), dim3(256), 0, s, delta, (const float*)x,
                           n, d, kind, scores);
    return launch_status();
}

}  // namespace dash
