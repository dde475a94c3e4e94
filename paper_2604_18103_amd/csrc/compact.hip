// Stream compaction of the surviving rows (Alg. 1 step 4; Sec. 3.4: each block runs on the
// compacted active sequence). HBM-bound: the row gather moves 2 * row_bytes per kept row.
//
// Layout: one workgroup per 64-row chunk (x column splits). The chunk's output offset is the sum of
// the kept counts of all earlier chunks (written by the decision kernel, one wave ballot each), so no
// cross-workgroup waiting is needed; ranks inside the chunk come from ballot + popcount.
#include "common.h"
#include "score_rows.h"

namespace dash {

__global__ __launch_bounds__(256) void chunk_counts_kernel(const uint8_t* __restrict__ halt, int n,
                                                           int32_t* __restrict__ counts) {
    const int chunk = (blockIdx.x * blockDim.x + threadIdx.x) / kWave;
    const int lane = threadIdx.x % kWave;
    const int n_chunks = (n + kChunkRows - 1) / kChunkRows;
    if (chunk >= n_chunks) return;
    const int row = chunk * kChunkRows + lane;
    const bool keep = row < n && halt[row] == 0;
    const unsigned long long m = __ballot(keep);
    if (lane == 0) counts[chunk] = __popcll(m);
}

__device__ __forceinline__ int wave_sum_int(int v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

constexpr int kCompactThreads = 256;
constexpr int kCompactWaves = kCompactThreads / kWave;

__global__ __launch_bounds__(kCompactThreads) void compact_kernel(
    const uint8_t* __restrict__ halt, const int32_t* __restrict__ counts,
    const int32_t* __restrict__ active_idx, const uint4* __restrict__ x_next, int n, int row_vecs,
    int vecs_per_split, uint4* __restrict__ x_compact, int32_t* __restrict__ new_idx,
    int32_t* __restrict__ n_out) {
    __shared__ int wave_part[kCompactWaves];
    __shared__ int kept_rows[kChunkRows];
    const int chunk = blockIdx.x;
    const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;

    // exclusive offset of this chunk: integer sum of earlier chunk counts (order does not matter)
    int part = 0;
    for (int c = tid; c < chunk; c += kCompactThreads) part += counts[c];
    part = wave_sum_int(part);
    if (lane == 0) wave_part[wave] = part;

    const int row = chunk * kChunkRows + lane;
    const bool keep = row < n && halt[row] == 0;
    const unsigned long long mask = __ballot(keep);
    const int rank = __popcll(mask & ((1ull << lane) - 1ull));
    const int cnt = __popcll(mask);
    if (wave == 0 && keep) kept_rows[rank] = row;
    __syncthreads();
    int base = 0;
#pragma unroll
    for (int w = 0; w < kCompactWaves; ++w) base += wave_part[w];

    if (blockIdx.y == 0 && wave == 0) {
        if (keep) new_idx[base + rank] = active_idx[row];
        if (chunk == (int)gridDim.x - 1 && lane == 0) *n_out = base + cnt;
    }

    // gather: a wave copies its kept rows four at a time (four independent 16-byte loads per lane in
    // flight before the first store); lanes stride over this split's vectors
    const int v0 = blockIdx.y * vecs_per_split;
    const int v1 = min(row_vecs, v0 + vecs_per_split);
    constexpr int R = 4;
    for (int r0 = wave * R; r0 < cnt; r0 += kCompactWaves * R) {
        const uint4* src[R];
        uint4* dst[R];
#pragma unroll
        for (int i = 0; i < R; ++i) {
            const int r = min(r0 + i, cnt - 1);  // a clamped duplicate rewrites the same bytes
            src[i] = x_next + (size_t)kept_rows[r] * row_vecs;
            dst[i] = x_compact + (size_t)(base + r) * row_vecs;
        }
        for (int c = v0 + lane; c < v1; c += kWave) {
            uint4 val[R];
#pragma unroll
            for (int i = 0; i < R; ++i) val[i] = src[i][c];
#pragma unroll
            for (int i = 0; i < R; ++i) dst[i][c] = val[i];
        }
    }
}

// ------------------------------------------------------------------------------------------------
// Score, threshold decision and compaction in ONE launch (rules NONE and THRESHOLD of the layer call).
//
// Grid (chunks of 64 rows, column splits), 256 threads. Workgroup (c, 0) finishes the scores of chunk c from the
// norm partials, writes scores and halt flags and PUBLISHES the chunk's kept mask and count; every workgroup
// (c, y) takes its chunk's mask and the counts of all earlier chunks from the published words, then gathers its
// columns of the kept rows as compact_kernel does. Nothing is computed twice and nothing waits for a kernel boundary.
//
// Published words: two 64-bit words per chunk, each valid on its own (a relaxed device-scope atomic store / load
// of one word: no fences, no ordering between words needed):
//   word 0 = kept mask bits 0..31 | kept count << 32 | READY      word 1 = kept mask bits 32..63 | READY
// They must be zero when the kernel starts (the attention kernel of the same layer call clears them).
// Waiting is safe: workgroups are dispatched in the order of their linear index (x fastest), a waiter (c, y) only
// waits for publishers (c', 0) with c' <= c, which have a smaller linear index, are therefore resident or done, and
// never wait themselves. The wait is bounded all the same: if a word never arrives the workgroup gives up, gathers
// nothing and the survivor count is written as -1.
// ------------------------------------------------------------------------------------------------
constexpr unsigned long long kPubReady = 1ull << 62;
constexpr int kPubSpinLimit = 1 << 20;

__device__ __forceinline__ unsigned long long wait_published(const unsigned long long* word, bool& bad) {
    unsigned long long v = __hip_atomic_load(word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    int spins = 0;
    while (!(v & kPubReady)) {
        __builtin_amdgcn_s_sleep(4);
        if (++spins > kPubSpinLimit) {
            bad = true;
            break;
        }
        v = __hip_atomic_load(word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    return v;
}

__global__ __launch_bounds__(kCompactThreads) void score_decide_compact_kernel(
    const float* __restrict__ partials, int P, int n, int score_kind, int rule, float tau, int n_first, int n_last,
    float* __restrict__ scores, uint8_t* __restrict__ halt, unsigned long long* __restrict__ published,
    const int32_t* __restrict__ active_idx, const uint4* __restrict__ x_next, int row_vecs, int vecs_per_split,
    uint4* __restrict__ x_compact, int32_t* __restrict__ new_idx, int32_t* __restrict__ n_out) {
    __shared__ float2 red[4][kChunkRows];
    __shared__ int wave_part[kCompactWaves];
    __shared__ int wave_bad[kCompactWaves];
    __shared__ int kept_rows[kChunkRows];
    const int chunk = blockIdx.x;
    const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
    const int row = chunk * kChunkRows + lane;
    bool bad = false;
    unsigned long long mask;
    if (blockIdx.y == 0) {
        // publisher: scores, flags, the chunk's kept mask
        const float2 t = row_sums_256(partials, P, n, chunk * kChunkRows, red);
        bool keep = false;
        if (row < n) {  // every wave holds the sums of the chunk's rows (row = lane): every wave gets the same mask
            const float sc = score_from_sums(t, score_kind);
            const bool h = rule == DASH_RULE_THRESHOLD && !row_protected(row, n, n_first, n_last) && sc < tau;
            keep = !h;
            if (wave == 0) {
                scores[row] = sc;
                halt[row] = h ? 1 : 0;
            }
        }
        mask = __ballot(keep);
        if (tid == 0) {
            const unsigned long long cnt = (unsigned long long)__popcll(mask);
            __hip_atomic_store(published + 2 * chunk, (mask & 0xFFFFFFFFull) | (cnt << 32) | kPubReady, __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(published + 2 * chunk + 1, (mask >> 32) | kPubReady, __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
        }
    } else {
        // the chunk's mask from its publisher (every lane reads the same two words: one request per wave)
        const unsigned long long w0 = wait_published(published + 2 * chunk, bad);
        const unsigned long long w1 = wait_published(published + 2 * chunk + 1, bad);
        mask = (w0 & 0xFFFFFFFFull) | ((w1 & 0xFFFFFFFFull) << 32);
    }
    // exclusive offset of this chunk: kept counts of all earlier chunks (integer sum, order does not matter)
    int part = 0;
    for (int c = tid; c < chunk; c += kCompactThreads)
        part += (int)((wait_published(published + 2 * c, bad) >> 32) & 0x7Full);
    part = wave_sum_int(part);
    const unsigned long long any_bad = __ballot(bad);
    if (lane == 0) {
        wave_part[wave] = part;
        wave_bad[wave] = any_bad != 0ull;
    }
    const bool keep = (mask >> lane) & 1ull;
    const int rank = __popcll(mask & ((1ull << lane) - 1ull));
    const int cnt = __popcll(mask);
    if (wave == 0 && keep) kept_rows[rank] = row;
    __syncthreads();
    int base = 0, failed = 0;
#pragma unroll
    for (int w = 0; w < kCompactWaves; ++w) {
        base += wave_part[w];
        failed |= wave_bad[w];
    }
    if (blockIdx.y == 0 && wave == 0) {
        if (keep && !failed) new_idx[base + rank] = active_idx[row];
        if (chunk == (int)gridDim.x - 1 && lane == 0) *n_out = failed ? -1 : base + cnt;
    }
    if (failed) return;  // uniform: every thread read the same LDS words
    const int v0 = ((int)gridDim.y - 1 - (int)blockIdx.y) * vecs_per_split;
    const int v1 = min(row_vecs, v0 + vecs_per_split);
    constexpr int R = 4;
    for (int r0 = wave * R; r0 < cnt; r0 += kCompactWaves * R) {
        const uint4* src[R];
        uint4* dst[R];
#pragma unroll
        for (int i = 0; i < R; ++i) {
            const int r = min(r0 + i, cnt - 1);  // a clamped duplicate rewrites the same bytes
            src[i] = x_next + (size_t)kept_rows[r] * row_vecs;
            dst[i] = x_compact + (size_t)(base + r) * row_vecs;
        }
        for (int c = v0 + lane; c < v1; c += kWave) {
            uint4 val[R];
#pragma unroll
            for (int i = 0; i < R; ++i) val[i] = src[i][c];
#pragma unroll
            for (int i = 0; i < R; ++i) dst[i][c] = val[i];
        }
    }
}

__global__ void write_zero_kernel(int32_t* p) { *p = 0; }

__global__ __launch_bounds__(256) void validate_idx_kernel(const int32_t* __restrict__ idx, int n, int N,
                                                           int32_t* __restrict__ violations) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int v = idx[i];
    bool bad = v < 0 || (N >= 0 && v >= N);
    if (i > 0 && idx[i - 1] >= v) bad = true;
    if (bad) atomicAdd(violations, 1);
}

// Column splits of the gather: whole wave-widths (64 vectors), enough workgroups to fill 256 CUs several times over.
static void gather_splits(int n_chunks, int row_vecs, int& splits, int& vecs_per_split) {
    const int wave_cols = (row_vecs + kWave - 1) / kWave;
    splits = (2048 + n_chunks - 1) / n_chunks;
    if (splits > wave_cols) splits = wave_cols;
    if (splits < 1) splits = 1;
    vecs_per_split = ((wave_cols + splits - 1) / splits) * kWave;
    splits = (row_vecs + vecs_per_split - 1) / vecs_per_split;
}

dash_status launch_chunk_counts(const uint8_t* halt, int n, int32_t* chunk_counts, hipStream_t s) {
    const int n_chunks = (n + kChunkRows - 1) / kChunkRows;
    if (n_chunks == 0) return DASH_OK;
    const int blocks = (n_chunks * kWave + 255) / 256;
    hipLaunchKernelGGL(chunk_counts_kernel, dim3(blocks), dim3(256), 0, s, halt, n, chunk_counts);
    return launch_status();
}

dash_status launch_compact(const uint8_t* halt, const int32_t* chunk_counts, const int32_t* active_idx,
                           const void* x_next, int n, int row_bytes, void* x_compact,
                           int32_t* new_active_idx, int32_t* n_active_out, hipStream_t s) {
    if (n == 0) {
        hipLaunchKernelGGL(write_zero_kernel, dim3(1), dim3(1), 0, s, n_active_out);
        return launch_status();
    }
    const int n_chunks = (n + kChunkRows - 1) / kChunkRows;
    const int row_vecs = row_bytes / 16;
    int splits, vecs_per_split;
    gather_splits(n_chunks, row_vecs, splits, vecs_per_split);
    hipLaunchKernelGGL(compact_kernel, dim3(n_chunks, splits), dim3(kCompactThreads), 0, s, halt,
                       chunk_counts, active_idx, (const uint4*)x_next, n, row_vecs, vecs_per_split,
                       (uint4*)x_compact, new_active_idx, n_active_out);
    return launch_status();
}

size_t published_bytes(int n) { return (size_t)((n + kChunkRows - 1) / kChunkRows) * 2 * sizeof(unsigned long long); }

// rules NONE and THRESHOLD: scores, decision and compaction in one launch. `published` (published_bytes(n), 8-byte
// aligned) must have been cleared on this stream before (launch_flash_fwd does it for the layer call).
dash_status launch_score_decide_compact(const dash_layer_params& p, const float* partials, int n_partials, int n,
                                        float* scores, uint8_t* halt, void* published, const int32_t* active_idx,
                                        const void* x_next, int row_bytes, void* x_compact, int32_t* new_active_idx,
                                        int32_t* n_active_out, hipStream_t s) {
    const int n_chunks = (n + kChunkRows - 1) / kChunkRows;
    const int row_vecs = row_bytes / 16;
    int splits, vecs_per_split;
    gather_splits(n_chunks, row_vecs, splits, vecs_per_split);
    hipLaunchKernelGGL(score_decide_compact_kernel, dim3(n_chunks, splits), dim3(kCompactThreads), 0, s, partials,
                       n_partials, n, p.score_kind, p.rule, p.tau, p.keep_first_n, p.keep_last_n, scores, halt,
                       (unsigned long long*)published, active_idx, (const uint4*)x_next, row_vecs, vecs_per_split,
                       (uint4*)x_compact, new_active_idx, n_active_out);
    return launch_status();
}

dash_status launch_validate_idx(const int32_t* idx, int n, int N, int32_t* violations, hipStream_t s) {
    hipLaunchKernelGGL(write_zero_kernel, dim3(1), dim3(1), 0, s, violations);
    if (n > 0)
        hipLaunchKernelGGL(validate_idx_kernel, dim3((n + 255) / 256), dim3(256), 0, s, idx, n, N,
                           violations);
    return launch_status();
}

// Halted tokens keep the state they had when they halted (Sec. 3.4): selected rows are written to a
// full-length buffer at their original positions. One wave per row, 16-byte vectors; rows whose position
// lies outside [0, N) are skipped.
template <typename T>
__global__ __launch_bounds__(256) void scatter_rows_kernel(const T* __restrict__ rows, const int32_t* __restrict__ idx,
                                                           const uint8_t* __restrict__ sel, int sel_value, int n,
                                                           int d, int N, T* __restrict__ full) {
    constexpr int VEC = 16 / (int)sizeof(T);
    const int row = (int)((blockIdx.x * (size_t)blockDim.x + threadIdx.x) / kWave);
    const int lane = threadIdx.x % kWave;
    if (row >= n) return;
    if (sel && sel[row] != (uint8_t)sel_value) return;
    const int p = idx[row];
    if (p < 0 || p >= N) return;
    const u32x4* src = reinterpret_cast<const u32x4*>(rows + (size_t)row * d);
    u32x4* dst = reinterpret_cast<u32x4*>(full + (size_t)p * d);
    for (int c = lane; c < d / VEC; c += kWave) dst[c] = src[c];
}

dash_status launch_scatter_rows(const void* rows, const int32_t* idx, const uint8_t* sel, int sel_value, int n,
                                int d, int dtype, int N, void* full, hipStream_t s) {
    if (n == 0) return DASH_OK;
    const int blocks = (int)(((size_t)n * kWave + 255) / 256);
    if (dtype == DASH_BF16)
        hipLaunchKernelGGL(scatter_rows_kernel<__bf16>, dim3(blocks), dim3(256), 0, s, (const __bf16*)rows, idx, sel,
                           sel_value, n, d, N, (__bf16*)full);
    else
        hipLaunchKernelGGL(scatter_rows_kernel<float>, dim3(blocks), dim3(256), 0, s, (const float*)rows, idx, sel,
                           sel_value, n, d, N, (float*)full);
    return launch_status();
}

}  // namespace dash
