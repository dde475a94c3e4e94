// Stream compaction of the surviving rows (Alg. 1 step 4; Sec. 3.4: each block runs on the
// compacted active sequence). HBM-bound: the row gather moves 2 * row_bytes per kept row.
//
// Layout: one workgroup per 64-row chunk (x column splits). The chunk's output offset is the sum of
// the kept counts of all earlier chunks (written by the decision kernel, one wave ballot each), so no
// cross-workgroup waiting is needed; ranks inside the chunk come from ballot + popcount.
#include "common.h"

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
    // column splits of whole wave-widths (64 vectors), enough workgroups to fill 256 CUs several times over
    const int wave_cols = (row_vecs + kWave - 1) / kWave;
    int splits = (2048 + n_chunks - 1) / n_chunks;
    if (splits > wave_cols) splits = wave_cols;
    if (splits < 1) splits = 1;
    const int vecs_per_split = ((wave_cols + splits - 1) / splits) * kWave;
    splits = (row_vecs + vecs_per_split - 1) / vecs_per_split;
    hipLaunchKernelGGL(compact_kernel, dim3(n_chunks, splits), dim3(kCompactThreads), 0, s, halt,
                       chunk_counts, active_idx, (const uint4*)x_next, n, row_vecs, vecs_per_split,
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
