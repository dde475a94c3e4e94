// Device helpers shared by the score/decision kernels and the fused score + decision + compaction kernel: the
// per-token score of Eq. 2 (or its relative form) finished from the per-row partial sums of squares that the
// projection stage took from its fp32 accumulators.
#pragma once

#include "common.h"

namespace dash {

// Sum of the P partial pairs of one row, taken by the four threads (row, q = 0..3) of a 256-thread
// workgroup that covers 64 rows: thread q adds partials q, q+4, ... in order, then the four sums are
// added in order q = 0..3 through LDS. Fixed order, so the score is bit-reproducible.
__device__ __forceinline__ float2 row_sums_256(const float* __restrict__ partials, int P, int n, int row_base,
                                               float2 (*red)[kChunkRows]) {
    const int r = threadIdx.x % kChunkRows, qd = threadIdx.x / kChunkRows;
    const int row = row_base + r;
    float sd = 0.f, sx = 0.f;
    if (row < n) {
#pragma unroll 4
        for (int p = qd; p < P; p += 4) {
            const float2 v = *reinterpret_cast<const float2*>(partials + ((size_t)p * n + row) * 2);
            sd += v.x;
            sx += v.y;
        }
    }
    red[qd][r] = make_float2(sd, sx);
    __syncthreads();
    float2 t = red[0][r];
#pragma unroll
    for (int k = 1; k < 4; ++k) {
        t.x += red[k][r].x;
        t.y += red[k][r].y;
    }
    return t;  // valid in every thread; callers use the copy of wave 0
}

__device__ __forceinline__ float score_from_sums(float2 t, int score_kind) {
    const float nd = sqrtf(t.x);
    if (score_kind == DASH_SCORE_ABS) return nd;
    return nd / fmaxf(sqrtf(t.y), kNormEps);
}

}  // namespace dash
