// Shared declarations of the libdash kernels (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dash.h"

namespace dash {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

constexpr int kWave = 64;
constexpr float kNormEps = 1e-30f;  // floor on ||x_t|| in the relative score
constexpr int kChunkRows = 64;      // rows per keep-count chunk (one wave ballot)

__device__ __forceinline__ float to_float(float v) { return v; }
__device__ __forceinline__ float to_float(__bf16 v) { return (float)v; }
template <typename T>
__device__ __forceinline__ T from_float(float v);
template <>
__device__ __forceinline__ float from_float<float>(float v) { return v; }
template <>
__device__ __forceinline__ __bf16 from_float<__bf16>(float v) { return (__bf16)v; }  // round to nearest even

// Row is in the protected prefix/suffix of the current active order (App. A).
__device__ __forceinline__ bool row_protected(int i, int n, int n_first, int n_last) {
    return i < n_first || i >= n - n_last;
}

#define DASH_HIP_CHECK(expr)                     \
    do {                                         \
        if ((expr) != hipSuccess) return DASH_ERR_HIP; \
    } while (0)

inline dash_status launch_status() { return hipGetLastError() == hipSuccess ? DASH_OK : DASH_ERR_HIP; }

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// ---- stage launchers (implemented in the .hip files; all arguments validated by the caller) ----

// one-time set-up of the MFMA kernels (idempotent; also run by the first launch)
dash_status init_flash_kernels();
dash_status init_gemm_kernels();

// flash_fwd.hip
// clear_words / n_clear: optional device words the launch sets to zero (its first workgroup does it), for the
// kernels that follow in the same layer call and need cleared scratch without a launch of their own
dash_status launch_flash_fwd(const dash_layer_params& p, const void* q, const void* k, const void* v,
                             const int32_t* active_idx, int n, void* o, uint32_t* clear_words, int n_clear,
                             hipStream_t s);
// wo_gemm.hip
int norm_partials_per_row(int d, int dtype);
// split_ws / split_bytes: optional device scratch that lets products with few output tiles split along K
size_t wo_splitk_bytes(const dash_layer_params& p, int n);
dash_status launch_wo_residual_rownorm(const dash_layer_params& p, const void* o, const void* w_o,
                                       const void* x, int n, void* x_next, float* partials,
                                       float* delta_dbg, void* split_ws, size_t split_bytes, hipStream_t s);
size_t qkv_workspace_bytes(const dash_layer_params& p, int n);
dash_status launch_rmsnorm_qkv(const dash_layer_params& p, const void* x, const void* w_q, const void* w_k,
                               const void* w_v, int n, void* q, void* k, void* v, void* h, void* split_ws,
                               size_t split_bytes, hipStream_t s);
dash_status launch_rmsnorm_qkv_fused(const dash_layer_params& p, const void* x, const void* w_qkv, int n, void* q,
                                     void* k, void* v, void* h, void* split_ws, size_t split_bytes, hipStream_t s);
// score_decide.hip
size_t decide_workspace_bytes();
constexpr int kStaticTopkMaxRows = 1 << 20;  // row limit of the allocation-free TopK entry point
dash_status topk_static_scratch_ptr(void** out);  // this device's copy of its file-scope scratch array
dash_status launch_score_decide(const dash_layer_params& p, const float* partials, int n_partials, int n,
                                float* scores, uint8_t* halt, int32_t* chunk_counts, void* ws,
                                hipStream_t s);
dash_status launch_score_rows(const float* delta, const void* x, int n, int d, int dtype, int kind,
                              float* scores, hipStream_t s);
// compact.hip
size_t published_bytes(int n);  // words the fused score + decision + compaction kernel publishes its chunks through
dash_status launch_score_decide_compact(const dash_layer_params& p, const float* partials, int n_partials, int n,
                                        float* scores, uint8_t* halt, void* published, const int32_t* active_idx,
                                        const void* x_next, int row_bytes, void* x_compact, int32_t* new_active_idx,
                                        int32_t* n_active_out, hipStream_t s);
dash_status launch_chunk_counts(const uint8_t* halt, int n, int32_t* chunk_counts, hipStream_t s);
dash_status launch_compact(const uint8_t* halt, const int32_t* chunk_counts, const int32_t* active_idx,
                           const void* x_next, int n, int row_bytes, void* x_compact,
                           int32_t* new_active_idx, int32_t* n_active_out, hipStream_t s);
size_t ffn_workspace_bytes(const dash_layer_params& p, int n, int m);
dash_status launch_ffn_swiglu(const dash_layer_params& p, const void* x, const void* w_gate_up, const void* w_down,
                              int n, int m, void* x_out, void* ws, hipStream_t s);
dash_status launch_scatter_rows(const void* rows, const int32_t* idx, const uint8_t* sel, int sel_value, int n,
                                int d, int dtype, int N, void* full, hipStream_t s);
dash_status launch_decide_topk(const dash_layer_params& p, const float* scores, int n, int keep_low, uint8_t* halt,
                               int32_t* chunk_counts, void* ws, bool one_launch_allowed, hipStream_t s);
dash_status launch_score_diff_rows(const void* x_new, const void* x_old, int n, int d, int dtype, int kind,
                                   float* scores, hipStream_t s);
dash_status launch_rope_qk(const dash_layer_params& p, void* q, void* k, const int32_t* active_idx, int n,
                           double theta, hipStream_t s);
// mfma_probe.hip
constexpr int kProbeThreadsPerGroup = 512;
dash_status launch_mfma_probe(int wide, int normal_data, int iters, int workgroups, float* sink, hipStream_t s);
dash_status launch_validate_idx(const int32_t* idx, int n, int N, int32_t* violations, hipStream_t s);

}  // namespace dash
