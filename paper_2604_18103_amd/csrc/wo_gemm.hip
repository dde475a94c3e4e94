// Output projection fused with the residual update and the row norms:
//   delta = O @ W_o            (completes U of Eq. 1: the attention output before the residual add)
//   x_next = x + delta         (Sec. 3.1, Alg. 1 step 6)
//   partial sums of delta^2 and x^2 per row, from the fp32 accumulators (feeds Eq. 2)
// delta never goes to HBM (unless the caller asks for the debug copy): the score is taken before the
// bf16 rounding of x_next, which would otherwise cancel catastrophically for large-norm rows.
//
// Also here: the front end used by a chain of layers (RMSNorm + q/k/v projections), which shares the
// MFMA main loop with a plain store epilogue.
//
// norm_partials layout: [P][n][2] fp32, P = column tiles (x wave columns) of the kernel in use.
#include "common.h"

namespace dash {

// ------------------------------------------------------------------------------------------------
// Plain tiled kernel (fp32 path): 64x64 tile, 16x16 threads, 4x4 outputs per thread.
// ------------------------------------------------------------------------------------------------
constexpr int kSimpleTile = 64;

template <typename T>
__global__ __launch_bounds__(256) void wo_simple_kernel(const T* __restrict__ A, const T* __restrict__ B,
                                                        const T* __restrict__ x, int M, int K, int N,
                                                        T* __restrict__ x_next, float* __restrict__ partials,
                                                        float* __restrict__ delta_dbg) {
    constexpr int BK = 16;
    __shared__ float As[kSimpleTile][BK + 1];
    __shared__ float Bs[BK][kSimpleTile + 1];
    __shared__ float red[2][kSimpleTile][17];
    const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
    const int m0 = blockIdx.y * kSimpleTile, n0 = blockIdx.x * kSimpleTile;
    float acc[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) acc[a][b] = 0.f;
    for (int k0 = 0; k0 < K; k0 += BK) {
        for (int e = threadIdx.x; e < kSimpleTile * BK; e += 256) {
            const int r = e / BK, c = e % BK;
            const int gm = m0 + r, gk = k0 + c;
            As[r][c] = (gm < M && gk < K) ? to_float(A[(size_t)gm * K + gk]) : 0.f;
        }
        for (int e = threadIdx.x; e < BK * kSimpleTile; e += 256) {
            const int r = e / kSimpleTile, c = e % kSimpleTile;
            const int gk = k0 + r, gn = n0 + c;
            Bs[r][c] = (gk < K && gn < N) ? to_float(B[(size_t)gk * N + gn]) : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < BK; ++kk) {
            float av[4], bv[4];
#pragma unroll
            for (int a = 0; a < 4; ++a) av[a] = As[ty * 4 + a][kk];
#pragma unroll
            for (int b = 0; b < 4; ++b) bv[b] = Bs[kk][tx * 4 + b];
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int b = 0; b < 4; ++b) acc[a][b] = fmaf(av[a], bv[b], acc[a][b]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int a = 0; a < 4; ++a) {
        const int gm = m0 + ty * 4 + a;
        float sd = 0.f, sx = 0.f;
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int gn = n0 + tx * 4 + b;
            if (gm < M && gn < N) {
                const float xv = to_float(x[(size_t)gm * N + gn]);
                const float dv = acc[a][b];
                x_next[(size_t)gm * N + gn] = from_float<T>(xv + dv);
                if (delta_dbg) delta_dbg[(size_t)gm * N + gn] = dv;
                sd = fmaf(dv, dv, sd);
                sx = fmaf(xv, xv, sx);
            }
        }
        red[0][ty * 4 + a][tx] = sd;
        red[1][ty * 4 + a][tx] = sx;
    }
    __syncthreads();
    if (threadIdx.x < kSimpleTile) {
        const int gm = m0 + threadIdx.x;
        if (gm < M) {
            float sd = 0.f, sx = 0.f;
            for (int c = 0; c < 16; ++c) {
                sd += red[0][threadIdx.x][c];
                sx += red[1][threadIdx.x][c];
            }
            float2* dst = reinterpret_cast<float2*>(partials + ((size_t)blockIdx.x * M + gm) * 2);
            *dst = make_float2(sd, sx);
        }
    }
}

// ------------------------------------------------------------------------------------------------
// MFMA kernel (bf16): C[M,N] = A[M,K] B[K,N], A and B row-major.
// Workgroup tile 256x256, K step 32; 4 waves in 2x2, each wave 128x128 = 4x4 MFMA 32x32x16 blocks
// (256 fp32 accumulator registers per lane). A fragments are 16-byte LDS reads from the [m][k] tile;
// B fragments come from the natural [k][n] tile through LDS transpose reads.
// ------------------------------------------------------------------------------------------------
constexpr int kGM = 256, kGN = 256, kGK = 64;
constexpr int kGAStr = kGK + 8;     // elements; 144-byte rows: 16 lanes x 16 B land in distinct banks
constexpr int kGBStr = kGN + 32;    // elements; 576-byte rows for the transpose reads
constexpr int kEpiStr = 128 + 4;    // fp32 words per staged epilogue row
constexpr int kGAElems = kGM * kGAStr, kGBElems = kGK * kGBStr;
constexpr int kGStageElems = kGAElems + kGBElems;
constexpr size_t kGemmSmemBytes = 2 * kGStageElems * sizeof(__bf16);  // two operand stages (147456 B)
static_assert(kGemmSmemBytes >= 4 * 32 * kEpiStr * sizeof(float), "epilogue staging must fit");

typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;

__device__ __forceinline__ s16x4 lds_read_tr16_b(const __bf16* p) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(p));
}

enum { EPI_RESIDUAL_NORM = 0, EPI_STORE = 1 };

// MB = 32-row blocks per wave: 4 gives the 256-row tile, 2 a 128-row half tile. Half tiles finish the
// grid: when the 256-row tiles do not fill a whole number of rounds over the compute units, the tiles of
// the last, partly filled round are cut in two so that twice as many units share them.
// Workgroup b handles tile first_tile + b (MB = 4) or half b % 2 of tile first_tile + b / 2 (MB = 2).
template <int EPI, int MB>
__global__ __launch_bounds__(256, 1) void gemm_mfma_kernel(const __bf16* __restrict__ A,
                                                           const __bf16* __restrict__ B, int M, int K, int N,
                                                           const __bf16* __restrict__ x,
                                                           __bf16* __restrict__ out,  // x_next or C
                                                           float* __restrict__ partials,
                                                           float* __restrict__ delta_dbg, int n_mtiles,
                                                           int first_tile) {
    constexpr int BM = 64 * MB;   // rows of this workgroup's tile
    constexpr int WM = 32 * MB;   // rows of a wave's tile
    extern __shared__ __attribute__((aligned(16))) unsigned char gemm_smem_raw[];
    __bf16* smem = reinterpret_cast<__bf16*>(gemm_smem_raw);
    const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    const int j = lane % 32, h = lane / 32;
    const int wm = wave / 2, wn = wave % 2;
    // consecutive workgroups walk down M inside one column tile, so the B panel stays hot in L2
    const int tile = first_tile + (MB == 4 ? (int)blockIdx.x : (int)blockIdx.x / 2);
    const int tile_m = tile % n_mtiles, tile_n = tile / n_mtiles;
    const int m0 = tile_m * kGM + (MB == 4 ? 0 : ((int)blockIdx.x % 2) * BM), n0 = tile_n * kGN;

    f32x16 acc[MB][4];
#pragma unroll
    for (int a = 0; a < MB; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

    // global -> register staging of the next K step: A tile 256x64 and B tile 64x256, 8 x 16 B each per thread
    constexpr int AL = BM * kGK / 8 / 256, BL = kGK * kGN / 8 / 256;
    u32x4 ra[AL], rb[BL];
    const int a_row = tid / 8, a_c8 = tid % 8;    // + 32 rows per step
    const int b_row = tid / 32, b_c8 = tid % 32;  // + 8 rows per step
    const int gn = min(n0 + b_c8 * 8, N - 8);  // columns beyond N are computed on clamped data and never stored
    auto load_tiles = [&](int k0) {
#pragma unroll
        for (int it = 0; it < AL; ++it) {
            const int gm = min(m0 + a_row + 32 * it, M - 1);
            ra[it] = *reinterpret_cast<const u32x4*>(A + (size_t)gm * K + k0 + a_c8 * 8);
        }
#pragma unroll
        for (int it = 0; it < BL; ++it) {
            const int gk = k0 + b_row + 8 * it;
            rb[it] = *reinterpret_cast<const u32x4*>(B + (size_t)gk * N + gn);
        }
    };
    auto store_tiles = [&](int stage) {
        __bf16* sa = smem + stage * kGStageElems;
        __bf16* sb = sa + kGAElems;
#pragma unroll
        for (int it = 0; it < AL; ++it)
            *reinterpret_cast<u32x4*>(&sa[(a_row + 32 * it) * kGAStr + a_c8 * 8]) = ra[it];
#pragma unroll
        for (int it = 0; it < BL; ++it)
            *reinterpret_cast<u32x4*>(&sb[(b_row + 8 * it) * kGBStr + b_c8 * 8]) = rb[it];
    };

    const int tg = lane / 16, ti = lane % 16;
    const int n_ksteps = K / kGK;
    // barrier that orders LDS traffic only: the global loads of the next step must stay in flight across it
    auto lds_barrier = [] {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
    };
    // 64 MFMAs of one K step on the operand stage `st`
    auto compute_step = [&](int st) {
        const __bf16* sa = smem + st * kGStageElems;
        const __bf16* sb = sa + kGAElems;
#pragma unroll
        for (int ks = 0; ks < kGK / 16; ++ks) {
            bf16x8 Af[MB], Bf[4];
#pragma unroll
            for (int a = 0; a < MB; ++a)
                Af[a] = *reinterpret_cast<const bf16x8*>(&sa[(wm * WM + 32 * a + j) * kGAStr + 16 * ks + 8 * h]);
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                // lane (tg, ti): rows k = 16ks + 8*(tg/2) + ti/4 (+4), columns wn*128 + 32b + 16*(tg%2) + 4*(ti%4)
                const int krow = 16 * ks + 8 * (tg / 2) + ti / 4;
                const int col = wn * 128 + 32 * b + 16 * (tg % 2) + 4 * (ti % 4);
                const s16x4 lo = lds_read_tr16_b(&sb[krow * kGBStr + col]);
                const s16x4 hi = lds_read_tr16_b(&sb[(krow + 4) * kGBStr + col]);
                Bf[b] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
            }
#pragma unroll
            for (int a = 0; a < MB; ++a)
#pragma unroll
                for (int b = 0; b < 4; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Af[a], Bf[b], acc[a][b], 0, 0, 0);
        }
    };
    load_tiles(0);
    store_tiles(0);
    __syncthreads();
    // Steady state: one straight-line block per K step with its issue order pinned - the fragment reads of
    // the first 16-wide slice up front, then every MFMA paired with one read for a later slice; the
    // global loads of the next step ride along the first MFMAs and its LDS writes along the last ones,
    // by which time the loads have had about 1500 cycles to land.
    for (int kt = 0; kt + 1 < n_ksteps; ++kt) {
        load_tiles((kt + 1) * kGK);
        compute_step(kt & 1);
        // the other stage was last read in step kt-1, which every wave left through the barrier below
        store_tiles((kt + 1) & 1);
        if (MB == 4) {
        __builtin_amdgcn_sched_group_barrier(0x100, 12, 0);
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
#pragma unroll
        for (int i = 0; i < 20; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, 12, 0);
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);
        }
        } else {
            // half tile, 32 MFMAs per step: 10 fragment reads per 16-wide slice, 12 loads, 12 LDS writes
            __builtin_amdgcn_sched_group_barrier(0x100, 10, 0);
#pragma unroll
            for (int i = 0; i < 12; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
            }
#pragma unroll
            for (int i = 0; i < 6; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
            __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
#pragma unroll
            for (int i = 0; i < 12; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);
            }
        }
        lds_barrier();
    }
    compute_step((n_ksteps - 1) & 1);
    __syncthreads();
    // all waves are past the last barrier: the operand stages are free and are reused by the epilogue

    // Epilogue, per 32-row block of the wave's 128x128 tile: stage the fp32 accumulators in LDS, then every
    // lane handles 8 consecutive columns of one row - 16-byte x loads, 16-byte x_next stores, in-row sums
    // over 16 lanes. The x vectors of the next block are fetched before the current one is processed.
    float* stage = reinterpret_cast<float*>(gemm_smem_raw) + wave * 32 * kEpiStr;
    const int e_row = lane / 16, e_c8 = lane % 16;
    const int gn_e = n0 + wn * 128 + 8 * e_c8;
    const bool col_ok = gn_e < N;
    bf16x8 xv[2][8];
    auto fetch_x = [&](int a, bf16x8* dst) {
#pragma unroll
        for (int step = 0; step < 8; ++step) {
            const int gm = min(m0 + wm * WM + 32 * a + 4 * step + e_row, M - 1);
            dst[step] = *reinterpret_cast<const bf16x8*>(x + (size_t)gm * N + min(gn_e, N - 8));
        }
    };
    if (EPI == EPI_RESIDUAL_NORM) fetch_x(0, xv[0]);
#pragma unroll
    for (int a = 0; a < MB; ++a) {
        if (EPI == EPI_RESIDUAL_NORM && a + 1 < MB) fetch_x(a + 1, xv[(a + 1) & 1]);
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r)  // accumulator register r: local row 8*(r/4) + 4h + r%4, column j
                stage[(8 * (r / 4) + 4 * h + r % 4) * kEpiStr + 32 * b + j] = acc[a][b][r];
        __syncthreads();  // every wave runs the same epilogue schedule, so the barrier is uniform
#pragma unroll
        for (int step = 0; step < 8; ++step) {
            const int lr = 4 * step + e_row;
            const int gm = m0 + wm * WM + 32 * a + lr;
            const f32x4 d0 = *reinterpret_cast<const f32x4*>(&stage[lr * kEpiStr + 8 * e_c8]);
            const f32x4 d1 = *reinterpret_cast<const f32x4*>(&stage[lr * kEpiStr + 8 * e_c8 + 4]);
            const float dv[8] = {d0[0], d0[1], d0[2], d0[3], d1[0], d1[1], d1[2], d1[3]};
            const bool ok = gm < M && col_ok;
            if (EPI == EPI_RESIDUAL_NORM) {
                float sd = 0.f, sx = 0.f;
                if (ok) {
                    const bf16x8 xr = xv[a & 1][step];
                    bf16x8 ov;
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const float xf = (float)xr[e];
                        ov[e] = (__bf16)(xf + dv[e]);
                        sd = fmaf(dv[e], dv[e], sd);
                        sx = fmaf(xf, xf, sx);
                    }
                    *reinterpret_cast<bf16x8*>(out + (size_t)gm * N + gn_e) = ov;
                    if (delta_dbg) {
                        *reinterpret_cast<f32x4*>(delta_dbg + (size_t)gm * N + gn_e) = d0;
                        *reinterpret_cast<f32x4*>(delta_dbg + (size_t)gm * N + gn_e + 4) = d1;
                    }
                }
#pragma unroll
                for (int off = 8; off > 0; off >>= 1) {
                    sd += __shfl_xor(sd, off);
                    sx += __shfl_xor(sx, off);
                }
                if (e_c8 == 0 && gm < M) {
                    const int p = tile_n * 2 + wn;
                    *reinterpret_cast<float2*>(partials + ((size_t)p * M + gm) * 2) = make_float2(sd, sx);
                }
            } else if (ok) {
                bf16x8 ov;
#pragma unroll
                for (int e = 0; e < 8; ++e) ov[e] = (__bf16)dv[e];
                *reinterpret_cast<bf16x8*>(out + (size_t)gm * N + gn_e) = ov;
            }
        }
        __syncthreads();
    }
}

// h = x / sqrt(mean(x^2) + 1e-6), unit gain; one wave per row.
__global__ __launch_bounds__(256) void rmsnorm_kernel(const __bf16* __restrict__ x, int n, int d,
                                                      __bf16* __restrict__ hout) {
    const int row = (blockIdx.x * blockDim.x + threadIdx.x) / kWave;
    const int lane = threadIdx.x % kWave;
    if (row >= n) return;
    const __bf16* xr = x + (size_t)row * d;
    float ss = 0.f;
    for (int c = lane * 8; c < d; c += kWave * 8) {
        const bf16x8 v = *reinterpret_cast<const bf16x8*>(xr + c);
#pragma unroll
        for (int e = 0; e < 8; ++e) ss = fmaf((float)v[e], (float)v[e], ss);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off);
    const float inv = 1.0f / sqrtf(ss / (float)d + 1e-6f);
    __bf16* hr = hout + (size_t)row * d;
    for (int c = lane * 8; c < d; c += kWave * 8) {
        const bf16x8 v = *reinterpret_cast<const bf16x8*>(xr + c);
        bf16x8 ov;
#pragma unroll
        for (int e = 0; e < 8; ++e) ov[e] = (__bf16)((float)v[e] * inv);
        *reinterpret_cast<bf16x8*>(hr + c) = ov;
    }
}

int norm_partials_per_row(int d, int dtype) {
    if (dtype == DASH_F32) return (d + kSimpleTile - 1) / kSimpleTile;
    return 2 * ((d + kGN - 1) / kGN);
}

// Number of compute units of the current device (queried once; the library serves one GPU).
static int compute_units() {
    static const int n = [] {
        int dev = 0, cu = 0;
        if (hipGetDevice(&dev) != hipSuccess) return 0;
        if (hipDeviceGetAttribute(&cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
        return cu;
    }();
    return n;
}

// 256x256 tiles for every whole round over the compute units; if the tiles left over would occupy at most
// half of the units, they are run as 128-row half tiles by a second launch (same kernel, MB = 2).
template <int EPI>
static dash_status launch_gemm(const __bf16* A, const __bf16* B, int M, int K, int N, const __bf16* x,
                               __bf16* out, float* partials, float* delta_dbg, hipStream_t s) {
    static const hipError_t attr4 = hipFuncSetAttribute((const void*)gemm_mfma_kernel<EPI, 4>,
                                                         hipFuncAttributeMaxDynamicSharedMemorySize,
                                                         (int)kGemmSmemBytes);
    static const hipError_t attr2 = hipFuncSetAttribute((const void*)gemm_mfma_kernel<EPI, 2>,
                                                         hipFuncAttributeMaxDynamicSharedMemorySize,
                                                         (int)kGemmSmemBytes);
    if (attr4 != hipSuccess || attr2 != hipSuccess) return DASH_ERR_HIP;
    const int mt = (M + kGM - 1) / kGM, nt = (N + kGN - 1) / kGN, tiles = mt * nt;
    const int cu = compute_units();
    int rest = cu > 0 ? tiles % cu : 0;
    if (2 * rest > cu) rest = 0;
    const int full = tiles - rest;
    if (full > 0)
        hipLaunchKernelGGL((gemm_mfma_kernel<EPI, 4>), dim3(full), dim3(256), kGemmSmemBytes, s, A, B, M, K, N, x,
                           out, partials, delta_dbg, mt, 0);
    if (rest > 0)
        hipLaunchKernelGGL((gemm_mfma_kernel<EPI, 2>), dim3(2 * rest), dim3(256), kGemmSmemBytes, s, A, B, M, K, N,
                           x, out, partials, delta_dbg, mt, full);
    return launch_status();
}

static dash_status launch_gemm_store(const __bf16* A, const __bf16* B, int M, int K, int N, __bf16* C,
                                     hipStream_t s) {
    return launch_gemm<EPI_STORE>(A, B, M, K, N, nullptr, C, nullptr, nullptr, s);
}

dash_status launch_wo_residual_rownorm(const dash_layer_params& p, const void* o, const void* w_o,
                                       const void* x, int n, void* x_next, float* partials,
                                       float* delta_dbg, hipStream_t s) {
    if (n == 0) return DASH_OK;
    const int K = p.n_q_heads * p.head_dim, N = p.d;
    if (p.dtype == DASH_F32) {
        dim3 grid((N + kSimpleTile - 1) / kSimpleTile, (n + kSimpleTile - 1) / kSimpleTile);
        hipLaunchKernelGGL(wo_simple_kernel<float>, grid, dim3(256), 0, s, (const float*)o, (const float*)w_o,
                           (const float*)x, n, K, N, (float*)x_next, partials, delta_dbg);
        return launch_status();
    }
    return launch_gemm<EPI_RESIDUAL_NORM>((const __bf16*)o, (const __bf16*)w_o, n, K, N, (const __bf16*)x,
                                          (__bf16*)x_next, partials, delta_dbg, s);
}

dash_status launch_rmsnorm_qkv(const dash_layer_params& p, const void* x, const void* w_q, const void* w_k,
                               const void* w_v, int n, void* q, void* k, void* v, void* hbuf,
                               hipStream_t s) {
    if (n == 0) return DASH_OK;
    const int d = p.d, Dq = p.n_q_heads * p.head_dim, Dkv = p.n_kv_heads * p.head_dim;
    const int blocks = (int)(((size_t)n * kWave + 255) / 256);
    hipLaunchKernelGGL(rmsnorm_kernel, dim3(blocks), dim3(256), 0, s, (const __bf16*)x, n, d, (__bf16*)hbuf);
    dash_status st = launch_gemm_store((const __bf16*)hbuf, (const __bf16*)w_q, n, d, Dq, (__bf16*)q, s);
    if (st != DASH_OK) return st;
    st = launch_gemm_store((const __bf16*)hbuf, (const __bf16*)w_k, n, d, Dkv, (__bf16*)k, s);
    if (st != DASH_OK) return st;
    return launch_gemm_store((const __bf16*)hbuf, (const __bf16*)w_v, n, d, Dkv, (__bf16*)v, s);
}

}  // namespace dash
