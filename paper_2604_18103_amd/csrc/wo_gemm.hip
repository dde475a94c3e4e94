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
// norm_partials layout: [P][n][2] fp32, P = column tiles of the kernel in use (256 columns; 64 in the fp32 kernel).
#include "common.h"
#include "lds_ops.h"
#include "staging_addr.h"

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
// Workgroup tile 256x256, K step 64; 8 waves in 2 (M) x 4 (N), two per SIMD, each wave 128x64 = 8x4 blocks of
// v_mfma_f32_16x16x32_bf16 (128 fp32 accumulator registers per lane). On normally distributed operands the part
// is power-limited, and this shape moves fewer accumulator registers per flop than 32x32x16: the same tiles and
// LDS traffic finish 1-2 % sooner end to end, although twice the MFMA instructions cost cycles at the full
// clock. A fragments are 16-byte LDS reads from the [m][k] tile; B fragments come from the natural [k][n] tile
// through LDS transpose reads.
// The tiles of a K step go from global memory straight into LDS (no registers in between). Such a load
// writes 1 KB of consecutive LDS per wave instruction, so rows cannot be padded; bank conflicts are avoided
// by an XOR swizzle of the 16-byte chunk index inside a row: A (128-byte rows, 16-byte reads of one chunk
// from 16 consecutive rows) by (row / 2) % 8, B (512-byte rows; 32 lanes read 4 k-rows and the 4 k-rows 8
// below them, 32 bytes of each) by 4 * (row % 4) + 2 * ((row / 8) % 2).
// ------------------------------------------------------------------------------------------------
constexpr int kGThreads = kGWaves * kWave;  // tile constants kGM, kGN, kGK: staging_addr.h
constexpr int kGBElems = kGK * kGN;
// Operand stages in LDS: a stage holds the A tile (64 MB rows) and the B tile of one K step. The 256-row tile has
// two stages (128 KB): the tiles of step k + 2 are requested once every wave is done with step k. The 128-row half
// tile has three (144 KB) and requests three steps ahead: its steps are half as long, and with only one step of
// lead it waited for memory latency at every step.
constexpr int gemm_stages(int MB) { return MB == 2 ? 3 : 2; }
constexpr int gemm_stage_elems(int MB) { return 64 * MB * kGK + kGBElems; }
constexpr size_t gemm_smem_bytes(int MB) { return (size_t)gemm_stages(MB) * gemm_stage_elems(MB) * sizeof(__bf16); }
constexpr int kEpiStr = 64 + 4;  // fp32 words per staged epilogue row (conflict-free 16-byte reads of two rows by 16 lanes)
static_assert(gemm_smem_bytes(4) >= 8 * 32 * kEpiStr * sizeof(float) + 4 * kGM * 2 * sizeof(float) &&
                  gemm_smem_bytes(2) >= 8 * 32 * kEpiStr * sizeof(float) + 4 * kGM * 2 * sizeof(float),
              "epilogue staging and the row-sum exchange must fit");


// EPI_SWIGLU: B holds gate and up columns interleaved in blocks of 32 (columns 64c..64c+31 = gate features
// 32c..32c+31, columns 64c+32..64c+63 = the up columns of the same features), so a wave's two 32-column
// accumulator blocks are gate and up of the same 32 features and the epilogue writes silu(gate) * up,
// N / 2 columns per row.
// EPI_SPLITK: the workgroup covers only the K steps of split blockIdx.y and writes its fp32 accumulators to
// f32_out[split][M][N]; a reduction kernel adds the splits in order and applies one of the other epilogues.
// EPI_QKV: a plain store whose columns are routed to three outputs (the q, k and v projections as one product
// over the concatenated weight).
enum { EPI_RESIDUAL_NORM = 0, EPI_STORE = 1, EPI_SWIGLU = 2, EPI_SPLITK = 3, EPI_QKV = 4 };

// Output routing of EPI_QKV: columns [0, Dq) go to `out` (row stride Dq), [Dq, Dq + Dkv) to k and the rest to v
// (row stride Dkv). Dq and Dkv are multiples of 8, so the 8 columns a lane stores never straddle two outputs.
struct QkvOut {
    __bf16* k;
    __bf16* v;
    int Dq, Dkv;
};
__device__ __forceinline__ __bf16* qkv_dst(__bf16* q, const QkvOut& o, int row, int col) {
    if (col < o.Dq) return q + (size_t)row * o.Dq + col;
    col -= o.Dq;
    if (col < o.Dkv) return o.k + (size_t)row * o.Dkv + col;
    return o.v + (size_t)row * o.Dkv + (col - o.Dkv);
}

// How the workgroups of a launch map to tiles (staging_addr.h: GemmPlan, gemm_index_of, gemm_tile_of).
struct GemmLaunch {
    int mt, nt, ksteps;
    int full, plain, seg;   // the launch of 256-row tiles (MB = 4): tile order and indices per XCD
    int first_tile;         // MB = 2: half tiles start at this tile index
    int ksteps_per_split;   // EPI_SPLITK: K steps per part (part = blockIdx.y)
};

// MB = 32-row blocks per wave: 4 gives the 256-row tile, 2 a 128-row half tile. Half tiles finish the
// grid: when the 256-row tiles do not fill a whole number of rounds over the compute units, the tiles of
// the last, partly filled round are cut in two so that twice as many units share them: workgroup b of that
// second launch handles half b % 2 of tile first_tile + b / 2.
template <int EPI, int MB>
__global__ __launch_bounds__(kGThreads, 1) void gemm_mfma_kernel(const __bf16* __restrict__ A,
                                                                 const __bf16* __restrict__ B, int M, int K,
                                                                 int N, const __bf16* __restrict__ x,
                                                                 __bf16* __restrict__ out,  // x_next or C
                                                                 float* __restrict__ partials,
                                                                 float* __restrict__ f32_out,  // delta (debug) or split sums
                                                                 GemmLaunch L, QkvOut qkv) {
    constexpr int BM = 64 * MB;   // rows of this workgroup's tile
    constexpr int WM = 32 * MB;   // rows of a wave's tile
    constexpr int NS = gemm_stages(MB), kAElems = BM * kGK, kStageElems = gemm_stage_elems(MB);
    extern __shared__ __attribute__((aligned(16))) unsigned char gemm_smem_raw[];
    __bf16* smem = reinterpret_cast<__bf16*>(gemm_smem_raw);
    const int tid = threadIdx.x, lane = tid % kWave;
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int wm = wave / 4, wn = wave % 4;
    // this workgroup's tile and K steps
    int tile_idx, ks0 = 0, n_ksteps = L.ksteps;
    if (EPI == EPI_SPLITK) {
        tile_idx = (int)blockIdx.x;
        ks0 = (int)blockIdx.y * L.ksteps_per_split;
        n_ksteps = min(L.ksteps_per_split, L.ksteps - ks0);
    } else if (MB == 2) {
        tile_idx = L.first_tile + (int)blockIdx.x / 2;
    } else {
        tile_idx = gemm_index_of((int)blockIdx.x, L.full, L.plain != 0, L.seg);
        if (tile_idx < 0) return;  // padding of the last stretch: the whole workgroup leaves
    }
    int tile_m, tile_n;
    gemm_tile_of(tile_idx, L.mt, L.nt, L.plain != 0, tile_m, tile_n);
    const int m0 = tile_m * kGM + (MB == 4 ? 0 : ((int)blockIdx.x % 2) * BM), n0 = tile_n * kGN;

    constexpr int RB = 2 * MB;  // 16-row blocks of the wave's tile; 4 column blocks of 16
    f32x4 acc[RB][4];
#pragma unroll
    for (int a = 0; a < RB; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[a][b][r] = 0.f;

    // Staging. A tile: BM rows of 128 bytes, one load instruction = 8 rows; B tile: 64 rows of 512 bytes,
    // one instruction = 2 rows. Lane l lands in physical chunk l % (chunks per row) of its row and therefore
    // fetches the logical chunk that the swizzle maps there. Rows beyond M and columns beyond N are clamped:
    // they are computed on valid data and never stored.
    // The address of a load is a scalar base (this workgroup's tile at the current K step, advanced by scalar
    // arithmetic) plus a 32-bit lane offset that never changes.
    constexpr int ADMA = gemm_adma(BM), BDMA = gemm_bdma();  // load instructions per wave and K step
    uint32_t a_off[ADMA], b_off[BDMA];
#pragma unroll
    for (int i = 0; i < ADMA; ++i) {
        const int row = gemm_a_row(wave, i, lane, ADMA);
        a_off[i] = gemm_a_off(m0, M, K, row, gemm_a_lchunk(row, lane));
    }
#pragma unroll
    for (int i = 0; i < BDMA; ++i) {
        const int row = gemm_b_row(wave, i, lane);
        b_off[i] = gemm_b_off(n0, N, row, gemm_b_lchunk(row, lane));
    }
    const char* a_base = reinterpret_cast<const char*>(A + gemm_a_base_elem(m0, M, K, ks0));
    const char* b_base = reinterpret_cast<const char*>(B + gemm_b_base_elem(n0, N, ks0));
    const size_t b_step = gemm_b_step_bytes(N);
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)gemm_smem_raw;
    const uint32_t lds_a = lds0 + (uint32_t)(wave * ADMA * 1024);
    const uint32_t lds_b = lds0 + (uint32_t)(kAElems * 2 + wave * BDMA * 1024);
    // K steps are fetched strictly in order; the A and the B tile of a step are requested separately
    auto dma_next_a = [&](int stage) {
        const uint32_t so = (uint32_t)(stage * kStageElems * 2);
#pragma unroll
        for (int i = 0; i < ADMA; ++i) dma_load16(a_base, a_off[i], lds_a + so + i * 1024);
        a_base += gemm_a_step_bytes();
    };
    auto dma_next_b = [&](int stage) {
        const uint32_t so = (uint32_t)(stage * kStageElems * 2);
#pragma unroll
        for (int i = 0; i < BDMA; ++i) dma_load16(b_base, b_off[i], lds_b + so + i * 1024);
        b_base += b_step;
    };

    // barrier that orders LDS traffic only
    auto lds_barrier = [] {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
    };
    // Fragments of one 32-wide slice for v_mfma_f32_16x16x32_bf16: RB A fragments (rows 16 rb + i, k-slots
    // 8 g .. 8 g + 7: one 16-byte read) and four B fragments (columns 16 cb + i, the same k-slots: two transpose
    // reads of a 4 x 16 block each), lane = 16 g + i.
    const int fi = lane % 16, fg = lane / 16;
    bf16x8 Af[2][RB], Bf[2][4];
    auto read_frags = [&](int st, int ks, bf16x8* af, bf16x8* bfr) {
        const __bf16* sa = smem + st * kStageElems;
        const __bf16* sb = sa + kAElems;
        // B first: the MFMAs of a slice go through the row blocks in order and need every B fragment at once
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int krow = 32 * ks + 8 * fg + fi / 4;  // and krow + 4: the same swizzle
            const int col = wn * 64 + 16 * b + 4 * (fi % 4);
            const int scol = ((col / 8) ^ gemm_b_swz(krow)) * 8 + col % 8;
            const s16x4 lo = lds_read_tr16(&sb[krow * kGN + scol]);
            const s16x4 hi = lds_read_tr16(&sb[(krow + 4) * kGN + scol]);
            bfr[b] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
        }
#pragma unroll
        for (int a = 0; a < RB; ++a) {
            const int row = wm * WM + 16 * a + fi;
            af[a] = *reinterpret_cast<const bf16x8*>(&sa[row * kGK + ((4 * ks + fg) ^ ((row / 2) % 8)) * 8]);
        }
    };
    auto mfma_slice = [&](const bf16x8* af, const bf16x8* bfr) {
#pragma unroll
        for (int a = 0; a < RB; ++a)
#pragma unroll
            for (int b = 0; b < 4; ++b)
                acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[a], bfr[b], acc[a][b], 0, 0, 0);
    };
    // issue order of one slice: the fragment reads of the slice after it spread between its MFMAs
    constexpr int RD = RB + 8, MF = 4 * RB;  // LDS reads and MFMAs per slice: 16 and 32, or 12 and 16
    auto pin_slice = [] {
#pragma unroll
        for (int i = 0; i < 2 * RD - MF; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
#pragma unroll
        for (int i = 0; i < MF - RD; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
    };
    constexpr int kStepLoads = ADMA + BDMA;
    const int n_pre = min(NS, n_ksteps);
    for (int j = 0; j < n_pre; ++j) {
        dma_next_a(j);
        dma_next_b(j);
    }
    if (n_pre == NS) {
        asm volatile("s_waitcnt vmcnt(%0)" : : "n"((NS - 1) * kStepLoads) : "memory");  // step 0 has landed
    } else {
        dma_wait();
    }
    __syncthreads();
    read_frags(0, 0, Af[0], Bf[0]);
    // One round per K step of two 32-wide slices. The fragments of a slice are read while the MFMAs of the slice
    // before it run, across the step boundary too: the wait for the next step's tiles and the barrier that
    // publishes them sit before the second slice's MFMAs, whose fragments are in registers by then, and the
    // first slice of the next step is read from the next stage while those MFMAs run. After that barrier every
    // wave is done reading this step's stage, so the tiles of step kt + NS are requested into it.
    //
    // Second half of a step. The tile requests are dealt out between its MFMAs, one every three: the compute
    // unit's one address unit takes 16 cycles per request and holds few of them, so after a burst of requests every
    // wave queues behind it and issues no MFMA meanwhile (a burst after the barrier: 5 % slower; one request per
    // MFMA, per 2, per 4: 3, 1.5 and 0.5 % slower than per 3). The requests are opaque to the compiler's scheduler
    // and fence its LDS reads, so this half is placed by hand: requests, the fragment reads of the next slice (B
    // first) at even distances, MFMAs, pinned in eight groups.
    auto read_b_frag = [&](int st, int ks, int b, bf16x8* bfr) {
        const __bf16* sb = smem + st * kStageElems + kAElems;
        const int krow = 32 * ks + 8 * fg + fi / 4;
        const int col = wn * 64 + 16 * b + 4 * (fi % 4);
        const int scol = ((col / 8) ^ gemm_b_swz(krow)) * 8 + col % 8;
        const s16x4 lo = lds_read_tr16(&sb[krow * kGN + scol]);
        const s16x4 hi = lds_read_tr16(&sb[(krow + 4) * kGN + scol]);
        bfr[b] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    };
    auto read_a_frag = [&](int st, int ks, int a, bf16x8* af) {
        const __bf16* sa = smem + st * kStageElems;
        const int row = wm * WM + 16 * a + fi;
        af[a] = *reinterpret_cast<const bf16x8*>(&sa[row * kGK + ((4 * ks + fg) ^ ((row / 2) % 8)) * 8]);
    };
    constexpr int kRequestEvery = 3;  // MFMAs from one tile request to the next
    static_assert((kStepLoads - 1) * kRequestEvery < MF, "the requests of a step fit into its second half");
    auto second_half = [&](int st_next, bool request, int st_free) {
        constexpr int UNITS = 4 + RB;  // fragments of the next slice: 4 B, RB A
        const uint32_t so = (uint32_t)(st_free * kStageElems * 2);
#pragma unroll
        for (int m = 0; m < MF; ++m) {
#pragma unroll
            for (int l = 0; l < kStepLoads; ++l)
                if (m == l * kRequestEvery && request) {
                    if (l < ADMA) dma_load16(a_base, a_off[l], lds_a + so + l * 1024);
                    else dma_load16(b_base, b_off[l - ADMA], lds_b + so + (l - ADMA) * 1024);
                }
#pragma unroll
            for (int u = 0; u < UNITS; ++u)  // fragment u before the first MFMA m with u * MF <= m * UNITS
                if (u * MF <= m * UNITS && (m == 0 || u * MF > (m - 1) * UNITS)) {
                    if (u < 4) read_b_frag(st_next, 0, u, Bf[0]);
                    else read_a_frag(st_next, 0, u - 4, Af[0]);
                }
            acc[m / 4][m % 4] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(Af[1][m / 4], Bf[1][m % 4], acc[m / 4][m % 4], 0, 0, 0);
            if (m % (MF / 8) == MF / 8 - 1) __builtin_amdgcn_sched_barrier(0);
        }
        if (request) {
            a_base += gemm_a_step_bytes();
            b_base += b_step;
        }
    };
    int kt = 0, st = 0;  // st = kt % NS
    for (; kt + NS < n_ksteps; ++kt) {
        const int st_next = st + 1 == NS ? 0 : st + 1;
        read_frags(st, 1, Af[1], Bf[1]);
        mfma_slice(Af[0], Bf[0]);
        pin_slice();
        // the tiles of step kt + 1 have landed; those of the steps after it may still be in flight
        asm volatile("s_waitcnt vmcnt(%0)" : : "n"((NS - 2) * kStepLoads) : "memory");
        asm volatile("s_waitcnt lgkmcnt(0)" : : : "memory");  // the second slice's fragments are in registers
        lds_barrier();
        second_half(st_next, true, st);
        st = st_next;
    }
    for (; kt < n_ksteps; ++kt) {  // the last NS steps request nothing
        const int st_next = st + 1 == NS ? 0 : st + 1;
        read_frags(st, 1, Af[1], Bf[1]);
        mfma_slice(Af[0], Bf[0]);
        pin_slice();
        dma_wait();
        asm volatile("s_waitcnt lgkmcnt(0)" : : : "memory");
        lds_barrier();
        second_half(st_next, false, st);  // after the last step the fragments read are stale data, never used
        st = st_next;
    }
    __syncthreads();  // the stale fragment reads of slower waves are harmless, but keep the epilogue's reuse simple
    // all waves are past the last barrier: the operand stages are free and are reused by the epilogue

    // Epilogue, per 32-row block of the wave's tile: stage the fp32 accumulators in LDS, then every lane
    // handles 8 consecutive columns of one row - 16-byte x loads, 16-byte x_next stores, in-row sums over
    // 8 lanes. The x vectors of the next block are fetched before the current one is processed.
    float* stage = reinterpret_cast<float*>(gemm_smem_raw) + wave * 32 * kEpiStr;
    float2* nrm = reinterpret_cast<float2*>(gemm_smem_raw + kGWaves * 32 * kEpiStr * sizeof(float));  // [4 wave columns][BM rows]
    const int e_row = lane / 8, e_c8 = lane % 8;
    const int gn_e = n0 + wn * 64 + 8 * e_c8;
    const bool col_ok = gn_e < N;
    bf16x8 xv[2][4];
    auto fetch_x = [&](int a, bf16x8* dst) {
#pragma unroll
        for (int step = 0; step < 4; ++step) {
            const int gm = min(m0 + wm * WM + 32 * a + 8 * step + e_row, M - 1);
            dst[step] = __builtin_nontemporal_load(reinterpret_cast<const bf16x8*>(x + (size_t)gm * N + min(gn_e, N - 8)));
        }
    };
    if (EPI == EPI_RESIDUAL_NORM) fetch_x(0, xv[0]);
#pragma unroll
    for (int a = 0; a < MB; ++a) {
        if (EPI == EPI_RESIDUAL_NORM && a + 1 < MB) fetch_x(a + 1, xv[(a + 1) & 1]);
#pragma unroll
        for (int sb = 0; sb < 2; ++sb)
#pragma unroll
            for (int b = 0; b < 4; ++b)
#pragma unroll
                for (int r = 0; r < 4; ++r)  // accumulator register r of a 16x16 block: row 4 g + r, column i
                    stage[(16 * sb + 4 * fg + r) * kEpiStr + 16 * b + fi] = acc[2 * a + sb][b][r];
        __syncthreads();  // every wave runs the same epilogue schedule, so the barrier is uniform
        if (EPI == EPI_SWIGLU) {
            // 4 lanes per row: lane c takes gate columns 8c..8c+7 and the up columns 32 + 8c..
            const int s_row = lane / 4, s_c = lane % 4;
            const int gcol = n0 / 2 + wn * 32 + 8 * s_c;  // output column
#pragma unroll
            for (int step = 0; step < 2; ++step) {
                const int lr = 16 * step + s_row;
                const int gm = m0 + wm * WM + 32 * a + lr;
                const f32x4 g0 = *reinterpret_cast<const f32x4*>(&stage[lr * kEpiStr + 8 * s_c]);
                const f32x4 g1 = *reinterpret_cast<const f32x4*>(&stage[lr * kEpiStr + 8 * s_c + 4]);
                const f32x4 u0 = *reinterpret_cast<const f32x4*>(&stage[lr * kEpiStr + 32 + 8 * s_c]);
                const f32x4 u1 = *reinterpret_cast<const f32x4*>(&stage[lr * kEpiStr + 32 + 8 * s_c + 4]);
                const float gv[8] = {g0[0], g0[1], g0[2], g0[3], g1[0], g1[1], g1[2], g1[3]};
                const float uv[8] = {u0[0], u0[1], u0[2], u0[3], u1[0], u1[1], u1[2], u1[3]};
                if (gm < M && gcol < N / 2) {
                    bf16x8 ov;
#pragma unroll
                    for (int e = 0; e < 8; ++e) ov[e] = (__bf16)(gv[e] / (1.0f + __expf(-gv[e])) * uv[e]);
                    *reinterpret_cast<bf16x8*>(out + (size_t)gm * (N / 2) + gcol) = ov;
                }
            }
            __syncthreads();
            continue;
        }
#pragma unroll
        for (int step = 0; step < 4; ++step) {
            const int lr = 8 * step + e_row;
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
                    if (f32_out) {
                        *reinterpret_cast<f32x4*>(f32_out + (size_t)gm * N + gn_e) = d0;
                        *reinterpret_cast<f32x4*>(f32_out + (size_t)gm * N + gn_e + 4) = d1;
                    }
                }
#pragma unroll
                for (int off = 4; off > 0; off >>= 1) {
                    sd += __shfl_xor(sd, off);
                    sx += __shfl_xor(sx, off);
                }
                // the four wave columns of the tile meet in LDS; one pair per row and tile is written after the loop
                if (e_c8 == 0) nrm[wn * BM + wm * WM + 32 * a + lr] = make_float2(sd, sx);
            } else if (EPI == EPI_SPLITK) {
                if (ok) {
                    float* dst = f32_out + ((size_t)blockIdx.y * M + gm) * N + gn_e;
                    *reinterpret_cast<f32x4*>(dst) = d0;
                    *reinterpret_cast<f32x4*>(dst + 4) = d1;
                }
            } else if (ok) {
                bf16x8 ov;
#pragma unroll
                for (int e = 0; e < 8; ++e) ov[e] = (__bf16)dv[e];
                __bf16* dst = EPI == EPI_QKV ? qkv_dst(out, qkv, gm, gn_e) : out + (size_t)gm * N + gn_e;
                *reinterpret_cast<bf16x8*>(dst) = ov;
            }
        }
        __syncthreads();
    }
    if (EPI == EPI_RESIDUAL_NORM) {
        // row sums of the tile's 256 columns: the wave columns in the fixed order 0..3
        for (int r = tid; r < BM; r += kGThreads) {
            const int gm = m0 + r;
            if (gm < M) {
                float2 t = nrm[r];
#pragma unroll
                for (int w = 1; w < 4; ++w) {
                    t.x += nrm[w * BM + r].x;
                    t.y += nrm[w * BM + r].y;
                }
                *reinterpret_cast<float2*>(partials + ((size_t)tile_n * M + gm) * 2) = t;
            }
        }
    }
}

// Second pass of a split-K product: adds the S split sums of sums[S][M][N] in the order s = 0..S-1 and applies
// the epilogue EPI (same results layout as the one-pass kernel). A wave works on one row; a lane owns 8
// consecutive columns, so the 32 lanes of a 256-column tile hold that tile's row sums for the norm partials.
template <int EPI>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* __restrict__ sums, int S, int M, int N,
                                                            const __bf16* __restrict__ x, __bf16* __restrict__ out,
                                                            float* __restrict__ partials, QkvOut qkv) {
    const int lane = threadIdx.x % kWave;
    const int wave_global = (int)((blockIdx.x * (size_t)blockDim.x + threadIdx.x) / kWave);
    if (EPI == EPI_SWIGLU) {
        // 4 lanes per 64-column group (32 gate + 32 up columns): 16 groups = 1024 input columns per wave
        const int segs = (N + 1023) / 1024;
        const int row = wave_global / segs, seg = wave_global % segs;
        if (row >= M) return;
        const int grp = seg * 16 + lane / 4, c = lane % 4;
        const int gcol = grp * 64 + 8 * c;  // gate columns gcol..gcol+7, up columns gcol+32..
        if (gcol >= N) return;
        float g[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f}, u[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        for (int sp = 0; sp < S; ++sp) {
            const float* src = sums + ((size_t)sp * M + row) * N + gcol;
            const f32x4 g0 = *reinterpret_cast<const f32x4*>(src), g1 = *reinterpret_cast<const f32x4*>(src + 4);
            const f32x4 u0 = *reinterpret_cast<const f32x4*>(src + 32), u1 = *reinterpret_cast<const f32x4*>(src + 36);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                g[e] += g0[e];
                g[4 + e] += g1[e];
                u[e] += u0[e];
                u[4 + e] += u1[e];
            }
        }
        bf16x8 ov;
#pragma unroll
        for (int e = 0; e < 8; ++e) ov[e] = (__bf16)(g[e] / (1.0f + __expf(-g[e])) * u[e]);
        *reinterpret_cast<bf16x8*>(out + (size_t)row * (N / 2) + grp * 32 + 8 * c) = ov;
        return;
    }
    const int segs = (N + 511) / 512;  // 8 groups of 64 columns per wave
    const int row = wave_global / segs, seg = wave_global % segs;
    if (row >= M) return;
    const int grp = seg * 8 + lane / 8;
    const int col = grp * 64 + 8 * (lane % 8);
    const bool ok = col < N;
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (ok) {
        for (int sp = 0; sp < S; ++sp) {
            const float* src = sums + ((size_t)sp * M + row) * N + col;
            const f32x4 a0 = *reinterpret_cast<const f32x4*>(src), a1 = *reinterpret_cast<const f32x4*>(src + 4);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                acc[e] += a0[e];
                acc[4 + e] += a1[e];
            }
        }
    }
    if (EPI == EPI_STORE || EPI == EPI_QKV) {
        if (ok) {
            bf16x8 ov;
#pragma unroll
            for (int e = 0; e < 8; ++e) ov[e] = (__bf16)acc[e];
            __bf16* dst = EPI == EPI_QKV ? qkv_dst(out, qkv, row, col) : out + (size_t)row * N + col;
            *reinterpret_cast<bf16x8*>(dst) = ov;
        }
        return;
    }
    float sd = 0.f, sx = 0.f;
    if (ok) {
        const bf16x8 xr = *reinterpret_cast<const bf16x8*>(x + (size_t)row * N + col);
        bf16x8 ov;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float xf = (float)xr[e];
            ov[e] = (__bf16)(xf + acc[e]);
            sd = fmaf(acc[e], acc[e], sd);
            sx = fmaf(xf, xf, sx);
        }
        *reinterpret_cast<bf16x8*>(out + (size_t)row * N + col) = ov;
    }
    // one partial pair per 256-column tile, as the one-pass kernel writes them: the 32 lanes of a tile in fixed order
#pragma unroll
    for (int off = 1; off < 32; off <<= 1) {
        sd += __shfl_xor(sd, off);
        sx += __shfl_xor(sx, off);
    }
    const int tile = seg * 2 + lane / 32;
    if (lane % 32 == 0 && tile < (N + kGN - 1) / kGN)
        *reinterpret_cast<float2*>(partials + ((size_t)tile * M + row) * 2) = make_float2(sd, sx);
}

// h = x / sqrt(mean(x^2) + 1e-6), unit gain; one wave per row. Rows of up to 512 * CH elements are held in
// registers between the two passes (one read of x); longer rows are read twice (CH = 0).
template <int CH>
__global__ __launch_bounds__(256) void rmsnorm_kernel(const __bf16* __restrict__ x, int n, int d,
                                                      __bf16* __restrict__ hout) {
    const int row = (blockIdx.x * blockDim.x + threadIdx.x) / kWave;
    const int lane = threadIdx.x % kWave;
    if (row >= n) return;
    const __bf16* xr = x + (size_t)row * d;
    __bf16* hr = hout + (size_t)row * d;
    float ss = 0.f;
    if (CH > 0) {
        bf16x8 v[CH > 0 ? CH : 1];
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const int c = (i * kWave + lane) * 8;
            if (c < d) {
                v[i] = *reinterpret_cast<const bf16x8*>(xr + c);
#pragma unroll
                for (int e = 0; e < 8; ++e) ss = fmaf((float)v[i][e], (float)v[i][e], ss);
            }
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off);
        const float inv = 1.0f / sqrtf(ss / (float)d + 1e-6f);
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const int c = (i * kWave + lane) * 8;
            if (c < d) {
                bf16x8 ov;
#pragma unroll
                for (int e = 0; e < 8; ++e) ov[e] = (__bf16)((float)v[i][e] * inv);
                *reinterpret_cast<bf16x8*>(hr + c) = ov;
            }
        }
        return;
    }
    for (int c = lane * 8; c < d; c += kWave * 8) {
        const bf16x8 v = *reinterpret_cast<const bf16x8*>(xr + c);
#pragma unroll
        for (int e = 0; e < 8; ++e) ss = fmaf((float)v[e], (float)v[e], ss);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off);
    const float inv = 1.0f / sqrtf(ss / (float)d + 1e-6f);
    for (int c = lane * 8; c < d; c += kWave * 8) {
        const bf16x8 v = *reinterpret_cast<const bf16x8*>(xr + c);
        bf16x8 ov;
#pragma unroll
        for (int e = 0; e < 8; ++e) ov[e] = (__bf16)((float)v[e] * inv);
        *reinterpret_cast<bf16x8*>(hr + c) = ov;
    }
}

static void launch_rmsnorm(const __bf16* x, int n, int d, __bf16* h, hipStream_t s) {
    const int blocks = (int)(((size_t)n * kWave + 255) / 256);
    if (d <= 512 * 4)
        hipLaunchKernelGGL(rmsnorm_kernel<4>, dim3(blocks), dim3(256), 0, s, x, n, d, h);
    else if (d <= 512 * 8)
        hipLaunchKernelGGL(rmsnorm_kernel<8>, dim3(blocks), dim3(256), 0, s, x, n, d, h);
    else
        hipLaunchKernelGGL(rmsnorm_kernel<0>, dim3(blocks), dim3(256), 0, s, x, n, d, h);
}

int norm_partials_per_row(int d, int dtype) {
    if (dtype == DASH_F32) return (d + kSimpleTile - 1) / kSimpleTile;
    return (d + kGN - 1) / kGN;
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

// One-time launch attribute of every instantiation of the MFMA kernel: its dynamic LDS (128 KB, half tiles 144 KB).
template <int EPI>
static hipError_t set_gemm_lds_size() {
    hipError_t e = hipFuncSetAttribute((const void*)gemm_mfma_kernel<EPI, 4>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)gemm_smem_bytes(4));
    if (e != hipSuccess) return e;
    return hipFuncSetAttribute((const void*)gemm_mfma_kernel<EPI, 2>, hipFuncAttributeMaxDynamicSharedMemorySize,
                               (int)gemm_smem_bytes(2));
}

dash_status init_gemm_kernels() {
    static const hipError_t err = [] {
        hipError_t e = set_gemm_lds_size<EPI_RESIDUAL_NORM>();
        if (e == hipSuccess) e = set_gemm_lds_size<EPI_STORE>();
        if (e == hipSuccess) e = set_gemm_lds_size<EPI_SWIGLU>();
        if (e == hipSuccess) e = set_gemm_lds_size<EPI_SPLITK>();
        if (e == hipSuccess) e = set_gemm_lds_size<EPI_QKV>();
        return e;
    }();
    return err == hipSuccess && compute_units() > 0 ? DASH_OK : DASH_ERR_HIP;
}

// Split-K (staging_addr.h: splitk_parts, gemm_plan): each part writes fp32 sums to scratch, and a second kernel
// adds the parts in a fixed order and applies the epilogue.
constexpr int kSplitSizingUnits = 256;  // unit count assumed when sizing the scratch (the launch uses the real one)

// Scratch bytes that let every product of up to M_cap rows with this K and N split as far as it would like to.
size_t gemm_splitk_bytes(int M_cap, int K, int N) {
    const int nt = (N + kGN - 1) / kGN, ksteps = K / kGK;
    size_t best = 0;
    for (int mt = 1; mt <= (M_cap + kGM - 1) / kGM; ++mt) {
        const int parts = splitk_parts(mt * nt, ksteps, kSplitSizingUnits);
        if (parts < 2) break;  // more row tiles only split less
        const size_t rows = (size_t)min(mt * kGM, M_cap);
        best = max(best, (size_t)parts * rows * N * sizeof(float));
    }
    return (best + 255) / 256 * 256;
}

// 256x256 tiles for every whole round over the compute units, in an order that keeps the tiles an XCD runs at one
// time close together (GemmPlan); if the tiles left over would occupy at most half of the units, they are run as
// 128-row half tiles by a second launch (same kernel, MB = 2). Products with few tiles are split along K when
// `split_ws` (device scratch of `split_bytes`) allows.
template <int EPI>
static dash_status launch_gemm(const __bf16* A, const __bf16* B, int M, int K, int N, const __bf16* x,
                               __bf16* out, float* partials, float* delta_dbg, void* split_ws, size_t split_bytes,
                               hipStream_t s, QkvOut qkv = QkvOut{nullptr, nullptr, 0, 0}) {
    // the staging loads address a tile with 32-bit lane offsets: 256 rows of A, 64 rows of B
    if ((size_t)kGM * K * 2 >= ((size_t)1 << 32) || (size_t)kGK * N * 2 + 2 * kGN >= ((size_t)1 << 32)) return DASH_ERR_UNSUPPORTED;
    if (init_gemm_kernels() != DASH_OK) return DASH_ERR_HIP;
    const GemmPlan g = gemm_plan(M, K, N, compute_units(), split_ws != nullptr && !delta_dbg, split_bytes);
    GemmLaunch L{};
    L.mt = g.mt;
    L.nt = g.nt;
    L.ksteps = g.ksteps;
    L.plain = g.plain;
    if (g.parts >= 2) {
        float* sums = reinterpret_cast<float*>(split_ws);
        L.ksteps_per_split = g.ksteps_per_part;
        hipLaunchKernelGGL((gemm_mfma_kernel<EPI_SPLITK, 4>), dim3(g.tiles, g.parts), dim3(kGThreads), gemm_smem_bytes(4), s,
                           A, B, M, K, N, nullptr, nullptr, nullptr, sums, L, qkv);
        const int cols_per_wave = EPI == EPI_SWIGLU ? 1024 : 512;
        const size_t waves = (size_t)M * ((N + cols_per_wave - 1) / cols_per_wave);
        hipLaunchKernelGGL((splitk_reduce_kernel<EPI>), dim3((unsigned)((waves * kWave + 255) / 256)), dim3(256), 0,
                           s, sums, g.parts, M, N, x, out, partials, qkv);
        return launch_status();
    }
    L.full = g.full;
    L.seg = g.seg;
    if (g.full > 0)
        hipLaunchKernelGGL((gemm_mfma_kernel<EPI, 4>), dim3(g.grid), dim3(kGThreads), gemm_smem_bytes(4), s, A, B, M, K, N, x,
                           out, partials, delta_dbg, L, qkv);
    if (g.rest > 0) {
        L.first_tile = g.full;
        hipLaunchKernelGGL((gemm_mfma_kernel<EPI, 2>), dim3(2 * g.rest), dim3(kGThreads), gemm_smem_bytes(2), s, A, B, M, K, N,
                           x, out, partials, delta_dbg, L, qkv);
    }
    return launch_status();
}

size_t wo_splitk_bytes(const dash_layer_params& p, int n) {
    if (p.dtype != DASH_BF16) return 0;
    return gemm_splitk_bytes(n, p.n_q_heads * p.head_dim, p.d);
}

dash_status launch_wo_residual_rownorm(const dash_layer_params& p, const void* o, const void* w_o,
                                       const void* x, int n, void* x_next, float* partials,
                                       float* delta_dbg, void* split_ws, size_t split_bytes, hipStream_t s) {
    if (n == 0) return DASH_OK;
    const int K = p.n_q_heads * p.head_dim, N = p.d;
    if (p.dtype == DASH_F32) {
        dim3 grid((N + kSimpleTile - 1) / kSimpleTile, (n + kSimpleTile - 1) / kSimpleTile);
        hipLaunchKernelGGL(wo_simple_kernel<float>, grid, dim3(256), 0, s, (const float*)o, (const float*)w_o,
                           (const float*)x, n, K, N, (float*)x_next, partials, delta_dbg);
        return launch_status();
    }
    return launch_gemm<EPI_RESIDUAL_NORM>((const __bf16*)o, (const __bf16*)w_o, n, K, N, (const __bf16*)x,
                                          (__bf16*)x_next, partials, delta_dbg, split_ws, split_bytes, s);
}

static size_t up256(size_t v) { return (v + 255) / 256 * 256; }

size_t ffn_workspace_bytes(const dash_layer_params& p, int n, int m) {
    return up256((size_t)n * p.d * 2) + up256((size_t)n * m * 2) +
           up256((size_t)n * norm_partials_per_row(p.d, p.dtype) * 2 * sizeof(float)) +
           max(gemm_splitk_bytes(n, p.d, 2 * m), gemm_splitk_bytes(n, m, p.d));
}

// out = x + (silu(h W_gate) * (h W_up)) W_down with h = RMSNorm(x) (Alg. 1 step 7): row norm, one GEMM over
// the interleaved gate/up weight with the gating in its epilogue, one GEMM with the residual epilogue.
dash_status launch_ffn_swiglu(const dash_layer_params& p, const void* x, const void* w_gate_up, const void* w_down,
                              int n, int m, void* x_out, void* ws, hipStream_t s) {
    if (n == 0) return DASH_OK;
    char* base = reinterpret_cast<char*>(ws);
    __bf16* h = reinterpret_cast<__bf16*>(base);
    __bf16* act = reinterpret_cast<__bf16*>(base + up256((size_t)n * p.d * 2));
    float* partials = reinterpret_cast<float*>(base + up256((size_t)n * p.d * 2) + up256((size_t)n * m * 2));
    char* split_ws = reinterpret_cast<char*>(partials) +
                     up256((size_t)n * norm_partials_per_row(p.d, p.dtype) * 2 * sizeof(float));
    const size_t split_bytes = max(gemm_splitk_bytes(n, p.d, 2 * m), gemm_splitk_bytes(n, m, p.d));
    launch_rmsnorm((const __bf16*)x, n, p.d, h, s);
    dash_status st = launch_gemm<EPI_SWIGLU>(h, (const __bf16*)w_gate_up, n, p.d, 2 * m, nullptr, act, nullptr,
                                             nullptr, split_ws, split_bytes, s);
    if (st != DASH_OK) return st;
    return launch_gemm<EPI_RESIDUAL_NORM>(act, (const __bf16*)w_down, n, m, p.d, (const __bf16*)x,
                                          (__bf16*)x_out, partials, nullptr, split_ws, split_bytes, s);
}

size_t qkv_workspace_bytes(const dash_layer_params& p, int n) {
    if (p.dtype != DASH_BF16) return 0;
    const int Dq = p.n_q_heads * p.head_dim, Dkv = p.n_kv_heads * p.head_dim;
    // the widest of the three separate projections, or the one product over the concatenated weight
    return max(gemm_splitk_bytes(n, p.d, Dq), gemm_splitk_bytes(n, p.d, Dq + 2 * Dkv));
}

dash_status launch_rmsnorm_qkv(const dash_layer_params& p, const void* x, const void* w_q, const void* w_k,
                               const void* w_v, int n, void* q, void* k, void* v, void* hbuf, void* split_ws,
                               size_t split_bytes, hipStream_t s) {
    if (n == 0) return DASH_OK;
    const int d = p.d, Dq = p.n_q_heads * p.head_dim, Dkv = p.n_kv_heads * p.head_dim;
    launch_rmsnorm((const __bf16*)x, n, d, (__bf16*)hbuf, s);
    const __bf16* h = (const __bf16*)hbuf;
    dash_status st = launch_gemm<EPI_STORE>(h, (const __bf16*)w_q, n, d, Dq, nullptr, (__bf16*)q, nullptr, nullptr,
                                            split_ws, split_bytes, s);
    if (st != DASH_OK) return st;
    st = launch_gemm<EPI_STORE>(h, (const __bf16*)w_k, n, d, Dkv, nullptr, (__bf16*)k, nullptr, nullptr, split_ws,
                                split_bytes, s);
    if (st != DASH_OK) return st;
    return launch_gemm<EPI_STORE>(h, (const __bf16*)w_v, n, d, Dkv, nullptr, (__bf16*)v, nullptr, nullptr, split_ws,
                                  split_bytes, s);
}

// The same front end as one product over w_qkv = [w_q | w_k | w_v] ([d, Dq + 2 Dkv]): one pass over the
// normalised rows instead of three, and no launches that fill a fraction of the chip for the narrow k and v.
dash_status launch_rmsnorm_qkv_fused(const dash_layer_params& p, const void* x, const void* w_qkv, int n, void* q,
                                     void* k, void* v, void* hbuf, void* split_ws, size_t split_bytes,
                                     hipStream_t s) {
    if (n == 0) return DASH_OK;
    const int d = p.d, Dq = p.n_q_heads * p.head_dim, Dkv = p.n_kv_heads * p.head_dim;
    launch_rmsnorm((const __bf16*)x, n, d, (__bf16*)hbuf, s);
    return launch_gemm<EPI_QKV>((const __bf16*)hbuf, (const __bf16*)w_qkv, n, d, Dq + 2 * Dkv, nullptr, (__bf16*)q,
                                nullptr, nullptr, split_ws, split_bytes, s, QkvOut{(__bf16*)k, (__bf16*)v, Dq, Dkv});
}

}  // namespace dash
