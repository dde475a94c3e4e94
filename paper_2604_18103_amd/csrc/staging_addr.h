// Address arithmetic of the direct global->LDS staging loads of the two MFMA kernels, and the way a GEMM is
// cut into launches. Plain C++ that compiles for the host and for the device: the kernels and launchers use
// these functions, and a host program (staging_check.cpp) enumerates every load of a launch with the same
// functions and checks it against the operand sizes, so a change of the addressing is checked on the CPU
// before it runs on a GPU.
#pragma once

#include <stddef.h>
#include <stdint.h>

#if defined(__HIPCC__)
#define DASH_HD __host__ __device__ __forceinline__
#else
#define DASH_HD inline
#endif

namespace dash {

DASH_HD int sa_min(int a, int b) { return a < b ? a : b; }
DASH_HD int sa_max(int a, int b) { return a > b ? a : b; }

// ------------------------------------------------------------------------------------------------
// GEMM: workgroup tile 256 x 256, K step 64, 8 waves. A tile rows are 128 bytes (one load instruction = 8
// rows), B tile rows 512 bytes (one instruction = 2 rows). A load's address is a uniform base (the tile at the
// current K step) plus a 32-bit lane offset that never changes.
// ------------------------------------------------------------------------------------------------
constexpr int kGM = 256, kGN = 256, kGK = 64;
constexpr int kGWaves = 8;

DASH_HD constexpr int gemm_adma(int BM) { return BM / 8 / 8; }   // A load instructions per wave and K step
DASH_HD constexpr int gemm_bdma() { return kGK / 2 / 8; }         // B load instructions per wave and K step

DASH_HD int gemm_a_row(int wave, int i, int lane, int adma) { return (wave * adma + i) * 8 + lane / 8; }
DASH_HD int gemm_b_row(int wave, int i, int lane) { return (wave * gemm_bdma() + i) * 2 + lane / 32; }
// logical 16-byte chunk that lands in physical chunk lane % (chunks per row) of the row (XOR swizzle)
DASH_HD int gemm_a_lchunk(int row, int lane) { return (lane % 8) ^ ((row / 2) % 8); }
DASH_HD int gemm_b_swz(int row) { return 4 * (row % 4) + 2 * ((row / 8) % 2); }
DASH_HD int gemm_b_lchunk(int row, int lane) { return (lane % 32) ^ gemm_b_swz(row); }

// First row of the A base. The second half tile of a last row tile may lie wholly beyond M: the base is
// clamped like the rows, so every lane offset stays non-negative. Rows beyond M and columns beyond N are
// computed on valid (clamped) data and never stored.
DASH_HD int gemm_a_base_row(int m0, int M) { return sa_min(m0, M - 1); }
DASH_HD size_t gemm_a_base_elem(int m0, int M, int K, int ks0) {
    return (size_t)gemm_a_base_row(m0, M) * K + (size_t)ks0 * kGK;
}
DASH_HD uint32_t gemm_a_off(int m0, int M, int K, int row, int lchunk) {
    return (uint32_t)(((size_t)(sa_min(m0 + row, M - 1) - gemm_a_base_row(m0, M)) * K + lchunk * 8) * 2);
}
DASH_HD size_t gemm_b_base_elem(int n0, int N, int ks0) { return (size_t)ks0 * kGK * N + n0; }
DASH_HD uint32_t gemm_b_off(int n0, int N, int row, int lchunk) {
    return (uint32_t)(((size_t)row * N + (sa_min(n0 + lchunk * 8, N - 8) - n0)) * 2);
}
DASH_HD size_t gemm_a_step_bytes() { return (size_t)kGK * 2; }
DASH_HD size_t gemm_b_step_bytes(int N) { return (size_t)kGK * N * 2; }

// Split-K: a product with few output tiles and a long contraction (few active rows) leaves most compute units
// idle and the few busy ones with a long serial loop. Such a product is cut along K into parts that run side
// by side. Used when the tiles would occupy at most half of the units; a part has at least kSplitMinSteps K steps.
constexpr int kSplitMinSteps = 4;
inline int splitk_parts(int tiles, int ksteps, int cu) {
    if (cu <= 0 || 2 * tiles > cu) return 1;
    const int s = sa_min(cu / tiles, ksteps / kSplitMinSteps);
    return s < 2 ? 1 : s;
}

// Order in which the output tiles of a product are handed out ("tile index" below), and which workgroup takes which
// index. Workgroup b of a launch runs on XCD b % 8, and each XCD has its own L2: what the 32 workgroups that an XCD
// runs at one time share in that L2 is decided here.
//  - row tiles a multiple of 8 ("plain"): tile index = column-major position (row tile fastest), workgroup b takes
//    index b. An XCD then holds row tiles b % 8, b % 8 + 8, ... of four consecutive tile columns: 8 A panels and
//    4 B panels for 32 tiles, and all XCDs are in the same four tile columns at the same time.
//  - otherwise: column panels of 4 tile columns (the last one narrower), row by row inside a panel, so that 32
//    consecutive indices are a block of 8 x 4 tiles; the indices are dealt to the XCDs as 8 contiguous stretches
//    (workgroup b takes index (b % 8) * seg + b / 8), equally many per XCD. With the plain order a row-tile count
//    that is not a multiple of 8 would scatter an XCD's 32 tiles over up to 32 row panels.
constexpr int kGPanel = 4;
DASH_HD void gemm_tile_of(int idx, int mt, int nt, bool plain, int& tile_m, int& tile_n) {
    if (plain) {
        tile_m = idx % mt;
        tile_n = idx / mt;
        return;
    }
    const int per_panel = mt * kGPanel, whole = nt / kGPanel;
    const int p = idx / per_panel;
    if (p < whole) {
        const int r = idx - p * per_panel;
        tile_m = r / kGPanel;
        tile_n = p * kGPanel + r % kGPanel;
    } else {
        const int w = nt - whole * kGPanel;  // >= 1: idx < mt * nt
        const int r = idx - whole * per_panel;
        tile_m = r / w;
        tile_n = whole * kGPanel + r % w;
    }
}

// How launch_gemm cuts a product into launches: either `parts` >= 2 split-K parts over all tiles, or `full`
// 256-row tiles (a grid of `grid` workgroups: gemm_index_of) followed by `rest` tiles run as 128-row half tiles
// (when the tiles left over after the whole rounds would occupy at most half of the units).
struct GemmPlan {
    int mt, nt, tiles, ksteps;
    int parts, ksteps_per_part;  // parts >= 2: split-K launch
    int full, rest;              // otherwise
    int plain, seg, grid;        // tile order of the whole tiles, indices per XCD, workgroups of their launch
};
inline GemmPlan gemm_plan(int M, int K, int N, int cu, bool may_split, size_t split_bytes) {
    GemmPlan g{};
    g.mt = (M + kGM - 1) / kGM;
    g.nt = (N + kGN - 1) / kGN;
    g.tiles = g.mt * g.nt;
    g.ksteps = K / kGK;
    g.parts = 1;
    g.ksteps_per_part = g.ksteps;
    g.plain = g.mt % 8 == 0 ? 1 : 0;
    if (may_split) {
        int parts = splitk_parts(g.tiles, g.ksteps, cu);
        const size_t per_part = (size_t)M * N * sizeof(float);
        if ((size_t)parts * per_part > split_bytes) parts = (int)(split_bytes / per_part);
        if (parts >= 2) {
            const int per = (g.ksteps + parts - 1) / parts;
            g.parts = (g.ksteps + per - 1) / per;  // every part has at least one K step
            g.ksteps_per_part = per;
            return g;
        }
    }
    g.rest = cu > 0 ? g.tiles % cu : 0;
    if (2 * g.rest > cu) g.rest = 0;
    g.full = g.tiles - g.rest;
    g.seg = (g.full + 7) / 8;
    g.grid = g.plain ? g.full : 8 * g.seg;
    return g;
}

// Tile index that workgroup b of the whole-tile launch takes, or -1 (padding of the last stretch: the workgroup leaves).
DASH_HD int gemm_index_of(int b, int full, bool plain, int seg) {
    if (plain) return b;
    const int idx = (b % 8) * seg + b / 8;
    return (b / 8 < seg && idx < sa_min(((b % 8) + 1) * seg, full)) ? idx : -1;
}

// ------------------------------------------------------------------------------------------------
// Attention: K/V tiles of 64 keys, rows of DH bf16, unpadded, 16-byte chunks XOR-swizzled inside a row. One
// load instruction moves 1 KB = 64 / CPR rows; lane l lands in physical chunk l % CPR of row l / CPR. The four
// waves of a group fetch a tile; a load's address is a uniform tile base plus a 32-bit lane offset that is the
// same for every whole tile; in the last, partly filled tile rows beyond the end are clamped to the last row.
// ------------------------------------------------------------------------------------------------
constexpr int kFaBN = 64;  // keys per tile

DASH_HD constexpr int fa_cpr(int DH) { return DH / 8; }            // 16-byte chunks per row
DASH_HD constexpr int fa_rp(int DH) { return 256 / (DH * 2); }     // rows per 256 bytes of LDS
DASH_HD constexpr int fa_k_swz(int row, int DH) { return (row / fa_rp(DH)) % fa_cpr(DH); }
DASH_HD constexpr int fa_v_swz(int row, int DH) { return 4 * ((row / fa_rp(DH)) % (fa_cpr(DH) / 4)); }
DASH_HD constexpr int fa_rows_per_dma(int DH) { return 64 / fa_cpr(DH); }
DASH_HD constexpr int fa_dmas(int DH) { return kFaBN / fa_rows_per_dma(DH) / 4; }  // per wave and tile

// row in the tile that load i of wave gw (0..3 inside its group) fetches for this lane
DASH_HD int fa_dma_row(int gw, int i, int lane, int DH) {
    return (gw * fa_dmas(DH) + i) * fa_rows_per_dma(DH) + lane / fa_cpr(DH);
}
// lane offset inside a whole tile: row r of the tile, KV head g, the logical chunk that the swizzle maps to
// this lane's physical chunk (is_k selects the K or the V swizzle)
DASH_HD uint32_t fa_dma_voff(int r, int lane, int g, int Hkv, int DH, bool is_k) {
    const int pchunk = lane % fa_cpr(DH);
    const int lchunk = pchunk ^ (is_k ? fa_k_swz(r, DH) : fa_v_swz(r, DH));
    return (uint32_t)r * ((uint32_t)Hkv * DH * 2u) + ((uint32_t)g * DH + lchunk * 8) * 2u;
}
// the same for a tile that holds only rows_left (1..63) rows
DASH_HD uint32_t fa_dma_voff_tail(uint32_t voff, int r, int rows_left, int Hkv, int DH) {
    const int beyond = sa_max(r - (rows_left - 1), 0);  // rows past the last one
    return voff - (uint32_t)beyond * ((uint32_t)Hkv * DH * 2u);
}
DASH_HD size_t fa_tile_bytes(int Hkv, int DH) { return (size_t)kFaBN * Hkv * DH * 2; }

}  // namespace dash
