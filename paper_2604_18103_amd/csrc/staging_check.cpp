// Host-side check of the staging addresses (test infrastructure, CPU only; built as its own small library).
// Enumerates the direct global->LDS loads of a GEMM or attention launch with the functions the kernels use
// (staging_addr.h), forms each address the way the hardware does (64-bit uniform base + zero-extended 32-bit
// lane offset) and compares it with the address stated from first principles: the clamped row and column of
// the operand the lane is meant to fetch. A wrapped offset, a wrong clamp or a load outside the operand fails.
#include <stdint.h>

#include <vector>

#include "staging_addr.h"

using namespace dash;

namespace {

struct Counter {
    long long loads = 0;
    int status = 0;
    void fail(int code) {
        if (status == 0) status = code;
    }
};

// one GEMM workgroup: tile (tile_m, tile_n), half (0/1, used when MB == 2), K steps ks0 .. ks0 + n_ksteps - 1
void check_gemm_workgroup(int M, int K, int N, int MB, int tile_m, int tile_n, int half, int ks0, int n_ksteps,
                          Counter& c) {
    const int BM = 64 * MB;
    const int m0 = tile_m * kGM + (MB == 4 ? 0 : half * BM), n0 = tile_n * kGN;
    const int adma = gemm_adma(BM), bdma = gemm_bdma();
    const uint64_t a_bytes = (uint64_t)M * K * 2, b_bytes = (uint64_t)K * N * 2;
    for (int wave = 0; wave < kGWaves; ++wave)
        for (int lane = 0; lane < 64; ++lane) {
            for (int i = 0; i < adma; ++i) {
                const int row = gemm_a_row(wave, i, lane, adma);
                const int lchunk = gemm_a_lchunk(row, lane);
                if (row < 0 || row >= BM || lchunk < 0 || lchunk >= 8) c.fail(1);
                const uint64_t off = gemm_a_off(m0, M, K, row, lchunk);
                for (int st = 0; st < n_ksteps; ++st) {
                    const uint64_t addr = gemm_a_base_elem(m0, M, K, ks0) * 2 + (uint64_t)st * gemm_a_step_bytes() + off;
                    const int grow = sa_min(m0 + row, M - 1);
                    const uint64_t want = ((uint64_t)grow * K + (uint64_t)(ks0 + st) * kGK + lchunk * 8) * 2;
                    if (addr != want) c.fail(2);
                    if (addr + 16 > a_bytes) c.fail(3);
                    ++c.loads;
                }
            }
            for (int i = 0; i < bdma; ++i) {
                const int row = gemm_b_row(wave, i, lane);
                const int lchunk = gemm_b_lchunk(row, lane);
                if (row < 0 || row >= kGK || lchunk < 0 || lchunk >= 32) c.fail(4);
                const uint64_t off = gemm_b_off(n0, N, row, lchunk);
                for (int st = 0; st < n_ksteps; ++st) {
                    const uint64_t addr = gemm_b_base_elem(n0, N, ks0) * 2 + (uint64_t)st * gemm_b_step_bytes(N) + off;
                    const int gcol = sa_min(n0 + lchunk * 8, N - 8);
                    const uint64_t want = ((uint64_t)((ks0 + st) * kGK + row) * N + gcol) * 2;
                    if (addr != want) c.fail(5);
                    if (addr + 16 > b_bytes) c.fail(6);
                    ++c.loads;
                }
            }
        }
}

// a tile index is checked when the launch is small, or when it is the first or last tile of its row or column range
bool sampled(int idx, int count, bool all) { return all || idx == 0 || idx == count - 1; }

}  // namespace

extern "C" {

// Checks the launches that the library makes for C[M,N] = A[M,K] B[K,N] on `cu` compute units (split_bytes > 0:
// scratch for split-K is available): that the tile order visits every tile once, that the workgroups of the
// whole-tile launch take every whole tile exactly once, equally many per XCD (workgroup b runs on XCD b % 8), and
// every staging load. Products with more than 4096 tiles have their loads checked on the first and last row and
// column tiles only (the addresses are affine in the tile indices); the coverage is always checked in full.
// Returns 0 when everything is right; *n_loads = loads checked.
int dash_check_gemm_staging(int M, int K, int N, int cu, unsigned long long split_bytes, long long* n_loads) {
    Counter c;
    if (M <= 0 || K <= 0 || K % kGK != 0 || N <= 0 || N % 8 != 0) return -1;
    const GemmPlan g = gemm_plan(M, K, N, cu, split_bytes > 0, (size_t)split_bytes);
    const bool all = g.tiles <= 4096;
    const bool plain = g.plain != 0;
    // the tile order is a bijection onto the tile grid
    {
        std::vector<char> seen((size_t)g.tiles, 0);
        for (int idx = 0; idx < g.tiles; ++idx) {
            int tm = -1, tn = -1;
            gemm_tile_of(idx, g.mt, g.nt, plain, tm, tn);
            if (tm < 0 || tm >= g.mt || tn < 0 || tn >= g.nt || seen[(size_t)tn * g.mt + tm]) {
                c.fail(9);
                break;
            }
            seen[(size_t)tn * g.mt + tm] = 1;
        }
    }
    auto loads_wanted = [&](int tm, int tn) { return sampled(tm, g.mt, all) || sampled(tn, g.nt, all); };
    if (g.parts >= 2) {
        for (int tile = 0; tile < g.tiles; ++tile) {
            int tm, tn;
            gemm_tile_of(tile, g.mt, g.nt, plain, tm, tn);
            if (!loads_wanted(tm, tn)) continue;
            for (int part = 0; part < g.parts; ++part) {
                const int ks0 = part * g.ksteps_per_part;
                const int nk = sa_min(g.ksteps_per_part, g.ksteps - ks0);
                if (nk <= 0) c.fail(7);
                check_gemm_workgroup(M, K, N, 4, tm, tn, 0, ks0, nk, c);
            }
        }
    } else {
        if (g.full + g.rest != g.tiles || g.full < 0 || g.rest < 0) c.fail(8);
        if (g.full > 0 && (g.grid < g.full || g.grid > g.full + 15)) c.fail(10);
        std::vector<int> taken((size_t)g.tiles, 0);
        int per_xcd[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        for (int b = 0; b < (g.full > 0 ? g.grid : 0); ++b) {
            const int idx = gemm_index_of(b, g.full, plain, g.seg);
            if (idx < 0) continue;
            if (idx >= g.full) {
                c.fail(11);
                continue;
            }
            ++taken[(size_t)idx];
            ++per_xcd[b % 8];
            int tm, tn;
            gemm_tile_of(idx, g.mt, g.nt, plain, tm, tn);
            if (loads_wanted(tm, tn) || idx == g.full - 1) check_gemm_workgroup(M, K, N, 4, tm, tn, 0, 0, g.ksteps, c);
        }
        for (int t = 0; t < g.full; ++t)
            if (taken[(size_t)t] != 1) c.fail(12);
        for (int x = 0; x < 8; ++x)  // no XCD has more than a stretch's worth, none is short by more than the padding
            if (per_xcd[x] > (g.full + 7) / 8 || per_xcd[x] + 8 < g.full / 8) c.fail(13);
        for (int b = 0; b < 2 * g.rest; ++b) {  // half tiles: workgroup b handles half b % 2 of tile full + b / 2
            int tm, tn;
            gemm_tile_of(g.full + b / 2, g.mt, g.nt, plain, tm, tn);
            check_gemm_workgroup(M, K, N, 2, tm, tn, b % 2, 0, g.ksteps, c);
        }
    }
    if (n_loads) *n_loads = c.loads;
    return c.status;
}

// The launch decomposition of a product as launch_gemm makes it: out[0..7] = tiles, K steps, parts (>= 2: split-K),
// K steps per part, whole 256-row tiles, tiles run as 128-row half tiles, plain tile order (1) or column panels
// dealt to the XCDs in stretches (0), workgroups of the whole-tile launch.
void dash_gemm_launch_plan(int M, int K, int N, int cu, unsigned long long split_bytes, int* out) {
    const GemmPlan g = gemm_plan(M, K, N, cu, split_bytes > 0, (size_t)split_bytes);
    out[0] = g.tiles; out[1] = g.ksteps; out[2] = g.parts; out[3] = g.ksteps_per_part; out[4] = g.full;
    out[5] = g.rest; out[6] = g.plain; out[7] = g.grid;
}

// Checks every K and V staging load of the attention launch over n rows (K, V: [n][Hkv][DH] bf16): for each
// query tile of 256 rows, the tiles of 64 keys it fetches. Returns 0 when all loads are right.
int dash_check_flash_staging(int n, int Hkv, int DH, int causal, long long* n_loads) {
    Counter c;
    if (n <= 0 || Hkv <= 0 || (DH != 64 && DH != 128)) return -1;
    const uint64_t kv_bytes = (uint64_t)n * Hkv * DH * 2;
    const int n_qtiles = (n + 255) / 256;
    const int dmas = fa_dmas(DH), cpr = fa_cpr(DH);
    // the tiles a query tile fetches are a prefix of those of the last query tile: the last two are checked
    for (int qt = n_qtiles - 1; qt >= 0 && qt >= n_qtiles - 2; --qt) {
        const int kv_end = causal ? sa_min(n, qt * 256 + 256) : n;
        const int n_tiles = (kv_end + kFaBN - 1) / kFaBN;
        for (int g = 0; g < Hkv; ++g)
            for (int is_k = 0; is_k < 2; ++is_k)
                for (int gw = 0; gw < 4; ++gw)
                    for (int lane = 0; lane < 64; ++lane)
                        for (int i = 0; i < dmas; ++i) {
                            const int r = fa_dma_row(gw, i, lane, DH);
                            if (r < 0 || r >= kFaBN) c.fail(1);
                            const uint32_t voff = fa_dma_voff(r, lane, g, Hkv, DH, is_k != 0);
                            const int swz = is_k ? fa_k_swz(r, DH) : fa_v_swz(r, DH);
                            const int lchunk = (lane % cpr) ^ swz;
                            if (lchunk < 0 || lchunk >= cpr) c.fail(2);
                            for (int t = 0; t < n_tiles; ++t) {
                                const int rows_left = n - t * kFaBN;
                                if (rows_left < 1) c.fail(3);
                                const uint32_t off = rows_left >= kFaBN ? voff : fa_dma_voff_tail(voff, r, rows_left, Hkv, DH);
                                const uint64_t addr = (uint64_t)t * fa_tile_bytes(Hkv, DH) + off;
                                const int grow = sa_min(t * kFaBN + r, n - 1);
                                const uint64_t want = ((uint64_t)grow * Hkv + g) * DH * 2 + (uint64_t)lchunk * 16;
                                if (addr != want) c.fail(4);
                                if (addr + 16 > kv_bytes) c.fail(5);
                                ++c.loads;
                            }
                        }
    }
    if (n_loads) *n_loads = c.loads;
    return c.status;
}

}  // extern "C"
