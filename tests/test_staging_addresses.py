"""CPU check of the staging addresses of the two MFMA kernels: a host library built from the same header the
kernels use (csrc/staging_addr.h) enumerates every direct global->LDS load of a launch and compares it with
the clamped row and column the lane is meant to fetch. Shapes: every GEMM and attention shape of the GPU
tests and the benches, ragged lengths around the tile edges, and seeded random ones."""
import ctypes
import os
import subprocess
import tempfile

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PKG = os.path.join(ROOT, "paper_2604_18103_amd")
CHECK_LIB = os.path.join(PKG, "libdash_staging_check.so")


def _load(path=CHECK_LIB):
    if not os.path.exists(path):
        pytest.fail("libdash_staging_check.so is not built: run `python -m paper_2604_18103_amd.build`")
    lib = ctypes.CDLL(path)
    lib.dash_check_gemm_staging.argtypes = [ctypes.c_int] * 4 + [ctypes.c_ulonglong, ctypes.POINTER(ctypes.c_longlong)]
    lib.dash_check_gemm_staging.restype = ctypes.c_int
    lib.dash_check_flash_staging.argtypes = [ctypes.c_int] * 4 + [ctypes.POINTER(ctypes.c_longlong)]
    lib.dash_check_flash_staging.restype = ctypes.c_int
    return lib


def _gemm(lib, M, K, N, cu=256, split_bytes=0):
    n = ctypes.c_longlong(0)
    st = lib.dash_check_gemm_staging(M, K, N, cu, split_bytes, ctypes.byref(n))
    return st, n.value


GEMM_SHAPES = [
    # (M, K, N): projections, gated feed-forward (N = 2 m), down projection, q/k/v as one product
    (300, 256, 1024), (300, 512, 256), (333, 256, 256), (1, 64, 64), (1, 3584, 3584), (64, 64, 8),
    (127, 128, 264), (128, 128, 264), (129, 128, 264), (255, 192, 520), (256, 192, 520), (257, 192, 520),
    (383, 64, 256), (384, 64, 256), (385, 64, 256), (511, 64, 256), (513, 64, 256),
    (8192, 3584, 3584), (16384, 3584, 3584), (16384, 3584, 4608), (10976, 3584, 4608), (10976, 18944, 3584),
    (10976, 3584, 37888), (32768, 3584, 37888), (32768, 18944, 3584), (52428, 4096, 4096), (82, 3584, 3584),
    (328, 18944, 3584), (2048, 3584, 512),
]


@pytest.mark.parametrize("M,K,N", GEMM_SHAPES)
def test_gemm_staging_loads_fetch_the_clamped_rows_and_columns(M, K, N):
    lib = _load()
    for cu in (256, 304, 64):
        for split_bytes in (0, 1 << 30):
            st, n_loads = _gemm(lib, M, K, N, cu, split_bytes)
            assert st == 0, (M, K, N, cu, split_bytes, st)
            assert n_loads > 0


def test_gemm_staging_seeded_random_shapes():
    lib = _load()
    rng = np.random.default_rng(20260418)
    for _ in range(60):
        M = int(rng.integers(1, 3000))
        K = 64 * int(rng.integers(1, 40))
        N = 8 * int(rng.integers(1, 600))
        st, _ = _gemm(lib, M, K, N, 256, int(rng.integers(0, 2)) << 30)
        assert st == 0, (M, K, N, st)


@pytest.mark.parametrize("n", [1, 2, 63, 64, 65, 127, 129, 255, 256, 257, 300, 333, 511, 513, 1000, 8192, 10976,
                               16384, 52428])
def test_flash_staging_loads_fetch_the_clamped_rows(n):
    lib = _load()
    for Hkv, DH in ((4, 128), (8, 128), (1, 64), (2, 64), (1, 128)):
        for causal in (1, 0):
            if n > 20000 and (causal == 0 or Hkv != 8):
                continue
            cnt = ctypes.c_longlong(0)
            st = lib.dash_check_flash_staging(n, Hkv, DH, causal, ctypes.byref(cnt))
            assert st == 0, (n, Hkv, DH, causal, st)
            assert cnt.value > 0


def test_checker_catches_an_unclamped_base_row():
    """The mistake is planted in a copy of the header on the CPU: with the A base row left unclamped, the second
    half tile of a 300-row product lies beyond M and its lane offsets wrap; the checker must say so."""
    src = open(os.path.join(PKG, "csrc", "staging_addr.h")).read()
    good = "DASH_HD int gemm_a_base_row(int m0, int M) { return sa_min(m0, M - 1); }"
    assert good in src
    bad = src.replace(good, "DASH_HD int gemm_a_base_row(int m0, int M) { return m0; }")
    with tempfile.TemporaryDirectory() as tmp:
        open(os.path.join(tmp, "staging_addr.h"), "w").write(bad)
        open(os.path.join(tmp, "staging_check.cpp"), "w").write(open(os.path.join(PKG, "csrc", "staging_check.cpp")).read())
        out = os.path.join(tmp, "libbad.so")
        subprocess.run(["g++", "-O1", "-std=c++17", "-fPIC", "-shared", os.path.join(tmp, "staging_check.cpp"),
                        "-o", out], check=True)
        lib = _load(out)
        st, _ = _gemm(lib, 300, 256, 1024)
        assert st != 0
        st, _ = _gemm(lib, 512, 256, 1024)      # whole tiles only: the mistake does not show
        assert st == 0


def test_gemm_launch_plan_whole_rounds_half_tiles_k_parts_and_tile_order():
    """How a product is cut into launches on 256 compute units: whole 256-row tiles for the whole rounds, the tiles
    left over as half tiles when they would fill at most half of the units, K parts when all tiles do; and which
    tile order the whole tiles take (plain when the row tiles are a multiple of 8, else column panels dealt to the
    XCDs in equal stretches, the grid padded to a multiple of 8)."""
    lib = _load()
    lib.dash_gemm_launch_plan.argtypes = [ctypes.c_int] * 4 + [ctypes.c_ulonglong, ctypes.POINTER(ctypes.c_int)]
    lib.dash_gemm_launch_plan.restype = None
    names = ("tiles", "ksteps", "parts", "per_part", "full", "rest", "plain", "grid")

    def plan(M, K, N, cu=256, split_bytes=0):
        out = (ctypes.c_int * 10)()
        lib.dash_gemm_launch_plan(M, K, N, cu, split_bytes, out)
        return dict(zip(names, out))

    # the bench's projection: 64 x 14 = 896 tiles = 3 whole rounds + 128 tiles as 256 half tiles; 64 row tiles: plain order
    assert plan(16384, 3584, 3584) == dict(tiles=896, ksteps=56, parts=1, per_part=56, full=768, rest=128, plain=1,
                                           grid=768)
    # 8192 rows: 448 tiles; the 192 left over would need more than half of the units twice over: all whole tiles
    p = plan(8192, 3584, 3584)
    assert (p["full"], p["rest"], p["plain"], p["grid"]) == (448, 0, 1, 448)
    # whole rounds only
    assert plan(32768, 3584, 3584)["rest"] == 0 and plan(32768, 3584, 37888)["rest"] == 0
    # 10976 rows (kept by the single shot): 43 row tiles -> panel order; 602 tiles = 2 rounds + 90: 512 whole tiles in
    # stretches of 64 per XCD, 90 tiles as 180 half tiles
    p = plan(10976, 3584, 3584)
    assert (p["full"], p["rest"], p["plain"], p["grid"]) == (512, 90, 0, 512)
    # 11469 rows: 45 x 14 = 630 = 2 rounds + 118; 13423 rows: 53 x 14 = 742 -> 230 left over: all whole, grid padded
    p = plan(11469, 3584, 3584)
    assert (p["full"], p["rest"], p["plain"]) == (512, 118, 0)
    p = plan(13423, 3584, 3584)
    assert (p["full"], p["rest"], p["plain"], p["grid"]) == (742, 0, 0, 744)
    # 177 rows of the down projection (K = 18944): 14 tiles on 256 units -> 18 K parts of at most 17 steps
    p = plan(177, 18944, 3584, split_bytes=1 << 30)
    assert p["tiles"] == 14 and p["parts"] == 18 and p["per_part"] == 17 and 17 * 18 >= 296
    # without scratch, or when the scratch holds one part only, no split
    assert plan(177, 18944, 3584)["parts"] == 1
    assert plan(177, 18944, 3584, split_bytes=177 * 3584 * 4)["parts"] == 1
    # a part never has fewer than 4 K steps: K = 256 (4 steps) cannot split
    assert plan(64, 256, 256, split_bytes=1 << 30)["parts"] == 1


def test_checker_catches_a_wrong_work_map():
    """A mistake planted in a copy of the header on the CPU: a stretch map that is off by one (a tile run twice,
    another never)."""
    src = open(os.path.join(PKG, "csrc", "staging_addr.h")).read()
    good = "    const int idx = (b % 8) * seg + b / 8;"
    assert good in src
    with tempfile.TemporaryDirectory() as tmp:
        open(os.path.join(tmp, "staging_addr.h"), "w").write(src.replace(good, "    const int idx = (b % 8) * seg + b / 8 + 1;"))
        open(os.path.join(tmp, "staging_check.cpp"), "w").write(open(os.path.join(PKG, "csrc", "staging_check.cpp")).read())
        out = os.path.join(tmp, "libbad.so")
        subprocess.run(["g++", "-O1", "-std=c++17", "-fPIC", "-shared", os.path.join(tmp, "staging_check.cpp"),
                        "-o", out], check=True)
        lib = _load(out)
        st, _ = _gemm(lib, 10976, 3584, 3584)          # 43 row tiles: the panel order with stretches
        assert st != 0
        st, _ = _gemm(lib, 16384, 3584, 3584)          # 64 row tiles: plain order, the mistake does not show
        assert st == 0
