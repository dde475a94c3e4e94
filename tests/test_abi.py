"""The C-ABI library loads on a CPU-only machine and exports every symbol the header declares.
No compute call is made here; host-only entry points (pure arithmetic) are exercised."""
import ctypes
import os
import re

import pytest

from paper_2604_18103_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "dash.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dash_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_expected_entry_points():
    syms = declared_symbols()
    for must in ("dash_attn_layer", "dash_flash_fwd", "dash_wo_residual_rownorm", "dash_score_decide",
                 "dash_compact", "dash_score_rows", "dash_keep_count", "dash_workspace_bytes"):
        assert must in syms


def test_library_exports_every_declared_symbol():
    if not os.path.exists(B.LIB_PATH):
        pytest.fail("libdash.so is not built: run `python -m paper_2604_18103_amd.build`")
    lib = ctypes.CDLL(B.LIB_PATH)
    missing = [s for s in declared_symbols() if not hasattr(lib, s)]
    assert not missing, missing


def test_keep_count_matches_both_rules():
    assert B.keep_count(16384, 0.667) == 5455                       # Eq. 3: floor((1 - rho) T)
    for n, n_hat in ((8192, 2792), (16384, 5520), (32768, 10976), (65536, 21888), (131072, 43711)):
        assert B.keep_count(n, 0.667, 64, 32, paper_impl_rounding=True) == n_hat   # App. A, Table 5
    assert B.keep_count(50, 0.5, 64, 32, paper_impl_rounding=True) == 50
    assert B.keep_count(10, 1.0) == -1 and B.keep_count(-1, 0.5) == -1


def test_host_helpers_validate_params():
    p = B.make_params(3584, 28, 4, 128)
    assert B.workspace_bytes(p, 16384) > 16384 * 3584 * 2
    assert B.norm_partials_per_row(p) > 0
    # 4 * dh * Hq * n(n+1)/2 + 2 * n * Da * d
    n = 1000
    want = 4 * 128 * 28 * n * (n + 1) / 2 + 2 * n * 3584 * 3584
    assert B.layer_flops(p, n) == want
    bad = B.make_params(3584, 28, 5, 128)
    assert B.workspace_bytes(bad, 100) == 0 and B.layer_flops(bad, 100) == 0.0
    assert B.lib().dash_status_string(-3).decode().startswith("workspace")


def test_schedule_host_helpers_agree_with_the_oracle():
    """Host arithmetic of the schedule driver (block lengths, App. A cost, comparable multi-shot ratio: bisection)
    against the oracle's own versions (plain scan)."""
    from oracle import reference as ref
    from paper_2604_18103_amd import single_shot as SS
    d, m, L = 3584, 18944, 28
    for n in (8192, 32768):
        assert SS.block_cost(n, d, m) == ref.flops_A(n, d, m)
        one = {11: 0.667}
        assert SS.schedule_lengths(n, L, one, 64, 32) == ref.schedule_lengths(n, L, one, 64, 32)
        target = ref.schedule_flops(ref.schedule_lengths(n, L, one, 64, 32), d, m)
        for layers in ([11], [11, 19], [11, 16, 22], [11, 15, 19, 23]):
            c = SS.comparable_multi_shot_ratio(n, L, layers, target, d, m, 64, 32)
            assert c == ref.comparable_multi_shot_ratio(n, L, layers, target, d, m, 64, 32)
            shots = {l: c for l in layers}
            assert SS.schedule_lengths(n, L, shots, 64, 32) == ref.schedule_lengths(n, L, shots, 64, 32)
    with pytest.raises(ValueError):
        SS.comparable_multi_shot_ratio(1000, 4, [1], 0.0, 64, 128)


def test_workspace_sizes_grow_with_capacity_and_hold_the_split_sums():
    """Host arithmetic of the workspace sizes: monotone in the capacity, and with room for at least two fp32
    [n, N] split sums wherever a product of n rows fills at most half of 256 compute units with its tiles."""
    p = B.make_params(3584, 28, 4, 128)
    prev = (0, 0, 0)
    for n in (0, 1, 64, 177, 256, 1000, 2304, 4096, 16384, 32768):
        cur = (B.workspace_bytes(p, n), B.ffn_workspace_bytes(p, n, 18944), B.qkv_workspace_bytes(p, n))
        assert all(c >= q for c, q in zip(cur, prev)), (n, cur, prev)
        prev = cur
    # 177 rows: the projection has 14 tiles, the q/k/v product 18, the FFN down projection 14
    assert B.workspace_bytes(p, 177) >= 2 * 177 * 3584 * 4
    assert B.qkv_workspace_bytes(p, 177) >= 2 * 177 * 4608 * 4
    assert B.ffn_workspace_bytes(p, 177, 18944) >= 177 * (3584 + 18944) * 2 + 2 * 177 * 3584 * 4
    # a capacity whose tiles fill the chip needs no room for split sums
    big = B.workspace_bytes(p, 32768)
    assert big < 32768 * 3584 * 2 + 32768 * 56 * 8 + (80 << 20)
    assert B.qkv_workspace_bytes(B.make_params(3584, 28, 4, 128, dtype=B.DASH_F32), 177) == 0


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2 and "ONE GPU" in r.stderr
