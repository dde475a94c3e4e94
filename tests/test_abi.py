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


# ---------------------------------------------------------------- argument errors are found on the host, before any launch

FAKE = 0x7F0000001000          # a 256-byte aligned, non-null "device pointer": never dereferenced on the host


def _layer_args(p, n_rows, ws_size, **over):
    """Positional arguments of dash_attn_layer after params, with fake device pointers."""
    a = dict(x=FAKE, q=FAKE, k=FAKE, v=FAKE, w_o=FAKE, active_idx=FAKE, n=n_rows, x_next=FAKE, scores=FAKE, halt=FAKE,
             x_compact=FAKE, new_idx=FAKE, n_out=FAKE, delta=None, ws=FAKE, ws_bytes=ws_size, profile=None,
             stream=None)
    a.update(over)
    return [a[k] for k in ("x", "q", "k", "v", "w_o", "active_idx", "n", "x_next", "scores", "halt", "x_compact",
                           "new_idx", "n_out", "delta", "ws", "ws_bytes", "profile", "stream")]


def test_layer_call_rejects_bad_arguments_without_launching():
    """Null pointers, a negative row count, misaligned pointers, a workspace sized for fewer rows than n_active,
    invalid parameter structs: every one returns its error code from the host-side checks (this machine has no
    GPU, so anything that reached a launch would fail differently)."""
    L = B.lib()
    p = B.make_params(3584, 28, 4, 128, rule=B.RULE_THRESHOLD, tau=0.1)
    n = 1000
    ws = B.workspace_bytes(p, n)
    INVALID, UNSUPPORTED, WORKSPACE = -1, -2, -3
    call = lambda params, **over: L.dash_attn_layer(ctypes.byref(params), *_layer_args(params, n, ws, **over))
    for name in ("x", "q", "k", "v", "w_o", "active_idx", "x_next", "scores", "halt", "x_compact", "new_idx", "n_out"):
        assert call(p, **{name: None}) == INVALID, name
    assert call(p, n=-1) == INVALID
    assert L.dash_attn_layer(None, *_layer_args(p, n, ws)) == INVALID
    for name in ("x", "q", "k", "v", "w_o", "x_next", "x_compact", "delta"):
        assert call(p, **{name: FAKE + 8}) == INVALID, name               # not 16-byte aligned
    # capacity: a workspace sized for fewer rows than n_active, none at all, or one that is not 256-byte aligned
    assert call(p, ws_bytes=B.workspace_bytes(p, n - 1) - 1) == WORKSPACE
    assert call(p, ws_bytes=B.workspace_bytes(p, 10)) == WORKSPACE
    assert call(p, ws=None) == WORKSPACE
    assert call(p, ws=FAKE + 16) == WORKSPACE
    # parameter structs
    bad = lambda **kw: B.make_params(**{**dict(d=3584, n_q_heads=28, n_kv_heads=4, head_dim=128), **kw})
    assert call(bad(n_kv_heads=5)) == INVALID                     # heads do not group
    assert call(bad(head_dim=96)) == UNSUPPORTED
    assert call(bad(d=3588)) == UNSUPPORTED                       # rows are not whole 16-byte vectors
    assert call(bad(dtype=7)) == INVALID
    assert call(bad(rule=5)) == INVALID
    assert call(bad(score_kind=2)) == INVALID
    assert call(bad(keep_first_n=-1)) == INVALID
    assert call(bad(rule=B.RULE_TOPK, k_keep=-1, rho=1.0)) == INVALID
    assert call(bad(rule=B.RULE_TOPK, k_keep=-1, rho=float("nan"))) == INVALID


def test_stage_calls_reject_bad_arguments_without_launching():
    L = B.lib()
    p = B.make_params(512, 4, 2, 128, rule=B.RULE_TOPK, k_keep=10)
    pp = ctypes.byref(p)
    INVALID, UNSUPPORTED, WORKSPACE = -1, -2, -3
    n = 300
    assert L.dash_flash_fwd(pp, None, FAKE, FAKE, FAKE, n, FAKE, None) == INVALID
    assert L.dash_flash_fwd(pp, FAKE, FAKE, FAKE, FAKE, -5, FAKE, None) == INVALID
    assert L.dash_flash_fwd(pp, FAKE, FAKE + 2, FAKE, FAKE, n, FAKE, None) == INVALID
    assert L.dash_wo_residual_rownorm(pp, FAKE, FAKE, FAKE, n, None, FAKE, None, None, 0, None) == INVALID
    assert L.dash_wo_residual_rownorm(pp, FAKE, FAKE, FAKE, -1, FAKE, FAKE, None, None, 0, None) == INVALID
    # TopK needs its selection scratch: 256 + 4 * ceil(n / 64) bytes
    assert L.dash_score_decide(pp, FAKE, n, FAKE, FAKE, FAKE, None, 0, None) == WORKSPACE
    assert L.dash_score_decide(pp, FAKE, n, FAKE, FAKE, FAKE, FAKE, 256 + 4 * 5 - 1, None) == WORKSPACE
    assert L.dash_score_decide(pp, None, n, FAKE, FAKE, FAKE, FAKE, 4096, None) == INVALID
    assert L.dash_decide_topk(pp, FAKE, n, 0, FAKE, FAKE, FAKE, 256 + 4 * 5 - 1, None) == WORKSPACE
    assert L.dash_decide_topk(pp, None, n, 0, FAKE, FAKE, FAKE, 4096, None) == INVALID
    p_rho = B.make_params(512, 4, 2, 128, rule=B.RULE_NONE, k_keep=-1, rho=1.5)
    assert L.dash_decide_topk(ctypes.byref(p_rho), FAKE, n, 0, FAKE, FAKE, FAKE, 4096, None) == INVALID
    assert L.dash_compact(pp, FAKE, FAKE, FAKE, FAKE, n, FAKE, FAKE, None, None, 0, None) == INVALID
    assert L.dash_compact(pp, FAKE, None, FAKE, FAKE, n, FAKE, FAKE, FAKE, None, 0, None) == WORKSPACE
    assert L.dash_compact(pp, None, FAKE, FAKE, FAKE, n, FAKE, FAKE, FAKE, None, 0, None) == INVALID
    assert L.dash_score_rows(FAKE, FAKE, n, 12, B.DASH_BF16, B.SCORE_REL, FAKE, None) == INVALID   # d % 8
    assert L.dash_score_rows(FAKE, None, n, 512, B.DASH_BF16, B.SCORE_REL, FAKE, None) == INVALID
    assert L.dash_score_diff_rows(FAKE, FAKE, n, 12, B.DASH_BF16, B.SCORE_REL, FAKE, None) == UNSUPPORTED
    assert L.dash_scatter_rows(None, FAKE, None, 0, n, 512, B.DASH_BF16, 1000, FAKE, None) == INVALID
    assert L.dash_scatter_rows(FAKE, FAKE, None, 0, n, 512, B.DASH_BF16, -1, FAKE, None) == INVALID
    assert L.dash_rope_qk(pp, FAKE, FAKE, FAKE, n, ctypes.c_double(0.5), None) == INVALID
    assert L.dash_rope_qk(pp, FAKE, None, FAKE, n, ctypes.c_double(1e6), None) == INVALID
    assert L.dash_ffn_swiglu(pp, FAKE, FAKE, FAKE, n, 100, FAKE, FAKE, 1 << 30, None) == UNSUPPORTED  # m % 64
    assert L.dash_ffn_swiglu(pp, FAKE, FAKE, FAKE, n, 128, FAKE, FAKE, 16, None) == WORKSPACE
    assert L.dash_ffn_swiglu(pp, FAKE, FAKE, FAKE, n, 128, FAKE, None, 1 << 30, None) == INVALID
    assert L.dash_rmsnorm_qkv_fused(pp, FAKE, None, n, FAKE, FAKE, FAKE, FAKE, None, 0, None) == INVALID
    assert L.dash_validate_active_idx(FAKE, n, 1000, None, None) == INVALID


def test_keep_count_for_decimal_ratios_is_exact():
    """Eq. 3 with the ratios a caller writes as decimals: floor((1 - rho) n) from exact rational arithmetic.
    The ratio travels as a double everywhere (a float 0.4 is slightly above 0.4 and would lose a row whenever
    (1 - rho) n is an integer)."""
    from fractions import Fraction
    from oracle import reference as ref
    for rho_txt in ("0.2", "0.3", "0.4", "0.6", "0.667", "0.75"):
        for n in (10, 1000, 16384, 100000, 131072):
            want = int((1 - Fraction(rho_txt)) * n // 1)
            assert B.keep_count(n, float(rho_txt)) == want, (rho_txt, n)
            assert ref.keep_count(n, float(rho_txt)) == want, (rho_txt, n)
    p = B.make_params(512, 4, 2, 128, rho=0.4)
    assert p.rho == 0.4                                        # the struct carries the double unchanged
    assert B.keep_count_quantile(1000, 0.2) == 800 and B.keep_count_quantile(32768, 0.2) == 26215
    assert B.keep_count_quantile(7, 0.0) == 7 and B.keep_count_quantile(7, 1.0) == 0
    assert B.keep_count_quantile(-1, 0.5) == -1 and B.keep_count_quantile(5, 1.5) == -1


def test_schedule_helpers_validate_arguments():
    import ctypes as C
    L = B.lib()
    out = (C.c_int64 * 8)()
    blocks, ratios = (C.c_int32 * 2)(3, 2), (C.c_double * 2)(0.5, 0.5)
    assert L.dash_schedule_lengths(100, 8, blocks, ratios, 2, 0, 0, out) == -1       # blocks not increasing
    blocks = (C.c_int32 * 2)(2, 9)
    assert L.dash_schedule_lengths(100, 8, blocks, ratios, 2, 0, 0, out) == -1       # block outside [0, L)
    assert L.dash_schedule_lengths(100, 8, None, None, 0, 0, 0, None) == -1
    assert L.dash_schedule_lengths(100, 8, None, None, 0, 0, 0, out) == 0 and list(out) == [100] * 8
    assert B.schedule_lengths(100, 4, {1: 0.5}) == [100, 100, 50, 50]
    assert B.schedule_lengths(1000, 3, {0: 0.5}, 64, 32) == [1000, 1000 - 452, 1000 - 452]   # round(0.5 * 904)
    assert B.block_cost(10, 4, 8) == 4 * 10 * 16 + 2 * 100 * 4 + 2 * 10 * 4 * 8                # App. A, Eq. 4 by hand
    assert B.schedule_cost([10, 10, 5], 4, 8) == 2 * B.block_cost(10, 4, 8) + B.block_cost(5, 4, 8)
    assert B.block_cost(-1, 4, 8) == -1.0


def test_sizes_beyond_the_32_bit_offsets_are_reported_as_unsupported():
    """The attention kernel adds 32-bit byte offsets to a 64-bit tile base, so K may hold at most 2^31 bytes; the
    products bound their K and N the same way. One row more than fits must return "unsupported" from the host-side
    checks; the largest accepted size gets past them (and fails at the launch here, where there is no GPU)."""
    L = B.lib()
    UNSUPPORTED, HIP = -2, -4
    p = B.make_params(3584, 28, 4, 128, rule=B.RULE_THRESHOLD, tau=0.1)
    limit = 2 ** 31 // (4 * 128 * 2)                       # rows whose K bytes reach 2^31
    for n, want in ((limit - 1, HIP), (limit, UNSUPPORTED), (3 * limit, UNSUPPORTED)):
        ws = B.workspace_bytes(p, n)
        assert L.dash_attn_layer(ctypes.byref(p), *_layer_args(p, n, ws)) == want, n
        assert L.dash_flash_fwd(ctypes.byref(p), FAKE, FAKE, FAKE, FAKE, n, FAKE, None) == want, n
    # a contraction too long for the 32-bit offsets inside a 256-row operand tile: Hq * dh = 2^23
    wide = B.make_params(3584, 65536, 65536, 128)
    assert L.dash_wo_residual_rownorm(ctypes.byref(wide), FAKE, FAKE, FAKE, 1000, FAKE, FAKE, None, None, 0,
                                      None) == UNSUPPORTED
