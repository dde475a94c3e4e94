"""Pins for the fp64 CPU oracle: what the paper and the mathematics fix.

None of these compares the oracle with itself: expected values come from literal
double loops written here, closed forms, exact identities, hand-worked vectors
and the numbers the paper prints (tests/golden/).
"""
import math
import os

import numpy as np
import pytest

from oracle import reference as ref

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def brute_force_attention(q, k, v, pos, causal, scale):
    """Textbook softmax attention with plain Python loops (Eq. 1's Attn, no projection)."""
    n, Hq, dh = q.shape
    Hkv = k.shape[1]
    group = Hq // Hkv
    out = np.zeros((n, Hq * dh))
    for i in range(n):
        for h in range(Hq):
            g = h // group
            vis = [j for j in range(n) if (not causal) or pos[j] <= pos[i]]
            logits = [scale * sum(q[i, h, c] * k[j, g, c] for c in range(dh)) for j in vis]
            m = max(logits)
            w = [math.exp(l - m) for l in logits]
            z = sum(w)
            for c in range(dh):
                out[i, h * dh + c] = sum(w[a] / z * v[j, g, c] for a, j in enumerate(vis))
    return out


@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("Hq,Hkv", [(1, 1), (4, 1), (4, 2)])
def test_attention_matches_brute_force(causal, Hq, Hkv):
    rng = np.random.default_rng(10 + Hq + Hkv)
    n, dh = 11, 6
    q = rng.standard_normal((n, Hq, dh))
    k = rng.standard_normal((n, Hkv, dh))
    v = rng.standard_normal((n, Hkv, dh))
    pos = np.sort(rng.choice(50, size=n, replace=False)).astype(np.int32)
    scale = 0.37
    got = ref.attention_rows(q, k, v, pos, causal=causal, scale=scale)
    want = brute_force_attention(q, k, v, pos, causal, scale)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-13)


def test_attention_default_scale_is_inverse_sqrt_head_dim():
    rng = np.random.default_rng(3)
    n, dh = 7, 16
    q, k, v = (rng.standard_normal((n, 2, dh)) for _ in range(3))
    pos = np.arange(n, dtype=np.int32)
    got = ref.attention_rows(q, k, v, pos)
    want = brute_force_attention(q, k, v, pos, True, 1.0 / math.sqrt(dh))
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-13)


def test_attention_masks_on_original_positions_not_ranks():
    # rows given in scrambled position order: visibility must follow pos, not the row index
    rng = np.random.default_rng(4)
    n, dh = 9, 4
    q, k, v = (rng.standard_normal((n, 1, dh)) for _ in range(3))
    pos = rng.permutation(n).astype(np.int32)
    got = ref.attention_rows(q, k, v, pos, causal=True, scale=0.5)
    want = brute_force_attention(q, k, v, pos, True, 0.5)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-13)
    # the row holding the smallest position sees only itself
    i0 = int(np.argmin(pos))
    np.testing.assert_allclose(got[i0], v[i0, 0], rtol=0, atol=1e-15)


def test_sorted_positions_equal_rank_mask():
    # strictly increasing original positions give the plain lower-triangular mask on ranks
    rng = np.random.default_rng(5)
    n, dh = 10, 4
    q, k, v = (rng.standard_normal((n, 2, dh)) for _ in range(3))
    pos = np.sort(rng.choice(1000, size=n, replace=False)).astype(np.int32)
    a = ref.attention_rows(q, k, v, pos)
    b = ref.attention_rows(q, k, v, np.arange(n, dtype=np.int32))
    assert np.array_equal(a, b)


def test_equal_keys_give_running_mean_of_values():
    rng = np.random.default_rng(6)
    n, dh = 13, 5
    q = rng.standard_normal((n, 3, dh))
    k = np.tile(rng.standard_normal((1, 1, dh)), (n, 1, 1))
    v = rng.standard_normal((n, 1, dh))
    got = ref.attention_rows(q, k, v, np.arange(n, dtype=np.int32))
    run_mean = np.cumsum(v[:, 0, :], axis=0) / np.arange(1, n + 1)[:, None]
    for h in range(3):
        np.testing.assert_allclose(got[:, h * dh:(h + 1) * dh], run_mean, rtol=1e-13, atol=1e-14)
    # non-causal: every row is the global mean
    got_nc = ref.attention_rows(q, k, v, np.arange(n, dtype=np.int32), causal=False)
    np.testing.assert_allclose(got_nc[:, :dh], np.tile(v[:, 0].mean(0), (n, 1)), rtol=1e-13, atol=1e-14)


def test_single_token_returns_its_value_and_matvec():
    rng = np.random.default_rng(7)
    dh, Hq, d = 4, 2, 5
    q = rng.standard_normal((1, Hq, dh))
    k = rng.standard_normal((1, 1, dh))
    v = rng.standard_normal((1, 1, dh))
    w_o = rng.standard_normal((Hq * dh, d))
    x = rng.standard_normal((1, d))
    res = ref.attn_layer(x, q, k, v, w_o, np.array([17], dtype=np.int32), tau=0.0)
    v_cat = np.concatenate([v[0, 0], v[0, 0]])
    want = np.array([sum(v_cat[a] * w_o[a, c] for a in range(Hq * dh)) for c in range(d)])
    np.testing.assert_allclose(res.delta[0], want, rtol=1e-14, atol=1e-15)


def test_softmax_is_stable_for_huge_logits():
    n, dh = 6, 2
    q = np.full((n, 1, dh), 400.0)
    k = np.zeros((n, 1, dh))
    k[:, 0, 0] = np.arange(n)  # logit grows with j: each row attends (almost) only to itself
    v = np.arange(n, dtype=np.float64).reshape(n, 1, 1) * np.ones((1, 1, dh))
    got = ref.attention_rows(q, k, v, np.arange(n, dtype=np.int32), scale=1.0)
    assert np.all(np.isfinite(got))
    np.testing.assert_allclose(got[:, 0], np.arange(n), atol=1e-12)


def test_projection_hand_example_and_orientation():
    O = np.array([[1.0, 2.0]])
    w = np.array([[1.0, 2.0, 3.0], [4.0, 5.0, 6.0]])  # [Da=2, d=3]: delta = O @ w
    np.testing.assert_array_equal(ref.project(O, w), np.array([[9.0, 12.0, 15.0]]))
    rng = np.random.default_rng(8)
    O = rng.standard_normal((5, 7))
    w = rng.standard_normal((7, 3))
    np.testing.assert_allclose(ref.project(O, w), O @ w, rtol=1e-13, atol=1e-14)


def test_residual_identity_exact():
    rng = np.random.default_rng(9)
    x = rng.integers(-1000, 1000, size=(6, 8)).astype(np.float64)
    delta = rng.integers(-1000, 1000, size=(6, 8)).astype(np.float64)
    xn = ref.residual(x, delta)
    assert np.array_equal(xn - x, delta)          # exact: integers
    x = rng.standard_normal((6, 8))
    delta = rng.standard_normal((6, 8))
    assert np.array_equal(ref.residual(x, delta), x + delta)


def test_scores_hand_values():
    delta = np.array([[3.0, 4.0], [0.0, 0.0], [1.0, 0.0]])
    x = np.array([[6.0, 8.0], [1.0, 1.0], [0.0, 0.0]])
    np.testing.assert_array_equal(ref.scores(delta, kind=ref.SCORE_ABS), [5.0, 0.0, 1.0])
    rel = ref.scores(delta, x, kind=ref.SCORE_REL)
    assert rel[0] == 0.5 and rel[1] == 0.0
    assert rel[2] == 1.0 / 1e-30       # zero input row, non-zero update: huge score, kept


def _small_layer(seed, n=24, Hq=4, Hkv=2, dh=8, d=12):
    rng = np.random.default_rng(seed)
    return dict(x=rng.standard_normal((n, d)) * np.exp(1.5 * rng.standard_normal((n, 1))),
                q=rng.standard_normal((n, Hq, dh)), k=rng.standard_normal((n, Hkv, dh)),
                v=rng.standard_normal((n, Hkv, dh)),
                w_o=rng.standard_normal((Hq * dh, d)) / math.sqrt(d),
                active_idx=np.sort(rng.choice(4 * n, size=n, replace=False)).astype(np.int32))


def test_zero_output_projection_gives_zero_scores():
    L = _small_layer(11)
    L["w_o"] = np.zeros_like(L["w_o"])
    res = ref.attn_layer(**L, tau=1e-6)
    assert np.all(res.scores == 0.0) and np.all(res.delta == 0.0)
    assert np.array_equal(res.x_next, L["x"])
    assert res.halt.all() and res.n_active_out == 0       # any tau > 0 halts every row
    res0 = ref.attn_layer(**L, tau=0.0)
    assert not res0.halt.any() and res0.n_active_out == len(L["active_idx"])  # tau = 0 never halts


def test_identity_output_projection_scores_attention_output():
    L = _small_layer(12, Hq=2, Hkv=1, dh=6, d=12)
    L["w_o"] = np.eye(12)
    res = ref.attn_layer(**L, tau=0.0)
    O = brute_force_attention(L["q"], L["k"], L["v"], L["active_idx"], True, 1 / math.sqrt(6))
    np.testing.assert_allclose(res.delta, O, rtol=1e-12, atol=1e-13)
    want = np.sqrt((O ** 2).sum(1)) / np.sqrt((L["x"] ** 2).sum(1))
    np.testing.assert_allclose(res.scores, want, rtol=1e-12)
    np.testing.assert_allclose(res.x_next, L["x"] + O, rtol=1e-12, atol=1e-13)


def test_relative_score_scales_inversely_with_row_norm():
    L = _small_layer(13)
    base_rel = ref.attn_layer(**L, tau=0.0).scores
    base_abs = ref.attn_layer(**L, tau=0.0, score_kind=ref.SCORE_ABS).scores
    L2 = dict(L)
    L2["x"] = L["x"].copy()
    L2["x"][5] *= 8.0
    rel = ref.attn_layer(**L2, tau=0.0).scores
    ab = ref.attn_layer(**L2, tau=0.0, score_kind=ref.SCORE_ABS).scores
    np.testing.assert_allclose(rel[5], base_rel[5] / 8.0, rtol=1e-14)
    assert np.array_equal(np.delete(rel, 5), np.delete(base_rel, 5))
    assert np.array_equal(ab, base_abs)


def test_row_sampled_layer_equals_full_rows():
    L = _small_layer(14)
    full = ref.attn_layer(**L, tau=0.0)
    rows = np.array([0, 3, 7, 23])
    part = ref.attn_layer(**L, tau=0.0, rows=rows)
    assert np.array_equal(part.x_next, full.x_next[rows])
    assert np.array_equal(part.scores, full.scores[rows])


# ---------------------------------------------------------------- decision (Eq. 3, Fig. 8)

def test_low_scores_halt_high_scores_stay():
    s = np.array([0.9, 0.1, 0.5, 0.05, 0.7])
    np.testing.assert_array_equal(ref.decide_threshold(s, 0.3), [0, 1, 0, 1, 0])
    np.testing.assert_array_equal(ref.decide_topk(s, 3), [0, 1, 0, 1, 0])
    np.testing.assert_array_equal(ref.decide_topk(s, 1), [0, 1, 1, 1, 1])
    np.testing.assert_array_equal(ref.decide_topk(s, 0), [1, 1, 1, 1, 1])
    np.testing.assert_array_equal(ref.decide_topk(s, 5), [0, 0, 0, 0, 0])
    np.testing.assert_array_equal(ref.decide_topk(s, 9), [0, 0, 0, 0, 0])


def test_threshold_is_strict_and_nan_is_kept():
    s = np.array([0.3, 0.29999, np.nan, 0.30001])
    np.testing.assert_array_equal(ref.decide_threshold(s, 0.3), [0, 1, 0, 0])


def test_topk_ties_keep_earlier_rows():
    s = np.array([0.5, 0.2, 0.5, 0.5, 0.9, 0.5])
    # K=3: 0.9 first, then the two earliest 0.5 rows (0 and 2)
    np.testing.assert_array_equal(ref.decide_topk(s, 3), [0, 1, 0, 1, 0, 1])


def test_topk_orders_nan_above_inf_and_ties_the_two_zeros():
    """Eq. 3 ranks real numbers; for NaN and signed zeros the reading is one total order
    -inf < ... < -0.0 = +0.0 < ... < +inf < NaN (all NaNs equal), ties by row. Expected masks written by hand."""
    inf, nan = np.inf, np.nan
    #             0     1    2     3     4    5     6     7
    s = np.array([0.0, nan, -0.0, inf, -1.0, nan, -inf, 0.0])
    # descending: NaN rows 1, 5 | +inf row 3 | zeros rows 0, 2, 7 (row order: the sign of zero does not rank) |
    # -1 row 4 | -inf row 6
    want_order = [1, 5, 3, 0, 2, 7, 4, 6]
    for K in range(9):
        want = np.ones(8, dtype=np.uint8)
        want[want_order[:K]] = 0
        np.testing.assert_array_equal(ref.decide_topk(s, K), want, err_msg=f"K={K}")
        # direction control: the lowest in the same order are kept, so NaN rows halt first
        want_low = np.ones(8, dtype=np.uint8)
        asc = [6, 4, 0, 2, 7, 3, 1, 5]
        want_low[asc[:K]] = 0
        np.testing.assert_array_equal(ref.decide_topk(s, K, keep_low=True), want_low, err_msg=f"low K={K}")
    # NaNs with different payloads and signs are one value
    weird = np.array([0x7FF8000000000001, 0xFFF8000000000000, 0x7FF0000000000001], dtype=np.uint64).view(np.float64)
    s2 = np.concatenate([[5.0], weird, [inf]])
    np.testing.assert_array_equal(ref.decide_topk(s2, 2), [1, 0, 0, 1, 1])
    np.testing.assert_array_equal(ref.decide_topk(s2, 4), [1, 0, 0, 0, 0])
    # a vector of NaNs only and of mixed zeros only: ties by row
    np.testing.assert_array_equal(ref.decide_topk(np.full(5, nan), 2), [0, 0, 1, 1, 1])
    np.testing.assert_array_equal(ref.decide_topk(np.array([-0.0, 0.0, -0.0, 0.0]), 3), [0, 0, 0, 1])
    np.testing.assert_array_equal(ref.decide_topk(np.array([-0.0, 0.0, -0.0, 0.0]), 3, keep_low=True), [0, 0, 0, 1])


def test_protected_prefix_and_suffix_never_halt():
    s = np.array([0.0, 0.0, 0.8, 0.1, 0.6, 0.2, 0.0, 0.0])
    np.testing.assert_array_equal(ref.decide_threshold(s, 0.5, 2, 1), [0, 0, 0, 1, 0, 1, 1, 0])
    # TopK: 3 protected rows count towards K=5, so two more of the unprotected are kept
    np.testing.assert_array_equal(ref.decide_topk(s, 5, 2, 1), [0, 0, 0, 1, 0, 1, 1, 0])
    # K not above the protected count: every unprotected row halts
    np.testing.assert_array_equal(ref.decide_topk(s, 2, 2, 1), [0, 0, 1, 1, 1, 1, 1, 0])
    # n <= n_first + n_last: nothing halts
    np.testing.assert_array_equal(ref.decide_threshold(s[:3], 9.0, 2, 2), [0, 0, 0])


def test_threshold_in_the_gap_equals_topk():
    rng = np.random.default_rng(15)
    s = rng.random(200)
    order = np.sort(s)[::-1]
    for K in (1, 17, 100, 199):
        tau = 0.5 * (order[K - 1] + order[K])
        assert np.array_equal(ref.decide_threshold(s, tau), ref.decide_topk(s, K))
        assert int((ref.decide_topk(s, K) == 0).sum()) == K


# ---------------------------------------------------------------- compaction (Alg. 1 step 4)

def test_compaction_is_stable_gather():
    halt = np.array([0, 1, 1, 0, 0, 1, 0], dtype=np.uint8)
    idx = np.array([2, 5, 9, 11, 30, 31, 40], dtype=np.int32)
    xn = np.arange(7 * 3, dtype=np.float64).reshape(7, 3)
    new_idx, xc, n_out = ref.compact(halt, idx, xn)
    assert n_out == 4
    np.testing.assert_array_equal(new_idx, [2, 11, 30, 40])
    np.testing.assert_array_equal(xc, xn[[0, 3, 4, 6]])
    e_idx, _, e_n = ref.compact(np.ones(7, np.uint8), idx, xn)
    assert e_n == 0 and e_idx.size == 0


def test_chain_active_set_only_shrinks_and_halted_rows_stay_frozen():
    rng = np.random.default_rng(16)
    n0, Hq, Hkv, dh, d = 40, 2, 1, 4, 8
    x = rng.standard_normal((n0, d)) * np.exp(1.5 * rng.standard_normal((n0, 1)))
    idx = np.arange(n0, dtype=np.int32)
    final = np.full((n0, d), np.nan)
    seen_halted = set()
    prev = set(idx.tolist())
    for layer in range(4):
        n = x.shape[0]
        wq, wk, wv = (rng.standard_normal((d, h * dh)) / math.sqrt(d) for h in (Hq, Hkv, Hkv))
        w_o = rng.standard_normal((Hq * dh, d)) / math.sqrt(d)
        q = (x @ wq).reshape(n, Hq, dh)
        k = (x @ wk).reshape(n, Hkv, dh)
        v = (x @ wv).reshape(n, Hkv, dh)
        res = ref.attn_layer(x, q, k, v, w_o, idx, rule=ref.RULE_TOPK, k_keep=n - n // 5)
        cur = set(res.new_active_idx.tolist())
        assert cur <= prev and res.n_active_out <= n
        halted_now = prev - cur
        assert not (halted_now & seen_halted)
        for r in np.nonzero(res.halt)[0]:
            final[idx[r]] = res.x_next[r]          # frozen at the last updated value
        seen_halted |= halted_now
        assert not (cur & seen_halted)             # a halted token never re-enters
        assert np.all(np.diff(res.new_active_idx) > 0)
        np.testing.assert_array_equal(res.x_compact, res.x_next[res.halt == 0])
        prev, x, idx = cur, res.x_compact, res.new_active_idx
    assert len(prev) < n0


# ---------------------------------------------------------------- kept length and FLOPs proxy (App. A)

def _table5():
    rows = []
    with open(os.path.join(GOLDEN, "table5_theoretical_flops.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                a = line.split()
                rows.append((int(a[0]), int(a[1]), float(a[2]), float(a[3])))
    return rows


def test_kept_length_matches_table5():
    for n, n_hat, _, _ in _table5():
        assert ref.keep_count(n, 0.667, 64, 32, paper_impl_rounding=True) == n_hat


def test_flops_ratios_match_table5():
    for n, n_hat, r_pct, s in _table5():
        r, sp = ref.flops_reduction_and_speedup(n, n_hat, d=3584, m=18944, L=28, l_s=11)
        assert abs(100.0 * r - r_pct) < 0.006          # printed to two decimals
        assert abs(sp - s) < 0.006


def test_flops_proxy_terms():
    # A(n) = 4 n d^2 + 2 n^2 d + 2 n d m: each term isolated
    assert ref.flops_A(1, 1, 0) == 4 + 2
    assert ref.flops_A(2, 3, 5) == 4 * 2 * 9 + 2 * 4 * 3 + 2 * 2 * 3 * 5


def test_eq3_keep_count_is_floor():
    assert ref.keep_count(16384, 0.667) == 5455          # differs from Table 5's 5520 by design
    assert ref.keep_count(10, 0.5) == 5
    assert ref.keep_count(7, 0.5) == 3
    assert ref.keep_count(100, 0.0) == 100
    # paper's quoted fixed active length floor((1-rho)T) in Sec. 3.4 for rho = 0.667, T = 16384
    assert ref.keep_count(16384, 0.667) == math.floor((1 - 0.667) * 16384)


def test_schedule_lengths_and_cost_reduce_to_single_shot_table5():
    """One shot at l_s = 11 of 28 blocks: 11 blocks at n, 17 at n_hat, and the cost ratio is Table 5's speedup."""
    for n, n_hat, r_pct, s in _table5():
        lengths = ref.schedule_lengths(n, 28, {11: 0.667}, 64, 32)
        assert lengths == [n] * 12 + [n_hat] * 16       # block 11 itself still runs on all n rows ...
        # ... while App. A's count charges blocks l_s..L-1 at n_hat (17 reduced blocks): its cost is the
        # schedule's with the decision taken one block earlier
        cost_app_a = ref.schedule_flops(ref.schedule_lengths(n, 28, {10: 0.667}, 64, 32), 3584, 18944)
        full = ref.schedule_flops([n] * 28, 3584, 18944)
        assert abs(full / cost_app_a - s) < 0.006
        assert abs(100.0 * (1.0 - cost_app_a / full) - r_pct) < 0.006


def test_schedule_lengths_multi_shot_by_hand():
    # 100 rows, ratio 0.5 at blocks 1 and 3, 4 + 2 protected: drop round(0.5 * 94) = 47 -> 53; then
    # drop round(0.5 * 47) = 24 (23.5 rounds half away from zero) -> 29
    assert ref.schedule_lengths(100, 5, {1: 0.5, 3: 0.5}, 4, 2) == [100, 100, 53, 53, 29]
    assert ref.schedule_lengths(100, 3, {}, 4, 2) == [100, 100, 100]
    assert ref.schedule_lengths(5, 3, {0: 0.9}, 4, 2) == [5, 5, 5]          # nothing outside the protected ranks
    assert ref.schedule_flops([2, 1], 3, 5) == ref.flops_A(2, 3, 5) + ref.flops_A(1, 3, 5)


def test_comparable_multi_shot_ratio_properties():
    n, L, d, m = 32768, 28, 3584, 18944
    single = ref.schedule_flops(ref.schedule_lengths(n, L, {11: 0.667}, 64, 32), d, m)
    # one shot at the same block: the ratio itself comes back
    assert ref.comparable_multi_shot_ratio(n, L, [11], single, d, m, 64, 32) == 0.667
    for layers in ([11, 19], [11, 16, 22], [11, 15, 19, 23]):
        c = ref.comparable_multi_shot_ratio(n, L, layers, single, d, m, 64, 32)
        lengths = ref.schedule_lengths(n, L, {l: c for l in layers}, 64, 32)
        assert ref.schedule_flops(lengths, d, m) <= single
        less = ref.schedule_lengths(n, L, {l: c - 1e-4 for l in layers}, 64, 32)
        assert ref.schedule_flops(less, d, m) > single                       # the smallest ratio on the grid
        assert 0.0 < c < 0.667                                               # each shot prunes less than the one shot
        assert lengths[-1] < 10976                                           # ... but ends shorter (n_hat of one shot)
        assert all(a >= b for a, b in zip(lengths, lengths[1:]))


# ---------------------------------------------------------------- chain front end (LN of Eq. 1)

def test_rmsnorm_closed_forms():
    eps = 1e-6
    x = np.array([[3.0, 4.0], [2.0, 2.0], [0.0, 0.0], [-5.0, 0.0]])
    got = ref.rmsnorm(x, eps)
    np.testing.assert_allclose(got[0], np.array([3.0, 4.0]) / math.sqrt(12.5 + eps), rtol=1e-15)
    np.testing.assert_allclose(got[1], np.array([2.0, 2.0]) / math.sqrt(4.0 + eps), rtol=1e-15)
    assert np.all(got[2] == 0.0)
    np.testing.assert_allclose(got[3], np.array([-5.0, 0.0]) / math.sqrt(12.5 + eps), rtol=1e-15)
    # unit RMS (up to eps) and scale invariance for rows far above eps
    rng = np.random.default_rng(20)
    y = rng.standard_normal((5, 64)) * 30.0
    h = ref.rmsnorm(y, eps)
    np.testing.assert_allclose(np.sqrt((h ** 2).mean(1)), 1.0, rtol=1e-8)
    np.testing.assert_allclose(ref.rmsnorm(7.0 * y, eps), h, rtol=1e-8)


def test_rmsnorm_qkv_is_norm_then_products():
    rng = np.random.default_rng(21)
    n, d, Hq, Hkv, dh = 6, 10, 4, 2, 3
    x = rng.standard_normal((n, d))
    wq, wk, wv = rng.standard_normal((d, Hq * dh)), rng.standard_normal((d, Hkv * dh)), rng.standard_normal((d, Hkv * dh))
    q, k, v = ref.rmsnorm_qkv(x, wq, wk, wv, Hq, Hkv, dh)
    h = x / np.sqrt((x ** 2).mean(1, keepdims=True) + 1e-6)
    np.testing.assert_allclose(q.reshape(n, -1), h @ wq, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(k.reshape(n, -1), h @ wk, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(v.reshape(n, -1), h @ wv, rtol=1e-12, atol=1e-13)
    assert q.shape == (n, Hq, dh) and k.shape == (n, Hkv, dh)


# ---------------------------------------------------------------- rotary embedding of the front end

def test_rope_is_a_rotation_by_position_times_frequency():
    """Each (i, i + dh/2) pair, read as a complex number, is multiplied by exp(j * pos * theta^(-2i/dh))."""
    rng = np.random.default_rng(30)
    m, heads, dh, theta = 7, 3, 8, 10000.0
    u = rng.standard_normal((m, heads, dh))
    pos = np.array([0, 1, 2, 5, 17, 1000, 131071], dtype=np.int32)
    got = ref.rope(u, pos, theta)
    z = u[..., : dh // 2] + 1j * u[..., dh // 2:]
    freq = theta ** (-np.arange(dh // 2) * 2.0 / dh)
    zr = z * np.exp(1j * pos[:, None, None].astype(np.float64) * freq[None, None, :])
    np.testing.assert_allclose(got[..., : dh // 2], zr.real, rtol=1e-9, atol=1e-9)
    np.testing.assert_allclose(got[..., dh // 2:], zr.imag, rtol=1e-9, atol=1e-9)
    # position 0 leaves the vector alone; every position preserves the norm of every head vector
    np.testing.assert_array_equal(got[0], u[0])
    np.testing.assert_allclose(np.linalg.norm(got, axis=-1), np.linalg.norm(u, axis=-1), rtol=1e-12)


def test_rope_hand_values():
    # dh = 2: a single frequency 1, so position p rotates (a, b) by p radians
    u = np.array([[[1.0, 0.0]], [[0.0, 2.0]], [[3.0, 4.0]]])
    pos = np.array([1, 2, 3], dtype=np.int32)
    got = ref.rope(u, pos, 10000.0)
    np.testing.assert_allclose(got[0, 0], [math.cos(1.0), math.sin(1.0)], rtol=1e-15)
    np.testing.assert_allclose(got[1, 0], [-2.0 * math.sin(2.0), 2.0 * math.cos(2.0)], rtol=1e-15)
    np.testing.assert_allclose(got[2, 0], [3 * math.cos(3.0) - 4 * math.sin(3.0), 3 * math.sin(3.0) + 4 * math.cos(3.0)],
                               rtol=1e-15)
    # dh = 4, theta = 100: frequencies 1 and 100^(-1/2) = 0.1; pairs are (0, 2) and (1, 3)
    u4 = np.array([[[1.0, 1.0, 0.0, 0.0]]])
    got4 = ref.rope(u4, np.array([10], dtype=np.int32), 100.0)
    np.testing.assert_allclose(got4[0, 0], [math.cos(10.0), math.cos(1.0), math.sin(10.0), math.sin(1.0)], rtol=1e-12)


def test_rope_scores_depend_on_relative_position_only():
    """The reason it must be fed original positions: q.k after rotation depends on pos_q - pos_k alone, so a
    compacted sequence scored with compacted ranks would see different attention logits."""
    rng = np.random.default_rng(31)
    dh, theta = 16, 1.0e6
    q = rng.standard_normal((1, 1, dh)); k = rng.standard_normal((1, 1, dh))
    def dot(pq, pk):
        return float((ref.rope(q, np.array([pq], dtype=np.int32), theta) *
                      ref.rope(k, np.array([pk], dtype=np.int32), theta)).sum())
    np.testing.assert_allclose(dot(100, 40), dot(5060, 5000), rtol=1e-9, atol=1e-9)
    np.testing.assert_allclose(dot(7, 7), float((q * k).sum()), rtol=1e-12)
    assert abs(dot(100, 40) - dot(100, 41)) > 1e-6      # and it does depend on the difference


def test_rmsnorm_qkv_with_rope_rotates_q_and_k_only():
    rng = np.random.default_rng(32)
    n, d, Hq, Hkv, dh = 5, 12, 4, 2, 6
    x = rng.standard_normal((n, d))
    wq, wk, wv = rng.standard_normal((d, Hq * dh)), rng.standard_normal((d, Hkv * dh)), rng.standard_normal((d, Hkv * dh))
    pos = np.array([0, 3, 4, 90, 91], dtype=np.int32)
    q0, k0, v0 = ref.rmsnorm_qkv(x, wq, wk, wv, Hq, Hkv, dh)
    q1, k1, v1 = ref.rmsnorm_qkv(x, wq, wk, wv, Hq, Hkv, dh, pos=pos, rope_theta=5.0e5)
    np.testing.assert_array_equal(v1, v0)
    np.testing.assert_allclose(q1, ref.rope(q0, pos, 5.0e5), rtol=1e-15)
    np.testing.assert_allclose(k1, ref.rope(k0, pos, 5.0e5), rtol=1e-15)
    np.testing.assert_array_equal(q1[0], q0[0])          # position 0
    assert np.abs(q1[1] - q0[1]).max() > 1e-3


# ---------------------------------------------------------------- second half of a block (Alg. 1 step 7)

def test_ffn_swiglu_scalar_closed_form_and_silu_values():
    # d = m = 1: LN(x) = x / sqrt(x^2 + eps) = sign(x) (eps -> 0), so out = x + silu(s wg) * (s wu) * wd
    for x0, wg, wu, wd in ((2.0, 1.0, 3.0, 0.5), (-4.0, 2.0, -1.0, 2.0), (1.0, 0.0, 5.0, 7.0)):
        got = ref.ffn_swiglu(np.array([[x0]]), np.array([[wg]]), np.array([[wu]]), np.array([[wd]]), eps=0.0)
        s = math.copysign(1.0, x0)
        g = s * wg
        want = x0 + g / (1.0 + math.exp(-g)) * (s * wu) * wd
        assert abs(got[0, 0] - want) <= 1e-15 * max(1.0, abs(want))
    # silu through the function: h = [1] (x = 1, eps = 0), w_up = 1, w_down = 1  ->  out - x = silu(w_gate)
    def silu_via(z):
        return ref.ffn_swiglu(np.array([[1.0]]), np.array([[z]]), np.array([[1.0]]), np.array([[1.0]]), eps=0.0)[0, 0] - 1.0
    assert silu_via(0.0) == 0.0
    assert abs(silu_via(1.0) - 1.0 / (1.0 + math.exp(-1.0))) < 1e-15
    assert abs(silu_via(40.0) - 40.0) < 1e-12 and abs(silu_via(-40.0)) < 1e-12
    assert abs(silu_via(-1.2784645427610738) - (-0.27846454276107374)) < 1e-12     # the minimum of silu


def test_ffn_swiglu_identities():
    rng = np.random.default_rng(41)
    rows, d, m = 6, 10, 14
    x = rng.standard_normal((rows, d)) * 3.0
    wg, wu, wd = rng.standard_normal((d, m)), rng.standard_normal((d, m)), rng.standard_normal((m, d))
    base = ref.ffn_swiglu(x, wg, wu, wd)
    # W_down = 0 or W_up = 0: the block is the identity
    np.testing.assert_array_equal(ref.ffn_swiglu(x, wg, wu, np.zeros_like(wd)), x)
    np.testing.assert_allclose(ref.ffn_swiglu(x, wg, np.zeros_like(wu), wd), x, atol=1e-15)
    # linear in W_up and in W_down
    np.testing.assert_allclose(ref.ffn_swiglu(x, wg, 2.0 * wu, wd) - x, 2.0 * (base - x), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(ref.ffn_swiglu(x, wg, wu, -3.0 * wd) - x, -3.0 * (base - x), rtol=1e-12, atol=1e-12)
    # the update does not see the scale of the row (LN), the residual does
    np.testing.assert_allclose(ref.ffn_swiglu(5.0 * x, wg, wu, wd) - 5.0 * x, base - x, rtol=1e-6, atol=1e-9)
    # built from the other oracle pieces and numpy: LN, two products, gate, product, add
    h = ref.rmsnorm(x)
    g, u = h @ wg, h @ wu
    np.testing.assert_allclose(base, x + (g / (1.0 + np.exp(-g)) * u) @ wd, rtol=1e-12, atol=1e-12)
    # rows are independent
    np.testing.assert_array_equal(ref.ffn_swiglu(x[2:3], wg, wu, wd), base[2:3])


def test_scatter_rows_writes_selected_rows_at_original_positions():
    rows = np.arange(12.0).reshape(4, 3)
    idx = np.array([1, 4, 5, 9], dtype=np.int32)
    full = -np.ones((10, 3))
    out = ref.scatter_rows(rows, idx, full)
    for t, p in enumerate(idx):
        np.testing.assert_array_equal(out[p], rows[t])
    untouched = np.setdiff1d(np.arange(10), idx)
    assert np.all(out[untouched] == -1.0) and np.all(full == -1.0)       # the input buffer is not modified
    halt = np.array([0, 1, 1, 0], dtype=np.uint8)
    out1 = ref.scatter_rows(rows, idx, full, sel=halt, sel_value=1)
    np.testing.assert_array_equal(out1[4], rows[1]); np.testing.assert_array_equal(out1[5], rows[2])
    assert np.all(out1[1] == -1.0) and np.all(out1[9] == -1.0)
    out0 = ref.scatter_rows(rows, idx, out1, sel=halt, sel_value=0)      # the survivors, later
    assert np.array_equal(out0[[1, 4, 5, 9]], rows)
    with pytest.raises(Exception):
        ref.scatter_rows(rows, np.array([1, 4, 5, 10], dtype=np.int32), full)


# ---------------------------------------------------------------- signal and direction variants (Sec. 5.4)

def test_topk_keep_low_hand_vectors_and_complement():
    s = np.array([0.5, 0.1, 0.9, 0.1, 0.7, 0.3])
    # keep the 3 lowest: 0.1 (row 1), 0.1 (row 3), 0.3 (row 5)
    np.testing.assert_array_equal(ref.decide_topk(s, 3, keep_low=True), [1, 0, 1, 0, 1, 0])
    # ties: the earlier row is kept first
    np.testing.assert_array_equal(ref.decide_topk(s, 1, keep_low=True), [1, 0, 1, 1, 1, 1])
    # protected rows count towards the budget and never halt
    np.testing.assert_array_equal(ref.decide_topk(s, 3, keep_first_n=1, keep_last_n=1, keep_low=True), [0, 0, 1, 1, 1, 0])
    np.testing.assert_array_equal(ref.decide_topk(s, 0, keep_low=True), [1] * 6)
    np.testing.assert_array_equal(ref.decide_topk(s, 6, keep_low=True), [0] * 6)
    # without ties: the rows kept when keeping the K lowest are exactly the rows halted when keeping the n-K highest
    rng = np.random.default_rng(80)
    r = rng.permutation(200).astype(np.float64)
    for K in (0, 1, 57, 199, 200):
        low = ref.decide_topk(r, K, keep_low=True)
        high = ref.decide_topk(r, 200 - K)
        np.testing.assert_array_equal(low, 1 - high)
    # negating the scores turns one rule into the other (no ties here)
    np.testing.assert_array_equal(ref.decide_topk(-r, 57, keep_low=True), ref.decide_topk(r, 57))


def test_score_block_is_eq2_on_the_block_change():
    rng = np.random.default_rng(81)
    a, b = rng.standard_normal((5, 7)), rng.standard_normal((5, 7))
    np.testing.assert_allclose(ref.score_block(b, a, ref.SCORE_ABS), np.linalg.norm(b - a, axis=1), rtol=1e-14)
    np.testing.assert_allclose(ref.score_block(b, a), np.linalg.norm(b - a, axis=1) / np.linalg.norm(a, axis=1), rtol=1e-14)
    assert np.all(ref.score_block(a, a) == 0.0)
    # a block that only adds the attention output has block signal == attention signal
    u = rng.standard_normal((5, 7))
    np.testing.assert_allclose(ref.score_block(a + u, a), ref.scores(u, a), rtol=1e-12)
