"""Second half of a block (gated feed-forward), scatter of halted rows, and the single-shot schedule of Alg. 1."""
import numpy as np
import pytest
import torch

from oracle import reference as ref
from paper_2604_18103_amd import binding as B
from paper_2604_18103_amd import inputs as I
from paper_2604_18103_amd import single_shot as SS

import parity_util as P

pytestmark = pytest.mark.gpu


def _dev(a):
    return B.to_device(a, B.DASH_BF16)


def _f(t):
    return t.float().cpu().numpy()


@pytest.mark.parametrize("shape", [(300, 256, 512), (517, 512, 1408), (64, 128, 64)], ids=lambda t: "n%d_d%d_m%d" % t)
def test_ffn_swiglu_matches_oracle(shape):
    n, d, m = shape
    cfg = I.LayerConfig("ffn", "bf16", n, n, d, 4, 2, 64, 0.3, seed=50 + n)
    x = I.make_hidden(cfg)
    W = I.make_ffn_weights(cfg, 0, m)
    p = P.params_for(cfg)
    wgu = B.interleave_gate_up(_dev(W["w_gate"]), _dev(W["w_up"]))
    out = torch.empty((n, d), dtype=torch.bfloat16, device="cuda")
    ws = torch.empty((B.ffn_workspace_bytes(p, n, m),), dtype=torch.uint8, device="cuda")
    gx = _dev(x)
    B.dash_ffn_swiglu(p, gx, wgu, _dev(W["w_down"]), n, m, out, ws)
    torch.cuda.synchronize()
    want = ref.ffn_swiglu(x, W["w_gate"], W["w_up"], W["w_down"])
    err = P.row_rel_err(_f(out), want)
    assert err.max() <= P.X_TOL["bf16"], err.max()
    # the update itself, not only the residual it rides on
    upd_err = np.abs((_f(out) - x) - (want - x)).max(axis=1) / np.maximum(np.abs(want).max(axis=1), 1e-30)
    assert upd_err.max() <= P.X_TOL["bf16"]
    assert np.abs(want - x).max() > 1e-2            # the FFN contributes at this scale
    # in place
    B.dash_ffn_swiglu(p, gx, wgu, _dev(W["w_down"]), n, m, gx, ws)
    torch.cuda.synchronize()
    assert torch.equal(gx, out)


# ---------------------------------------------------------------- few active rows: products split along K

@pytest.mark.parametrize("shape", [(177, 56, 64, 3584), (64, 9, 64, 256), (300, 8, 128, 512), (1, 16, 64, 128)],
                         ids=lambda t: "n%d_hq%d_dh%d_d%d" % t)
def test_projection_split_along_k_matches_oracle_and_one_pass(shape):
    """With scratch the output projection of a short active sequence is cut along the contraction (here 14, 2,
    4 and 4 parts, the last part shorter where K steps do not divide evenly): x_next and the row sums of squares
    against the oracle, and against the one-pass product of the same library (no scratch)."""
    n, hq, dh, d = shape
    K = hq * dh
    rng = np.random.default_rng(200 + n)
    o = I.round_to_bf16(rng.standard_normal((n, K)))
    w = I.round_to_bf16(rng.standard_normal((K, d)) / np.sqrt(K))
    x = I.round_to_bf16(rng.standard_normal((n, d)) * np.exp(0.5 * rng.standard_normal((n, 1))))
    p = B.make_params(d, hq, hq, dh)
    P_ = B.norm_partials_per_row(p)
    ws = torch.empty((B.workspace_bytes(p, n),), dtype=torch.uint8, device="cuda")
    assert ws.numel() >= 2 * n * d * 4                   # room for at least two parts
    delta = ref.project(o, w)
    want = ref.residual(x, delta)
    got = {}
    for name, scratch in (("split", ws), ("one_pass", None)):
        xn = torch.empty((n, d), dtype=torch.bfloat16, device="cuda")
        parts = torch.full((P_, n, 2), float("nan"), dtype=torch.float32, device="cuda")
        B.dash_wo_residual_rownorm(p, _dev(o), _dev(w), _dev(x), n, xn, parts, None, scratch)
        torch.cuda.synchronize()
        sums = parts.double().sum(dim=0).cpu().numpy()   # every partial slot written (no NaN left)
        assert P.row_rel_err(_f(xn), want).max() <= P.X_TOL["bf16"]
        np.testing.assert_allclose(sums[:, 0], (delta ** 2).sum(axis=1), rtol=1e-4)
        np.testing.assert_allclose(sums[:, 1], (x ** 2).sum(axis=1), rtol=1e-5)
        got[name] = (_f(xn), sums)
    # the two differ only in the order of fp32 additions: at most one bf16 step of the result, plus the fp32
    # difference itself where x and delta cancel
    a, b = got["split"][0], got["one_pass"][0]
    assert np.all(np.abs(a - b) <= 2.0 ** -7 * np.maximum(np.abs(a), np.abs(b)) + 1e-4 * (np.abs(x) + np.abs(delta)))
    np.testing.assert_allclose(got["split"][1], got["one_pass"][1], rtol=1e-5)


@pytest.mark.parametrize("shape", [(150, 512, 576), (40, 1024, 2048)], ids=lambda t: "n%d_d%d_m%d" % t)
def test_ffn_and_front_end_with_few_rows_split_along_k(shape):
    """Short sequences through the feed-forward (both products split: K = d and K = m, m / 64 odd in the first
    case) and the q/k/v projections with scratch, against the oracle."""
    n, d, m = shape
    cfg = I.LayerConfig("ffn_small", "bf16", n, n, d, 8, 2, 64, 0.3, seed=300 + n)
    x = I.make_hidden(cfg)
    W = I.make_ffn_weights(cfg, 0, m)
    p = P.params_for(cfg)
    out = torch.empty((n, d), dtype=torch.bfloat16, device="cuda")
    ws = torch.empty((B.ffn_workspace_bytes(p, n, m),), dtype=torch.uint8, device="cuda")
    B.dash_ffn_swiglu(p, _dev(x), B.interleave_gate_up(_dev(W["w_gate"]), _dev(W["w_up"])), _dev(W["w_down"]), n, m,
                      out, ws)
    torch.cuda.synchronize()
    want = ref.ffn_swiglu(x, W["w_gate"], W["w_up"], W["w_down"])
    assert P.row_rel_err(_f(out), want).max() <= P.X_TOL["bf16"]
    upd_err = np.abs((_f(out) - x) - (want - x)).max(axis=1) / np.maximum(np.abs(want).max(axis=1), 1e-30)
    assert upd_err.max() <= P.X_TOL["bf16"]
    Wp = I.make_projection_weights(cfg, 0)
    q = torch.empty((n, cfg.n_q_heads, cfg.head_dim), dtype=torch.bfloat16, device="cuda")
    k = torch.empty((n, cfg.n_kv_heads, cfg.head_dim), dtype=torch.bfloat16, device="cuda")
    v = torch.empty_like(k)
    h = torch.empty((n, d), dtype=torch.bfloat16, device="cuda")
    qws = torch.empty((B.qkv_workspace_bytes(p, n),), dtype=torch.uint8, device="cuda")
    assert qws.numel() >= 2 * n * cfg.n_q_heads * cfg.head_dim * 4
    B.dash_rmsnorm_qkv(p, _dev(x), _dev(Wp["w_q"]), _dev(Wp["w_k"]), _dev(Wp["w_v"]), n, q, k, v, h, qws)
    torch.cuda.synchronize()
    oq, ok, ov = ref.rmsnorm_qkv(x, Wp["w_q"], Wp["w_k"], Wp["w_v"], cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim)
    for got, want_ in ((q, oq), (k, ok), (v, ov)):
        assert P.row_rel_err(_f(got).reshape(n, -1), want_.reshape(n, -1)).max() <= 2e-2


def test_seeded_random_shapes_of_the_products_against_oracle():
    """Sixteen seeded draws of (rows, hidden, heads, head_dim, FFN width) around the tile, half-tile and split
    boundaries: the front end as three products and as one, the projection with residual and row sums, and the
    feed-forward, each with scratch for splitting along K, against the oracle."""
    rng = np.random.default_rng(7)
    for case in range(16):
        n = int(rng.choice([1, 2, 31, 64, 65, 127, 128, 129, 177, 255, 256, 257, 300, 511, 513, 700]))
        dh = int(rng.choice([64, 128]))
        hkv = int(rng.choice([1, 2, 4]))
        hq = hkv * int(rng.choice([1, 2, 4]))
        d = int(rng.choice([128, 256, 512, 1024, 1536]))
        m = int(rng.choice([64, 192, 576, 1024]))
        what = dict(case=case, n=n, d=d, hq=hq, hkv=hkv, dh=dh, m=m)
        cfg = I.LayerConfig("rnd", "bf16", n, n, d, hq, hkv, dh, 0.3, seed=1000 + case)
        x = I.make_hidden(cfg)
        Wp = I.make_projection_weights(cfg, 0)
        Wf = I.make_ffn_weights(cfg, 0, m)
        p = P.params_for(cfg)
        q = torch.empty((n, hq, dh), dtype=torch.bfloat16, device="cuda")
        k = torch.empty((n, hkv, dh), dtype=torch.bfloat16, device="cuda")
        v = torch.empty_like(k)
        h = torch.empty((n, d), dtype=torch.bfloat16, device="cuda")
        ws = torch.empty((max(B.qkv_workspace_bytes(p, n), 256),), dtype=torch.uint8, device="cuda")
        oq, ok, ov = ref.rmsnorm_qkv(x, Wp["w_q"], Wp["w_k"], Wp["w_v"], hq, hkv, dh)
        for one_product in (False, True):
            for t in (q, k, v):
                t.fill_(float("nan"))
            if one_product:
                B.dash_rmsnorm_qkv_fused(p, _dev(x), B.concat_qkv(_dev(Wp["w_q"]), _dev(Wp["w_k"]), _dev(Wp["w_v"])), n,
                                         q, k, v, h, ws)
            else:
                B.dash_rmsnorm_qkv(p, _dev(x), _dev(Wp["w_q"]), _dev(Wp["w_k"]), _dev(Wp["w_v"]), n, q, k, v, h, ws)
            torch.cuda.synchronize()
            for got, want in ((q, oq), (k, ok), (v, ov)):
                assert P.row_rel_err(_f(got).reshape(n, -1), want.reshape(n, -1)).max() <= 2e-2, what
        o = I.round_to_bf16(rng.standard_normal((n, hq * dh)))
        wsl = torch.empty((B.workspace_bytes(p, n),), dtype=torch.uint8, device="cuda")
        xn = torch.empty((n, d), dtype=torch.bfloat16, device="cuda")
        parts = torch.full((B.norm_partials_per_row(p), n, 2), float("nan"), dtype=torch.float32, device="cuda")
        B.dash_wo_residual_rownorm(p, _dev(o), _dev(Wp["w_o"]), _dev(x), n, xn, parts, None, wsl)
        torch.cuda.synchronize()
        delta = ref.project(o, Wp["w_o"])
        assert P.row_rel_err(_f(xn), ref.residual(x, delta)).max() <= P.X_TOL["bf16"], what
        sums = parts.double().sum(dim=0).cpu().numpy()
        np.testing.assert_allclose(sums[:, 0], (delta ** 2).sum(axis=1), rtol=2e-4, err_msg=str(what))
        np.testing.assert_allclose(sums[:, 1], (x ** 2).sum(axis=1), rtol=1e-5, err_msg=str(what))
        out = torch.empty((n, d), dtype=torch.bfloat16, device="cuda")
        wsf = torch.empty((B.ffn_workspace_bytes(p, n, m),), dtype=torch.uint8, device="cuda")
        B.dash_ffn_swiglu(p, _dev(x), B.interleave_gate_up(_dev(Wf["w_gate"]), _dev(Wf["w_up"])), _dev(Wf["w_down"]), n,
                          m, out, wsf)
        torch.cuda.synchronize()
        want = ref.ffn_swiglu(x, Wf["w_gate"], Wf["w_up"], Wf["w_down"])
        assert P.row_rel_err(_f(out), want).max() <= P.X_TOL["bf16"], what


def test_scatter_rows_matches_oracle():
    n, d, N = 333, 256, 1000
    rng = np.random.default_rng(60)
    rows = I.round_to_bf16(rng.standard_normal((n, d)))
    idx = np.sort(rng.choice(N, size=n, replace=False)).astype(np.int32)
    sel = (rng.random(n) < 0.4).astype(np.uint8)
    full0 = I.round_to_bf16(rng.standard_normal((N, d)))
    g_full = _dev(full0)
    B.dash_scatter_rows(_dev(rows), torch.from_numpy(idx).cuda(), torch.from_numpy(sel).cuda(), 1, n, d, B.DASH_BF16,
                        N, g_full)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(_f(g_full), ref.scatter_rows(rows, idx, full0, sel=sel, sel_value=1))
    B.dash_scatter_rows(_dev(rows), torch.from_numpy(idx).cuda(), None, 0, n, d, B.DASH_BF16, N, g_full)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(_f(g_full), ref.scatter_rows(rows, idx, full0))
    # positions outside the buffer are skipped, nothing else is touched
    bad = idx.copy(); bad[5] = N + 3; bad[6] = -1
    g2 = _dev(full0)
    B.dash_scatter_rows(_dev(rows), torch.from_numpy(bad).cuda(), None, 0, n, d, B.DASH_BF16, N, g2)
    torch.cuda.synchronize()
    keep = np.ones(n, dtype=np.uint8); keep[5] = keep[6] = 0
    np.testing.assert_array_equal(_f(g2), ref.scatter_rows(rows, np.where(keep == 1, bad, 0).astype(np.int32), full0,
                                                           sel=keep, sel_value=1))


def test_single_shot_schedule_teacher_forced_against_oracle():
    """Alg. 1 on four blocks with the decision at l_s = 1 (App. A's protected prefix/suffix and rounding):
    every block is checked against the oracle run on the block's actual GPU input; the decision against the
    oracle's TopK; the full-length result against the states the rows had when they stopped."""
    N, d, m, L, l_s, theta = 700, 256, 512, 4, 1, 1.0e6
    cfg = I.LayerConfig("blocks", "bf16", N, N, d, 4, 2, 64, 0.667, seed=70)
    Wnp = []
    for l in range(L):
        w = I.make_projection_weights(cfg, l)
        w.update(I.make_ffn_weights(cfg, l, m))
        Wnp.append(w)
    Wdev = []
    for w in Wnp:
        dw = {k: _dev(w[k]) for k in ("w_q", "w_k", "w_v", "w_o", "w_down")}
        dw["w_gate_up"] = B.interleave_gate_up(_dev(w["w_gate"]), _dev(w["w_up"]))
        Wdev.append(dw)
    st = SS.alloc_blocks(d, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, m, N)
    st.params.keep_first_n, st.params.keep_last_n = 64, 32
    k_keep = B.keep_count(N, 0.667, 64, 32, paper_impl_rounding=True)
    assert k_keep == N - round(0.667 * (N - 96))
    x0 = I.make_hidden(cfg)
    seen = {}

    def check(l, x_in, idx, n, st_, x_out):
        xs, idx_np = _f(x_in[:n]), idx[:n].cpu().numpy()
        W = Wnp[l]
        oq, ok, ov = ref.rmsnorm_qkv(xs, W["w_q"], W["w_k"], W["w_v"], cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim,
                                     pos=idx_np, rope_theta=theta)
        qs, ks, vs = _f(st_.q[:n]), _f(st_.k[:n]), _f(st_.v[:n])
        assert P.row_rel_err(qs.reshape(n, -1), oq.reshape(n, -1)).max() <= 2e-2
        assert P.row_rel_err(ks.reshape(n, -1), ok.reshape(n, -1)).max() <= 2e-2
        rule = ref.RULE_TOPK if l == l_s else ref.RULE_NONE
        o = ref.attn_layer(xs, qs, ks, vs, W["w_o"], idx_np, rule=rule, k_keep=k_keep, keep_first_n=64, keep_last_n=32)
        h_next = ref.ffn_swiglu(o.x_next, W["w_gate"], W["w_up"], W["w_down"])
        assert P.row_rel_err(_f(x_out[:n]), h_next).max() <= P.X_TOL["bf16"]
        if l == l_s:
            halt = st_.buf.halt_mask[:n].cpu().numpy()
            assert int((halt == 0).sum()) == k_keep == o.n_active_out
            assert not halt[:64].any() and not halt[-32:].any()                      # App. A's protected ranges
            thr = np.sort(o.scores[64:n - 32])[::-1][k_keep - 96 - 1]
            band = np.abs(o.scores - thr) <= P.BAND_REL * thr
            assert np.array_equal(halt[~band], o.halt[~band])
            seen.update(halt=halt, state=_f(x_out[:n]).copy(), band=int(band.sum()))
        seen["last_n"] = n

    res = SS.run_single_shot(st, _dev(x0), Wdev, l_s, k_keep, rope_theta=theta, on_block=check)
    torch.cuda.synchronize()
    assert res["n_after"] == k_keep == seen["last_n"]
    final = _f(res["final"])
    halt = seen["halt"]
    # halted tokens: the state they had at the end of block l_s, bit for bit; survivors: the last block's output
    np.testing.assert_array_equal(final[halt == 1], seen["state"][halt == 1])
    surv = res["idx"][:k_keep].cpu().numpy()
    np.testing.assert_array_equal(surv, np.nonzero(halt == 0)[0])
    last = st.x_a if (L - 1) % 2 == 0 else st.x_b
    np.testing.assert_array_equal(final[surv], _f(last[:k_keep]))
    assert not np.array_equal(final[surv], seen["state"][halt == 0])                # they did move on
    print("single shot: kept", k_keep, "of", N, "band rows", seen["band"])


def test_multi_shot_schedule_teacher_forced_against_oracle():
    """Decisions after blocks 1 and 3 of five (App. D's multi-shot variant; protected ranks in the current active
    order): every block against the oracle on the block's actual GPU input, each decision against the oracle's
    TopK on the rows still active, and the full-length result: a token holds the state of the block at whose
    end it stopped."""
    N, d, m, L, theta = 650, 256, 512, 5, 1.0e6
    first, last = 16, 8
    cfg = I.LayerConfig("blocks_ms", "bf16", N, N, d, 4, 2, 64, 0.4, seed=72)
    Wnp = []
    for l in range(L):
        w = I.make_projection_weights(cfg, l)
        w.update(I.make_ffn_weights(cfg, l, m))
        Wnp.append(w)
    Wdev = []
    for w in Wnp:
        dw = {k: _dev(w[k]) for k in ("w_q", "w_k", "w_v", "w_o", "w_down")}
        dw["w_gate_up"] = B.interleave_gate_up(_dev(w["w_gate"]), _dev(w["w_up"]))
        Wdev.append(dw)
    for dw in Wdev:                       # front end as one product over [w_q | w_k | w_v]
        dw["w_qkv"] = B.concat_qkv(dw["w_q"], dw["w_k"], dw["w_v"])
    st = SS.alloc_blocks(d, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, m, N)
    st.params.keep_first_n, st.params.keep_last_n = first, last
    lengths = SS.schedule_lengths(N, L, {1: 0.4, 3: 0.5}, first, last)
    assert lengths == ref.schedule_lengths(N, L, {1: 0.4, 3: 0.5}, first, last)
    shots = {1: lengths[2], 3: lengths[4]}
    assert N > shots[1] > shots[3] > first + last
    seen = {"n_in": [], "stopped": {}, "active": np.arange(N)}

    def check(l, x_in, idx, n, st_, x_out):
        xs, idx_np = _f(x_in[:n]), idx[:n].cpu().numpy()
        np.testing.assert_array_equal(idx_np, seen["active"])
        seen["n_in"].append(n)
        W = Wnp[l]
        oq, ok, ov = ref.rmsnorm_qkv(xs, W["w_q"], W["w_k"], W["w_v"], cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim,
                                     pos=idx_np, rope_theta=theta)
        qs, ks, vs = _f(st_.q[:n]), _f(st_.k[:n]), _f(st_.v[:n])
        assert P.row_rel_err(qs.reshape(n, -1), oq.reshape(n, -1)).max() <= 2e-2
        assert P.row_rel_err(ks.reshape(n, -1), ok.reshape(n, -1)).max() <= 2e-2
        k_keep = shots.get(l, n)
        rule = ref.RULE_TOPK if l in shots else ref.RULE_NONE
        o = ref.attn_layer(xs, qs, ks, vs, W["w_o"], idx_np, rule=rule, k_keep=k_keep, keep_first_n=first,
                           keep_last_n=last)
        h_next = ref.ffn_swiglu(o.x_next, W["w_gate"], W["w_up"], W["w_down"])
        assert P.row_rel_err(_f(x_out[:n]), h_next).max() <= P.X_TOL["bf16"]
        if l in shots:
            halt = st_.buf.halt_mask[:n].cpu().numpy()
            assert int((halt == 0).sum()) == k_keep == o.n_active_out
            assert not halt[:first].any() and not halt[n - last:].any()       # ranks in the current order
            thr = np.sort(o.scores[first:n - last])[::-1][k_keep - first - last - 1]
            band = np.abs(o.scores - thr) <= P.BAND_REL * thr
            assert np.array_equal(halt[~band], o.halt[~band])
            state = _f(x_out[:n])
            for r in np.nonzero(halt == 1)[0]:
                seen["stopped"][int(idx_np[r])] = state[r].copy()
            seen["active"] = idx_np[halt == 0]

    res = SS.run_schedule(st, _dev(I.make_hidden(cfg)), Wdev, shots, rope_theta=theta, on_block=check)
    torch.cuda.synchronize()
    assert seen["n_in"] == lengths and res["n_after"] == shots[3]
    final = _f(res["final"])
    assert len(seen["stopped"]) == N - shots[3]
    for pos, state in seen["stopped"].items():
        np.testing.assert_array_equal(final[pos], state)
    surv = res["idx"][:shots[3]].cpu().numpy()
    np.testing.assert_array_equal(surv, seen["active"])
    last_buf = st.x_a if (L - 1) % 2 == 0 else st.x_b
    np.testing.assert_array_equal(final[surv], _f(last_buf[:shots[3]]))


def test_graphed_schedule_replays_match_eager_runs():
    """A two-shot schedule captured in a HIP graph: every replay, with eager work of the same library and
    synchronisations in between and with the prompt's contents changed in place, equals the eager run on the same
    contents bit for bit (all kernels are deterministic)."""
    N, d, m, L, theta = 600, 256, 512, 4, 1.0e6
    cfg = I.LayerConfig("blocks_graph", "bf16", N, N, d, 4, 2, 64, 0.4, seed=73)
    Wdev = []
    for l in range(L):
        w = I.make_projection_weights(cfg, l)
        w.update(I.make_ffn_weights(cfg, l, m))
        dw = {k: _dev(w[k]) for k in ("w_q", "w_k", "w_v", "w_o", "w_down")}
        dw["w_gate_up"] = B.interleave_gate_up(_dev(w["w_gate"]), _dev(w["w_up"]))
        Wdev.append(dw)
    shots = {0: 400, 2: 150}
    xa = _dev(I.make_hidden(cfg))
    xb = _dev(I.make_hidden(I.scaled(cfg, N, N=N, seed=74)))
    st_e = SS.alloc_blocks(d, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, m, N)
    st_g = SS.alloc_blocks(d, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, m, N)
    for st in (st_e, st_g):
        st.params.keep_first_n, st.params.keep_last_n = 8, 4

    def eager(x):
        r = SS.run_schedule(st_e, x, Wdev, shots, rope_theta=theta)
        torch.cuda.synchronize()
        assert r["n_after"] == 150
        return r["final"].clone(), r["idx"][:150].clone()

    fa, ia = eager(xa)
    fb, ib = eager(xb)
    assert not torch.equal(fa, fb) and not torch.equal(ia, ib)
    x_in = xa.clone()
    gs = SS.GraphedSchedule(st_g, x_in, Wdev, shots, rope_theta=theta)
    assert gs.n_after == 150
    for contents, (want_f, want_i) in ((xa, (fa, ia)), (xb, (fb, ib)), (xb, (fb, ib)), (xa, (fa, ia))):
        x_in.copy_(contents)
        gs.final.zero_()
        gs.replay()
        torch.cuda.synchronize()
        assert torch.equal(gs.final, want_f)
        assert torch.equal(gs.idx[:150], want_i)
        assert int(st_g.buf.n_active_out.item()) == 150
        f2, _ = eager(xb if contents is xa else xa)          # eager work between the replays
        assert torch.equal(f2, fb if contents is xa else fa)
    with pytest.raises(ValueError):
        SS.run_schedule(st_g, x_in, Wdev, {0: 5}, rope_theta=theta, read_counts=False)


def test_single_shot_without_halting_is_the_plain_model():
    """l_s = None: every block on every row; the result is the last block's output at every position."""
    N, d, m, L = 200, 128, 128, 2
    cfg = I.LayerConfig("blocks_full", "bf16", N, N, d, 2, 1, 64, 0.0, seed=71)
    Wdev = []
    for l in range(L):
        w = I.make_projection_weights(cfg, l)
        w.update(I.make_ffn_weights(cfg, l, m))
        dw = {k: _dev(w[k]) for k in ("w_q", "w_k", "w_v", "w_o", "w_down")}
        dw["w_gate_up"] = B.interleave_gate_up(_dev(w["w_gate"]), _dev(w["w_up"]))
        Wdev.append(dw)
    st = SS.alloc_blocks(d, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, m, N)
    res = SS.run_single_shot(st, _dev(I.make_hidden(cfg)), Wdev, None, N, rope_theta=5.0e5)
    torch.cuda.synchronize()
    assert res["n_after"] == N
    assert torch.equal(res["final"], st.x_b[:N])


# ---------------------------------------------------------------- signal and direction variants (Sec. 5.4)

@pytest.mark.parametrize("n", [1, 63, 64, 1000, 4097])
def test_decide_topk_on_given_scores_both_directions(n):
    """TopK on caller-provided scores: integer work, compared bit for bit. Random scores are the random-halting
    control; keep_low is the high-Delta control. Heavy ties included."""
    rng = np.random.default_rng(90 + n)
    p = B.make_params(256, 4, 2, 64)
    ws = torch.empty((256 + 4 * ((n + 63) // 64) + 64,), dtype=torch.uint8, device="cuda")
    for case in range(6):
        s = rng.random(n).astype(np.float32)
        if case % 2:
            s = np.round(s * 7) / 7                      # many exact ties
        if case == 4:
            s = -s
        first, last = ((0, 0), (3, 2), (64, 32))[case % 3]
        k_keep = int(rng.integers(0, n + 1))
        p.k_keep, p.keep_first_n, p.keep_last_n = k_keep, first, last
        gs = torch.from_numpy(s).cuda()
        for keep_low in (False, True):
            halt = torch.empty((n,), dtype=torch.uint8, device="cuda")
            counts = torch.empty(((n + 63) // 64,), dtype=torch.int32, device="cuda")
            B.dash_decide_topk(p, gs, n, keep_low, halt, counts, ws)
            torch.cuda.synchronize()
            want = ref.decide_topk(s.astype(np.float64), k_keep, first, last, keep_low=keep_low)
            np.testing.assert_array_equal(halt.cpu().numpy(), want)
            kept = (want == 0).astype(np.int64)
            np.testing.assert_array_equal(counts.cpu().numpy(), np.add.reduceat(kept, np.arange(0, n, 64)))


@pytest.mark.parametrize("dt", ["bf16", "f32"])
def test_score_diff_rows_matches_oracle(dt):
    n, d = 333, 512
    rng = np.random.default_rng(95)
    a = rng.standard_normal((n, d)) * np.exp(rng.standard_normal((n, 1)))
    b = a + 0.05 * rng.standard_normal((n, d)) * np.abs(a).mean(1, keepdims=True)
    b[7] = a[7]
    if dt == "bf16":
        a, b = I.round_to_bf16(a), I.round_to_bf16(b)
    else:
        a, b = a.astype(np.float32).astype(np.float64), b.astype(np.float32).astype(np.float64)
    code = B.DASH_BF16 if dt == "bf16" else B.DASH_F32
    ga, gb = B.to_device(a, code), B.to_device(b, code)
    for kind in (ref.SCORE_REL, ref.SCORE_ABS):
        out = torch.empty((n,), dtype=torch.float32, device="cuda")
        B.dash_score_diff_rows(gb, ga, n, d, code, kind, out)
        torch.cuda.synchronize()
        want = ref.score_block(b, a, kind)
        np.testing.assert_allclose(out.cpu().numpy(), want, rtol=2e-5, atol=1e-30)
        assert out[7].item() == 0.0
