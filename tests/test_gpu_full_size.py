"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times.

Config 2 (N = 8192, all rows active) is compared with the oracle on EVERY row. At the two larger sizes the oracle
cannot finish all rows within seconds, so it evaluates a sample of query rows (both ends, rows around the tile
boundaries, the ragged tail, the rest seeded-uniform: 2048 rows at N = 32768 / 50 %, 512 rows at N = 131072 / 40 %)
against ALL keys/values: exact for those rows because attention rows are independent. tau comes from the GPU's own
scores by the percentile rule and is given to both sides. On those rows x_next, the score and the halt flag are
compared, and so is delta itself, element by element (a second run with the debug output: x_next on a row with a
large norm hides an error in delta). Compaction is checked in full against the GPU's own mask, and the TopK rule of
the layer call is checked in full, bit for bit, against the oracle's TopK on the GPU's own fp32 scores (pure integer
work once the scores are fixed).
"""
import time

import numpy as np
import pytest
import torch

from oracle import reference as ref
from paper_2604_18103_amd import binding as B
from paper_2604_18103_amd import inputs as I

import parity_util as P

pytestmark = pytest.mark.gpu

DELTA_TOL = 1e-2      # per-row max |delta_gpu - delta_oracle| / max |delta_oracle| (bf16 O and P roundings: ~3e-3)


def oracle_rows(L, cfg, rows):
    """The layer on the sampled query rows against all keys/values, converting only what the rows need."""
    t0 = time.perf_counter()
    O = ref.attention_rows(L["q"], L["k"], L["v"], L["active_idx"], rows=rows, causal=cfg.causal)
    delta = ref.project(O, L["w_o"])
    x_rows = L["x"][rows].astype(np.float64)
    res = ref.LayerResult(rows, delta, ref.residual(x_rows, delta), ref.scores(delta, x_rows), None, None, None, None)
    return res, time.perf_counter() - t0


def finish_full(o, tau, active_idx):
    """Every row was evaluated: the oracle's own decision and compaction, for the comparison of the index sets."""
    o.halt = ref.decide_threshold(o.scores, tau)
    o.new_active_idx, o.x_compact, o.n_active_out = ref.compact(o.halt, active_idx, o.x_next)
    return o


@pytest.mark.parametrize("name,n_rows", [("qwen_8k", None), ("qwen_32k_half", 2048), ("llama_128k_40", 512)])
def test_full_size_against_oracle(name, n_rows):
    cfg = I.CONFIGS[name]
    n = cfg.n
    L = I.make_layer_inputs(cfg)
    D = P.device_inputs(cfg, L)
    buf = B.alloc_layer_buffers(P.params_for(cfg), n)
    g0 = P.run_gpu_layer(cfg, P.params_for(cfg, rule=B.RULE_NONE), D, buf=buf)
    tau, h = I.percentile_tau(g0.scores, cfg.halt_frac)
    gpu_scores = g0.scores.copy()
    del g0
    g = P.run_gpu_layer(cfg, P.params_for(cfg, rule=B.RULE_THRESHOLD, tau=tau), D, buf=buf)
    P.check_self_consistency(g, L["active_idx"], n)
    assert g.n_active_out == n - h
    assert set(g.new_active_idx.tolist()) <= set(L["active_idx"].tolist())
    assert np.array_equal(g.scores, gpu_scores)                      # run to run: the same bits
    x_next_no_dbg = g.x_next

    rows = np.arange(n, dtype=np.int64) if n_rows is None else I.sample_rows(n, n_rows, seed=cfg.seed, tile=256)
    o, secs = oracle_rows(L, cfg, rows)
    if n_rows is None:
        finish_full(o, tau, L["active_idx"])
    rep = P.compare_with_oracle(cfg, g, o, tau, L["active_idx"], rows=rows)
    del g

    # delta itself on the same rows (debug output of the projection)
    buf_d = B.alloc_layer_buffers(P.params_for(cfg), n, with_delta=True)
    gd = P.run_gpu_layer(cfg, P.params_for(cfg, rule=B.RULE_THRESHOLD, tau=tau), D, with_delta=True, buf=buf_d)
    assert np.array_equal(gd.x_next, x_next_no_dbg)                  # the debug copy changes nothing else
    derr = P.row_rel_err(gd.delta[rows], o.delta)
    assert derr.max() <= DELTA_TOL, f"delta rel err {derr.max():.3e} at row {rows[derr.argmax()]}"
    # x_next minus x is delta up to the rounding of x_next: half a bf16 step of the larger of the two
    upd = gd.x_next[rows].astype(np.float64) - L["x"][rows]
    # (half a bf16 step, plus the fp32 rounding of the sum before it)
    bound = 2.0 ** -8 * np.abs(gd.x_next[rows]) * (1 + 1e-4) + np.abs(gd.delta[rows] - o.delta) * (1 + 1e-6) + 1e-30
    n_bad = int((np.abs(upd - o.delta) > bound).sum())
    assert n_bad == 0, f"{n_bad} elements of x_next - x differ from delta by more than the rounding of x_next"
    rep["delta_max_rel"] = float(derr.max())
    del gd, buf_d, x_next_no_dbg

    # the TopK rule of the layer call, in full, on the GPU's own scores
    for first, last in ((0, 0), (64, 32)):
        k_keep = n - h
        gt = P.run_gpu_layer(cfg, P.params_for(cfg, rule=B.RULE_TOPK, k_keep=k_keep, keep_first_n=first,
                                               keep_last_n=last), D, buf=buf)
        assert np.array_equal(gt.scores, gpu_scores)
        want = ref.decide_topk(gpu_scores.astype(np.float64), k_keep, first, last)
        np.testing.assert_array_equal(gt.halt, want)
        assert gt.n_active_out == k_keep
        np.testing.assert_array_equal(gt.new_active_idx, L["active_idx"][want == 0])
        P.check_self_consistency(gt, L["active_idx"], n)
        del gt
    print(name, "n", n, "kept", n - h, "oracle rows", len(rows), f"oracle {secs:.1f} s", rep)


def test_full_size_block_half_and_front_end_sampled_rows():
    """The steps around the layer at the size the end-to-end workloads run them (Qwen2.5-7B shapes, 32768 rows,
    FFN width 18944): rows are independent in the feed-forward, the projections and the rotary embedding, so the
    oracle on a sample of rows is exact for those rows. The same feed-forward on the first 177 rows alone (the
    length left after 99 % of an 8192-token prompt halts) takes the path that cuts both products along K."""
    cfg = I.CONFIGS["qwen_32k_chain"]
    n, d, m, theta = cfg.n, cfg.d, 18944, 1.0e6
    x = I.make_hidden(cfg)
    Wf = I.make_ffn_weights(cfg, 0, m)
    Wp = I.make_projection_weights(cfg, 0)
    p = P.params_for(cfg)
    dev = lambda a: B.to_device(a, B.DASH_BF16)
    f = lambda t: t.float().cpu().numpy()
    rows = I.sample_rows(n, 256, seed=cfg.seed, tile=256)
    small = rows[rows < 177]
    gx = dev(x)
    wgu, wd = B.interleave_gate_up(dev(Wf["w_gate"]), dev(Wf["w_up"])), dev(Wf["w_down"])
    want = ref.ffn_swiglu(x[rows], Wf["w_gate"], Wf["w_up"], Wf["w_down"])
    out = torch.empty((n, d), dtype=torch.bfloat16, device="cuda")
    ws = torch.empty((B.ffn_workspace_bytes(p, n, m),), dtype=torch.uint8, device="cuda")
    B.dash_ffn_swiglu(p, gx, wgu, wd, n, m, out, ws)
    torch.cuda.synchronize()
    err = P.row_rel_err(f(out[torch.from_numpy(rows).cuda()]), want)
    assert err.max() <= P.X_TOL["bf16"], err.max()
    out_s = torch.empty((177, d), dtype=torch.bfloat16, device="cuda")
    B.dash_ffn_swiglu(p, gx, wgu, wd, 177, m, out_s, ws)
    torch.cuda.synchronize()
    assert len(small) >= 8
    err_s = P.row_rel_err(f(out_s)[small], want[: len(small)])
    assert err_s.max() <= P.X_TOL["bf16"], err_s.max()
    del ws, out, wgu, wd
    # front end: RMSNorm + q/k/v projections + rotary embedding at positions up to 131071
    pos = np.sort(np.random.default_rng(5).choice(131072, size=n, replace=False)).astype(np.int32)
    q = torch.empty((n, cfg.n_q_heads, cfg.head_dim), dtype=torch.bfloat16, device="cuda")
    k = torch.empty((n, cfg.n_kv_heads, cfg.head_dim), dtype=torch.bfloat16, device="cuda")
    v = torch.empty_like(k)
    h = torch.empty((n, d), dtype=torch.bfloat16, device="cuda")
    B.dash_rmsnorm_qkv(p, gx, dev(Wp["w_q"]), dev(Wp["w_k"]), dev(Wp["w_v"]), n, q, k, v, h)
    B.dash_rope_qk(p, q, k, torch.from_numpy(pos).cuda(), n, theta)
    torch.cuda.synchronize()
    oq, ok, ov = ref.rmsnorm_qkv(x[rows], Wp["w_q"], Wp["w_k"], Wp["w_v"], cfg.n_q_heads, cfg.n_kv_heads,
                                 cfg.head_dim, pos=pos[rows], rope_theta=theta)
    sel = torch.from_numpy(rows).cuda()
    for got, want_ in ((q, oq), (k, ok), (v, ov)):
        e = P.row_rel_err(f(got[sel]).reshape(len(rows), -1), want_.reshape(len(rows), -1))
        assert e.max() <= 2e-2, e.max()
    print("block half: ffn err", float(err.max()), "split-K", float(err_s.max()))
