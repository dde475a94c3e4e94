"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times.

The oracle cannot run these sizes in full within seconds, so it evaluates a sample of query rows
(both ends, tile boundaries, the ragged tail, the rest seeded-uniform) against ALL keys/values: exact
for those rows because attention rows are independent. tau comes from the GPU's own scores by the
percentile rule and is given to both sides. Compaction is checked in full against the GPU's own mask.
"""
import numpy as np
import pytest

from oracle import reference as ref
from paper_2604_18103_amd import binding as B
from paper_2604_18103_amd import inputs as I

import parity_util as P

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,n_rows", [("qwen_8k", 96), ("qwen_32k_half", 96), ("llama_128k_40", 64)])
def test_full_size_sampled_rows(name, n_rows):
    cfg = I.CONFIGS[name]
    n = cfg.n
    L = I.make_layer_inputs(cfg)
    D = P.device_inputs(cfg, L)
    buf = B.alloc_layer_buffers(P.params_for(cfg), n)
    g0 = P.run_gpu_layer(cfg, P.params_for(cfg, rule=B.RULE_NONE), D, buf=buf)
    tau, h = I.percentile_tau(g0.scores, cfg.halt_frac)
    del g0
    g = P.run_gpu_layer(cfg, P.params_for(cfg, rule=B.RULE_THRESHOLD, tau=tau), D, buf=buf)
    P.check_self_consistency(g, L["active_idx"], n)
    assert g.n_active_out == n - h
    assert set(g.new_active_idx.tolist()) <= set(L["active_idx"].tolist())
    rows = I.sample_rows(n, n_rows, seed=cfg.seed)
    o = ref.attn_layer(L["x"], L["q"], L["k"], L["v"], L["w_o"], L["active_idx"], causal=cfg.causal, rows=rows)
    rep = P.compare_with_oracle(cfg, g, o, tau, L["active_idx"], rows=rows)
    print(name, "n", n, "kept", g.n_active_out, rep)


def test_full_size_block_half_and_front_end_sampled_rows():
    """The steps around the layer at the size the end-to-end workloads run them (Qwen2.5-7B shapes, 32768 rows,
    FFN width 18944): rows are independent in the feed-forward, the projections and the rotary embedding, so the
    oracle on a sample of rows is exact for those rows. The same feed-forward on the first 177 rows alone (the
    length left after 99 % of an 8192-token prompt halts) takes the path that cuts both products along K."""
    import torch
    cfg = I.CONFIGS["qwen_32k_chain"]
    n, d, m, theta = cfg.n, cfg.d, 18944, 1.0e6
    x = I.make_hidden(cfg)
    Wf = I.make_ffn_weights(cfg, 0, m)
    Wp = I.make_projection_weights(cfg, 0)
    p = P.params_for(cfg)
    dev = lambda a: B.to_device(a, B.DASH_BF16)
    f = lambda t: t.float().cpu().numpy()
    rows = I.sample_rows(n, 64, seed=cfg.seed)
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
