"""GPU parity: the HIP path, called through the C ABI, against the fp64 CPU oracle."""
import numpy as np
import pytest
import torch

from oracle import reference as ref
from paper_2604_18103_amd import binding as B
from paper_2604_18103_amd import inputs as I

import parity_util as P

pytestmark = pytest.mark.gpu

TINY = I.CONFIGS["tiny_f32"]
QWEN = I.CONFIGS["qwen_8k"]
LLAMA = I.CONFIGS["llama_128k_40"]
# a narrow bf16 layer: several query/key tiles and ragged tails at little oracle cost
NARROW = I.LayerConfig("narrow_bf16", "bf16", 4000, 1333, 512, 4, 2, 128, 0.4, seed=11)
NARROW64 = I.LayerConfig("narrow_bf16_hd64", "bf16", 2000, 777, 256, 4, 1, 64, 0.5, seed=12)


def test_tiny_fp32_config_full():
    """Benchmark configuration 1 in full: fp32, N=512, hidden 256, 4/1 heads, head_dim 64."""
    rep, g, o = P.full_parity(TINY, check_delta=True)
    assert g.n_active_out == o.n_active_out == 256 or rep["band_rows"] > 0
    print("tiny_f32", rep)


@pytest.mark.parametrize("cfg", [NARROW, NARROW64], ids=lambda c: c.name)
def test_bf16_narrow_layer(cfg):
    rep, g, o = P.full_parity(cfg, check_delta=True)
    print(cfg.name, rep)


@pytest.mark.parametrize("heads", [(6, 3), (32, 16), (8, 8)], ids=lambda h: f"hq{h[0]}_hkv{h[1]}")
def test_bf16_head_layouts(heads):
    """Head counts that take the other branches of the attention kernel's work map: 3 KV heads (no
    XCD-aligned map), 16 KV heads (two KV heads per XCD), and plain multi-head attention (group size 1)."""
    hq, hkv = heads
    cfg = I.LayerConfig(f"heads_{hq}_{hkv}", "bf16", 2500, 700, 256, hq, hkv, 64, 0.3, seed=21 + hq)
    rep, g, o = P.full_parity(cfg)
    print(cfg.name, rep)


@pytest.mark.parametrize("halt_frac", [0.75, 0.9, 0.99, 0.999])
def test_extreme_reduction_ratios(halt_frac):
    """The aggressive budgets of the vision-language setting (Sec. 4.3: up to 99 % of the tokens dropped): the
    decision, the counts and the compaction with very few survivors, threshold and TopK alike."""
    cfg = I.scaled(NARROW, 1333, N=4000, halt_frac=halt_frac)
    rep, g, o = P.full_parity(cfg)
    assert g.n_active_out == o.n_active_out or rep["band_rows"] > 0
    assert o.n_active_out <= int(round((1 - halt_frac) * cfg.n)) + 1
    rep2, g2, o2 = P.full_parity(cfg, rule=B.RULE_TOPK)
    assert g2.n_active_out == o2.n_active_out == cfg.n - int(halt_frac * cfg.n)
    print(cfg.name, halt_frac, rep, rep2)


def test_bf16_qwen_shape_ragged():
    """Qwen2.5-7B layer shape (hidden 3584, 28/4 heads, head_dim 128) at a length that is not a
    multiple of any tile (query tile 128, key tile 64, GEMM tile 256)."""
    cfg = I.scaled(QWEN, 715, N=3000)
    rep, g, o = P.full_parity(cfg)
    print(cfg.name, rep)


def test_bf16_llama_shape_ragged():
    cfg = I.scaled(LLAMA, 389, N=1000)
    rep, g, o = P.full_parity(cfg)
    print(cfg.name, rep)


def test_non_causal():
    cfg = I.scaled(NARROW, 300, N=900, causal=False)
    P.full_parity(cfg)
    cfg32 = I.scaled(TINY, 200, N=200, causal=False)
    P.full_parity(cfg32)


def test_absolute_score_kind():
    P.full_parity(I.scaled(NARROW, 260, N=800), score_kind=B.SCORE_ABS)
    P.full_parity(I.scaled(TINY, 130, N=130), score_kind=B.SCORE_ABS)


@pytest.mark.parametrize("n", [1, 2, 63, 64, 65, 127, 128, 129, 257])
def test_edge_lengths_bf16(n):
    P.full_parity(I.scaled(NARROW, n, N=4 * n + 3))


@pytest.mark.parametrize("n", [1, 63, 64, 65])
def test_edge_lengths_fp32(n):
    P.full_parity(I.scaled(TINY, n, N=n))


def test_rule_none_halts_nothing():
    P.full_parity(I.scaled(NARROW, 200, N=700), rule=B.RULE_NONE)


@pytest.mark.parametrize("cfg", [I.scaled(NARROW, 900, N=3000), I.scaled(TINY, 300, N=300)],
                         ids=["bf16", "f32"])
def test_topk_rule(cfg):
    rep, g, o = P.full_parity(cfg, rule=B.RULE_TOPK)
    assert g.n_active_out == cfg.n - int(np.floor(cfg.halt_frac * cfg.n))


def test_protected_prefix_suffix():
    cfg = I.scaled(NARROW, 500, N=2000, halt_frac=0.7)
    P.full_parity(cfg, keep_first_n=64, keep_last_n=32)
    P.full_parity(cfg, rule=B.RULE_TOPK, keep_first_n=64, keep_last_n=32)


def _stage_setup(cfg):
    L = I.make_layer_inputs(cfg)
    D = P.device_inputs(cfg, L)
    return L, D


def test_all_halt_none_halt_and_empty():
    cfg = I.scaled(NARROW, 150, N=600)
    L, D = _stage_setup(cfg)
    for tau, want in ((0.0, cfg.n), (float("inf"), 0)):
        params = P.params_for(cfg, rule=B.RULE_THRESHOLD, tau=tau)
        g = P.run_gpu_layer(cfg, params, D)
        P.check_self_consistency(g, L["active_idx"], cfg.n)
        assert g.n_active_out == want
    # n_active = 0 is a valid no-op that reports zero survivors
    params = P.params_for(cfg, rule=B.RULE_THRESHOLD, tau=0.5)
    buf = B.alloc_layer_buffers(params, 0)
    buf.n_active_out.fill_(77)
    B.dash_attn_layer(params, D["x"], D["q"], D["k"], D["v"], D["w_o"], D["active_idx"], 0, buf)
    torch.cuda.synchronize()
    assert int(buf.n_active_out.item()) == 0


def test_zero_output_projection_scores_are_zero():
    cfg = I.scaled(NARROW, 200, N=500)
    L, D = _stage_setup(cfg)
    D["w_o"].zero_()
    params = P.params_for(cfg, rule=B.RULE_THRESHOLD, tau=1e-6)
    g = P.run_gpu_layer(cfg, params, D)
    assert np.all(g.scores == 0.0) and g.n_active_out == 0 and g.halt.all()
    assert np.array_equal(g.x_next, L["x"])


def test_threshold_and_topk_agree_and_runs_are_bit_reproducible():
    cfg = I.scaled(NARROW, 1000, N=3000)
    L, D = _stage_setup(cfg)
    g0 = P.run_gpu_layer(cfg, P.params_for(cfg, rule=B.RULE_NONE), D)
    tau, h = I.percentile_tau(g0.scores, 0.35)
    ga = P.run_gpu_layer(cfg, P.params_for(cfg, rule=B.RULE_THRESHOLD, tau=tau), D)
    gb = P.run_gpu_layer(cfg, P.params_for(cfg, rule=B.RULE_TOPK, k_keep=cfg.n - h), D)
    gc = P.run_gpu_layer(cfg, P.params_for(cfg, rule=B.RULE_THRESHOLD, tau=tau), D)
    assert np.array_equal(ga.halt, gb.halt) and ga.n_active_out == gb.n_active_out == cfg.n - h
    for f in ("x_next", "scores", "halt", "x_compact", "new_active_idx"):
        assert np.array_equal(getattr(ga, f), getattr(gc, f)), f
    # rho form of Eq. 3: K = floor((1 - rho) n)
    gd = P.run_gpu_layer(cfg, P.params_for(cfg, rule=B.RULE_TOPK, k_keep=-1, rho=0.667), D)
    assert gd.n_active_out == int(np.floor((1 - np.float64(np.float32(0.667))) * cfg.n))


def test_topk_ties_keep_earliest_rows():
    """Stage-level: hand-made partial sums with many equal scores."""
    cfg = I.scaled(NARROW, 300, N=300)
    params = P.params_for(cfg, rule=B.RULE_TOPK, k_keep=120, score_kind=B.SCORE_ABS)
    Pn = B.norm_partials_per_row(params)
    n = cfg.n
    rng = np.random.default_rng(0)
    vals = rng.integers(1, 6, size=n).astype(np.float32)          # scores sqrt(1..5): heavy ties
    partials = np.zeros((Pn, n, 2), np.float32)
    partials[0, :, 0] = vals
    partials[:, :, 1] = 1.0
    dp = torch.from_numpy(partials).cuda()
    scores = torch.empty(n, dtype=torch.float32, device="cuda")
    halt = torch.empty(n, dtype=torch.uint8, device="cuda")
    counts = torch.empty((n + 63) // 64, dtype=torch.int32, device="cuda")
    ws = torch.empty(4096, dtype=torch.uint8, device="cuda")
    B.dash_score_decide(params, dp, n, scores, halt, counts, ws)
    torch.cuda.synchronize()
    want = ref.decide_topk(np.sqrt(vals.astype(np.float64)), 120)
    assert np.array_equal(halt.cpu().numpy(), want)
    assert int(counts.sum().item()) == 120
    np.testing.assert_allclose(scores.cpu().numpy(), np.sqrt(vals), rtol=1e-6)


def test_compact_stage_alone_and_score_rows():
    cfg = I.scaled(NARROW, 1000, N=5000)
    n, d = cfg.n, cfg.d
    rng = np.random.default_rng(1)
    params = P.params_for(cfg)
    halt_np = (rng.random(n) < 0.6).astype(np.uint8)
    idx_np = I.make_active_idx(cfg.N, n, 3)
    xn = torch.randn(n, d, device="cuda").to(torch.bfloat16)
    halt = torch.from_numpy(halt_np).cuda()
    idx = torch.from_numpy(idx_np).cuda()
    xc = torch.empty_like(xn)
    new_idx = torch.empty(n, dtype=torch.int32, device="cuda")
    n_out = torch.zeros(1, dtype=torch.int32, device="cuda")
    ws = torch.empty(4096, dtype=torch.uint8, device="cuda")
    B.dash_compact(params, halt, None, idx, xn, n, xc, new_idx, n_out, ws)
    torch.cuda.synchronize()
    want_idx, _, want_n = ref.compact(halt_np, idx_np)
    assert int(n_out.item()) == want_n
    assert np.array_equal(new_idx[:want_n].cpu().numpy(), want_idx)
    assert torch.equal(xc[:want_n], xn[torch.from_numpy(halt_np == 0).cuda()])
    # standalone score of Eq. 2 from a stored delta
    delta = torch.randn(n, d, device="cuda")
    s = torch.empty(n, dtype=torch.float32, device="cuda")
    for kind in (B.SCORE_REL, B.SCORE_ABS):
        B.dash_score_rows(delta, xn, n, d, B.DASH_BF16, kind, s)
        torch.cuda.synchronize()
        want = ref.scores(delta.cpu().numpy(), xn.float().cpu().numpy(), kind=kind)
        np.testing.assert_allclose(s.cpu().numpy(), want, rtol=2e-6)


def test_validate_active_idx_counts_violations():
    idx = torch.tensor([0, 3, 3, 9, 8, 50], dtype=torch.int32, device="cuda")
    viol = torch.zeros(1, dtype=torch.int32, device="cuda")
    B.dash_validate_active_idx(idx, 6, 40, viol)
    torch.cuda.synchronize()
    assert int(viol.item()) == 3        # repeated 3, descending 8, out-of-range 50
    good = torch.arange(0, 100, 3, dtype=torch.int32, device="cuda")
    B.dash_validate_active_idx(good, good.numel(), -1, viol)
    torch.cuda.synchronize()
    assert int(viol.item()) == 0


def test_invalid_arguments_are_rejected_without_launch():
    cfg = I.scaled(NARROW, 64, N=64)
    L, D = _stage_setup(cfg)
    params = P.params_for(cfg, tau=0.1)
    buf = B.alloc_layer_buffers(params, cfg.n)
    small = B.LayerBuffers(**{**buf.__dict__, "workspace": buf.workspace[:256]})
    with pytest.raises(B.DashError, match="workspace"):
        B.dash_attn_layer(params, D["x"], D["q"], D["k"], D["v"], D["w_o"], D["active_idx"], cfg.n, small)
    bad = P.params_for(cfg, tau=0.1)
    bad.head_dim = 96
    with pytest.raises(B.DashError, match="unsupported"):
        B.dash_attn_layer(bad, D["x"], D["q"], D["k"], D["v"], D["w_o"], D["active_idx"], cfg.n, buf)
    bad2 = P.params_for(cfg, tau=0.1)
    bad2.n_kv_heads = 3
    with pytest.raises(B.DashError, match="invalid"):
        B.dash_attn_layer(bad2, D["x"], D["q"], D["k"], D["v"], D["w_o"], D["active_idx"], cfg.n, buf)
    mis = D["x"].view(-1)[1:1 + (cfg.n - 1) * cfg.d].view(cfg.n - 1, cfg.d)   # 2-byte offset
    with pytest.raises(B.DashError, match="invalid"):
        B.dash_attn_layer(params, mis, D["q"], D["k"], D["v"], D["w_o"], D["active_idx"], cfg.n - 1, buf)


@pytest.mark.parametrize("slope", [0.0, 8.0, 40.0, -40.0], ids=lambda s: "slope%g" % s)
@pytest.mark.parametrize("dh", [64, 128])
def test_flash_softmax_reference_moves_with_the_scores(dh, slope):
    """Scores that drift along the key axis by `slope` (natural-log units) per 64-key tile, up to hundreds over
    the sequence: the kernel's softmax reference is not the running maximum and moves only when a row sum leaves
    a modest range, so drifting scores exercise every branch of it (move at nearly every tile when they rise
    steeply, never after the first tile when they fall, underflow of everything but the newest keys). The
    attention output against the oracle on the same bf16 inputs."""
    import torch
    n, hq, hkv = 777, 4, 2
    rng = np.random.default_rng(400 + dh + int(slope))
    u = rng.standard_normal(dh)
    u /= np.linalg.norm(u)
    ramp = (np.arange(n) / 64.0) * slope                          # target drift of the logit along the keys
    q = rng.standard_normal((n, hq, dh)) * 0.5 + 4.0 * u          # q . u = 4 (+ noise)
    k = rng.standard_normal((n, hkv, dh)) * 0.5 + (ramp * np.sqrt(dh) / 4.0)[:, None, None] * u
    v = rng.standard_normal((n, hkv, dh))
    q, k, v = I.round_to_bf16(q), I.round_to_bf16(k), I.round_to_bf16(v)
    pos = np.arange(n, dtype=np.int32)
    p = B.make_params(hq * dh, hq, hkv, dh, causal=True)
    for causal in (True, False):
        p.causal = int(causal)
        o = torch.empty((n, hq * dh), dtype=torch.bfloat16, device="cuda")
        B.dash_flash_fwd(p, B.to_device(q, B.DASH_BF16), B.to_device(k, B.DASH_BF16), B.to_device(v, B.DASH_BF16),
                         torch.from_numpy(pos).cuda(), n, o)
        torch.cuda.synchronize()
        want = ref.attention_rows(q, k, v, pos, causal=causal)
        got = o.float().cpu().numpy()
        assert np.isfinite(got).all()
        err = P.row_rel_err(got, want)
        print("drift", dh, slope, causal, float(err.max()))
        assert err.max() <= P.X_TOL["bf16"], (causal, float(err.max()))


@pytest.mark.parametrize("n,d,prot", [(1, 256, (0, 0)), (63, 256, (3, 2)), (65, 256, (0, 0)), (1333, 512, (64, 32)),
                                      (20001, 256, (0, 0)), (131072, 128, (5, 7))],
                         ids=lambda v: str(v).replace(" ", ""))
def test_layer_call_in_one_launch_equals_the_staged_calls(n, d, prot):
    """Under the rules NONE and THRESHOLD the layer call finishes scores, decision and compaction in one launch whose
    workgroups hand each other the chunks' kept masks and counts; the stage-level calls (score + decision, then
    compaction, two launches) compute the same from the same norm partials. Every output must be bit-identical,
    from one chunk to 2048 chunks (n = 131072), twice in a row on the same buffers (the published words of the
    first call are cleared by the second)."""
    rng = np.random.default_rng(n)
    hq, dh = d // 64, 64
    p = B.make_params(d, hq, hq, dh, rule=B.RULE_THRESHOLD, keep_first_n=prot[0], keep_last_n=prot[1])
    N = 3 * n + 5
    idx = torch.from_numpy(np.sort(rng.choice(N, size=n, replace=False)).astype(np.int32)).cuda()
    bf = torch.bfloat16
    g = torch.Generator(device="cuda").manual_seed(n)
    rnd = lambda *shape: torch.randn(shape, generator=g, device="cuda", dtype=torch.float32)
    x = (rnd(n, d) * torch.exp(1.5 * rnd(n, 1))).to(bf)
    w_o = (rnd(hq * dh, d) / d ** 0.5).to(bf)
    o = rnd(n, hq * dh).to(bf)                      # any attention output: only to draw a threshold from real scores
    P_ = B.norm_partials_per_row(p)
    # staged: projection, score + decision, compaction
    x_next = torch.empty((n, d), dtype=bf, device="cuda")
    partials = torch.empty((P_, n, 2), dtype=torch.float32, device="cuda")
    B.dash_wo_residual_rownorm(p, o, w_o, x, n, x_next, partials, None, None)
    scores = torch.empty((n,), dtype=torch.float32, device="cuda")
    halt = torch.empty((n,), dtype=torch.uint8, device="cuda")
    counts = torch.empty(((n + 63) // 64,), dtype=torch.int32, device="cuda")
    p.rule = B.RULE_NONE
    B.dash_score_decide(p, partials, n, scores, halt, counts)
    torch.cuda.synchronize()
    tau, h = I.percentile_tau(scores.cpu().numpy(), 0.37)
    for rule, tau_ in ((B.RULE_THRESHOLD, tau), (B.RULE_NONE, 0.0), (B.RULE_THRESHOLD, float("inf")),
                       (B.RULE_THRESHOLD, tau)):
        p.rule, p.tau = rule, tau_
        x_c = torch.full((n, d), float("nan"), dtype=bf, device="cuda")
        new_idx = torch.full((n,), -1, dtype=torch.int32, device="cuda")
        n_out = torch.full((1,), -7, dtype=torch.int32, device="cuda")
        buf = B.alloc_layer_buffers(p, n, with_delta=True)   # the debug output keeps both paths off split-K
        q = rnd(n, hq, dh).to(bf)
        kk = rnd(n, hq, dh).to(bf)
        v = rnd(n, hq, dh).to(bf)
        B.dash_attn_layer(p, x, q, kk, v, w_o, idx, n, buf)
        B.dash_attn_layer(p, x, q, kk, v, w_o, idx, n, buf)          # again on the same workspace
        o2 = torch.empty((n, hq * dh), dtype=bf, device="cuda")
        B.dash_flash_fwd(p, q, kk, v, idx, n, o2)
        B.dash_wo_residual_rownorm(p, o2, w_o, x, n, x_next, partials, buf.delta_dbg, None)
        B.dash_score_decide(p, partials, n, scores, halt, counts)
        x_c.fill_(float("nan"))
        B.dash_compact(p, halt, counts, idx, x_next, n, x_c, new_idx, n_out)
        torch.cuda.synchronize()
        k = int(n_out.item())
        assert int(buf.n_active_out.item()) == k
        assert torch.equal(buf.x_next[:n], x_next)
        assert torch.equal(buf.scores[:n], scores) and torch.equal(buf.halt_mask[:n], halt)
        assert torch.equal(buf.new_active_idx[:k], new_idx[:k])
        assert torch.equal(buf.x_compact[:k], x_c[:k])
        if rule == B.RULE_NONE:
            assert k == n
        if tau_ == float("inf"):
            assert k == min(n, prot[0] + prot[1])


@pytest.mark.parametrize("rule", ["threshold", "topk", "none"])
def test_layer_call_in_a_hip_graph_replays_like_eager_calls(rule):
    """The layer call records only kernels (the words its one-launch score/decision/compaction hands chunks over
    with are cleared by the attention kernel of the same call, not by a memset), so it can be captured in a HIP
    graph. Every replay, with eager calls of the same library on other buffers and synchronisations in between and
    with the inputs changed in place, must equal the eager call on the same contents bit for bit."""
    cfg = I.LayerConfig("graph_layer", "bf16", 4000, 1500, 256, 4, 2, 64, 0.45, seed=81)
    n = cfg.n
    L1 = I.make_layer_inputs(cfg)
    L2 = I.make_layer_inputs(I.scaled(cfg, n, N=cfg.N, seed=82))
    D1, D2 = P.device_inputs(cfg, L1), P.device_inputs(cfg, L2)
    g0 = P.run_gpu_layer(cfg, P.params_for(cfg, rule=B.RULE_NONE), D1)
    tau, h = I.percentile_tau(g0.scores, cfg.halt_frac)
    p = {"threshold": P.params_for(cfg, rule=B.RULE_THRESHOLD, tau=tau, keep_first_n=8, keep_last_n=4),
         "topk": P.params_for(cfg, rule=B.RULE_TOPK, k_keep=n - h, keep_first_n=8, keep_last_n=4),
         "none": P.params_for(cfg, rule=B.RULE_NONE)}[rule]
    outs = ("x_next", "scores", "halt_mask", "x_compact", "new_active_idx", "n_active_out")

    def eager(D):
        buf = B.alloc_layer_buffers(p, n)
        buf.x_compact.zero_()                      # rows past n_active_out are not written: compare like with like
        buf.new_active_idx.zero_()
        B.dash_attn_layer(p, D["x"], D["q"], D["k"], D["v"], D["w_o"], D["active_idx"], n, buf)
        torch.cuda.synchronize()
        return {k: getattr(buf, k).clone() for k in outs}

    want1, want2 = eager(D1), eager(D2)
    assert not torch.equal(want1["scores"], want2["scores"])
    assert 0 < int(want1["n_active_out"].item()) <= n
    G = {k: v.clone() for k, v in D1.items()}      # the graph's own input buffers
    gbuf = B.alloc_layer_buffers(p, n)
    B.init()
    B.dash_attn_layer(p, G["x"], G["q"], G["k"], G["v"], G["w_o"], G["active_idx"], n, gbuf)   # eager once
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        B.dash_attn_layer(p, G["x"], G["q"], G["k"], G["v"], G["w_o"], G["active_idx"], n, gbuf)
    for D, want in ((D1, want1), (D2, want2), (D2, want2), (D1, want1)):
        for k in G:
            G[k].copy_(D[k])
        gbuf.x_compact.zero_()
        gbuf.new_active_idx.zero_()
        graph.replay()
        torch.cuda.synchronize()
        for k in outs:
            assert torch.equal(getattr(gbuf, k), want[k]), k
        other = eager(D2 if D is D1 else D1)        # eager work between the replays
        assert torch.equal(other["scores"], (want2 if D is D1 else want1)["scores"])
