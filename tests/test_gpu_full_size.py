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
