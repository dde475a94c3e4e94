"""Front end (RMSNorm + q/k/v projections, rotary embedding) and the layer chain with halting after every layer."""
import numpy as np
import pytest
import torch

from oracle import reference as ref
from paper_2604_18103_amd import binding as B
from paper_2604_18103_amd import chain as CH
from paper_2604_18103_amd import inputs as I

import parity_util as P

pytestmark = pytest.mark.gpu

CFG = I.LayerConfig("chain_small", "bf16", 900, 900, 512, 4, 2, 128, 0.2, seed=31)


def _dev(a):
    return B.to_device(a, B.DASH_BF16)


@pytest.mark.parametrize("d", [512, 2560, 4160], ids=lambda v: "d%d" % v)
def test_rmsnorm_qkv_matches_oracle(d):
    """Rows of 512, 2560 and 4160 elements: held in registers (4 or 8 chunks of 512) or read twice."""
    cfg = I.scaled(CFG, 333 if d == 512 else 70, N=333, d=d)
    x = I.make_hidden(cfg)
    W = I.make_projection_weights(cfg, 0)
    p = P.params_for(cfg)
    n = cfg.n
    q = torch.empty((n, cfg.n_q_heads, cfg.head_dim), dtype=torch.bfloat16, device="cuda")
    k = torch.empty((n, cfg.n_kv_heads, cfg.head_dim), dtype=torch.bfloat16, device="cuda")
    v = torch.empty_like(k)
    h = torch.empty((n, cfg.d), dtype=torch.bfloat16, device="cuda")
    B.dash_rmsnorm_qkv(p, _dev(x), _dev(W["w_q"]), _dev(W["w_k"]), _dev(W["w_v"]), n, q, k, v, h)
    torch.cuda.synchronize()
    oq, ok, ov = ref.rmsnorm_qkv(x, W["w_q"], W["w_k"], W["w_v"], cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim)
    for got, want in ((q, oq), (k, ok), (v, ov)):
        err = P.row_rel_err(got.float().cpu().numpy().reshape(n, -1), want.reshape(n, -1))
        assert err.max() <= 2e-2, err.max()
    herr = P.row_rel_err(h.float().cpu().numpy(), ref.rmsnorm(x))
    assert herr.max() <= 8e-3          # one bf16 rounding
    # the same as one product over [w_q | w_k | w_v] (k and v start inside a 256-column tile when Hq*dh is not a
    # multiple of 256), without and with scratch for splitting along K
    wqkv = B.concat_qkv(_dev(W["w_q"]), _dev(W["w_k"]), _dev(W["w_v"]))
    for ws in (None, torch.empty((max(B.qkv_workspace_bytes(p, n), 256),), dtype=torch.uint8, device="cuda")):
        q2, k2, v2 = torch.full_like(q, float("nan")), torch.full_like(k, float("nan")), torch.full_like(v, float("nan"))
        B.dash_rmsnorm_qkv_fused(p, _dev(x), wqkv, n, q2, k2, v2, h, ws)
        torch.cuda.synchronize()
        for got, want in ((q2, oq), (k2, ok), (v2, ov)):
            err = P.row_rel_err(got.float().cpu().numpy().reshape(n, -1), want.reshape(n, -1))
            assert err.max() <= 2e-2, err.max()
        if ws is None:                 # same tiles, same order of additions: the same bits as three products
            assert torch.equal(q2, q) and torch.equal(k2, k) and torch.equal(v2, v)


@pytest.mark.parametrize("shape", [(28, 4, 128), (6, 3, 64), (5, 1, 128), (8, 8, 64)], ids=lambda t: "hq%d_hkv%d_dh%d" % t)
def test_rope_qk_matches_oracle(shape):
    """In-place rotary embedding of q and k with original positions up to 131071 (config 5's prompt length):
    fp64 angles in the kernel, so the only rounding left is that of the bf16 outputs."""
    hq, hkv, dh = shape
    n, N = 517, 131072
    rng = np.random.default_rng(40 + hq)
    pos = np.sort(rng.choice(N, size=n, replace=False)).astype(np.int32)
    pos[0], pos[-1] = 0, N - 1
    q = I.round_to_bf16(rng.standard_normal((n, hq, dh)))
    k = I.round_to_bf16(rng.standard_normal((n, hkv, dh)) * 3.0)
    p = B.make_params(hq * dh, hq, hkv, dh)
    gq, gk = _dev(q), _dev(k)
    B.dash_rope_qk(p, gq, gk, torch.from_numpy(pos).cuda(), n, 1.0e6)
    torch.cuda.synchronize()
    for got, src in ((gq, q), (gk, k)):
        want = ref.rope(src, pos, 1.0e6)
        g = got.float().cpu().numpy()
        half = dh // 2
        mag = np.abs(src[..., :half]) + np.abs(src[..., half:])        # |a| + |b| bounds each output
        mag = np.concatenate([mag, mag], axis=-1)
        assert np.all(np.abs(g - want) <= 2.0 ** -8 * mag + 1e-30), float(np.abs(g - want).max())
    assert np.array_equal(gq[0].float().cpu().numpy(), q[0])                # position 0: untouched


@pytest.mark.parametrize("rope_theta", [None, 1.0e6], ids=["no_rope", "rope"])
def test_chain_teacher_forced_against_oracle(rope_theta):
    """Four layers; at every layer the oracle is run on the GPU's actual layer input and active set, so
    band flips cannot compound. Also: the active set only shrinks, halted tokens never return, TopK keeps
    exactly k_keep."""
    cfg = CFG
    n_layers = 4
    weights_np = [I.make_projection_weights(cfg, l) for l in range(n_layers)]
    weights = [{k: _dev(v) for k, v in W.items()} for W in weights_np]
    if rope_theta is not None:            # this variant runs the front end as one product over [w_q | w_k | w_v]
        for W in weights:
            W["w_qkv"] = B.concat_qkv(W["w_q"], W["w_k"], W["w_v"])
    state = CH.alloc_chain(cfg.d, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.n)
    x0 = _dev(I.make_hidden(cfg))
    idx0 = torch.from_numpy(I.make_active_idx(cfg.N, cfg.n, cfg.seed)).cuda()
    seen = {"prev": set(idx0.cpu().numpy().tolist()), "halted": set(), "band": 0}

    def check(l, x, idx, n, q, k, v, buf):
        f = lambda t: t.float().cpu().numpy()
        xs, qs, ks, vs = f(x[:n]), f(q[:n]), f(k[:n]), f(v[:n])
        idx_np = idx[:n].cpu().numpy()
        W = weights_np[l]
        # front end of this layer
        oq, ok, ov = ref.rmsnorm_qkv(xs, W["w_q"], W["w_k"], W["w_v"], cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim,
                                     pos=idx_np, rope_theta=rope_theta)
        assert P.row_rel_err(qs.reshape(n, -1), oq.reshape(n, -1)).max() <= 2e-2
        assert P.row_rel_err(ks.reshape(n, -1), ok.reshape(n, -1)).max() <= 2e-2
        assert P.row_rel_err(vs.reshape(n, -1), ov.reshape(n, -1)).max() <= 2e-2
        # the path proper, on the values the GPU kernels actually consumed
        k_keep = n - int(cfg.halt_frac * n)
        o = ref.attn_layer(xs, qs, ks, vs, W["w_o"], idx_np, rule=ref.RULE_TOPK, k_keep=k_keep)
        n_out = int(buf.n_active_out.item())
        g = P.GpuResult(f(buf.x_next[:n]), buf.scores[:n].cpu().numpy(), buf.halt_mask[:n].cpu().numpy(),
                        f(buf.x_compact[:n_out]), buf.new_active_idx[:n_out].cpu().numpy(), n_out, None)
        P.check_self_consistency(g, idx_np, n)
        assert n_out == k_keep == o.n_active_out
        assert P.row_rel_err(g.x_next, o.x_next).max() <= P.X_TOL["bf16"]
        thr = np.sort(o.scores)[::-1][k_keep - 1]
        band = np.abs(o.scores - thr) <= P.BAND_REL * thr
        assert np.array_equal(g.halt[~band], o.halt[~band])
        seen["band"] += int(band.sum())
        cur = set(g.new_active_idx.tolist())
        assert cur <= seen["prev"] and not (cur & seen["halted"])
        seen["halted"] |= seen["prev"] - cur
        seen["prev"] = cur

    recs = CH.run_chain(state, x0, idx0, cfg.n, weights, cfg.halt_frac, on_layer=check, rope_theta=rope_theta)
    ns = [r["n_in"] for r in recs] + [recs[-1]["n_out"]]
    assert all(a > b for a, b in zip(ns, ns[1:])), ns
    print("chain n_active:", ns, "band rows:", seen["band"])
