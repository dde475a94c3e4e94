"""GPU parity at the sizes the benchmarks run, for the parts the small cases do not reach:
the TopK decision on 16384 ... 131072 rows (bit for bit against the oracle, integer work), the 8-layer chain of
benchmark configuration 4 from N = 32768 (teacher-forced, Alg. 1 steps 4-13), and the epilogues of the 256-row
GEMM tiles on every row of a product with more than 256 tiles."""
import time

import numpy as np
import pytest
import torch

from oracle import reference as ref
from paper_2604_18103_amd import binding as B
from paper_2604_18103_amd import chain as CH
from paper_2604_18103_amd import inputs as I

import parity_util as P

pytestmark = pytest.mark.gpu


def _dev(a):
    return B.to_device(a, B.DASH_BF16)


def _f(t):
    return t.float().cpu().numpy()


def _decide_and_compact(p, s, n, keep_low, idx):
    """dash_decide_topk then dash_compact (on a 16-byte row per token, so the gather is exercised as well)."""
    gs = torch.from_numpy(s).cuda()
    halt = torch.empty((n,), dtype=torch.uint8, device="cuda")
    counts = torch.empty(((n + 63) // 64,), dtype=torch.int32, device="cuda")
    ws = torch.empty((256 + 4 * ((n + 63) // 64) + 64,), dtype=torch.uint8, device="cuda")
    B.dash_decide_topk(p, gs, n, keep_low, halt, counts, ws)
    pc = B.make_params(8, 1, 1, 64)                       # rows of 8 bf16 = 16 bytes
    rows = torch.arange(n * 8, dtype=torch.float32, device="cuda").reshape(n, 8).to(torch.bfloat16)
    x_c = torch.empty_like(rows)
    new_idx = torch.empty((n,), dtype=torch.int32, device="cuda")
    n_out = torch.zeros((1,), dtype=torch.int32, device="cuda")
    B.dash_compact(pc, halt, counts, idx, rows, n, x_c, new_idx, n_out)
    torch.cuda.synchronize()
    k = int(n_out.item())
    return halt.cpu().numpy(), counts.cpu().numpy(), new_idx[:k].cpu().numpy(), k, x_c[:k], rows


@pytest.mark.parametrize("n", [16384, 32768, 52428, 131072])
def test_decide_topk_at_benchmark_sizes_bit_exact(n):
    """Eq. 3 on given fp32 scores at the row counts of the benchmark configurations: the mask, the kept counts per
    64-row chunk, the survivor count and the new index list equal the oracle's bit for bit. Scores with the
    workload's heavy tail (a lognormal row factor), with heavy ties (quantised), negative, and with the special
    values (NaN, signed zeros, infinities); no protection, a few protected ranks, and App. A's 64 + 32."""
    rng = np.random.default_rng(700 + n % 1000)
    p = B.make_params(256, 4, 2, 64)
    N = 4 * n
    idx_np = np.sort(rng.choice(N, size=n, replace=False)).astype(np.int32)
    idx = torch.from_numpy(idx_np).cuda()
    base = (np.abs(rng.standard_normal(n)) * np.exp(1.5 * rng.standard_normal(n))).astype(np.float32)
    cases = [
        ("heavy tail", base, (0, 0), B.keep_count_quantile(n, 0.2)),
        ("heavy tail, protected", base, (64, 32), B.keep_count(n, 0.667, 64, 32, paper_impl_rounding=True)),
        ("ties", (np.round(base * 4) / 4).astype(np.float32), (3, 2), n // 2),
        ("few values", rng.integers(0, 3, size=n).astype(np.float32), (64, 32), n // 3),
        ("negative", -base, (0, 0), n - 1),
        ("all equal", np.full(n, 0.25, dtype=np.float32), (0, 0), n // 7),
        ("keep none", base, (0, 0), 0),
        ("keep all", base, (0, 0), n),
        ("keep one", base, (0, 0), 1),
    ]
    special = base.copy()
    special[rng.choice(n, size=n // 50, replace=False)] = np.nan
    special[rng.choice(n, size=n // 50, replace=False)] = 0.0
    special[rng.choice(n, size=n // 50, replace=False)] = -0.0
    special[rng.choice(n, size=n // 100, replace=False)] = np.inf
    special[rng.choice(n, size=n // 100, replace=False)] = -np.inf
    nan_bits = special.view(np.uint32)
    nan_rows = np.nonzero(np.isnan(special))[0]
    nan_bits[nan_rows[::2]] = 0xFFC00001                  # negative NaNs with a payload rank like any NaN
    cases.append(("special values", special, (0, 0), n // 50 + n // 200))          # cuts inside the NaN rows ...
    cases.append(("special values, zeros", special, (5, 5), n - n // 100 - n // 50))   # ... and inside the zeros
    for name, s, (first, last), k_keep in cases:
        p.k_keep, p.keep_first_n, p.keep_last_n = int(k_keep), first, last
        for keep_low in (False, True):
            halt, counts, new_idx, k, x_c, rows = _decide_and_compact(p, s, n, keep_low, idx)
            want = ref.decide_topk(s.astype(np.float64), k_keep, first, last, keep_low=keep_low)
            np.testing.assert_array_equal(halt, want, err_msg=f"{name} keep_low={keep_low}")
            kept = (want == 0).astype(np.int64)
            np.testing.assert_array_equal(counts, np.add.reduceat(kept, np.arange(0, n, 64)), err_msg=name)
            want_idx, _, want_k = ref.compact(want, idx_np)
            assert k == want_k == max(int(k_keep), min(n, first + last)), name
            np.testing.assert_array_equal(new_idx, want_idx, err_msg=name)
            assert torch.equal(x_c, rows[torch.from_numpy(np.nonzero(want == 0)[0]).cuda()]), name


@pytest.mark.parametrize("n,rho_txt", [(1000, "0.2"), (1000, "0.4"), (100000, "0.2"), (100000, "0.4"),
                                       (1000, "0.667"), (16384, "0.667")])
def test_topk_keeps_floor_one_minus_rho_n_rows(n, rho_txt):
    """The rho form of Eq. 3 (k_keep < 0): K = floor((1 - rho) n) as exact arithmetic on the decimal gives it."""
    from fractions import Fraction
    want_k = int((1 - Fraction(rho_txt)) * n // 1)
    rng = np.random.default_rng(n)
    s = rng.random(n).astype(np.float32)
    p = B.make_params(256, 4, 2, 64, k_keep=-1, rho=float(rho_txt))
    idx = torch.arange(n, dtype=torch.int32, device="cuda")
    halt, counts, new_idx, k, _, _ = _decide_and_compact(p, s, n, False, idx)
    assert k == want_k == int((halt == 0).sum()) == int(counts.sum())
    np.testing.assert_array_equal(halt, ref.decide_topk(s.astype(np.float64), want_k))


# ------------------------------------------------------------ epilogues of the 256-row tiles, every row

N_ROWS_TILES = 4864          # 19 row tiles x 14 column tiles = 266 tiles: 256 whole tiles and 10 run as half tiles


def test_residual_norm_epilogue_of_whole_tiles_every_row():
    """W_o projection with 3584 output columns and a contraction of 256: x_next, delta (debug copy) and the row sums
    of squares on every one of the 4864 rows against the oracle's product."""
    n, hq, dh, d = N_ROWS_TILES, 2, 128, 3584
    rng = np.random.default_rng(801)
    o = I.round_to_bf16(rng.standard_normal((n, hq * dh)))
    w = I.round_to_bf16(rng.standard_normal((hq * dh, d)) / np.sqrt(hq * dh))
    x = I.round_to_bf16(rng.standard_normal((n, d)) * np.exp(0.7 * rng.standard_normal((n, 1))))
    p = B.make_params(d, hq, hq, dh)
    P_ = B.norm_partials_per_row(p)
    delta = ref.project(o, w)
    want = ref.residual(x, delta)
    go, gw, gx = _dev(o), _dev(w), _dev(x)
    outs = []
    for with_delta in (False, True):
        xn = torch.empty((n, d), dtype=torch.bfloat16, device="cuda")
        parts = torch.full((P_, n, 2), float("nan"), dtype=torch.float32, device="cuda")
        dd = torch.full((n, d), float("nan"), dtype=torch.float32, device="cuda") if with_delta else None
        B.dash_wo_residual_rownorm(p, go, gw, gx, n, xn, parts, dd, None)
        torch.cuda.synchronize()
        sums = parts.double().sum(dim=0).cpu().numpy()                # no NaN left: every slot written
        assert P.row_rel_err(_f(xn), want).max() <= P.X_TOL["bf16"]
        np.testing.assert_allclose(sums[:, 0], (delta ** 2).sum(axis=1), rtol=1e-4)
        np.testing.assert_allclose(sums[:, 1], (x ** 2).sum(axis=1), rtol=1e-5)
        if with_delta:
            got = dd.cpu().numpy()
            # fp32 accumulation of 256 exact bf16 products
            assert np.abs(got - delta).max() <= 1e-5 * np.abs(delta).max()
            upd = _f(xn).astype(np.float64) - x
            assert np.all(np.abs(upd - delta) <= 2.0 ** -8 * np.abs(want) + 1e-5 * np.abs(delta).max())
        outs.append((xn, parts))
    assert torch.equal(outs[0][0], outs[1][0]) and torch.equal(outs[0][1], outs[1][1])


@pytest.mark.parametrize("k_steps", [1, 2, 3, 4, 5, 7])
def test_products_with_few_k_steps_through_whole_and_half_tiles(k_steps):
    """The operand pipeline of the product kernel: the 256-row tiles keep two stages of operand tiles and request two
    K steps ahead, the 128-row half tiles three stages and three steps ahead; prologue, steady state and the last
    steps without requests all change with the number of K steps. A contraction of 1 ... 7 steps of 64, 512 output
    columns and 33280 + 100 rows (260 whole tiles: 256 run as 256-row tiles, the rest and the ragged last row tile as
    half tiles): delta on every row against the oracle's product, element by element."""
    hq, dh, d = k_steps, 64, 512
    n = 256 * 130 + 100
    rng = np.random.default_rng(810 + k_steps)
    o = I.round_to_bf16(rng.standard_normal((n, hq * dh)))
    w = I.round_to_bf16(rng.standard_normal((hq * dh, d)) / np.sqrt(hq * dh))
    x = I.round_to_bf16(rng.standard_normal((n, d)))
    p = B.make_params(d, hq, hq, dh)
    P_ = B.norm_partials_per_row(p)
    delta = ref.project(o, w)
    xn = torch.empty((n, d), dtype=torch.bfloat16, device="cuda")
    parts = torch.full((P_, n, 2), float("nan"), dtype=torch.float32, device="cuda")
    dd = torch.full((n, d), float("nan"), dtype=torch.float32, device="cuda")
    B.dash_wo_residual_rownorm(p, _dev(o), _dev(w), _dev(x), n, xn, parts, dd, None)
    torch.cuda.synchronize()
    got = dd.cpu().numpy()
    assert np.abs(got - delta).max() <= 1e-5 * np.abs(delta).max()      # fp32 sums of exact bf16 products
    assert P.row_rel_err(_f(xn), ref.residual(x, delta)).max() <= P.X_TOL["bf16"]
    sums = parts.double().sum(dim=0).cpu().numpy()
    np.testing.assert_allclose(sums[:, 0], (delta ** 2).sum(axis=1), rtol=1e-4)


def test_gated_epilogue_of_whole_tiles_every_row():
    """Feed-forward with hidden 256 and width 1792: the gate/up product has 3584 columns (266 tiles, gating in the
    epilogue of 256-row tiles); every row against the oracle."""
    n, d, m = N_ROWS_TILES, 256, 1792
    cfg = I.LayerConfig("ffn_tiles", "bf16", n, n, d, 2, 2, 128, 0.3, seed=802)
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
    # the update itself: what is left of it after x_out was rounded to bf16 (half a step of |x_out|) agrees with the
    # oracle's update to 2e-2 of the row's largest update
    upd, upd_want = _f(out).astype(np.float64) - x, want - x
    assert np.all(np.abs(upd - upd_want) <= 2.0 ** -8 * np.abs(want) + 2e-2 * np.abs(upd_want).max(axis=1, keepdims=True))
    # the gated activations themselves (the epilogue's output), every row: a = silu(h W_gate) * (h W_up)
    h = ref.rmsnorm(x)
    gate, up = ref.project(I.round_to_bf16(h), W["w_gate"]), ref.project(I.round_to_bf16(h), W["w_up"])
    act_want = gate / (1.0 + np.exp(-gate)) * up
    act = ws[n * d * 2:][: n * m * 2].view(torch.bfloat16).reshape(n, m)     # second region of the workspace
    assert (n * d * 2) % 256 == 0
    assert P.row_rel_err(_f(act), act_want).max() <= 1e-2


def test_store_and_routing_epilogues_of_whole_tiles_every_row():
    """Front end with hidden 256, 20 query and 4 key/value heads of 128: the q product has 190 tiles (all whole),
    the product over [w_q | w_k | w_v] 3584 columns = 266 tiles with k and v starting inside a column tile; every
    row of q, k, v against the oracle, and both ways bit-identical."""
    n, d, hq, hkv, dh = N_ROWS_TILES, 256, 20, 4, 128
    cfg = I.LayerConfig("qkv_tiles", "bf16", n, n, d, hq, hkv, dh, 0.3, seed=803)
    x = I.make_hidden(cfg)
    W = I.make_projection_weights(cfg, 0)
    p = P.params_for(cfg)
    mk = lambda heads: torch.full((n, heads, dh), float("nan"), dtype=torch.bfloat16, device="cuda")
    q, k, v, q2, k2, v2 = mk(hq), mk(hkv), mk(hkv), mk(hq), mk(hkv), mk(hkv)
    h = torch.empty((n, d), dtype=torch.bfloat16, device="cuda")
    gx = _dev(x)
    B.dash_rmsnorm_qkv(p, gx, _dev(W["w_q"]), _dev(W["w_k"]), _dev(W["w_v"]), n, q, k, v, h)
    B.dash_rmsnorm_qkv_fused(p, gx, B.concat_qkv(_dev(W["w_q"]), _dev(W["w_k"]), _dev(W["w_v"])), n, q2, k2, v2, h)
    torch.cuda.synchronize()
    oq, ok, ov = ref.rmsnorm_qkv(x, W["w_q"], W["w_k"], W["w_v"], hq, hkv, dh)
    for got, got2, want in ((q, q2, oq), (k, k2, ok), (v, v2, ov)):
        assert P.row_rel_err(_f(got).reshape(n, -1), want.reshape(n, -1)).max() <= 2e-2
        assert torch.equal(got, got2)


# ------------------------------------------------------------ benchmark configuration 4 at its real size

def test_chain_of_eight_layers_from_32768_teacher_forced():
    """Eight attention-only layers from N = 32768 with the lowest 20 % of the scores halted after every layer
    (on-device TopK), rotary embedding at the original positions. Teacher-forced: at every layer the oracle gets
    the GPU's actual layer input, q/k/v and active set. Per layer: the front end, x_next, delta-free score and
    halt flag on 256 sampled rows (against all keys); the TopK decision, chunk counts, survivor count and new
    index list in full, bit for bit, on the GPU's own scores; compaction as the stable gather of the GPU's mask;
    the active set only shrinks and halted tokens never return. The free-running survivor counts are printed."""
    cfg = I.CONFIGS["qwen_32k_chain"]
    n_layers, theta, n_sample = 8, 1.0e6, 256
    t_start = time.perf_counter()
    weights_np = [I.make_projection_weights(cfg, l) for l in range(n_layers)]
    weights = []
    for W in weights_np:
        weights.append({"w_qkv": B.concat_qkv(_dev(W["w_q"]), _dev(W["w_k"]), _dev(W["w_v"])), "w_o": _dev(W["w_o"])})
    state = CH.alloc_chain(cfg.d, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.n)
    x0 = _dev(I.make_hidden(cfg))
    idx0 = torch.from_numpy(I.make_active_idx(cfg.N, cfg.n, cfg.seed)).cuda()
    seen = {"prev": None, "halted": np.zeros(cfg.N, dtype=bool), "band": 0, "oracle_s": 0.0, "xerr": 0.0, "serr": 0.0}

    def check(l, x, idx, n, q, k, v, buf):
        W = weights_np[l]
        idx_np = idx[:n].cpu().numpy()
        rows = I.sample_rows(n, n_sample, seed=cfg.seed + l, tile=256)
        sel = torch.from_numpy(rows).cuda()
        k_keep = B.keep_count_quantile(n, cfg.halt_frac)
        assert k_keep == n - int(np.floor(cfg.halt_frac * n))
        # front end on the sampled rows
        xs = _f(x[:n][sel])
        oq, ok, ov = ref.rmsnorm_qkv(xs, W["w_q"], W["w_k"], W["w_v"], cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim,
                                     pos=idx_np[rows], rope_theta=theta)
        for got, want in ((q, oq), (k, ok), (v, ov)):
            assert P.row_rel_err(_f(got[:n][sel]).reshape(len(rows), -1), want.reshape(len(rows), -1)).max() <= 2e-2
        # the path proper on the sampled rows, on the values the GPU kernels consumed
        t0 = time.perf_counter()
        O = ref.attention_rows(_f(q[:n]), _f(k[:n]), _f(v[:n]), idx_np, rows=rows)
        delta = ref.project(O, W["w_o"])
        x_next = ref.residual(xs, delta)
        s = ref.scores(delta, xs)
        seen["oracle_s"] += time.perf_counter() - t0
        xerr = P.row_rel_err(_f(buf.x_next[:n][sel]), x_next)
        assert xerr.max() <= P.X_TOL["bf16"], (l, xerr.max())
        gpu_scores = buf.scores[:n].cpu().numpy()
        serr = P.check_scores(cfg, gpu_scores[rows], s)
        seen["xerr"], seen["serr"] = max(seen["xerr"], float(xerr.max())), max(seen["serr"], float(serr.max()))
        # the decision in full on the GPU's own scores: integer work, bit for bit
        halt = buf.halt_mask[:n].cpu().numpy()
        want_halt = ref.decide_topk(gpu_scores.astype(np.float64), k_keep)
        np.testing.assert_array_equal(halt, want_halt)
        n_out = int(buf.n_active_out.item())
        want_idx, _, want_n = ref.compact(want_halt, idx_np)
        assert n_out == want_n == k_keep
        new_idx = buf.new_active_idx[:n_out].cpu().numpy()
        np.testing.assert_array_equal(new_idx, want_idx)
        # on the sampled rows the oracle's own scores give the same flags outside the band around the cut
        thr = np.sort(gpu_scores)[::-1][k_keep - 1]
        band = np.abs(s - thr) <= P.BAND_REL * thr
        assert np.array_equal(halt[rows][~band], (s < thr).astype(np.uint8)[~band])
        seen["band"] += int(band.sum())
        # compaction: bitwise copies of the kept rows, in order
        kept = torch.from_numpy(np.nonzero(halt == 0)[0]).cuda()
        assert torch.equal(buf.x_compact[:n_out], buf.x_next[:n][kept])
        # the active set only shrinks; halted tokens never return
        if seen["prev"] is not None:
            np.testing.assert_array_equal(idx_np, seen["prev"])
        assert not seen["halted"][new_idx].any()
        seen["halted"][idx_np[halt == 1]] = True
        seen["prev"] = new_idx

    recs = CH.run_chain(state, x0, idx0, cfg.n, weights, cfg.halt_frac, on_layer=check, rope_theta=theta)
    ns = [r["n_in"] for r in recs] + [recs[-1]["n_out"]]
    assert ns == [32768, 26215, 20972, 16778, 13423, 10739, 8592, 6874, 5500], ns
    print("chain n_active:", ns, "band rows on the samples:", seen["band"], f"x_next err {seen['xerr']:.2e}",
          f"score err {seen['serr']:.2e}", f"oracle {seen['oracle_s']:.1f} s", f"total {time.perf_counter() - t_start:.1f} s")
