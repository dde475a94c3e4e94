#!/usr/bin/env python3
"""Benchmark of the DASH hot path on one MI355X.

A step = one pass of the whole path (flash attention over the active rows, W_o + residual + row
norms, score + halting decision, stream compaction) over one batch of synthetic input already
resident in HBM. Prints ONE JSON line:
  value     active tokens/s of the whole step (headline workload: Qwen2.5-7B-shaped layer, N=32K, 50% active)
  roofline  the dominant kernel (flash attention forward) against the dense bf16 MFMA peak, its
            duration measured with HIP events on the launch stream inside the timed region
  cpu_baseline  the fp64 CPU oracle timed on a bounded row sample of the same workload
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16
HBM_PEAK_GBS = 8000.0
# HBM-side bytes per launch of the dominant kernel, from rocprofv3 FETCH_SIZE + WRITE_SIZE scaled by a
# copy kernel of known size (see profiles/hbm_traffic_and_pipe_counters_qwen_32k_half.md); offline
# measurements, so only the workload they were taken on has one.
FLASH_TRAFFIC_BYTES = {"qwen_32k_half": 398e6 + 117e6}


def measure_mfma_peak(seconds_per_case=0.25):
    """What the matrix pipe sustains on this machine with nothing else running: the library's register-only MFMA loop
    (dash_mfma_probe: no memory traffic, 8 waves per compute unit) in the two instruction shapes the kernels use,
    on zero operands (the published peak's conditions) and on N(0,1) operands (the workloads' data: the part
    lowers its clock under the power the operand bits draw). TFLOP/s per case, each from one launch of about
    `seconds_per_case` timed with events on the launch stream."""
    import torch
    from paper_2604_18103_amd import binding as B
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    sink = torch.empty((cus * 512,), dtype=torch.float32, device="cuda")
    out = {}
    for shape, sname in ((0, "32x32x16"), (1, "16x16x32")):
        for normal, dname in ((False, "zeros"), (True, "normal")):
            B.dash_mfma_probe(shape, normal, 20000, cus, sink)          # warm-up, and a first rate estimate
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            flops = B.dash_mfma_probe(shape, normal, 20000, cus, sink)
            e1.record()
            torch.cuda.synchronize()
            rate = flops / (e0.elapsed_time(e1) * 1e-3)
            iters = max(20000, min(4000000, int(20000 * seconds_per_case * rate / flops)))
            e0.record()
            flops = B.dash_mfma_probe(shape, normal, iters, cus, sink)
            e1.record()
            torch.cuda.synchronize()
            out[f"{sname}_{dname}"] = flops / (e0.elapsed_time(e1) * 1e-3) / 1e12
    return out


def run_mfma_peak_bench(args):
    """`--workload mfma_peak`: the probe alone, one second per case."""
    peak = measure_mfma_peak(1.0)
    best = peak["32x32x16_zeros"]
    print(json.dumps({
        "metric": "sustained bf16 MFMA rate of a register-only loop (32x32x16, zero operands)",
        "value": best, "unit": "TFLOP/s", "n_gpus": 1, "steps": 1, "warmup": 1, "ms_per_step": 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "mfma_peak"},
        "roofline": {"bound": "mfma", "achieved": best, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": best / MFMA_BF16_PEAK_TFLOPS, "traffic": None},
        "measured_peak_tflops": peak}))


def attention_flops(cfg, n):
    pairs = n * (n + 1) / 2 if cfg.causal else n * n
    return 4.0 * cfg.head_dim * cfg.n_q_heads * pairs


def wo_flops(cfg, n):
    return 2.0 * n * cfg.D_a * cfg.d


def score_compact_bytes(cfg, n, n_kept, partials_per_row, elem):
    """Algorithmic HBM bytes of score+decision and compaction: per active row one pair of norm partials per 256
    output columns read (`partials_per_row` of them: what the GEMM epilogue writes per row),
    score (4) and mask (1) written, index (4) read; per kept row the hidden row read and written plus the index
    written."""
    per_row = 8 * ((cfg.d + 255) // 256) + 4 + 1 + 4
    per_kept = 2 * cfg.d * elem + 4
    return n * per_row + n_kept * per_kept


def cpu_baseline(cfg, L, rows_target=3072, full=False):
    """The oracle as it stands on a bounded uniform sample of query rows (cost per row grows with its
    rank, so a uniform sample gives the mean per-row cost); all keys/values, full layer per row. full=True times
    every row of the configuration instead (a minute or more of CPU work at the headline size)."""
    import numpy as np
    from oracle import reference as ref
    n = cfg.n
    rng = np.random.default_rng(12345)
    rows = np.arange(n) if full else np.sort(rng.choice(n, size=min(rows_target, n), replace=False))
    t0 = time.perf_counter()
    ref.attn_layer(L["x"], L["q"], L["k"], L["v"], L["w_o"], L["active_idx"], causal=cfg.causal, rows=rows)
    dt = time.perf_counter() - t0
    what = (f"the FULL configuration: all {n} query rows" if len(rows) == n else
            f"SAMPLED, not the full configuration: {len(rows)} uniformly sampled query rows of the same workload")
    return {"value": len(rows) / dt, "unit": "active tokens/s", "cores": ref.num_threads(), "kind": "oracle",
            "sampled": len(rows) != n,
            "sample": f"{what} against all {n} keys/values, full layer per row, {dt:.1f} s; tokens/s = rows / seconds"}


def run_chain_bench(args, cfg, n_layers=8):
    """Eight attention-only layers (RMSNorm + q/k/v projections + rotary embedding at the original positions
    + the layer step), halting the lowest 20 %
    of the active scores after every layer (on-device TopK), the compacted output of one layer feeding the
    next. A step = the whole chain; per-layer n_active and time are reported."""
    import numpy as np
    import torch
    from paper_2604_18103_amd import binding as B
    from paper_2604_18103_amd import chain as CH
    from paper_2604_18103_amd import inputs as I

    weights = []
    for l in range(n_layers):
        W = {k: B.to_device(v, B.DASH_BF16) for k, v in I.make_projection_weights(cfg, l).items()}
        weights.append({"w_qkv": B.concat_qkv(W["w_q"], W["w_k"], W["w_v"]), "w_o": W["w_o"]})
    x0 = B.to_device(I.make_hidden(cfg), B.DASH_BF16)
    idx0 = torch.from_numpy(I.make_active_idx(cfg.N, cfg.n, cfg.seed)).cuda()
    state = CH.alloc_chain(cfg.d, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.n)
    rope_theta = 1.0e6   # Qwen2.5
    for _ in range(max(1, args.warmup)):
        CH.run_chain(state, x0, idx0, cfg.n, weights, cfg.halt_frac, rope_theta=rope_theta)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        CH.run_chain(state, x0, idx0, cfg.n, weights, cfg.halt_frac, rope_theta=rope_theta)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    layers = CH.run_chain(state, x0, idx0, cfg.n, weights, cfg.halt_frac, time_layers=True, rope_theta=rope_theta)
    flops = 0.0
    for r in layers:
        n = r["n_in"]
        r["flops"] = (attention_flops(cfg, n) + wo_flops(cfg, n)
                      + 2.0 * n * cfg.d * (cfg.D_a + 2 * cfg.n_kv_heads * cfg.head_dim))
        r["tflops"] = r["flops"] / (r["ms"] * 1e-3) / 1e12
        flops += r["flops"]
    tokens = sum(r["n_in"] for r in layers)
    ms = 1e3 * elapsed / args.steps
    print(json.dumps({
        "metric": "active tokens/s over a chain of 8 attention-only layers with halting after every layer, "
                  "Qwen2.5-7B-shaped, N=32768",
        "value": tokens / (elapsed / args.steps), "unit": "active tokens/s (sum over layers)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": cfg.name, "N": cfg.N, "layers": n_layers, "halt_frac_per_layer": cfg.halt_frac,
                   "hidden": cfg.d, "q_heads": cfg.n_q_heads, "kv_heads": cfg.n_kv_heads, "head_dim": cfg.head_dim,
                   "rope_theta": rope_theta},
        "chain_tflops": flops / (ms * 1e-3) / 1e12,
        "roofline": {"bound": "mfma", "achieved": flops / (ms * 1e-3) / 1e12, "peak": MFMA_BF16_PEAK_TFLOPS,
                     "unit": "TFLOP/s", "frac": flops / (ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, "traffic": None},
        "layers": layers}))


QWEN_BLOCKS = dict(L=28, m=18944, start_block=11, first=64, last=32, rope_theta=1.0e6)   # App. A's setting


def _blocks_setup(cfg):
    """Synthetic weights of 28 Qwen2.5-7B-shaped blocks (generated on the device), the prompt's hidden rows and
    the buffers of the schedule driver."""
    import torch
    from paper_2604_18103_amd import binding as B
    from paper_2604_18103_amd import inputs as I
    from paper_2604_18103_amd import single_shot as SS

    L, m = QWEN_BLOCKS["L"], QWEN_BLOCKS["m"]
    N, d, dh, Hq, Hkv = cfg.N, cfg.d, cfg.head_dim, cfg.n_q_heads, cfg.n_kv_heads
    g = torch.Generator(device="cuda").manual_seed(cfg.seed)
    bf = torch.bfloat16

    def rnd(rows, cols, fan):
        return (torch.randn((rows, cols), generator=g, device="cuda", dtype=torch.float32) * fan ** -0.5).to(bf)

    weights = []
    for _ in range(L):
        weights.append(dict(w_qkv=B.concat_qkv(rnd(d, Hq * dh, d), rnd(d, Hkv * dh, d), rnd(d, Hkv * dh, d)),
                            w_o=rnd(Hq * dh, d, d), w_down=rnd(m, d, m),
                            w_gate_up=B.interleave_gate_up(rnd(d, m, d), rnd(d, m, d))))
    x0 = B.to_device(I.make_hidden(cfg), B.DASH_BF16)
    st = SS.alloc_blocks(d, Hq, Hkv, dh, m, N)
    st.params.keep_first_n, st.params.keep_last_n = QWEN_BLOCKS["first"], QWEN_BLOCKS["last"]
    final = torch.empty_like(x0)

    def timed(shots, reps, warm, graph=False):
        """Mean seconds of one prefill under the schedule `shots` {block: rows kept after it}: every launch
        enqueued from the host, or (graph) the whole schedule captured once in a HIP graph and replayed."""
        kw = dict(rope_theta=QWEN_BLOCKS["rope_theta"], final=final)
        if graph:
            gs = SS.GraphedSchedule(st, x0, weights, shots, **kw)
            run = gs.replay
        else:
            run = lambda: SS.run_schedule(st, x0, weights, shots, **kw)
        for _ in range(warm):
            run()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            res = run()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / reps, res

    def block_flops(n):   # what the kernels execute: causal attention, GQA projections, three FFN matrices
        return (attention_flops(cfg, n) + wo_flops(cfg, n) + 2.0 * n * d * (Hq + 2 * Hkv) * dh + 6.0 * n * d * m)

    return timed, block_flops


def run_single_shot_bench(args, cfg):
    """The single-shot schedule of Alg. 1 end to end on synthetic weights, in the setting of the paper's table of
    theoretical prefill FLOPs (App. A): Qwen2.5-7B shapes, L = 28 blocks, hidden 3584, FFN width 18944, decision
    after the 11th block, reduction ratio 0.667 with 64 + 32 protected tokens. A step = one whole prefill with
    halting; the full model (no halting) is timed beside it and the ratio reported next to the paper's analytic
    one."""
    from paper_2604_18103_amd import binding as B
    from paper_2604_18103_amd import single_shot as SS

    L, m, start_block, first, last = (QWEN_BLOCKS[k] for k in ("L", "m", "start_block", "first", "last"))
    rho = 0.667
    N, d, dh, Hq, Hkv = cfg.N, cfg.d, cfg.head_dim, cfg.n_q_heads, cfg.n_kv_heads
    k_keep = B.keep_count(N, rho, first, last, paper_impl_rounding=True)
    timed, block_flops = _blocks_setup(cfg)
    t_dash, res = timed({start_block - 1: k_keep}, args.steps, max(1, args.warmup))
    assert res["n_after"] == k_keep
    t_full, _ = timed({}, max(2, args.steps // 4), 1)
    paper_A = lambda n: SS.block_cost(n, d, m)       # App. A: A(n) = 4 n d^2 + 2 n^2 d + 2 n d m
    flops_full = L * block_flops(N)
    flops_dash = start_block * block_flops(N) + (L - start_block) * block_flops(k_keep)
    print(json.dumps({
        "metric": "prompt tokens/s of a 28-block prefill with single-shot halting after block 11 "
                  "(Qwen2.5-7B shapes, N=32768, 66.7 % of the unprotected tokens halted)",
        "value": N / t_dash, "unit": "prompt tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": 1e3 * t_dash, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": "qwen_32k_single_shot", "N": N, "blocks": L, "start_block": start_block,
                   "reduction_ratio": rho, "protected": [first, last], "n_kept": k_keep, "hidden": d, "ffn": m,
                   "q_heads": Hq, "kv_heads": Hkv, "head_dim": dh, "rope_theta": QWEN_BLOCKS["rope_theta"]},
        "full_model_ms": 1e3 * t_full, "speedup_vs_full_model": t_full / t_dash,
        "speedup_of_executed_flops": flops_full / flops_dash,
        "speedup_paper_formula": L * paper_A(N) / (start_block * paper_A(N) + (L - start_block) * paper_A(k_keep)),
        "roofline": {"bound": "mfma", "achieved": flops_dash / t_dash / 1e12, "peak": MFMA_BF16_PEAK_TFLOPS,
                     "unit": "TFLOP/s", "frac": flops_dash / t_dash / 1e12 / MFMA_BF16_PEAK_TFLOPS, "traffic": None},
        "full_model_tflops": flops_full / t_full / 1e12}))


def run_schedule_sweep_bench(args, cfg, workload):
    """Two sweeps over halting schedules of the 28-block model, every schedule timed end to end beside the full
    model:
      qwen_32k_multi_shot   1-, 2-, 3- and 4-shot schedules under the same App. A budget as the single shot
                            (same per-shot ratio, smallest one on a 1e-4 grid whose cost does not exceed it)
      qwen_vl_8k_extreme    one shot at the reduction ratios of the paper's vision-language table (75 % ... 99 %) on
                            an 8192-token prompt (Qwen2-VL-7B has the shapes of Qwen2.5-7B): short surviving
                            sequences, where launch gaps and occupancy, not the matrix pipe, set the time
    A step = one prefill under the first schedule of the sweep, replayed from a HIP graph that holds the whole
    schedule (the launch-by-launch time is reported beside it); `value` is its prompt tokens/s."""
    from paper_2604_18103_amd import single_shot as SS

    L, m, start_block, first, last = (QWEN_BLOCKS[k] for k in ("L", "m", "start_block", "first", "last"))
    N, d = cfg.N, cfg.d
    l0 = start_block - 1                      # index of the block after which the first decision is taken
    if workload == "qwen_32k_multi_shot":
        single = sum(SS.block_cost(t, d, m) for t in SS.schedule_lengths(N, L, {l0: 0.667}, first, last))
        plans = []
        for layers in ([l0], [l0, 18], [l0, 15, 21], [l0, 14, 18, 22]):
            c = SS.comparable_multi_shot_ratio(N, L, layers, single, d, m, first, last)
            plans.append((f"{len(layers)}-shot", layers, c))
    else:
        plans = [(f"{100 * c:.2f} % halted", [l0], c) for c in (0.75, 0.8889, 0.9375, 0.96, 0.99)]
    timed, block_flops = _blocks_setup(cfg)
    t_full, _ = timed({}, max(2, args.steps // 2), 1, graph=True)
    rows = []
    for name, layers, c in plans:
        lengths = SS.schedule_lengths(N, L, {l: c for l in layers}, first, last)
        shots = {l: lengths[l + 1] for l in layers}
        t_eager, res = timed(shots, args.steps, max(1, args.warmup))
        assert res["n_after"] == lengths[-1]
        t, _ = timed(shots, args.steps, max(1, args.warmup), graph=True)
        flops = sum(block_flops(t_) for t_ in lengths)
        rows.append({"schedule": name, "decision_after_blocks": [l + 1 for l in layers], "ratio_per_shot": c,
                     "rows_per_block": sorted(set(lengths), reverse=True), "ms": 1e3 * t,
                     "ms_launch_by_launch": 1e3 * t_eager,
                     "speedup_vs_full_model": t_full / t,
                     "speedup_of_executed_flops": L * block_flops(N) / flops,
                     "speedup_paper_formula": L * SS.block_cost(N, d, m) / sum(SS.block_cost(t_, d, m) for t_ in lengths),
                     "tflops": flops / t / 1e12,
                     "ms_per_block_after_last_decision": 1e3 * (t - t_full * (layers[-1] + 1) / L) / (L - layers[-1] - 1)
                     if len(layers) == 1 else None})
    t0 = rows[0]["ms"] * 1e-3
    print(json.dumps({
        "metric": "prompt tokens/s of a 28-block prefill under the first schedule of the sweep "
                  f"({rows[0]['schedule']}), Qwen2.5-7B shapes, N={N}",
        "value": N / t0, "unit": "prompt tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": 1e3 * t0, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": workload, "N": N, "blocks": L, "protected": [first, last], "hidden": d, "ffn": m,
                   "q_heads": cfg.n_q_heads, "kv_heads": cfg.n_kv_heads, "head_dim": cfg.head_dim,
                   "rope_theta": QWEN_BLOCKS["rope_theta"]},
        "full_model_ms": 1e3 * t_full, "full_model_tflops": L * block_flops(N) / t_full / 1e12,
        "roofline": {"bound": "mfma", "achieved": rows[0]["tflops"], "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": rows[0]["tflops"] / MFMA_BF16_PEAK_TFLOPS, "traffic": None},
        "schedules": rows}))


def run_aux_kernels_bench(args, cfg):
    """The HBM-bound kernels beside the layer, each launched 50 times back to back between two events on operands
    that rotate over three buffers (more than the last-level cache holds): the standalone score of Eq. 2 from a
    stored delta, the block-level signal of the ablation (Sec. 5.4), the scatter of halted rows, the rotary
    embedding, and the TopK decision on given scores (latency-bound: microseconds only). Sizes of the headline
    workload (16384 active rows of a 32768-token prompt, hidden 3584). `value` is the mean fraction of the HBM peak
    over the four bandwidth-bound kernels."""
    import torch
    from paper_2604_18103_amd import binding as B

    n, N, d, Hq, Hkv, dh = cfg.n, cfg.N, cfg.d, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    p = B.make_params(d, Hq, Hkv, dh, causal=True, rule=B.RULE_TOPK, k_keep=B.keep_count_quantile(n, cfg.halt_frac))
    g = torch.Generator(device="cuda").manual_seed(cfg.seed)
    bf = torch.bfloat16
    rnd = lambda *shape: torch.randn(shape, generator=g, device="cuda", dtype=torch.float32)
    xs = [rnd(n, d).to(bf) for _ in range(3)]
    ys = [(xs[i].float() + 0.05 * rnd(n, d)).to(bf) for i in range(3)]
    deltas = [rnd(n, d) for _ in range(3)]
    fulls = [torch.empty((N, d), dtype=bf, device="cuda") for _ in range(3)]
    qs = [rnd(n, Hq, dh).to(bf) for _ in range(3)]
    ks = [rnd(n, Hkv, dh).to(bf) for _ in range(3)]
    idx = torch.sort(torch.randperm(N, generator=g, device="cuda")[:n]).values.to(torch.int32)
    scores = torch.empty((n,), dtype=torch.float32, device="cuda")
    halt = torch.empty((n,), dtype=torch.uint8, device="cuda")
    counts = torch.empty(((n + 63) // 64,), dtype=torch.int32, device="cuda")
    ws = torch.empty((256 + 4 * ((n + 63) // 64) + 64,), dtype=torch.uint8, device="cuda")
    reps = 50

    def timed(fn):
        for i in range(5):
            fn(i)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for i in range(reps):
            fn(i)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps * 1e3     # microseconds per launch

    cases = [
        ("score_rows_kernel (Eq. 2 from stored fp32 delta and x)", n * d * (4 + 2) + 4 * n,
         lambda i: B.dash_score_rows(deltas[i % 3], xs[i % 3], n, d, B.DASH_BF16, B.SCORE_REL, scores)),
        ("score_diff_rows_kernel (block-level signal)", n * d * (2 + 2) + 4 * n,
         lambda i: B.dash_score_diff_rows(ys[i % 3], xs[i % 3], n, d, B.DASH_BF16, B.SCORE_REL, scores)),
        ("scatter_rows_kernel (all rows to their original positions)", 2 * n * d * 2 + 4 * n,
         lambda i: B.dash_scatter_rows(xs[i % 3], idx, None, 0, n, d, B.DASH_BF16, N, fulls[i % 3])),
        ("rope_qk_kernel (q and k in place)", 2 * n * (Hq + Hkv) * dh * 2 + 4 * n,
         lambda i: B.dash_rope_qk(p, qs[i % 3], ks[i % 3], idx, n, 1.0e6)),
    ]
    rows = []
    for name, nbytes, fn in cases:
        us = timed(fn)
        rows.append({"kernel": name, "bytes": nbytes, "us": us, "GB/s": nbytes / us / 1e3,
                     "frac_of_hbm_peak": nbytes / us / 1e3 / HBM_PEAK_GBS})
    B.dash_score_rows(deltas[0], xs[0], n, d, B.DASH_BF16, B.SCORE_REL, scores)
    us_topk = timed(lambda i: B.dash_decide_topk(p, scores, n, False, halt, counts, ws))
    rows.append({"kernel": "topk_decide_small_kernel (TopK decision on 16384 given scores, one launch)",
                 "bytes": 4 * n * 2 + n, "us": us_topk, "GB/s": None, "frac_of_hbm_peak": None})
    mean_frac = sum(r["frac_of_hbm_peak"] for r in rows[:4]) / 4
    print(json.dumps({
        "metric": "mean fraction of the HBM peak over the bandwidth-bound kernels beside the layer",
        "value": mean_frac, "unit": "fraction of 8 TB/s", "n_gpus": 1, "steps": reps, "warmup": 5,
        "ms_per_step": sum(r["us"] for r in rows) * 1e-3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": "aux_kernels", "N": N, "n_active": n, "hidden": d, "q_heads": Hq, "kv_heads": Hkv,
                   "head_dim": dh},
        "roofline": {"bound": "hbm", "achieved": mean_frac * HBM_PEAK_GBS, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": mean_frac, "traffic": None},
        "kernels": rows}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="qwen_32k_half",
                    help="a key of paper_2604_18103_amd.inputs.CONFIGS (single-layer workloads; qwen_32k_chain is "
                         "the 8-layer chain), qwen_32k_single_shot (28 full blocks, one halting decision), "
                         "qwen_32k_multi_shot (1- to 4-shot schedules under one budget) or qwen_vl_8k_extreme "
                         "(one shot, 75 % to 99 % of the tokens halted), aux_kernels (the bandwidth-bound kernels "
                         "beside the layer, one by one) or mfma_peak (the register-only MFMA probe alone)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-baseline-full", action="store_true",
                    help="time the oracle on every row of the configuration instead of a 3072-row sample")
    ap.add_argument("--copy-calibration-mib", type=int, default=0,
                    help="also run device-to-device copies of this many MiB (a plain copy kernel of known "
                         "size, to scale rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
              "(no collectives or sharding are part of it).", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2604_18103_amd import binding as B
    from paper_2604_18103_amd import inputs as I

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    B.lib()  # fail loudly if the HIP library is missing
    if args.workload == "qwen_32k_single_shot":
        run_single_shot_bench(args, I.CONFIGS["qwen_32k_chain"])
        return
    if args.workload == "mfma_peak":
        run_mfma_peak_bench(args)
        return
    if args.workload == "aux_kernels":
        run_aux_kernels_bench(args, I.CONFIGS["qwen_32k_half"])
        return
    if args.workload == "qwen_32k_multi_shot":
        run_schedule_sweep_bench(args, I.CONFIGS["qwen_32k_chain"], args.workload)
        return
    if args.workload == "qwen_vl_8k_extreme":
        run_schedule_sweep_bench(args, I.scaled(I.CONFIGS["qwen_32k_chain"], 8192, N=8192), args.workload)
        return
    cfg = I.CONFIGS[args.workload]
    if args.workload == "qwen_32k_chain":
        run_chain_bench(args, cfg)
        return
    dt_code = B.DASH_BF16 if cfg.dtype == "bf16" else B.DASH_F32
    elem = 2 if cfg.dtype == "bf16" else 4
    L = I.make_layer_inputs(cfg)
    D = {k: B.to_device(L[k], dt_code) for k in ("x", "q", "k", "v", "w_o")}
    D["active_idx"] = torch.from_numpy(L["active_idx"]).cuda()
    n = cfg.n

    def params(**kw):
        return B.make_params(cfg.d, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, dtype=dt_code,
                             causal=cfg.causal, **kw)

    # tau at the workload's percentile of the active-token scores (one untimed pass, no halting)
    buf = B.alloc_layer_buffers(params(), n)
    B.dash_attn_layer(params(rule=B.RULE_NONE), D["x"], D["q"], D["k"], D["v"], D["w_o"], D["active_idx"], n, buf)
    torch.cuda.synchronize()
    tau, h = I.percentile_tau(buf.scores[:n].cpu().numpy(), cfg.halt_frac)
    p = params(rule=B.RULE_THRESHOLD, tau=tau)

    stream = torch.cuda.current_stream()
    for _ in range(args.warmup):
        B.dash_attn_layer(p, D["x"], D["q"], D["k"], D["v"], D["w_o"], D["active_idx"], n, buf)
    profiles = [B.Profile() for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        B.dash_attn_layer(p, D["x"], D["q"], D["k"], D["v"], D["w_o"], D["active_idx"], n, buf, profiles[s])
    stream.synchronize()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    n_kept = int(buf.n_active_out.item())

    if args.copy_calibration_mib > 0:
        src = torch.empty(args.copy_calibration_mib << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()

    # The two small stages again, on their own: 100 back-to-back launch pairs between two events, the rows they
    # gather rotating over three copies (3 x n x d x elem bytes, more than the 256 MB last-level cache), so the
    # figure carries neither the event overhead of the in-step intervals nor cache-resident rows.
    P_ = B.norm_partials_per_row(p)
    partials = torch.empty((P_, n, 2), dtype=torch.float32, device="cuda")
    o = torch.empty((n, cfg.D_a), dtype=buf.x_next.dtype, device="cuda")
    rot = [torch.empty_like(buf.x_next) for _ in range(3)]
    rot_out = [torch.empty_like(buf.x_compact) for _ in range(3)]
    counts = torch.empty(((n + 63) // 64,), dtype=torch.int32, device="cuda")
    B.dash_flash_fwd(p, D["q"], D["k"], D["v"], D["active_idx"], n, o)
    B.dash_wo_residual_rownorm(p, o, D["w_o"], D["x"], n, rot[0], partials, None, buf.workspace)
    rot[1].copy_(rot[0])
    rot[2].copy_(rot[0])
    pairs = 100
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for i in range(pairs + 5):
        if i == 5:
            ev0.record()
        B.dash_score_decide(p, partials, n, buf.scores, buf.halt_mask, counts, buf.workspace)
        B.dash_compact(p, buf.halt_mask, counts, D["active_idx"], rot[i % 3], n, rot_out[i % 3], buf.new_active_idx,
                       buf.n_active_out, buf.workspace)
    ev1.record()
    torch.cuda.synchronize()
    loop_ms = ev0.elapsed_time(ev1) / pairs
    assert int(buf.n_active_out.item()) == n_kept

    stage_ms = np.array([pr.read_ms() for pr in profiles])       # [steps, 4]
    mean_ms = stage_ms.mean(axis=0)
    ms_per_step = 1e3 * elapsed / args.steps
    fa_tflops = attention_flops(cfg, n) / (mean_ms[0] * 1e-3) / 1e12
    wo_tflops = wo_flops(cfg, n) / (mean_ms[1] * 1e-3) / 1e12
    both_tflops = (attention_flops(cfg, n) + wo_flops(cfg, n)) / ((mean_ms[0] + mean_ms[1]) * 1e-3) / 1e12
    sc_bytes = score_compact_bytes(cfg, n, n_kept, B.norm_partials_per_row(p), elem)
    sc_gbs = sc_bytes / ((mean_ms[2] + mean_ms[3]) * 1e-3) / 1e9

    peak = measure_mfma_peak()        # after the timed region: what the matrix pipe sustains on this machine
    out = {
        "metric": "active tokens/s, one DASH attention layer step (attention + W_o/residual + score/halting "
                  "+ compaction), Qwen2.5-7B-shaped layer" if args.workload.startswith("qwen")
                  else "active tokens/s, one DASH attention layer step",
        "value": n / (elapsed / args.steps),
        "unit": "active tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": cfg.name, "N": cfg.N, "n_active": n, "hidden": cfg.d,
                   "q_heads": cfg.n_q_heads, "kv_heads": cfg.n_kv_heads, "head_dim": cfg.head_dim,
                   "causal": cfg.causal, "halt_frac": cfg.halt_frac, "n_kept": n_kept, "tau": tau},
        "roofline": {"kernel": "flash_fwd_mfma", "bound": "mfma", "achieved": fa_tflops,
                     "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": fa_tflops / MFMA_BF16_PEAK_TFLOPS,
                     "traffic": FLASH_TRAFFIC_BYTES.get(cfg.name),
                     "traffic_source": "offline constant: rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE runs of this "
                                       "command, scaled by a copy of known size (profiles/); not measured in this run",
                     "algorithmic_flops_per_launch": attention_flops(cfg, n),
                     "kernel_ms": float(mean_ms[0]),
                     "measured_peak": peak,
                     "measured_peak_note": "TFLOP/s of a register-only MFMA loop on this box, measured in this run: "
                                           "zero operands reach the published peak, N(0,1) operands (the workload's "
                                           "data) hold the part at its power limit",
                     "frac_of_measured_peak_on_normal_data": fa_tflops / peak["32x32x16_normal"]},
        "stages_ms": dict(zip(B.STAGE_NAMES, [float(v) for v in mean_ms])),
        "roofline_wo": {"kernel": "gemm_mfma_kernel", "bound": "mfma", "achieved": wo_tflops,
                        "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                        "frac": wo_tflops / MFMA_BF16_PEAK_TFLOPS,
                        "frac_of_measured_peak_on_normal_data": wo_tflops / peak["16x16x32_normal"]},
        "roofline_attn_plus_wo": {"bound": "mfma", "achieved": both_tflops, "peak": MFMA_BF16_PEAK_TFLOPS,
                                  "unit": "TFLOP/s", "frac": both_tflops / MFMA_BF16_PEAK_TFLOPS},
        "roofline_score_compact": {"bound": "hbm", "achieved": sc_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                   "frac": sc_gbs / HBM_PEAK_GBS, "bytes": sc_bytes,
                                   "timing": "event interval around the one launch (scores, decision, compaction) inside "
                                             "the timed steps, launch gap and event records included",
                                   "loop": {"launch_pairs": pairs, "ms_per_pair": loop_ms,
                                            "achieved": sc_bytes / (loop_ms * 1e-3) / 1e9,
                                            "frac": sc_bytes / (loop_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                                            "timing": "score+decision and compaction launched back to back 100 "
                                                      "times between two events, gathered rows rotating over "
                                                      "three buffers (larger than the last-level cache)"}},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, L, full=args.cpu_baseline_full)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
