"""ctypes front end of the fp64 CPU oracle (oracle/dash_oracle.c).

Test infrastructure, not product code: only tests, the smoke check and the
CPU-baseline leg of the benchmark may import this module. It imports nothing
from the GPU package.

The functions mirror the steps of the layer in the paper's order
(Eq. 1 -> Sec. 3.1 residual -> Eq. 2 score -> Eq. 3 decision -> Alg. 1 step 4 gather);
`attn_layer` chains them. Inputs are whatever values the caller has (already
rounded to bf16 or fp32 if that is what the GPU sees); everything is upcast
exactly to fp64 here and no intermediate is rounded.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import numpy as np

from . import build as _build

SCORE_REL = 0  # ||U_t|| / ||H_t||  (the "relative" form named in the caption of Fig. 1)
SCORE_ABS = 1  # ||U_t||            (Eq. 2)

RULE_NONE = 0
RULE_THRESHOLD = 1
RULE_TOPK = 2

_lib = None


def _load():
    global _lib
    if _lib is not None:
        return _lib
    path = _build.LIB
    if not os.path.exists(path):
        path = _build.build_oracle(force=True)
    lib = C.CDLL(path)
    dp, i32p, i64p, u8p = (C.POINTER(C.c_double), C.POINTER(C.c_int32), C.POINTER(C.c_int64),
                           C.POINTER(C.c_uint8))
    lib.dash_oracle_num_threads.restype = C.c_int
    lib.dash_oracle_attention_rows.argtypes = [dp, dp, dp, i32p, C.c_int64, C.c_int32, C.c_int32,
                                               C.c_int32, C.c_int32, C.c_double, i64p, C.c_int64, dp]
    lib.dash_oracle_project.argtypes = [dp, dp, C.c_int64, C.c_int32, C.c_int32, dp]
    lib.dash_oracle_residual.argtypes = [dp, dp, C.c_int64, C.c_int32, dp]
    lib.dash_oracle_rmsnorm.argtypes = [dp, C.c_int64, C.c_int32, C.c_double, dp]
    lib.dash_oracle_rope.argtypes = [dp, i32p, C.c_int64, C.c_int32, C.c_int32, C.c_double, dp]
    lib.dash_oracle_ffn_swiglu.argtypes = [dp, dp, dp, dp, C.c_int64, C.c_int32, C.c_int32, C.c_double, dp]
    lib.dash_oracle_scatter_rows.argtypes = [dp, i32p, u8p, C.c_int32, C.c_int64, C.c_int32, C.c_int64, dp]
    lib.dash_oracle_scores.argtypes = [dp, dp, C.c_int64, C.c_int32, C.c_int32, dp]
    lib.dash_oracle_decide_threshold.argtypes = [dp, C.c_int64, C.c_double, C.c_int64, C.c_int64, u8p]
    lib.dash_oracle_decide_topk.argtypes = [dp, C.c_int64, C.c_int64, C.c_int64, C.c_int64, u8p]
    lib.dash_oracle_decide_topk_keep_low.argtypes = [dp, C.c_int64, C.c_int64, C.c_int64, C.c_int64, u8p]
    lib.dash_oracle_compact.argtypes = [u8p, i32p, dp, C.c_int64, C.c_int32, i32p, dp, i64p]
    lib.dash_oracle_keep_count.argtypes = [C.c_int64, C.c_double, C.c_int64, C.c_int64, C.c_int32]
    lib.dash_oracle_keep_count.restype = C.c_int64
    for name, nargs in (("dash_oracle_flops_A", 3), ("dash_oracle_flops_full", 4),
                        ("dash_oracle_flops_single_shot", 6)):
        fn = getattr(lib, name)
        fn.argtypes = [C.c_double] * nargs
        fn.restype = C.c_double
    _lib = lib
    return lib


def num_threads() -> int:
    return int(_load().dash_oracle_num_threads())


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def _ptr(a: np.ndarray, ctype):
    return a.ctypes.data_as(C.POINTER(ctype))


def _check(rc: int, what: str):
    if rc != 0:
        raise ValueError(f"oracle {what} failed with code {rc}")


def attention_rows(q, k, v, pos, rows=None, causal=True, scale=None) -> np.ndarray:
    """Eq. 1's Attn before the output projection, for the query rows in `rows`
    (default: all) against all keys. q [n,Hq,dh], k,v [n,Hkv,dh], pos [n] original
    positions. Returns [len(rows), Hq*dh] fp64."""
    q, k, v = _f64(q), _f64(k), _f64(v)
    n, Hq, dh = q.shape
    Hkv = k.shape[1]
    assert k.shape == (n, Hkv, dh) and v.shape == (n, Hkv, dh)
    pos = np.ascontiguousarray(np.asarray(pos, dtype=np.int32))
    assert pos.shape == (n,)
    rows = np.arange(n, dtype=np.int64) if rows is None else np.ascontiguousarray(np.asarray(rows, dtype=np.int64))
    if scale is None:
        scale = 1.0 / np.sqrt(float(dh))
    out = np.empty((rows.shape[0], Hq * dh), dtype=np.float64)
    rc = _load().dash_oracle_attention_rows(_ptr(q, C.c_double), _ptr(k, C.c_double), _ptr(v, C.c_double),
                                            _ptr(pos, C.c_int32), n, Hq, Hkv, dh, int(bool(causal)),
                                            float(scale), _ptr(rows, C.c_int64), rows.shape[0],
                                            _ptr(out, C.c_double))
    _check(rc, "attention_rows")
    return out


def project(O, w_o) -> np.ndarray:
    """U = O @ W_o with W_o [Da, d] (Sec. 3.1: attention output before the residual add)."""
    O, w_o = _f64(O), _f64(w_o)
    m, Da = O.shape
    assert w_o.shape[0] == Da
    d = w_o.shape[1]
    delta = np.empty((m, d), dtype=np.float64)
    _check(_load().dash_oracle_project(_ptr(O, C.c_double), _ptr(w_o, C.c_double), m, Da, d,
                                       _ptr(delta, C.c_double)), "project")
    return delta


def rmsnorm(x, eps=1e-6) -> np.ndarray:
    """LN of Eq. 1 as unit-gain RMS normalisation: x / sqrt(mean(x^2) + eps) per row."""
    x = _f64(x)
    m, d = x.shape
    out = np.empty_like(x)
    _check(_load().dash_oracle_rmsnorm(_ptr(x, C.c_double), m, d, float(eps), _ptr(out, C.c_double)), "rmsnorm")
    return out


def rope(u, pos, theta) -> np.ndarray:
    """Rotary position embedding (rotate-half pairing) of u [m, heads, dh] with original positions pos [m]."""
    u = _f64(u)
    m, heads, dh = u.shape
    pos = np.ascontiguousarray(pos, dtype=np.int32)
    assert pos.shape == (m,)
    out = np.empty_like(u)
    _check(_load().dash_oracle_rope(_ptr(u, C.c_double), _ptr(pos, C.c_int32), m, heads, dh, float(theta),
                                    _ptr(out, C.c_double)), "rope")
    return out


def rmsnorm_qkv(x, w_q, w_k, w_v, n_q_heads, n_kv_heads, head_dim, eps=1e-6, pos=None, rope_theta=None):
    """Front end of a layer in a chain: h = rmsnorm(x); q, k, v = h @ W_q, h @ W_k, h @ W_v; with
    rope_theta, q and k are then rotated by their original positions pos."""
    h = rmsnorm(x, eps)
    n = h.shape[0]
    q = project(h, w_q).reshape(n, n_q_heads, head_dim)
    k = project(h, w_k).reshape(n, n_kv_heads, head_dim)
    v = project(h, w_v).reshape(n, n_kv_heads, head_dim)
    if rope_theta is not None:
        q, k = rope(q, pos, rope_theta), rope(k, pos, rope_theta)
    return q, k, v


def ffn_swiglu(x, w_gate, w_up, w_down, eps=1e-6) -> np.ndarray:
    """Alg. 1 step 7: x + (silu(LN(x) W_gate) * (LN(x) W_up)) W_down."""
    x, w_gate, w_up, w_down = _f64(x), _f64(w_gate), _f64(w_up), _f64(w_down)
    rows, d = x.shape
    m = w_gate.shape[1]
    assert w_gate.shape == (d, m) and w_up.shape == (d, m) and w_down.shape == (m, d)
    out = np.empty_like(x)
    _check(_load().dash_oracle_ffn_swiglu(_ptr(x, C.c_double), _ptr(w_gate, C.c_double), _ptr(w_up, C.c_double),
                                          _ptr(w_down, C.c_double), rows, d, m, float(eps),
                                          _ptr(out, C.c_double)), "ffn_swiglu")
    return out


def scatter_rows(rows, idx, full, sel=None, sel_value=1) -> np.ndarray:
    """full[idx[t]] = rows[t] for the selected t (all if sel is None); returns the updated copy of full."""
    rows = _f64(rows)
    full = np.array(full, dtype=np.float64, order="C", copy=True)
    n, d = rows.shape
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    sp = None
    if sel is not None:
        sel = np.ascontiguousarray(sel, dtype=np.uint8)
        sp = _ptr(sel, C.c_uint8)
    _check(_load().dash_oracle_scatter_rows(_ptr(rows, C.c_double), _ptr(idx, C.c_int32), sp, int(sel_value), n, d,
                                            full.shape[0], _ptr(full, C.c_double)), "scatter_rows")
    return full


def residual(x, delta) -> np.ndarray:
    """H~ = H + U (Sec. 3.1, Alg. 1 step 6)."""
    x, delta = _f64(x), _f64(delta)
    assert x.shape == delta.shape
    m, d = x.shape
    out = np.empty_like(x)
    _check(_load().dash_oracle_residual(_ptr(x, C.c_double), _ptr(delta, C.c_double), m, d,
                                        _ptr(out, C.c_double)), "residual")
    return out


def scores(delta, x=None, kind=SCORE_REL) -> np.ndarray:
    """Eq. 2 (ABS) or its relative form (REL)."""
    delta = _f64(delta)
    m, d = delta.shape
    xs = _f64(x) if x is not None else None
    out = np.empty((m,), dtype=np.float64)
    xp = _ptr(xs, C.c_double) if xs is not None else None
    _check(_load().dash_oracle_scores(_ptr(delta, C.c_double), xp, m, d, int(kind),
                                      _ptr(out, C.c_double)), "scores")
    return out


def decide_threshold(s, tau, keep_first_n=0, keep_last_n=0) -> np.ndarray:
    s = _f64(s)
    halt = np.empty((s.shape[0],), dtype=np.uint8)
    _check(_load().dash_oracle_decide_threshold(_ptr(s, C.c_double), s.shape[0], float(tau),
                                                int(keep_first_n), int(keep_last_n),
                                                _ptr(halt, C.c_uint8)), "decide_threshold")
    return halt


def decide_topk(s, k_keep, keep_first_n=0, keep_last_n=0, keep_low=False) -> np.ndarray:
    """Eq. 3; keep_low=True is the direction control of Sec. 5.4 (the K LOWEST scores are kept)."""
    s = _f64(s)
    halt = np.empty((s.shape[0],), dtype=np.uint8)
    fn = _load().dash_oracle_decide_topk_keep_low if keep_low else _load().dash_oracle_decide_topk
    _check(fn(_ptr(s, C.c_double), s.shape[0], int(k_keep), int(keep_first_n), int(keep_last_n),
              _ptr(halt, C.c_uint8)), "decide_topk")
    return halt


def score_block(x_new, x_old, kind=SCORE_REL) -> np.ndarray:
    """The block-level signal of the ablation (Sec. 5.4): Eq. 2 applied to the change of the representation
    across the whole block, ||H^(l+1)_t - H^(l)_t||_2, optionally relative to ||H^(l)_t||_2."""
    x_new, x_old = _f64(x_new), _f64(x_old)
    return scores(x_new - x_old, x_old, kind)


def compact(halt, active_idx, x_next=None):
    """Stable gather of surviving rows (Alg. 1 step 4). Returns (new_idx, x_compact|None, n_out)."""
    halt = np.ascontiguousarray(np.asarray(halt, dtype=np.uint8))
    active_idx = np.ascontiguousarray(np.asarray(active_idx, dtype=np.int32))
    n = halt.shape[0]
    assert active_idx.shape == (n,)
    new_idx = np.empty((n,), dtype=np.int32)
    n_out = C.c_int64(0)
    if x_next is not None:
        xn = _f64(x_next)
        d = xn.shape[1]
        xc = np.empty_like(xn)
        xn_p, xc_p = _ptr(xn, C.c_double), _ptr(xc, C.c_double)
    else:
        d, xc, xn_p, xc_p = 1, None, None, None
    _check(_load().dash_oracle_compact(_ptr(halt, C.c_uint8), _ptr(active_idx, C.c_int32), xn_p, n, d,
                                       _ptr(new_idx, C.c_int32), xc_p, C.byref(n_out)), "compact")
    k = int(n_out.value)
    return new_idx[:k].copy(), (xc[:k].copy() if xc is not None else None), k


def keep_count(n, rho, keep_first_n=0, keep_last_n=0, paper_impl_rounding=False) -> int:
    return int(_load().dash_oracle_keep_count(int(n), float(rho), int(keep_first_n), int(keep_last_n),
                                              int(bool(paper_impl_rounding))))


def flops_A(n, d, m) -> float:
    return float(_load().dash_oracle_flops_A(float(n), float(d), float(m)))


def flops_reduction_and_speedup(n, n_hat, d, m, L, l_s):
    """(r_FLOPs, s_FLOPs) of App. A, Eq. 8-9."""
    lib = _load()
    full = lib.dash_oracle_flops_full(float(n), float(d), float(m), float(L))
    ours = lib.dash_oracle_flops_single_shot(float(n), float(n_hat), float(d), float(m), float(L), float(l_s))
    return 1.0 - ours / full, full / ours


def schedule_lengths(n, L, shots, n_first=0, n_last=0):
    """Sequence length each of the L blocks runs on when halting decisions are taken at several blocks.
    `shots` maps a block index to the compression ratio c applied to the rows that enter that block: the block
    itself still runs on all of them (Alg. 1 takes the decision after the block's FFN) and the blocks after it on
    the kept ones, whose number follows App. A's rule on the current length (protected first/last ranks in the
    current order). One entry at l_s is the single-shot schedule of Alg. 1."""
    lengths, cur = [], int(n)
    for l in range(int(L)):
        lengths.append(cur)
        if l in shots:
            cur = keep_count(cur, shots[l], n_first, n_last, paper_impl_rounding=True)
    return lengths


def schedule_flops(lengths, d, m) -> float:
    """Prefill FLOPs of a schedule under the per-block proxy A of App. A: the sum of A over the blocks' lengths
    (for one shot at l_s this is l_s A(n) + (L - l_s) A(n_hat))."""
    return float(sum(flops_A(t, d, m) for t in lengths))


def comparable_multi_shot_ratio(n, L, shot_layers, target_flops, d, m, n_first=0, n_last=0, grid=10000):
    """Per-shot compression ratio of a multi-shot schedule with a budget comparable to a single-shot one
    (App. D compares them under comparable pruning budgets without saying how the budget is split; reading:
    every shot uses the same ratio c, a multiple of 1/grid, and c is the smallest one whose schedule costs no
    more than `target_flops`). Plain scan over the grid."""
    for i in range(grid + 1):
        c = i / grid
        lengths = schedule_lengths(n, L, {l: c for l in shot_layers}, n_first, n_last)
        if schedule_flops(lengths, d, m) <= target_flops:
            return c
    raise ValueError("no ratio on the grid meets the budget")


@dataclass
class LayerResult:
    rows: np.ndarray          # query rows that were evaluated (indices into the active order)
    delta: np.ndarray         # [len(rows), d]
    x_next: np.ndarray        # [len(rows), d]
    scores: np.ndarray        # [len(rows)]
    halt: np.ndarray | None   # [n] uint8 (only when all rows were evaluated)
    new_active_idx: np.ndarray | None
    x_compact: np.ndarray | None
    n_active_out: int | None


def attn_layer(x, q, k, v, w_o, active_idx, *, causal=True, scale=None, score_kind=SCORE_REL,
               rule=RULE_THRESHOLD, tau=0.0, k_keep=None, keep_first_n=0, keep_last_n=0,
               rows=None) -> LayerResult:
    """One attention layer over the active tokens, then score, decision and compaction.

    With `rows` given only those query rows are evaluated (exact for them, since
    rows of attention are independent); decision and compaction need every row
    and are returned as None in that case.
    """
    x = _f64(x)
    n = x.shape[0]
    full = rows is None
    rows_arr = np.arange(n, dtype=np.int64) if full else np.asarray(rows, dtype=np.int64)
    O = attention_rows(q, k, v, active_idx, rows=rows_arr, causal=causal, scale=scale)
    delta = project(O, w_o)
    x_rows = x[rows_arr]
    x_next = residual(x_rows, delta)
    s = scores(delta, x_rows, kind=score_kind)
    if not full:
        return LayerResult(rows_arr, delta, x_next, s, None, None, None, None)
    if rule == RULE_NONE:
        halt = np.zeros((n,), dtype=np.uint8)
    elif rule == RULE_THRESHOLD:
        halt = decide_threshold(s, tau, keep_first_n, keep_last_n)
    elif rule == RULE_TOPK:
        halt = decide_topk(s, k_keep, keep_first_n, keep_last_n)
    else:
        raise ValueError("unknown rule")
    new_idx, xc, n_out = compact(halt, active_idx, x_next)
    return LayerResult(rows_arr, delta, x_next, s, halt, new_idx, xc, n_out)
