"""Chain of attention-only layers with halting after every layer (a multi-shot schedule).

Host driver only: every step runs in the HIP kernels behind the C ABI. Per layer l:
    q, k, v = RMSNorm(x_l) W_q, W_k, W_v          dash_rmsnorm_qkv   (LN of Eq. 1 and the projections)
    q, k    = RoPE(q, k; original positions S_l)  dash_rope_qk       (optional: rope_theta)
    x_next, scores, halt, x_{l+1}, S_{l+1}, n_{l+1} = dash_attn_layer(..., rule = TOPK, k_keep = n_l - floor(f n_l))
The compacted output of one layer is the input of the next (Alg. 1 step 4); the survivor count is read back
once per layer (4 bytes) to size the next launch.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import torch

from . import binding as B


@dataclass
class ChainState:
    n_capacity: int
    params: B.LayerParams
    bufs: list            # two LayerBuffers, ping-pong: layer l writes bufs[l & 1]
    q: torch.Tensor
    k: torch.Tensor
    v: torch.Tensor
    h: torch.Tensor
    qkv_ws: torch.Tensor
    per_layer: list = field(default_factory=list)


def alloc_chain(d, n_q_heads, n_kv_heads, head_dim, n_capacity, device="cuda") -> ChainState:
    p = B.make_params(d, n_q_heads, n_kv_heads, head_dim, dtype=B.DASH_BF16, causal=True, rule=B.RULE_TOPK)
    bf = torch.bfloat16
    return ChainState(
        n_capacity=n_capacity, params=p,
        bufs=[B.alloc_layer_buffers(p, n_capacity, device=device) for _ in range(2)],
        q=torch.empty((n_capacity, n_q_heads, head_dim), dtype=bf, device=device),
        k=torch.empty((n_capacity, n_kv_heads, head_dim), dtype=bf, device=device),
        v=torch.empty((n_capacity, n_kv_heads, head_dim), dtype=bf, device=device),
        h=torch.empty((n_capacity, d), dtype=bf, device=device),
        qkv_ws=torch.empty((max(B.qkv_workspace_bytes(p, n_capacity), 256),), dtype=torch.uint8, device=device))


def run_chain(state: ChainState, x0: torch.Tensor, active_idx0: torch.Tensor, n0: int, weights: list,
              halt_frac: float, on_layer=None, time_layers=False, rope_theta=None) -> list:
    """Run len(weights) layers. weights[l] = dict(w_q, w_k, w_v, w_o) or dict(w_qkv, w_o) of device tensors.
    Returns per-layer dicts {n_in, n_out, ms}. `on_layer(l, x, idx, n, q, k, v, buf)` is called after each
    layer (after a device synchronisation) with that layer's inputs and outputs, for checks.
    With rope_theta, q and k get the backbone's rotary embedding at the tokens' original positions."""
    p = state.params
    x, idx, n = x0, active_idx0, int(n0)
    out = []
    for l, W in enumerate(weights):
        buf = state.bufs[l & 1]
        p.k_keep = B.keep_count_quantile(n, halt_frac)        # halt the floor(f n) lowest scores
        if time_layers:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
        if "w_qkv" in W:      # one product over the concatenated weight
            B.dash_rmsnorm_qkv_fused(p, x, W["w_qkv"], n, state.q, state.k, state.v, state.h, state.qkv_ws)
        else:
            B.dash_rmsnorm_qkv(p, x, W["w_q"], W["w_k"], W["w_v"], n, state.q, state.k, state.v, state.h, state.qkv_ws)
        if rope_theta is not None:
            B.dash_rope_qk(p, state.q, state.k, idx, n, rope_theta)
        B.dash_attn_layer(p, x, state.q, state.k, state.v, W["w_o"], idx, n, buf)
        if time_layers:
            e1.record()
        n_out = int(buf.n_active_out.item())      # the one host read per layer (synchronises)
        rec = dict(layer=l, n_in=n, n_out=n_out, k_keep=int(p.k_keep))
        if time_layers:
            rec["ms"] = float(e0.elapsed_time(e1))
        if on_layer is not None:
            on_layer(l, x, idx, n, state.q, state.k, state.v, buf)
        out.append(rec)
        x, idx, n = buf.x_compact, buf.new_active_idx, n_out
    state.per_layer = out
    return out
