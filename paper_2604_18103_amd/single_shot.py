"""Driver of the halting schedules over L full blocks: the single-shot schedule of Alg. 1 (one decision at the
start layer l_s) and multi-shot schedules (decisions at several blocks, App. D).

Every step of a block runs in the HIP library:
    q, k, v      = RMSNorm(H) W_q, W_k, W_v ; RoPE at the original positions        dash_rmsnorm_qkv, dash_rope_qk
    U, H~        = Attn(.) W_o, H + U                                                dash_flash_fwd + dash_wo_residual_rownorm,
                                                                                     or dash_attn_layer at l = l_s
    H_next       = H~ + FFN(LN(H~))                                                  dash_ffn_swiglu
At l = l_s the layer call also scores the rows (Eq. 2) and picks S* = TopK (Eq. 3). The block still finishes
on all rows (Alg. 1 step 7 comes before the selection takes effect); then the rows that halt are written to the
full-length result at their original positions (they keep their last updated state, Sec. 3.4) and the kept rows
are gathered for the blocks l > l_s. The survivors are written to the result after the last block. One 4-byte
read-back per decision sizes the later launches.
"""
from __future__ import annotations

import dataclasses

import torch

from . import binding as B


@dataclasses.dataclass
class BlockState:
    params: B.LayerParams
    m: int
    buf: B.LayerBuffers
    q: torch.Tensor
    k: torch.Tensor
    v: torch.Tensor
    h: torch.Tensor
    o: torch.Tensor
    partials: torch.Tensor
    chunk_counts: torch.Tensor
    x_a: torch.Tensor
    x_b: torch.Tensor
    ffn_ws: torch.Tensor
    qkv_ws: torch.Tensor
    idx0: torch.Tensor | None = None      # positions 0..N-1 of a full prompt, and two buffers for the
    idx_spare: list | None = None         # survivors' positions after successive decisions


def alloc_blocks(d, n_q_heads, n_kv_heads, head_dim, m, n_capacity, device="cuda") -> BlockState:
    p = B.make_params(d, n_q_heads, n_kv_heads, head_dim, dtype=B.DASH_BF16, causal=True, rule=B.RULE_NONE)
    bf = torch.bfloat16
    cap = int(n_capacity)
    return BlockState(
        params=p, m=int(m), buf=B.alloc_layer_buffers(p, cap, device=device),
        q=torch.empty((cap, n_q_heads, head_dim), dtype=bf, device=device),
        k=torch.empty((cap, n_kv_heads, head_dim), dtype=bf, device=device),
        v=torch.empty((cap, n_kv_heads, head_dim), dtype=bf, device=device),
        h=torch.empty((cap, d), dtype=bf, device=device),
        o=torch.empty((cap, n_q_heads * head_dim), dtype=bf, device=device),
        partials=torch.empty((B.norm_partials_per_row(p), cap, 2), dtype=torch.float32, device=device),
        chunk_counts=torch.empty(((cap + 63) // 64,), dtype=torch.int32, device=device),
        x_a=torch.empty((cap, d), dtype=bf, device=device),
        x_b=torch.empty((cap, d), dtype=bf, device=device),
        ffn_ws=torch.empty((max(B.ffn_workspace_bytes(p, cap, m), 256),), dtype=torch.uint8, device=device),
        qkv_ws=torch.empty((max(B.qkv_workspace_bytes(p, cap), 256),), dtype=torch.uint8, device=device))


def run_schedule(st: BlockState, x0: torch.Tensor, weights: list, shots: dict, rope_theta=None,
                 final: torch.Tensor | None = None, on_block=None, read_counts: bool = True) -> dict:
    """Run len(weights) blocks on x0 [N, d] (all N tokens active at the start). weights[l] = dict(w_q, w_k, w_v,
    w_o, w_gate_up, w_down) of device tensors (w_qkv = binding.concat_qkv(w_q, w_k, w_v) may replace the three). `shots` maps a block index to the number of rows kept after that
    block: one entry is the single-shot schedule of Alg. 1, several entries are a multi-shot schedule (every
    decision ranks the rows still active by their Delta_attn in that block), none is the full model. `final`
    [N, d] receives every token's last state. `on_block(l, x_in, idx, n, st, x_out)` is called after every block
    (after a device synchronisation) for checks. One 4-byte read-back per decision sizes the later launches;
    with read_counts = False the host does not wait for it and takes the requested count instead (TopK keeps
    exactly that many rows), so the whole schedule is enqueued without a host synchronisation and can be
    captured in a HIP graph (capture_schedule). Returns {n_after, final, idx}."""
    p, buf = st.params, st.buf
    N, d = x0.shape
    if not read_counts:
        if on_block is not None:
            raise ValueError("on_block needs the host to wait for every block: use read_counts=True")
        cur = N
        for l in sorted(shots):
            # TopK never halts a protected row: a smaller request would keep more rows than asked for
            if int(shots[l]) < min(cur, p.keep_first_n + p.keep_last_n) or int(shots[l]) < 0:
                raise ValueError(f"block {l}: cannot keep {shots[l]} of {cur} rows with the protected ranks")
            cur = min(int(shots[l]), cur)
    if final is None:
        final = torch.empty_like(x0)
    if st.idx0 is None or st.idx0.numel() != N:
        st.idx0 = torch.arange(N, dtype=torch.int32, device=x0.device)
        st.idx_spare = [torch.empty_like(st.idx0), torch.empty_like(st.idx0)]
    idx, idx_spare = st.idx0, st.idx_spare
    n_shot = 0
    x, n = x0, N
    spare = [st.x_a, st.x_b]
    for l, W in enumerate(weights):
        x_out = spare[l & 1]
        if "w_qkv" in W:      # one product over the concatenated weight
            B.dash_rmsnorm_qkv_fused(p, x, W["w_qkv"], n, st.q, st.k, st.v, st.h, st.qkv_ws)
        else:
            B.dash_rmsnorm_qkv(p, x, W["w_q"], W["w_k"], W["w_v"], n, st.q, st.k, st.v, st.h, st.qkv_ws)
        if rope_theta is not None:
            B.dash_rope_qk(p, st.q, st.k, idx, n, rope_theta)
        if l in shots:
            p.rule, p.k_keep = B.RULE_TOPK, int(shots[l])
            B.dash_attn_layer(p, x, st.q, st.k, st.v, W["w_o"], idx, n, buf)     # H~ in buf.x_next, mask, S*
            p.rule = B.RULE_NONE
            B.dash_ffn_swiglu(p, buf.x_next, W["w_gate_up"], W["w_down"], n, st.m, buf.x_next, st.ffn_ws)
            # the rows that halt now keep this state; the kept rows go on (gathered from the finished block)
            B.dash_scatter_rows(buf.x_next, idx, buf.halt_mask, 1, n, d, p.dtype, N, final)
            old_idx = idx
            idx = idx_spare[n_shot & 1]
            n_shot += 1
            B.dash_compact(p, buf.halt_mask, None, old_idx, buf.x_next, n, x_out, idx, buf.n_active_out,
                           buf.workspace)
            n_new = int(buf.n_active_out.item()) if read_counts else min(int(shots[l]), n)   # the one host read
            if on_block is not None:
                on_block(l, x, old_idx, n, st, buf.x_next)
            x, n = x_out, n_new
        else:
            B.dash_flash_fwd(p, st.q, st.k, st.v, idx, n, st.o)
            B.dash_wo_residual_rownorm(p, st.o, W["w_o"], x, n, x_out, st.partials, None, buf.workspace)
            B.dash_ffn_swiglu(p, x_out, W["w_gate_up"], W["w_down"], n, st.m, x_out, st.ffn_ws)
            if on_block is not None:
                torch.cuda.synchronize()
                on_block(l, x, idx, n, st, x_out)
            x = x_out
    B.dash_scatter_rows(x, idx, None, 0, n, d, p.dtype, N, final)
    return {"n_after": n, "final": final, "idx": idx}


class GraphedSchedule:
    """A whole schedule (every block, every decision, the final scatter) captured once in a HIP graph and
    replayed with one launch: with a short surviving sequence a block is a dozen launches of a few microseconds
    each, and enqueueing them one by one from the host takes longer than running them. The graph reads x0 and
    the weights at the addresses given at capture and writes `final`; new prompt contents are copied into x0
    before a replay. Valid while the BlockState, x0, the weights and `final` are alive and not reallocated."""

    def __init__(self, st: BlockState, x0: torch.Tensor, weights: list, shots: dict, rope_theta=None,
                 final: torch.Tensor | None = None):
        self.final = torch.empty_like(x0) if final is None else final
        args = dict(rope_theta=rope_theta, final=self.final, read_counts=False)
        B.init()                                               # one-time set-up of the library, outside the capture
        run_schedule(st, x0, weights, shots, **args)           # eager once: torch's own lazy set-up
        torch.cuda.synchronize()
        self.graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(self.graph):
            self.result = run_schedule(st, x0, weights, shots, **args)
        self.n_after = self.result["n_after"]
        self.idx = self.result["idx"]
        self._keep = (st, x0, weights)

    def replay(self) -> dict:
        self.graph.replay()
        return self.result


def run_single_shot(st: BlockState, x0: torch.Tensor, weights: list, l_s: int | None, k_keep: int,
                    rope_theta=None, final: torch.Tensor | None = None, on_block=None) -> dict:
    """Alg. 1: one decision after block l_s keeping k_keep rows; l_s = None runs the full model."""
    shots = {} if l_s is None else {int(l_s): int(k_keep)}
    return run_schedule(st, x0, weights, shots, rope_theta=rope_theta, final=final, on_block=on_block)


# Host arithmetic of App. A's cost model and of the schedules lives in the library (include/dash.h); these names
# are kept for the callers of this module.
block_cost = B.block_cost
schedule_lengths = B.schedule_lengths
comparable_multi_shot_ratio = B.comparable_multi_shot_ratio
