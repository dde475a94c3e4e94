"""MI355X-native hot path of DASH (Delta Attention Selective Halting).

One prefill self-attention layer over the still-active tokens: causal GQA flash
attention, the W_o projection fused with the residual update and row norms, the
per-token delta-attention score, the halting decision and the stream compaction.
All compute runs in hand-written HIP kernels (csrc/) behind a C-ABI library;
`binding` marshals torch device tensors into it.
"""
__all__ = ["inputs", "binding", "build"]
