"""Thin ctypes binding of libdash.so: argument marshalling only.

Every step of the path runs in the HIP kernels behind the C ABI (include/dash.h);
torch is used for device memory and streams. There is no CPU fallback: if the
library is missing or cannot be loaded, importing the symbols raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libdash.so")

DASH_BF16, DASH_F32 = 0, 1
RULE_NONE, RULE_THRESHOLD, RULE_TOPK = 0, 1, 2
SCORE_REL, SCORE_ABS = 0, 1
N_STAGES = 4
STAGE_NAMES = ("flash_fwd", "wo_residual_rownorm", "score_decide", "compact")
CHUNK_ROWS = 64


class DashError(RuntimeError):
    pass


class LayerParams(C.Structure):
    _fields_ = [("d", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("dtype", C.c_int32), ("causal", C.c_int32),
                ("softmax_scale", C.c_float), ("rule", C.c_int32), ("score_kind", C.c_int32),
                ("tau", C.c_float), ("k_keep", C.c_int32), ("rho", C.c_double),
                ("keep_first_n", C.c_int32), ("keep_last_n", C.c_int32)]


_lib = None
_vp = C.c_void_p


def lib() -> C.CDLL:
    """Load libdash.so (built in-tree by paper_2604_18103_amd.build). Fails loudly if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise DashError(f"{LIB_PATH} not found: build it with `python -m paper_2604_18103_amd.build` "
                        "(there is no fallback path)")
    L = C.CDLL(LIB_PATH)
    pp = C.POINTER(LayerParams)
    L.dash_status_string.restype = C.c_char_p
    L.dash_status_string.argtypes = [C.c_int]
    L.dash_version.restype = C.c_char_p
    L.dash_keep_count.restype = C.c_int64
    L.dash_keep_count.argtypes = [C.c_int64, C.c_double, C.c_int32, C.c_int32, C.c_int32]
    L.dash_init.restype = C.c_int
    L.dash_init.argtypes = []
    L.dash_keep_count_quantile.restype = C.c_int64
    L.dash_keep_count_quantile.argtypes = [C.c_int64, C.c_double]
    L.dash_block_cost.restype = C.c_double
    L.dash_block_cost.argtypes = [C.c_double] * 3
    L.dash_schedule_lengths.restype = C.c_int
    L.dash_schedule_lengths.argtypes = [C.c_int64, C.c_int32, C.POINTER(C.c_int32), C.POINTER(C.c_double), C.c_int32,
                                        C.c_int32, C.c_int32, C.POINTER(C.c_int64)]
    L.dash_schedule_cost.restype = C.c_double
    L.dash_schedule_cost.argtypes = [C.POINTER(C.c_int64), C.c_int32, C.c_double, C.c_double]
    L.dash_comparable_multi_shot_ratio.restype = C.c_double
    L.dash_comparable_multi_shot_ratio.argtypes = [C.c_int64, C.c_int32, C.POINTER(C.c_int32), C.c_int32, C.c_double,
                                                   C.c_double, C.c_double, C.c_int32, C.c_int32, C.c_int32]
    L.dash_layer_flops.restype = C.c_double
    L.dash_layer_flops.argtypes = [pp, C.c_int64]
    L.dash_norm_partials_per_row.restype = C.c_int32
    L.dash_norm_partials_per_row.argtypes = [pp]
    L.dash_workspace_bytes.restype = C.c_size_t
    L.dash_workspace_bytes.argtypes = [pp, C.c_int32]
    L.dash_profile_create.restype = _vp
    L.dash_profile_create.argtypes = []
    L.dash_profile_destroy.restype = None
    L.dash_profile_destroy.argtypes = [_vp]
    L.dash_profile_read.argtypes = [_vp, C.POINTER(C.c_float)]
    L.dash_attn_layer.argtypes = [pp] + [_vp] * 6 + [C.c_int32] + [_vp] * 8 + [C.c_size_t, _vp, _vp]
    L.dash_flash_fwd.argtypes = [pp, _vp, _vp, _vp, _vp, C.c_int32, _vp, _vp]
    L.dash_wo_residual_rownorm.argtypes = [pp, _vp, _vp, _vp, C.c_int32, _vp, _vp, _vp, _vp, C.c_size_t, _vp]
    L.dash_score_decide.argtypes = [pp, _vp, C.c_int32, _vp, _vp, _vp, _vp, C.c_size_t, _vp]
    L.dash_compact.argtypes = [pp, _vp, _vp, _vp, _vp, C.c_int32, _vp, _vp, _vp, _vp, C.c_size_t, _vp]
    L.dash_score_rows.argtypes = [_vp, _vp, C.c_int32, C.c_int32, C.c_int32, C.c_int32, _vp, _vp]
    L.dash_rmsnorm_qkv.argtypes = [pp, _vp, _vp, _vp, _vp, C.c_int32, _vp, _vp, _vp, _vp, _vp, C.c_size_t, _vp]
    L.dash_rmsnorm_qkv_fused.argtypes = [pp, _vp, _vp, C.c_int32, _vp, _vp, _vp, _vp, _vp, C.c_size_t, _vp]
    L.dash_rmsnorm_qkv_fused.restype = C.c_int
    L.dash_qkv_workspace_bytes.restype = C.c_size_t
    L.dash_qkv_workspace_bytes.argtypes = [pp, C.c_int32]
    L.dash_rope_qk.argtypes = [pp, _vp, _vp, _vp, C.c_int32, C.c_double, _vp]
    L.dash_validate_active_idx.argtypes = [_vp, C.c_int32, C.c_int32, _vp, _vp]
    L.dash_score_diff_rows.argtypes = [_vp, _vp, C.c_int32, C.c_int32, C.c_int32, C.c_int32, _vp, _vp]
    L.dash_decide_topk.argtypes = [pp, _vp, C.c_int32, C.c_int32, _vp, _vp, _vp, C.c_size_t, _vp]
    L.dash_mfma_probe.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_int32, _vp, _vp]
    L.dash_mfma_probe.restype = C.c_int
    L.dash_mfma_probe_flops.argtypes = [C.c_int32, C.c_int32]
    L.dash_mfma_probe_flops.restype = C.c_double
    L.dash_decide_topk_static.argtypes = [pp, _vp, C.c_int32, C.c_int32, _vp, _vp, _vp]
    L.dash_decide_topk_static.restype = C.c_int
    L.dash_ffn_workspace_bytes.restype = C.c_size_t
    L.dash_ffn_workspace_bytes.argtypes = [pp, C.c_int32, C.c_int32]
    L.dash_ffn_swiglu.argtypes = [pp, _vp, _vp, _vp, C.c_int32, C.c_int32, _vp, _vp, C.c_size_t, _vp]
    L.dash_scatter_rows.argtypes = [_vp, _vp, _vp, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32, _vp, _vp]
    for name in ("dash_attn_layer", "dash_flash_fwd", "dash_wo_residual_rownorm", "dash_score_decide",
                 "dash_compact", "dash_score_rows", "dash_rmsnorm_qkv", "dash_rope_qk", "dash_validate_active_idx",
                 "dash_profile_read", "dash_ffn_swiglu", "dash_scatter_rows", "dash_score_diff_rows", "dash_decide_topk"):
        getattr(L, name).restype = C.c_int
    _lib = L
    return L


def _check(status: int, what: str):
    if status != 0:
        raise DashError(f"{what}: {lib().dash_status_string(status).decode()} ({status})")


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _p(t: torch.Tensor | None):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device tensors must be contiguous"
    return t.data_ptr()


def torch_dtype(dtype: int) -> torch.dtype:
    return torch.bfloat16 if dtype == DASH_BF16 else torch.float32


def make_params(d, n_q_heads, n_kv_heads, head_dim, dtype=DASH_BF16, causal=True, softmax_scale=0.0,
                rule=RULE_THRESHOLD, score_kind=SCORE_REL, tau=0.0, k_keep=-1, rho=0.0, keep_first_n=0,
                keep_last_n=0) -> LayerParams:
    return LayerParams(int(d), int(n_q_heads), int(n_kv_heads), int(head_dim), int(dtype), int(bool(causal)),
                       float(softmax_scale), int(rule), int(score_kind), float(tau), int(k_keep), float(rho),
                       int(keep_first_n), int(keep_last_n))


def keep_count(n, rho, keep_first_n=0, keep_last_n=0, paper_impl_rounding=False) -> int:
    return int(lib().dash_keep_count(int(n), float(rho), int(keep_first_n), int(keep_last_n),
                                     int(bool(paper_impl_rounding))))


def init() -> None:
    """One-time set-up of the library on the current device (needed before capturing calls in a HIP graph)."""
    _check(lib().dash_init(), "dash_init")


def keep_count_quantile(n, halt_frac) -> int:
    return int(lib().dash_keep_count_quantile(int(n), float(halt_frac)))


def block_cost(n, d, m) -> float:
    return float(lib().dash_block_cost(float(n), float(d), float(m)))


def schedule_lengths(n, L, ratios: dict, keep_first_n=0, keep_last_n=0) -> list:
    """Rows each of L blocks runs on when the decision after block l applies compression ratio ratios[l]."""
    blocks = sorted(int(l) for l in ratios)
    nb = len(blocks)
    b_arr = (C.c_int32 * max(nb, 1))(*blocks)
    r_arr = (C.c_double * max(nb, 1))(*[float(ratios[l]) for l in blocks])
    out = (C.c_int64 * max(int(L), 1))()
    _check(lib().dash_schedule_lengths(int(n), int(L), b_arr, r_arr, nb, int(keep_first_n), int(keep_last_n), out),
           "dash_schedule_lengths")
    return [int(out[l]) for l in range(int(L))]


def schedule_cost(lengths, d, m) -> float:
    arr = (C.c_int64 * max(len(lengths), 1))(*[int(t) for t in lengths])
    return float(lib().dash_schedule_cost(arr, len(lengths), float(d), float(m)))


def comparable_multi_shot_ratio(n, L, shot_blocks, target_cost, d, m, keep_first_n=0, keep_last_n=0,
                                grid=10000) -> float:
    blocks = sorted(int(l) for l in shot_blocks)
    b_arr = (C.c_int32 * max(len(blocks), 1))(*blocks)
    c = float(lib().dash_comparable_multi_shot_ratio(int(n), int(L), b_arr, len(blocks), float(target_cost), float(d),
                                                     float(m), int(keep_first_n), int(keep_last_n), int(grid)))
    if c < 0.0:
        raise ValueError("no ratio on the grid meets the budget")
    return c


def layer_flops(params: LayerParams, n: int) -> float:
    return float(lib().dash_layer_flops(C.byref(params), int(n)))


def norm_partials_per_row(params: LayerParams) -> int:
    return int(lib().dash_norm_partials_per_row(C.byref(params)))


def workspace_bytes(params: LayerParams, n_capacity: int) -> int:
    return int(lib().dash_workspace_bytes(C.byref(params), int(n_capacity)))


class Profile:
    """Per-stage HIP-event timing of dash_attn_layer on its launch stream."""

    def __init__(self):
        self.handle = lib().dash_profile_create()
        if not self.handle:
            raise DashError("dash_profile_create failed")

    def read_ms(self) -> list[float]:
        buf = (C.c_float * N_STAGES)()
        _check(lib().dash_profile_read(self.handle, buf), "dash_profile_read")
        return [float(v) for v in buf]

    def __del__(self):
        try:
            if self.handle:
                lib().dash_profile_destroy(self.handle)
                self.handle = None
        except Exception:
            pass


@dataclass
class LayerBuffers:
    """Caller-owned outputs and workspace of dash_attn_layer for up to `capacity` rows."""
    capacity: int
    x_next: torch.Tensor
    scores: torch.Tensor
    halt_mask: torch.Tensor
    x_compact: torch.Tensor
    new_active_idx: torch.Tensor
    n_active_out: torch.Tensor
    workspace: torch.Tensor
    delta_dbg: torch.Tensor | None = None


def alloc_layer_buffers(params: LayerParams, capacity: int, device="cuda", with_delta=False) -> LayerBuffers:
    dt = torch_dtype(params.dtype)
    cap = max(int(capacity), 1)
    ws = max(workspace_bytes(params, capacity), 256)
    return LayerBuffers(
        capacity=int(capacity),
        x_next=torch.empty((cap, params.d), dtype=dt, device=device),
        scores=torch.empty((cap,), dtype=torch.float32, device=device),
        halt_mask=torch.empty((cap,), dtype=torch.uint8, device=device),
        x_compact=torch.empty((cap, params.d), dtype=dt, device=device),
        new_active_idx=torch.empty((cap,), dtype=torch.int32, device=device),
        n_active_out=torch.zeros((1,), dtype=torch.int32, device=device),
        workspace=torch.empty((ws,), dtype=torch.uint8, device=device),
        delta_dbg=torch.empty((cap, params.d), dtype=torch.float32, device=device) if with_delta else None,
    )


def dash_attn_layer(params: LayerParams, x, q, k, v, w_o, active_idx, n_active: int, buf: LayerBuffers,
                    profile: Profile | None = None) -> None:
    """Enqueue the whole layer step on the current stream; results land in `buf`."""
    assert n_active <= buf.capacity
    st = lib().dash_attn_layer(C.byref(params), _p(x), _p(q), _p(k), _p(v), _p(w_o), _p(active_idx),
                               int(n_active), _p(buf.x_next), _p(buf.scores), _p(buf.halt_mask),
                               _p(buf.x_compact), _p(buf.new_active_idx), _p(buf.n_active_out),
                               _p(buf.delta_dbg), _p(buf.workspace), buf.workspace.numel(),
                               profile.handle if profile else None, _stream())
    _check(st, "dash_attn_layer")


def dash_flash_fwd(params, q, k, v, active_idx, n, o) -> None:
    _check(lib().dash_flash_fwd(C.byref(params), _p(q), _p(k), _p(v), _p(active_idx), int(n), _p(o),
                                _stream()), "dash_flash_fwd")


def dash_wo_residual_rownorm(params, o, w_o, x, n, x_next, norm_partials, delta_dbg=None, workspace=None) -> None:
    ws_n = workspace.numel() if workspace is not None else 0
    _check(lib().dash_wo_residual_rownorm(C.byref(params), _p(o), _p(w_o), _p(x), int(n), _p(x_next),
                                          _p(norm_partials), _p(delta_dbg), _p(workspace), ws_n, _stream()),
           "dash_wo_residual_rownorm")


def dash_score_decide(params, norm_partials, n, scores, halt_mask, chunk_keep_counts, workspace=None) -> None:
    ws_n = workspace.numel() if workspace is not None else 0
    _check(lib().dash_score_decide(C.byref(params), _p(norm_partials), int(n), _p(scores), _p(halt_mask),
                                   _p(chunk_keep_counts), _p(workspace), ws_n, _stream()),
           "dash_score_decide")


def dash_compact(params, halt_mask, chunk_keep_counts, active_idx, x_next, n, x_compact, new_active_idx,
                 n_active_out, workspace=None) -> None:
    ws_n = workspace.numel() if workspace is not None else 0
    _check(lib().dash_compact(C.byref(params), _p(halt_mask), _p(chunk_keep_counts), _p(active_idx),
                              _p(x_next), int(n), _p(x_compact), _p(new_active_idx), _p(n_active_out),
                              _p(workspace), ws_n, _stream()), "dash_compact")


def dash_score_rows(delta, x, n, d, dtype, score_kind, scores) -> None:
    _check(lib().dash_score_rows(_p(delta), _p(x), int(n), int(d), int(dtype), int(score_kind), _p(scores),
                                 _stream()), "dash_score_rows")


def dash_score_diff_rows(x_new, x_old, n, d, dtype, score_kind, scores) -> None:
    _check(lib().dash_score_diff_rows(_p(x_new), _p(x_old), int(n), int(d), int(dtype), int(score_kind), _p(scores),
                                      _stream()), "dash_score_diff_rows")


def dash_decide_topk(params, scores, n, keep_low, halt_mask, chunk_keep_counts, workspace) -> None:
    _check(lib().dash_decide_topk(C.byref(params), _p(scores), int(n), int(bool(keep_low)), _p(halt_mask),
                                  _p(chunk_keep_counts), _p(workspace), workspace.numel(), _stream()),
           "dash_decide_topk")


def dash_mfma_probe(shape: int, normal_data: bool, iters: int, workgroups: int, sink) -> float:
    """Enqueue the register-only MFMA loop (measurement aid); returns the flops of the launch."""
    _check(lib().dash_mfma_probe(int(shape), int(bool(normal_data)), int(iters), int(workgroups), _p(sink), _stream()),
           "dash_mfma_probe")
    return float(lib().dash_mfma_probe_flops(int(iters), int(workgroups)))


TOPK_STATIC_MAX_ROWS = 1 << 20


def dash_decide_topk_static(params, scores, n, keep_low, halt_mask, chunk_keep_counts) -> None:
    """dash_decide_topk without a workspace argument (the library's static device scratch); allocates nothing."""
    _check(lib().dash_decide_topk_static(C.byref(params), _p(scores), int(n), int(bool(keep_low)), _p(halt_mask),
                                         _p(chunk_keep_counts), _stream()), "dash_decide_topk_static")


def ffn_workspace_bytes(params: LayerParams, n_capacity: int, m: int) -> int:
    return int(lib().dash_ffn_workspace_bytes(C.byref(params), int(n_capacity), int(m)))


def dash_ffn_swiglu(params, x, w_gate_up, w_down, n, m, x_out, workspace) -> None:
    _check(lib().dash_ffn_swiglu(C.byref(params), _p(x), _p(w_gate_up), _p(w_down), int(n), int(m), _p(x_out),
                                 _p(workspace), workspace.numel(), _stream()), "dash_ffn_swiglu")


def dash_scatter_rows(rows, idx, select, select_value, n, d, dtype, N, full) -> None:
    _check(lib().dash_scatter_rows(_p(rows), _p(idx), _p(select), int(select_value), int(n), int(d), int(dtype),
                                   int(N), _p(full), _stream()), "dash_scatter_rows")


def interleave_gate_up(w_gate: torch.Tensor, w_up: torch.Tensor) -> torch.Tensor:
    """Weight layout dash_ffn_swiglu expects: [d, 2m] with blocks of 32 gate columns followed by the 32 up
    columns of the same features. Layout preparation done once when weights are loaded."""
    d, m = w_gate.shape
    assert w_up.shape == (d, m) and m % 32 == 0
    return torch.stack((w_gate.reshape(d, m // 32, 32), w_up.reshape(d, m // 32, 32)), dim=2).reshape(d, 2 * m).contiguous()


def dash_rope_qk(params, q, k, active_idx, n, theta_base) -> None:
    _check(lib().dash_rope_qk(C.byref(params), _p(q), _p(k), _p(active_idx), int(n), float(theta_base), _stream()),
           "dash_rope_qk")


def qkv_workspace_bytes(params, n_capacity: int) -> int:
    return int(lib().dash_qkv_workspace_bytes(C.byref(params), int(n_capacity)))


def dash_rmsnorm_qkv(params, x, w_q, w_k, w_v, n, q, k, v, h_scratch, workspace=None) -> None:
    ws_n = workspace.numel() if workspace is not None else 0
    _check(lib().dash_rmsnorm_qkv(C.byref(params), _p(x), _p(w_q), _p(w_k), _p(w_v), int(n), _p(q), _p(k),
                                  _p(v), _p(h_scratch), _p(workspace), ws_n, _stream()), "dash_rmsnorm_qkv")


def concat_qkv(w_q: torch.Tensor, w_k: torch.Tensor, w_v: torch.Tensor) -> torch.Tensor:
    """[w_q | w_k | w_v] as one contiguous [d, (Hq + 2 Hkv) * dh] weight for dash_rmsnorm_qkv_fused."""
    return torch.cat([w_q, w_k, w_v], dim=1).contiguous()


def dash_rmsnorm_qkv_fused(params, x, w_qkv, n, q, k, v, h_scratch, workspace=None) -> None:
    ws_n = workspace.numel() if workspace is not None else 0
    _check(lib().dash_rmsnorm_qkv_fused(C.byref(params), _p(x), _p(w_qkv), int(n), _p(q), _p(k), _p(v),
                                        _p(h_scratch), _p(workspace), ws_n, _stream()), "dash_rmsnorm_qkv_fused")


def dash_validate_active_idx(active_idx, n, N, violations) -> None:
    _check(lib().dash_validate_active_idx(_p(active_idx), int(n), int(N), _p(violations), _stream()),
           "dash_validate_active_idx")


def to_device(a, dtype: int, device="cuda") -> torch.Tensor:
    """float32 numpy array (values exact in the storage type) -> contiguous device tensor."""
    return torch.from_numpy(a).to(device=device, dtype=torch_dtype(dtype)).contiguous()
