"""Thin ctypes binding of libteam_moe.so (include/team_moe.h).

Argument marshalling only: every function takes PyTorch-ROCm device tensors (used purely as device memory),
passes their pointers and the current HIP stream to the C entry point of the same name, and raises on a
non-zero status.  There is no Python or PyTorch fallback: if the library is missing, import of this module's
``lib()`` fails loudly.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libteam_moe.so")

TEAM_F32, TEAM_BF16 = 0, 1
STATUS_OK = 0

EXPORTS = ["team_moe_workspace_size", "team_moe_route", "team_moe_build_dispatch", "team_moe_expert_ffn",
           "team_moe_combine", "team_moe_layer_forward", "team_moe_route_two_round", "team_moe_layer_forward_two_round",
           "team_moe_classify_tokens", "team_moe_layer_forward_rows", "team_moe_layer_forward_unique_rows",
           "team_moe_expert_ffn_w8", "team_moe_layer_forward_w8", "team_moe_dequantize_w8", "team_moe_layer_forward_ex",
           "team_moe_layer_forward_static", "team_moe_workspace_status", "team_moe_internal_set", "team_moe_internal_get", "team_moe_internal_stream_read",
           "team_moe_status_string"]


class LayerArgs(C.Structure):
    """team_moe_layer_args of include/team_moe.h."""
    _fields_ = [("x", C.c_void_p), ("y", C.c_void_p), ("T", C.c_int32), ("n_rows", C.c_int32), ("row_index", C.c_void_p),
                ("w_router", C.c_void_p), ("w_gate", C.c_void_p), ("w_up", C.c_void_p), ("w_down", C.c_void_p),
                ("scale_gate", C.c_void_p), ("scale_up", C.c_void_p), ("scale_down", C.c_void_p),
                ("expert_mask", C.c_void_p), ("token_class", C.c_void_p), ("activated_mask_out", C.c_void_p),
                ("n_activated_out", C.c_void_p), ("unique_rows", C.c_int32), ("reserved", C.c_int32),
                ("row_rep_out", C.c_void_p), ("n_unique_out", C.c_void_p), ("workspace", C.c_void_p), ("ws_bytes", C.c_size_t),
                ("stream", C.c_void_p), ("ffn_begin_event", C.c_void_p), ("ffn_end_event", C.c_void_p)]


class TeamMoeError(RuntimeError):
    def __init__(self, status: int, what: str):
        super().__init__(f"{what}: status {status} ({status_string(status)})")
        self.status = status


class Config(C.Structure):
    _fields_ = [("hidden", C.c_int32), ("inter", C.c_int32), ("num_experts", C.c_int32), ("top_k", C.c_int32),
                ("dtype", C.c_int32), ("renormalize", C.c_int32), ("max_tokens", C.c_int32), ("reserved", C.c_int32)]


def make_config(hidden: int, inter: int, num_experts: int, top_k: int, dtype: str, renormalize: int = 1,
                max_tokens: int = 256) -> Config:
    return Config(hidden, inter, num_experts, top_k, {"f32": TEAM_F32, "bf16": TEAM_BF16}[dtype], renormalize, max_tokens, 0)


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is not built; run `python -m paper_2602_08404_amd.build` "
                              "(there is no fallback implementation)")
        L = C.CDLL(LIB_PATH)
        vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
        cfgp = C.POINTER(Config)
        L.team_moe_workspace_size.argtypes = [cfgp, C.POINTER(sz)]
        L.team_moe_route.argtypes = [cfgp, vp, i32, vp, vp, vp, vp, vp, vp, sz, vp]
        L.team_moe_build_dispatch.argtypes = [cfgp, vp, i32, vp, vp, vp, vp, vp, vp, sz, vp]
        L.team_moe_expert_ffn.argtypes = [cfgp, vp, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.team_moe_combine.argtypes = [cfgp, vp, vp, vp, i32, vp, vp]
        L.team_moe_layer_forward.argtypes = [cfgp, vp, i32, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.team_moe_workspace_status.argtypes = [vp, sz, vp]
        L.team_moe_internal_set.argtypes = [C.c_char_p, C.c_int]
        L.team_moe_internal_get.argtypes = [C.c_char_p, C.POINTER(C.c_int)]
        L.team_moe_internal_stream_read.argtypes = [vp, sz, vp, i32, vp]
        L.team_moe_layer_forward_static.argtypes = [cfgp, vp, i32, vp, vp, vp, vp, vp, vp, vp]
        L.team_moe_route_two_round.argtypes = [cfgp, vp, i32, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.team_moe_layer_forward_two_round.argtypes = [cfgp, vp, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.team_moe_classify_tokens.argtypes = [vp, vp, i32, i32, vp, i32, C.c_float, i32, vp, vp]
        L.team_moe_layer_forward_rows.argtypes = [cfgp, vp, vp, i32, vp, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.team_moe_layer_forward_unique_rows.argtypes = [cfgp, vp, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.team_moe_expert_ffn_w8.argtypes = [cfgp, vp, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.team_moe_layer_forward_w8.argtypes = [cfgp, vp, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.team_moe_dequantize_w8.argtypes = [vp, vp, C.c_int64, C.c_int64, vp, vp]
        L.team_moe_layer_forward_ex.argtypes = [cfgp, C.POINTER(LayerArgs)]
        L.team_moe_status_string.argtypes = [C.c_int]
        L.team_moe_status_string.restype = C.c_char_p
        for name in EXPORTS[:-1]:
            getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().team_moe_status_string(int(status)).decode()


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream() -> int:
    import torch
    return torch.cuda.current_stream().cuda_stream


def _check(status: int, what: str) -> None:
    if status != STATUS_OK:
        raise TeamMoeError(status, what)


def team_moe_workspace_size(cfg: Config) -> int:
    n = C.c_size_t(0)
    _check(lib().team_moe_workspace_size(C.byref(cfg), C.byref(n)), "team_moe_workspace_size")
    return int(n.value)


def team_moe_route(cfg: Config, x, T: int, w_router, expert_mask, topk_idx, topk_gate, logits_out=None, workspace=None,
                   stream=None) -> None:
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().team_moe_route(C.byref(cfg), _ptr(x), T, _ptr(w_router), _ptr(expert_mask), _ptr(topk_idx), _ptr(topk_gate),
                                _ptr(logits_out), _ptr(workspace), ws_bytes, stream if stream is not None else _stream()),
           "team_moe_route")


def team_moe_build_dispatch(cfg: Config, topk_idx, T: int, expert_offsets, sorted_token, inv_pos, active_experts, n_active,
                            workspace=None, stream=None) -> None:
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().team_moe_build_dispatch(C.byref(cfg), _ptr(topk_idx), T, _ptr(expert_offsets), _ptr(sorted_token), _ptr(inv_pos),
                                         _ptr(active_experts), _ptr(n_active), _ptr(workspace), ws_bytes,
                                         stream if stream is not None else _stream()), "team_moe_build_dispatch")


def team_moe_expert_ffn(cfg: Config, x, T: int, expert_offsets, sorted_token, active_experts, n_active, w_gate, w_up, w_down,
                        expert_out, workspace, stream=None) -> None:
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().team_moe_expert_ffn(C.byref(cfg), _ptr(x), T, _ptr(expert_offsets), _ptr(sorted_token), _ptr(active_experts),
                                     _ptr(n_active), _ptr(w_gate), _ptr(w_up), _ptr(w_down), _ptr(expert_out), _ptr(workspace),
                                     ws_bytes, stream if stream is not None else _stream()), "team_moe_expert_ffn")


def team_moe_combine(cfg: Config, expert_out, topk_gate, inv_pos, T: int, y, stream=None) -> None:
    _check(lib().team_moe_combine(C.byref(cfg), _ptr(expert_out), _ptr(topk_gate), _ptr(inv_pos), T, _ptr(y),
                                  stream if stream is not None else _stream()), "team_moe_combine")


def team_moe_layer_forward(cfg: Config, x, T: int, w_router, w_gate, w_up, w_down, expert_mask, y, workspace, stream=None) -> None:
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().team_moe_layer_forward(C.byref(cfg), _ptr(x), T, _ptr(w_router), _ptr(w_gate), _ptr(w_up), _ptr(w_down),
                                        _ptr(expert_mask), _ptr(y), _ptr(workspace), ws_bytes,
                                        stream if stream is not None else _stream()), "team_moe_layer_forward")


def team_moe_layer_forward_static(cfg: Config, x, T: int, w_router, w_gate, w_up, w_down, expert_mask, y, stream=None) -> None:
    _check(lib().team_moe_layer_forward_static(C.byref(cfg), _ptr(x), T, _ptr(w_router), _ptr(w_gate), _ptr(w_up), _ptr(w_down),
                                               _ptr(expert_mask), _ptr(y), stream if stream is not None else _stream()),
           "team_moe_layer_forward_static")


def team_moe_workspace_status(workspace, stream=None) -> int:
    """Returns the team_status (0: no wait gave up; -5: one did, reported once).  Synchronises the stream.  workspace None: the
    static array of team_moe_layer_forward_static."""
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    return int(lib().team_moe_workspace_status(_ptr(workspace), ws_bytes, stream if stream is not None else _stream()))


def internal_set(key: str, value: int) -> None:
    """Tuning / testing knob of include/team_moe_internal.h."""
    _check(lib().team_moe_internal_set(key.encode(), int(value)), f"team_moe_internal_set({key})")


def internal_stream_read(src, nbytes: int, sink, workgroups: int, stream=None) -> None:
    _check(lib().team_moe_internal_stream_read(_ptr(src), nbytes, _ptr(sink), workgroups, stream if stream is not None else _stream()),
           "team_moe_internal_stream_read")


def internal_get(key: str) -> int:
    v = C.c_int(0)
    _check(lib().team_moe_internal_get(key.encode(), C.byref(v)), f"team_moe_internal_get({key})")
    return int(v.value)


def team_moe_route_two_round(cfg: Config, x, T: int, w_router, token_class, activated_mask_out, n_activated_out, topk_idx, topk_gate,
                             logits_out=None, workspace=None, stream=None) -> None:
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().team_moe_route_two_round(C.byref(cfg), _ptr(x), T, _ptr(w_router), _ptr(token_class), _ptr(activated_mask_out),
                                          _ptr(n_activated_out), _ptr(topk_idx), _ptr(topk_gate), _ptr(logits_out), _ptr(workspace),
                                          ws_bytes, stream if stream is not None else _stream()), "team_moe_route_two_round")


def team_moe_layer_forward_two_round(cfg: Config, x, T: int, w_router, w_gate, w_up, w_down, token_class, activated_mask_out,
                                     n_activated_out, y, workspace, stream=None) -> None:
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().team_moe_layer_forward_two_round(C.byref(cfg), _ptr(x), T, _ptr(w_router), _ptr(w_gate), _ptr(w_up), _ptr(w_down),
                                                  _ptr(token_class), _ptr(activated_mask_out), _ptr(n_activated_out), _ptr(y),
                                                  _ptr(workspace), ws_bytes, stream if stream is not None else _stream()),
           "team_moe_layer_forward_two_round")


def team_moe_classify_tokens(conf, state, n_rows: int, block_len: int, live_index, T: int, tau_h: float, L_h: int, token_class,
                             stream=None) -> None:
    _check(lib().team_moe_classify_tokens(_ptr(conf), _ptr(state), n_rows, block_len, _ptr(live_index), T, float(tau_h), L_h,
                                          _ptr(token_class), stream if stream is not None else _stream()), "team_moe_classify_tokens")


def team_moe_layer_forward_rows(cfg: Config, x_rows, y_rows, n_rows: int, row_index, T: int, w_router, w_gate, w_up, w_down,
                                expert_mask, token_class, activated_mask_out, n_activated_out, workspace, stream=None) -> None:
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().team_moe_layer_forward_rows(C.byref(cfg), _ptr(x_rows), _ptr(y_rows), n_rows, _ptr(row_index), T, _ptr(w_router),
                                             _ptr(w_gate), _ptr(w_up), _ptr(w_down), _ptr(expert_mask), _ptr(token_class),
                                             _ptr(activated_mask_out), _ptr(n_activated_out), _ptr(workspace), ws_bytes,
                                             stream if stream is not None else _stream()), "team_moe_layer_forward_rows")


def team_moe_layer_forward_unique_rows(cfg: Config, x, T: int, w_router, w_gate, w_up, w_down, expert_mask, y, row_rep_out,
                                       n_unique_out, workspace, stream=None) -> None:
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().team_moe_layer_forward_unique_rows(C.byref(cfg), _ptr(x), T, _ptr(w_router), _ptr(w_gate), _ptr(w_up), _ptr(w_down),
                                                    _ptr(expert_mask), _ptr(y), _ptr(row_rep_out), _ptr(n_unique_out),
                                                    _ptr(workspace), ws_bytes, stream if stream is not None else _stream()),
           "team_moe_layer_forward_unique_rows")


def team_moe_expert_ffn_w8(cfg: Config, x, T: int, expert_offsets, sorted_token, active_experts, n_active, w_gate_q, w_up_q, w_down_q,
                           scale_gate, scale_up, scale_down, expert_out, workspace, stream=None) -> None:
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().team_moe_expert_ffn_w8(C.byref(cfg), _ptr(x), T, _ptr(expert_offsets), _ptr(sorted_token), _ptr(active_experts),
                                        _ptr(n_active), _ptr(w_gate_q), _ptr(w_up_q), _ptr(w_down_q), _ptr(scale_gate), _ptr(scale_up),
                                        _ptr(scale_down), _ptr(expert_out), _ptr(workspace), ws_bytes,
                                        stream if stream is not None else _stream()), "team_moe_expert_ffn_w8")


def team_moe_layer_forward_w8(cfg: Config, x, T: int, w_router, w_gate_q, w_up_q, w_down_q, scale_gate, scale_up, scale_down,
                              expert_mask, y, workspace, stream=None) -> None:
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().team_moe_layer_forward_w8(C.byref(cfg), _ptr(x), T, _ptr(w_router), _ptr(w_gate_q), _ptr(w_up_q), _ptr(w_down_q),
                                           _ptr(scale_gate), _ptr(scale_up), _ptr(scale_down), _ptr(expert_mask), _ptr(y),
                                           _ptr(workspace), ws_bytes, stream if stream is not None else _stream()),
           "team_moe_layer_forward_w8")


def team_moe_dequantize_w8(codes, scale, rows: int, cols: int, out, stream=None) -> None:
    _check(lib().team_moe_dequantize_w8(_ptr(codes), _ptr(scale), rows, cols, _ptr(out), stream if stream is not None else _stream()),
           "team_moe_dequantize_w8")


def team_moe_layer_forward_ex(cfg: Config, x, y, T: int, w_router, w_gate, w_up, w_down, workspace, *, row_index=None, n_rows: int = 0,
                              scales=None, expert_mask=None, token_class=None, activated_mask_out=None, n_activated_out=None,
                              unique_rows: bool = False, row_rep_out=None, n_unique_out=None, stream=None, ffn_events=None) -> None:
    """Keyword arguments select the variants; `scales` = (scale_gate, scale_up, scale_down) tensors for 8-bit weights;
    `ffn_events` = (begin, end) hipEvent_t handles recorded around the expert FFN kernel."""
    sg, su, sd = scales if scales is not None else (None, None, None)
    a = LayerArgs(_ptr(x), _ptr(y), T, n_rows, _ptr(row_index), _ptr(w_router), _ptr(w_gate), _ptr(w_up), _ptr(w_down), _ptr(sg), _ptr(su),
                  _ptr(sd), _ptr(expert_mask), _ptr(token_class), _ptr(activated_mask_out), _ptr(n_activated_out), 1 if unique_rows else 0, 0,
                  _ptr(row_rep_out), _ptr(n_unique_out), _ptr(workspace),
                  0 if workspace is None else workspace.numel() * workspace.element_size(), stream if stream is not None else _stream(),
                  None if ffn_events is None else ffn_events[0], None if ffn_events is None else ffn_events[1])
    _check(lib().team_moe_layer_forward_ex(C.byref(cfg), C.byref(a)), "team_moe_layer_forward_ex")
