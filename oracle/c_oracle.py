"""ctypes wrapper of the plain-C oracle (oracle/team_moe_oracle.c).  TEST INFRASTRUCTURE ONLY.

All arrays are host NumPy arrays; x and weights are fp32 values (bf16-stored tensors widened exactly by the
caller); results come back in fp64.
"""
from __future__ import annotations

import ctypes as C
from typing import Optional, Tuple

import numpy as np

from . import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(_build.build(force=False))
        _lib.oracle_max_threads.restype = C.c_int
        _lib.oracle_classify_tokens.argtypes = [C.POINTER(C.c_float), C.POINTER(C.c_uint8), C.c_int, C.c_int, C.POINTER(C.c_int32),
                                                C.c_int, C.c_float, C.c_int, C.POINTER(C.c_uint8)]
        _lib.oracle_row_representatives.argtypes = [C.c_void_p, C.c_int, C.c_int, C.POINTER(C.c_int32)]
    return _lib


def _p(a, ty):
    return a.ctypes.data_as(C.POINTER(ty)) if a is not None else None


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def max_threads() -> int:
    return int(lib().oracle_max_threads())


def router_logits(x, w_router) -> np.ndarray:
    x, w_router = _f32(x), _f32(w_router)
    T, H = x.shape
    E = w_router.shape[0]
    out = np.empty((T, E), np.float32)
    lib().oracle_router_logits(_p(x, C.c_float), _p(w_router, C.c_float), T, H, E, _p(out, C.c_float))
    return out


def route_from_logits(logits, k: int, renormalize: int = 1, mask: Optional[np.ndarray] = None) -> Tuple[np.ndarray, np.ndarray]:
    logits = _f32(logits)
    T, E = logits.shape
    idx = np.empty((T, k), np.int32)
    gate = np.empty((T, k), np.float64)
    m = None if mask is None else np.ascontiguousarray(mask, dtype=np.uint8)
    lib().oracle_route_from_logits(_p(logits, C.c_float), T, E, k, int(renormalize), _p(m, C.c_uint8),
                                   _p(idx, C.c_int32), _p(gate, C.c_double))
    return idx, gate


def route(x, w_router, k: int, renormalize: int = 1, mask=None):
    logits = router_logits(x, w_router)
    idx, gate = route_from_logits(logits, k, renormalize, mask)
    return idx, gate, logits


def route_two_round(logits, k: int, first_round, renormalize: int = 1):
    """Algorithm 1: returns (activated mask uint8 [E], topk_idx int32 [T,k], topk_gate fp64 [T,k])."""
    logits = _f32(logits)
    T, E = logits.shape
    fr = np.ascontiguousarray(first_round, dtype=np.uint8)
    assert fr.shape == (T,)
    mask = np.zeros(E, np.uint8)
    idx = np.empty((T, k), np.int32)
    gate = np.empty((T, k), np.float64)
    lib().oracle_route_two_round(_p(logits, C.c_float), T, E, k, int(renormalize), _p(fr, C.c_uint8), _p(mask, C.c_uint8),
                                 _p(idx, C.c_int32), _p(gate, C.c_double))
    return mask, idx, gate


def classify_tokens(conf, state, block_len: int, tau_h: float, L_h: int, live_index=None):
    """Step 1 of Algorithm 1 / Eq. 4: uint8 [T], 1 = first-round token (newly accepted or hot), 0 = cold."""
    conf = _f32(conf)
    state = np.ascontiguousarray(state, dtype=np.uint8)
    n = conf.shape[0]
    assert state.shape == (n,)
    if live_index is None:
        T, li = n, None
    else:
        li = np.ascontiguousarray(live_index, dtype=np.int32)
        T = li.shape[0]
    out = np.empty(T, np.uint8)
    lib().oracle_classify_tokens(_p(conf, C.c_float), _p(state, C.c_uint8), n, int(block_len),
                                 None if li is None else _p(li, C.c_int32), T, float(tau_h), int(L_h), _p(out, C.c_uint8))
    return out


def row_representatives(x_stored: np.ndarray) -> np.ndarray:
    """rep[t] = first row with the same stored bytes as row t (x_stored: [T,H] array of the storage type, e.g. uint16 bf16 bits)."""
    x_stored = np.ascontiguousarray(x_stored)
    T = x_stored.shape[0]
    row_bytes = x_stored.strides[0]
    rep = np.empty(T, np.int32)
    lib().oracle_row_representatives(x_stored.ctypes.data_as(C.c_void_p), T, int(row_bytes), _p(rep, C.c_int32))
    return rep


def dispatch(topk_idx, E: int):
    topk_idx = np.ascontiguousarray(topk_idx, dtype=np.int32)
    T, k = topk_idx.shape
    offsets = np.empty(E + 1, np.int32)
    sorted_token = np.empty(T * k, np.int32)
    inv_pos = np.empty((T, k), np.int32)
    active = np.empty(E, np.int32)
    n_active = np.zeros(1, np.int32)
    lib().oracle_dispatch(_p(topk_idx, C.c_int32), T, k, E, _p(offsets, C.c_int32), _p(sorted_token, C.c_int32),
                          _p(inv_pos, C.c_int32), _p(active, C.c_int32), _p(n_active, C.c_int32))
    return offsets, sorted_token, inv_pos, active, int(n_active[0])


def expert_rows(x, w_gate, w_up, w_down, topk_idx, threads: int = 0) -> np.ndarray:
    """o[t,s,:] = output of expert topk_idx[t,s] applied to token t (zeros for padded slots)."""
    x, w_gate, w_up, w_down = _f32(x), _f32(w_gate), _f32(w_up), _f32(w_down)
    topk_idx = np.ascontiguousarray(topk_idx, dtype=np.int32)
    T, H = x.shape
    k = topk_idx.shape[1]
    I = w_gate.shape[1]
    o = np.empty((T, k, H), np.float64)
    lib().oracle_expert_rows(_p(x, C.c_float), T, H, I, k, _p(w_gate, C.c_float), _p(w_up, C.c_float),
                             _p(w_down, C.c_float), _p(topk_idx, C.c_int32), _p(o, C.c_double), int(threads))
    return o


def combine(o, topk_gate, topk_idx) -> np.ndarray:
    o = np.ascontiguousarray(o, dtype=np.float64)
    topk_gate = np.ascontiguousarray(topk_gate, dtype=np.float64)
    topk_idx = np.ascontiguousarray(topk_idx, dtype=np.int32)
    T, k, H = o.shape
    y = np.empty((T, H), np.float64)
    lib().oracle_combine(_p(o, C.c_double), _p(topk_gate, C.c_double), _p(topk_idx, C.c_int32), T, k, H, _p(y, C.c_double))
    return y


def moe_layer(x, w_router, w_gate, w_up, w_down, k: int, renormalize: int = 1, mask=None, threads: int = 0):
    """The whole layer from the definition. Returns (y fp64 [T,H], topk_idx int32 [T,k], topk_gate fp64 [T,k])."""
    x, w_router, w_gate, w_up, w_down = _f32(x), _f32(w_router), _f32(w_gate), _f32(w_up), _f32(w_down)
    T, H = x.shape
    E, I = w_gate.shape[0], w_gate.shape[1]
    assert w_router.shape == (E, H) and w_up.shape == (E, I, H) and w_down.shape == (E, H, I)
    m = None if mask is None else np.ascontiguousarray(mask, dtype=np.uint8)
    y = np.empty((T, H), np.float64)
    idx = np.empty((T, k), np.int32)
    gate = np.empty((T, k), np.float64)
    lib().oracle_moe_layer(_p(x, C.c_float), T, H, E, k, I, int(renormalize), _p(w_router, C.c_float),
                           _p(w_gate, C.c_float), _p(w_up, C.c_float), _p(w_down, C.c_float), _p(m, C.c_uint8),
                           _p(y, C.c_double), _p(idx, C.c_int32), _p(gate, C.c_double), int(threads))
    return y, idx, gate
