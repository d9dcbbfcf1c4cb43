"""Second oracle: the masked top-k MoE layer in vectorised NumPy fp64.  TEST INFRASTRUCTURE ONLY.

Written independently of the C oracle (different language, different control flow: array ops over all tokens
instead of a per-token loop, a stable sort instead of repeated arg-max) so that agreement between the two
pins both.  Follows the same passages of the paper: Algorithm 1 (routing confined to the activated set E_A)
and the per-token gating of a MoE layer.
"""
from __future__ import annotations

import numpy as np


def moe_layer_numpy(x, w_router, w_gate, w_up, w_down, k, renormalize=1, mask=None):
    x64 = np.asarray(x, np.float64)
    T, H = x64.shape
    E = w_router.shape[0]
    # selection happens on fp32 logits (the precision the decision is taken in)
    logits = (x64 @ np.asarray(w_router, np.float64).T).astype(np.float32)
    allowed = np.ones(E, bool) if mask is None else np.asarray(mask) != 0
    k_eff = min(k, int(allowed.sum()))
    key = np.where(allowed[None, :], logits, -np.inf)
    order = np.argsort(-key, axis=1, kind="stable")[:, :k_eff]      # stable: equal logits keep ascending id
    idx = np.full((T, k), -1, np.int32)
    idx[:, :k_eff] = order
    gate = np.zeros((T, k), np.float64)
    if k_eff > 0:
        sel = np.take_along_axis(logits, order, axis=1).astype(np.float64)
        if renormalize:
            w = np.exp(sel - sel.max(axis=1, keepdims=True))
            gate[:, :k_eff] = w / w.sum(axis=1, keepdims=True)
        else:
            z = logits.astype(np.float64)
            m = z.max(axis=1, keepdims=True)
            gate[:, :k_eff] = np.exp(sel - m) / np.exp(z - m).sum(axis=1, keepdims=True)
    y = np.zeros((T, H), np.float64)
    for e in np.unique(order) if k_eff > 0 else []:
        tok, slot = np.nonzero(order == e)
        xe = x64[tok]
        g = xe @ np.asarray(w_gate[e], np.float64).T
        u = xe @ np.asarray(w_up[e], np.float64).T
        h = g / (1.0 + np.exp(-g)) * u
        y[tok] += gate[tok, slot][:, None] * (h @ np.asarray(w_down[e], np.float64).T)
    return y, idx, gate
