"""Shared helpers of the GPU parity tests: upload seeded inputs, call the C-ABI through the binding, and compare
with the CPU oracle under the documented bars.

Bars (stated here, used by every parity test):
  * integer outputs (dispatch tables) are bit-exact;
  * top-k indices are bit-exact for every token whose oracle gap between the k-th and (k+1)-th allowed logit
    exceeds GAP = 1e-4 (compared as sets; as ordered lists when all adjacent gaps among the top k+1 exceed GAP);
  * floating-point outputs: per row, max|gpu - ref| / max|ref| <= 2e-2 for bf16 storage, 1e-5 for fp32 storage;
  * tokens inside the gap band are checked against the oracle's FFN + combine run on the GPU's own selection.
Also reported, without a bar of its own (the stated bar is the row form): the element-wise error
max |gpu - ref| / max(|ref|, 1e-3 * rms(ref)).  The achieved errors of the tests that call record() are written to
parity_errors.json when the test session ends (tests/conftest.py says where).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, Optional

import numpy as np
import torch

import paper_2602_08404_amd as tm
from oracle import c_oracle as orc
from paper_2602_08404_amd import inputs as gen

GAP = 1e-4
TOL = {"bf16": 2e-2, "f32": 1e-5}
DEV = "cuda:0"
ELEM_FLOOR = 1e-3            # floor of the element-wise error's denominator, in units of rms(ref)

RECORDS = {}                 # name -> achieved errors (written out by tests/conftest.py at the end of the session)


def record(name: str, report: dict) -> None:
    RECORDS[name] = {k: (float(v) if isinstance(v, (float, np.floating)) else v) for k, v in report.items()}


def to_dev(a: Optional[np.ndarray]):
    """Host array in storage dtype -> device tensor (uint16 bit patterns become torch.bfloat16)."""
    if a is None:
        return None
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(DEV).view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def y_to_host(y: torch.Tensor) -> np.ndarray:
    return y.float().cpu().numpy().astype(np.float64)


@dataclass
class Case:
    shape: gen.MoEShape
    x: np.ndarray                 # storage dtype
    w: Dict[str, np.ndarray]      # storage dtype
    xf: np.ndarray                # fp32 views for the oracle
    wf: Dict[str, np.ndarray]
    d_x: torch.Tensor
    d_w: Dict[str, torch.Tensor]
    cfg: tm.Config

    @staticmethod
    def make(shape: gen.MoEShape, x: np.ndarray, w: Dict[str, np.ndarray], wf=None, d_w=None, max_tokens=None) -> "Case":
        wf = wf or {n: gen.as_f32(a) for n, a in w.items()}
        d_w = d_w or {n: to_dev(a) for n, a in w.items()}
        cfg = tm.make_config(shape.H, shape.I, shape.E, shape.k, shape.dtype, shape.renormalize, max_tokens or shape.T)
        return Case(shape, x, w, gen.as_f32(x), wf, to_dev(x), d_w, cfg)

    def with_x(self, shape: gen.MoEShape, x: np.ndarray) -> "Case":
        return Case.make(shape, x, self.w, self.wf, self.d_w)


def out_dtype(shape):
    return torch.bfloat16 if shape.dtype == "bf16" else torch.float32


# ----------------------------------------------------------------------------- GPU calls
def gpu_route(case: Case, mask: Optional[np.ndarray], want_logits=True):
    s = case.shape
    idx = torch.full((s.T, s.k), -7, dtype=torch.int32, device=DEV)
    gate = torch.full((s.T, s.k), -7.0, dtype=torch.float32, device=DEV)
    logits = torch.empty((s.T, s.E), dtype=torch.float32, device=DEV) if want_logits else None
    ws = None if want_logits else torch.empty(tm.team_moe_workspace_size(case.cfg), dtype=torch.uint8, device=DEV)
    d_mask = None if mask is None else torch.from_numpy(mask).to(DEV)
    tm.team_moe_route(case.cfg, case.d_x, s.T, case.d_w["router"], d_mask, idx, gate, logits, ws)
    torch.cuda.synchronize()
    return idx.cpu().numpy(), gate.cpu().numpy(), (logits.cpu().numpy() if want_logits else None)


def gpu_dispatch(case: Case, idx: np.ndarray):
    s = case.shape
    A = s.T * s.k
    d_idx = torch.from_numpy(np.ascontiguousarray(idx, np.int32)).to(DEV)
    offsets = torch.full((s.E + 1,), -7, dtype=torch.int32, device=DEV)
    sorted_token = torch.full((A,), -7, dtype=torch.int32, device=DEV)
    inv_pos = torch.full((s.T, s.k), -7, dtype=torch.int32, device=DEV)
    active = torch.full((s.E,), -7, dtype=torch.int32, device=DEV)
    n_active = torch.full((1,), -7, dtype=torch.int32, device=DEV)
    tm.team_moe_build_dispatch(case.cfg, d_idx, s.T, offsets, sorted_token, inv_pos, active, n_active)
    torch.cuda.synchronize()
    return (offsets.cpu().numpy(), sorted_token.cpu().numpy(), inv_pos.cpu().numpy(), active.cpu().numpy(),
            int(n_active.cpu().numpy()[0]))


def gpu_expert_ffn(case: Case, offsets, sorted_token, active, n_active):
    s = case.shape
    A = s.T * s.k
    ws = torch.empty(tm.team_moe_workspace_size(case.cfg), dtype=torch.uint8, device=DEV)
    out = torch.full((A, s.H), float("nan"), dtype=torch.float32, device=DEV)
    tm.team_moe_expert_ffn(case.cfg, case.d_x, s.T, torch.from_numpy(offsets).to(DEV), torch.from_numpy(sorted_token).to(DEV),
                           torch.from_numpy(active).to(DEV), torch.tensor([n_active], dtype=torch.int32, device=DEV),
                           case.d_w["gate"], case.d_w["up"], case.d_w["down"], out, ws)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def gpu_combine(case: Case, expert_out: np.ndarray, gate: np.ndarray, inv_pos: np.ndarray):
    s = case.shape
    y = torch.empty((s.T, s.H), dtype=out_dtype(s), device=DEV)
    tm.team_moe_combine(case.cfg, torch.from_numpy(np.ascontiguousarray(expert_out, np.float32)).to(DEV),
                        torch.from_numpy(np.ascontiguousarray(gate, np.float32)).to(DEV),
                        torch.from_numpy(np.ascontiguousarray(inv_pos, np.int32)).to(DEV), s.T, y)
    torch.cuda.synchronize()
    return y_to_host(y)


def gpu_layer(case: Case, mask: Optional[np.ndarray], ws=None) -> np.ndarray:
    s = case.shape
    if ws is None:
        ws = torch.empty(tm.team_moe_workspace_size(case.cfg), dtype=torch.uint8, device=DEV)
    y = torch.empty((s.T, s.H), dtype=out_dtype(s), device=DEV)
    d_mask = None if mask is None else torch.from_numpy(mask).to(DEV)
    tm.team_moe_layer_forward(case.cfg, case.d_x, s.T, case.d_w["router"], case.d_w["gate"], case.d_w["up"], case.d_w["down"],
                              d_mask, y, ws)
    torch.cuda.synchronize()
    return y_to_host(y), y


def gpu_route_two_round(case: Case, token_class: np.ndarray, want_logits=True, ws=None):
    s = case.shape
    idx = torch.full((s.T, s.k), -7, dtype=torch.int32, device=DEV)
    gate = torch.full((s.T, s.k), -7.0, dtype=torch.float32, device=DEV)
    mask = torch.full((s.E,), 9, dtype=torch.uint8, device=DEV)
    n_act = torch.full((1,), -7, dtype=torch.int32, device=DEV)
    logits = torch.empty((s.T, s.E), dtype=torch.float32, device=DEV) if want_logits else None
    if ws is None:
        ws = torch.empty(tm.team_moe_workspace_size(case.cfg), dtype=torch.uint8, device=DEV)
    tm.team_moe_route_two_round(case.cfg, case.d_x, s.T, case.d_w["router"], torch.from_numpy(token_class).to(DEV), mask, n_act,
                                idx, gate, logits, ws)
    torch.cuda.synchronize()
    return (idx.cpu().numpy(), gate.cpu().numpy(), mask.cpu().numpy(), int(n_act.cpu().numpy()[0]),
            logits.cpu().numpy() if want_logits else None)


def gpu_layer_two_round(case: Case, token_class: np.ndarray, ws=None):
    s = case.shape
    if ws is None:
        ws = torch.empty(tm.team_moe_workspace_size(case.cfg), dtype=torch.uint8, device=DEV)
    y = torch.empty((s.T, s.H), dtype=out_dtype(s), device=DEV)
    mask = torch.full((s.E,), 9, dtype=torch.uint8, device=DEV)
    n_act = torch.full((1,), -7, dtype=torch.int32, device=DEV)
    tm.team_moe_layer_forward_two_round(case.cfg, case.d_x, s.T, case.d_w["router"], case.d_w["gate"], case.d_w["up"],
                                        case.d_w["down"], torch.from_numpy(token_class).to(DEV), mask, n_act, y, ws)
    torch.cuda.synchronize()
    return y_to_host(y), y, mask.cpu().numpy(), int(n_act.cpu().numpy()[0])


def gpu_classify_tokens(conf: np.ndarray, state: np.ndarray, block_len: int, tau_h: float, L_h: int, live_index=None) -> np.ndarray:
    n = conf.shape[0]
    T = n if live_index is None else live_index.shape[0]
    out = torch.full((T,), 9, dtype=torch.uint8, device=DEV)
    d_live = None if live_index is None else torch.from_numpy(np.ascontiguousarray(live_index, np.int32)).to(DEV)
    tm.team_moe_classify_tokens(torch.from_numpy(conf).to(DEV), torch.from_numpy(state).to(DEV), n, block_len, d_live, T, tau_h, L_h, out)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def gpu_layer_rows(case: Case, x_rows: np.ndarray, row_index: np.ndarray, mask=None, token_class=None, ws=None, max_tokens=None):
    """team_moe_layer_forward_rows over rows `row_index` of x_rows [n_rows, H] (storage dtype); returns y_rows (device tensor,
    pre-filled with a sentinel so that untouched rows can be recognised), E_A and its size (two-round mode)."""
    s = case.shape
    T, n_rows = int(row_index.shape[0]), int(x_rows.shape[0])
    cfg = tm.make_config(s.H, s.I, s.E, s.k, s.dtype, s.renormalize, max_tokens or max(T, 1))
    if ws is None:
        ws = torch.empty(tm.team_moe_workspace_size(cfg), dtype=torch.uint8, device=DEV)
    y = torch.full((n_rows, s.H), 7.0, dtype=out_dtype(s), device=DEV)
    d_mask = None if mask is None else torch.from_numpy(mask).to(DEV)
    d_cls = None if token_class is None else torch.from_numpy(token_class).to(DEV)
    e_a = torch.full((s.E,), 9, dtype=torch.uint8, device=DEV)
    n_act = torch.full((1,), -7, dtype=torch.int32, device=DEV)
    tm.team_moe_layer_forward_rows(cfg, to_dev(x_rows), y, n_rows, torch.from_numpy(np.ascontiguousarray(row_index, np.int32)).to(DEV), T,
                                   case.d_w["router"], case.d_w["gate"], case.d_w["up"], case.d_w["down"], d_mask, d_cls, e_a, n_act, ws)
    torch.cuda.synchronize()
    return y, e_a.cpu().numpy(), int(n_act.cpu().numpy()[0])


def gpu_layer_unique_rows(case: Case, mask: Optional[np.ndarray], want_tables=True, ws=None):
    """team_moe_layer_forward_unique_rows; returns (y host fp64, y device, row_rep, n_unique) (tables None when not requested)."""
    s = case.shape
    if ws is None:
        ws = torch.empty(tm.team_moe_workspace_size(case.cfg), dtype=torch.uint8, device=DEV)
    y = torch.full((s.T, s.H), 7.0, dtype=out_dtype(s), device=DEV)
    d_mask = None if mask is None else torch.from_numpy(mask).to(DEV)
    rep = torch.full((s.T,), -7, dtype=torch.int32, device=DEV) if want_tables else None
    n_unique = torch.full((1,), -7, dtype=torch.int32, device=DEV) if want_tables else None
    tm.team_moe_layer_forward_unique_rows(case.cfg, case.d_x, s.T, case.d_w["router"], case.d_w["gate"], case.d_w["up"],
                                          case.d_w["down"], d_mask, y, rep, n_unique, ws)
    torch.cuda.synchronize()
    if not want_tables:
        return y_to_host(y), y, None, None
    return y_to_host(y), y, rep.cpu().numpy(), int(n_unique.cpu().numpy()[0])


# ----------------------------------------------------------------------------- 8-bit weights
@dataclass
class W8:
    """Expert weights of a Case re-stored as E4M3 codes with row scales; `case` carries the exactly dequantised weights
    for the oracle (and the bf16 router), `q` / `scale` are the device tensors the library reads."""
    case: Case
    q: Dict[str, torch.Tensor]
    scale: Dict[str, torch.Tensor]

    @staticmethod
    def make(base: Case) -> "W8":
        q, scale, wf = {}, {}, {"router": base.wf["router"]}
        for n in ("gate", "up", "down"):
            code, sc = gen.quantize_rows_e4m3(base.wf[n])
            wf[n] = gen.dequantize_rows_e4m3(code, sc)
            q[n] = torch.from_numpy(code).to(DEV)
            scale[n] = torch.from_numpy(sc).to(DEV)
        case = Case(base.shape, base.x, base.w, base.xf, wf, base.d_x, base.d_w, base.cfg)
        return W8(case, q, scale)

    def with_x(self, shape: gen.MoEShape, x: np.ndarray) -> "W8":
        c = self.case
        cfg = tm.make_config(shape.H, shape.I, shape.E, shape.k, shape.dtype, shape.renormalize, shape.T)
        return W8(Case(shape, x, c.w, gen.as_f32(x), c.wf, to_dev(x), c.d_w, cfg), self.q, self.scale)


def gpu_layer_w8(w8: W8, mask: Optional[np.ndarray], ws=None):
    c, s = w8.case, w8.case.shape
    if ws is None:
        ws = torch.empty(tm.team_moe_workspace_size(c.cfg), dtype=torch.uint8, device=DEV)
    y = torch.empty((s.T, s.H), dtype=out_dtype(s), device=DEV)
    d_mask = None if mask is None else torch.from_numpy(mask).to(DEV)
    tm.team_moe_layer_forward_w8(c.cfg, c.d_x, s.T, c.d_w["router"], w8.q["gate"], w8.q["up"], w8.q["down"], w8.scale["gate"],
                                 w8.scale["up"], w8.scale["down"], d_mask, y, ws)
    torch.cuda.synchronize()
    return y_to_host(y), y


def gpu_expert_ffn_w8(w8: W8, offsets, sorted_token, active, n_active):
    c, s = w8.case, w8.case.shape
    A = s.T * s.k
    ws = torch.empty(tm.team_moe_workspace_size(c.cfg), dtype=torch.uint8, device=DEV)
    out = torch.full((A, s.H), float("nan"), dtype=torch.float32, device=DEV)
    tm.team_moe_expert_ffn_w8(c.cfg, c.d_x, s.T, torch.from_numpy(offsets).to(DEV), torch.from_numpy(sorted_token).to(DEV),
                              torch.from_numpy(active).to(DEV), torch.tensor([n_active], dtype=torch.int32, device=DEV),
                              w8.q["gate"], w8.q["up"], w8.q["down"], w8.scale["gate"], w8.scale["up"], w8.scale["down"], out, ws)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def w8_parity(w8: W8, mask, threads=0):
    """The expert FFN and the whole layer on E4M3 weights against the oracle's plain layer on the exactly dequantised
    weights (same bars as for bf16 weights: the weights are inputs, the arithmetic is the same)."""
    c, s = w8.case, w8.case.shape
    tol = TOL[s.dtype]
    o_y, o_idx, o_gate = oracle_layer(c, mask, threads)
    o_logits = oracle_logits(c)
    g_idx, g_gate, _ = gpu_route(c, mask)
    set_safe, _ = safe_tokens(o_logits, mask, s.k)
    offsets, sorted_token, inv_pos, active, n_active = orc.dispatch(o_idx, s.E)
    g_out = gpu_expert_ffn_w8(w8, offsets, sorted_token, active, n_active)
    o_rows = orc.expert_rows(c.xf, c.wf["gate"], c.wf["up"], c.wf["down"], o_idx, threads)
    valid = inv_pos >= 0
    ref_out = np.zeros((s.T * s.k, s.H))
    ref_out[inv_pos[valid]] = o_rows[valid]
    n_rows = int(offsets[s.E])
    ffn_err = row_rel_err(g_out[:n_rows].astype(np.float64), ref_out[:n_rows]).max() if n_rows else 0.0
    assert ffn_err <= tol, ffn_err
    assert np.isnan(g_out[n_rows:]).all()
    y_gpu, _ = gpu_layer_w8(w8, mask)
    layer_err, n_band = check_layer(c, mask, y_gpu, g_idx, g_gate, o_y, o_idx, set_safe)
    return {"ffn_err": float(ffn_err), "layer_err": layer_err, "band_tokens": n_band, "n_active": n_active}


# ----------------------------------------------------------------------------- oracle side
def oracle_layer(case: Case, mask, threads=0):
    s = case.shape
    return orc.moe_layer(case.xf, case.wf["router"], case.wf["gate"], case.wf["up"], case.wf["down"], s.k, s.renormalize, mask,
                         threads=threads)


def oracle_logits(case: Case):
    return orc.router_logits(case.xf, case.wf["router"])


def safe_tokens(logits: np.ndarray, mask: Optional[np.ndarray], k: int):
    """Per token: (set_safe, order_safe) from the oracle's allowed logits.
    set_safe: gap between the k-th and (k+1)-th allowed logit > GAP (or fewer than k+1 allowed experts).
    order_safe: all adjacent gaps among the top min(k+1, |S|) allowed logits > GAP."""
    T, E = logits.shape
    allowed = np.ones(E, bool) if mask is None else mask != 0
    z = np.sort(logits[:, allowed].astype(np.float64), axis=1)[:, ::-1]
    n = z.shape[1]
    k_eff = min(k, n)
    if n == 0:
        return np.ones(T, bool), np.ones(T, bool)
    top = z[:, :min(k_eff + 1, n)]
    gaps = top[:, :-1] - top[:, 1:] if top.shape[1] > 1 else np.full((T, 1), np.inf)
    set_safe = np.ones(T, bool) if n <= k_eff else (z[:, k_eff - 1] - z[:, k_eff]) > GAP
    order_safe = (gaps > GAP).all(axis=1)
    return set_safe, order_safe & set_safe


def row_rel_err(got: np.ndarray, ref: np.ndarray) -> np.ndarray:
    """Per row: max|got-ref| / max|ref| (rows whose reference is all zero must match exactly -> 0 or inf)."""
    num = np.abs(got - ref).max(axis=1)
    den = np.abs(ref).max(axis=1)
    out = np.where(den > 0, num / np.where(den > 0, den, 1.0), np.where(num == 0, 0.0, np.inf))
    return out


def elem_rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    """Element-wise error with a floor: max |got - ref| / max(|ref|, ELEM_FLOOR * rms(ref))."""
    rms = float(np.sqrt(np.mean(ref * ref))) if ref.size else 0.0
    if rms == 0.0:
        return 0.0 if not np.abs(got - ref).any() else float("inf")
    return float((np.abs(got - ref) / np.maximum(np.abs(ref), ELEM_FLOOR * rms)).max())


def check_route(case: Case, mask, g_idx, g_gate, g_logits, o_idx, o_gate, o_logits):
    s = case.shape
    set_safe, order_safe = safe_tokens(o_logits, mask, s.k)
    if g_logits is not None:
        assert np.abs(g_logits.astype(np.float64) - o_logits).max() <= 2e-5 * max(1.0, np.abs(o_logits).max())
    for t in range(s.T):
        if order_safe[t]:
            assert g_idx[t].tolist() == o_idx[t].tolist(), (t, g_idx[t], o_idx[t])
            assert np.abs(g_gate[t] - o_gate[t]).max() <= 2e-6, (t, g_gate[t], o_gate[t])
        elif set_safe[t]:
            assert sorted(g_idx[t].tolist()) == sorted(o_idx[t].tolist()), (t, g_idx[t], o_idx[t])
    # properties that hold for every token, safe or not
    allowed = np.ones(s.E, bool) if mask is None else mask != 0
    k_eff = min(s.k, int(allowed.sum()))
    assert (g_idx[:, k_eff:] == -1).all() and (g_gate[:, k_eff:] == 0).all()
    if k_eff:
        assert allowed[g_idx[:, :k_eff]].all()
        assert all(len(set(r[:k_eff].tolist())) == k_eff for r in g_idx)
        if s.renormalize:
            assert np.abs(g_gate.sum(1) - 1.0).max() <= 1e-5
    return set_safe, order_safe


def check_layer(case: Case, mask, y_gpu: np.ndarray, g_idx, g_gate, o_y, o_idx, set_safe, metrics: Optional[dict] = None):
    """Rows with the oracle's selection: compare with the oracle's y.  Rows in the gap band: compare with the
    oracle's FFN + combine evaluated on the GPU's own selection and gates.  `metrics` receives the element-wise error."""
    s = case.shape
    tol = TOL[s.dtype]
    same = np.array([sorted(g_idx[t].tolist()) == sorted(o_idx[t].tolist()) for t in range(s.T)])
    assert same[set_safe].all()
    ref = o_y.copy()
    if (~same).any():
        rows = np.nonzero(~same)[0]
        o = orc.expert_rows(case.xf[rows], case.wf["gate"], case.wf["up"], case.wf["down"], g_idx[rows])
        ref[rows] = orc.combine(o, g_gate[rows].astype(np.float64), g_idx[rows])
    err = row_rel_err(y_gpu, ref)
    assert err.max() <= tol, (err.max(), int(err.argmax()))
    if metrics is not None:
        metrics["layer_err_elem"] = elem_rel_err(y_gpu, ref)
    return float(err.max()), int((~same).sum())


def full_parity(case: Case, mask, threads=0):
    """All five entry points against the oracle for one (inputs, mask). Returns a small report dict."""
    s = case.shape
    tol = TOL[s.dtype]
    o_y, o_idx, o_gate = oracle_layer(case, mask, threads)
    o_logits = oracle_logits(case)
    # route
    g_idx, g_gate, g_logits = gpu_route(case, mask)
    set_safe, order_safe = check_route(case, mask, g_idx, g_gate, g_logits, o_idx, o_gate, o_logits)
    # dispatch on the oracle's routing table: bit-exact
    o_disp = orc.dispatch(o_idx, s.E)
    g_disp = gpu_dispatch(case, o_idx)
    for a, b, name in zip(g_disp, o_disp, ("offsets", "sorted_token", "inv_pos", "active", "n_active")):
        assert np.array_equal(np.asarray(a), np.asarray(b)), name
    # expert FFN on the oracle's tables
    offsets, sorted_token, inv_pos, active, n_active = o_disp
    g_out = gpu_expert_ffn(case, offsets, sorted_token, active, n_active)
    o_rows = orc.expert_rows(case.xf, case.wf["gate"], case.wf["up"], case.wf["down"], o_idx, threads)     # [T,k,H]
    valid = inv_pos >= 0
    ref_out = np.zeros((s.T * s.k, s.H))
    ref_out[inv_pos[valid]] = o_rows[valid]
    n_rows = int(offsets[s.E])
    ffn_err = row_rel_err(g_out[:n_rows].astype(np.float64), ref_out[:n_rows]).max() if n_rows else 0.0
    assert ffn_err <= tol, ffn_err
    ffn_err_elem = elem_rel_err(g_out[:n_rows].astype(np.float64), ref_out[:n_rows]) if n_rows else 0.0
    assert np.isnan(g_out[n_rows:]).all()                      # rows beyond the table are left untouched
    # combine on the oracle's expert outputs (as float) and gates
    y_c = gpu_combine(case, ref_out.astype(np.float32), o_gate.astype(np.float32), inv_pos)
    ref_c = orc.combine(o_rows.astype(np.float32).astype(np.float64), o_gate.astype(np.float32).astype(np.float64), o_idx)
    comb_tol = 2.0 ** -8 if s.dtype == "bf16" else 1e-6
    assert row_rel_err(y_c, ref_c).max() <= comb_tol
    # whole layer
    y_gpu, _ = gpu_layer(case, mask)
    m = {}
    layer_err, n_band = check_layer(case, mask, y_gpu, g_idx, g_gate, o_y, o_idx, set_safe, m)
    logit_err = float(np.abs(g_logits.astype(np.float64) - o_logits).max())
    gate_err = float(np.abs(g_gate[order_safe] - o_gate[order_safe]).max()) if order_safe.any() else 0.0
    return {"ffn_err": float(ffn_err), "ffn_err_elem": ffn_err_elem, "layer_err": layer_err, "layer_err_elem": m["layer_err_elem"],
            "logit_abs_err": logit_err, "gate_abs_err": gate_err, "band_tokens": n_band, "unsafe": int((~set_safe).sum()),
            "n_active": n_active, "bar_row_rel": tol}


def unique_rows_parity(case: Case, mask, threads=0):
    """team_moe_layer_forward_unique_rows: the table of first equal rows is bit-exact against the oracle's byte-wise
    definition; y is compared, for every row, with the oracle's plain layer over all rows; repeated rows carry the bits of
    their first occurrence; the call without the optional outputs gives the same bits."""
    s = case.shape
    o_rep = orc.row_representatives(case.x)
    y_gpu, y_dev, rep, n_unique = gpu_layer_unique_rows(case, mask)
    assert np.array_equal(rep, o_rep)
    assert n_unique == int((o_rep == np.arange(s.T)).sum())
    assert torch.equal(y_dev, y_dev[torch.from_numpy(o_rep).long().to(DEV)])
    _, y_dev2, _, _ = gpu_layer_unique_rows(case, mask, want_tables=False)
    assert torch.equal(y_dev, y_dev2)
    o_y, o_idx, _ = oracle_layer(case, mask, threads)
    o_logits = oracle_logits(case)
    g_idx, g_gate, _ = gpu_route(case, mask)
    set_safe, _ = safe_tokens(o_logits, mask, s.k)
    layer_err, n_band = check_layer(case, mask, y_gpu, g_idx, g_gate, o_y, o_idx, set_safe)
    return {"n_unique": n_unique, "layer_err": layer_err, "band_tokens": n_band}


def two_round_parity(case: Case, token_class: np.ndarray, threads=0):
    """team_moe_route_two_round and team_moe_layer_forward_two_round against the oracle's Algorithm 1.

    E_A is the union of the first-round picks, so a first-round token inside the gap band may legitimately move one
    expert in or out of it.  What is compared: every first-round token against the oracle's free routing; the GPU's E_A
    against the union of the GPU's own first-round picks (always) and against the oracle's E_A (when no first-round
    token is in the band); every cold token against the oracle's routing confined to the GPU's E_A; the layer output
    against the oracle's layer under the GPU's E_A, and bitwise against team_moe_layer_forward given that E_A."""
    import dataclasses
    from types import SimpleNamespace
    s = case.shape
    first = np.nonzero(token_class)[0]
    cold = np.nonzero(token_class == 0)[0]
    o_logits = oracle_logits(case)
    o_mask, o_idx, o_gate = orc.route_two_round(o_logits, s.k, token_class, s.renormalize)
    g_idx, g_gate, g_mask, g_n, g_logits = gpu_route_two_round(case, token_class)
    assert set(np.unique(g_mask).tolist()) <= {0, 1} and g_n == int(g_mask.sum())
    # first round
    sub = lambda rows: SimpleNamespace(shape=dataclasses.replace(s, T=len(rows)))
    first_safe = True
    if len(first):
        set_safe, _ = check_route(sub(first), None, g_idx[first], g_gate[first], g_logits[first], o_idx[first], o_gate[first],
                                  o_logits[first])
        first_safe = bool(set_safe.all())
    union = np.zeros(s.E, np.uint8)
    picks = g_idx[first]
    union[np.unique(picks[picks >= 0])] = 1
    assert np.array_equal(g_mask, union)
    if first_safe:
        assert np.array_equal(g_mask, o_mask)
    # second round, inside the GPU's E_A
    if len(cold):
        c_idx, c_gate = orc.route_from_logits(o_logits[cold], s.k, s.renormalize, g_mask)
        check_route(sub(cold), g_mask, g_idx[cold], g_gate[cold], g_logits[cold], c_idx, c_gate, o_logits[cold])
    # scores kept in the workspace: same tables
    g2 = gpu_route_two_round(case, token_class, want_logits=False)
    assert np.array_equal(g2[0], g_idx) and np.array_equal(g2[1], g_gate) and np.array_equal(g2[2], g_mask)
    # whole layer
    y_gpu, y_dev, l_mask, l_n = gpu_layer_two_round(case, token_class)
    assert np.array_equal(l_mask, g_mask) and l_n == g_n
    _, y_ref_dev = gpu_layer(case, g_mask)
    assert torch.equal(y_dev, y_ref_dev)
    o_y, o_idx_m, _ = oracle_layer(case, g_mask, threads)
    set_safe_m, _ = safe_tokens(o_logits, g_mask, s.k)
    layer_err, n_band = check_layer(case, g_mask, y_gpu, g_idx, g_gate, o_y, o_idx_m, set_safe_m)
    return {"n_first": int(len(first)), "n_activated": g_n, "first_safe": first_safe, "layer_err": layer_err, "band_tokens": n_band}


def two_round_unique_rows_parity(case: Case, token_class: np.ndarray, scatter_seed: Optional[int] = None, threads=0):
    """team_moe_layer_forward_ex with the two-round router and the repeated-row search together (and, with scatter_seed, the
    tokens scattered over the rows of a larger tensor and reached through a row index).  The search changes no token's
    result: the table of first equal rows is bit-exact against the oracle's byte-wise definition, E_A is the one the
    two-round router finds without the search, y is compared row by row with the oracle's layer over all tokens under that
    E_A, repeated rows carry the bits of their first occurrence and rows outside the call are not written."""
    s = case.shape
    T = s.T
    if scatter_seed is None:
        n_rows, rows, d_x = 0, None, case.d_x
    else:
        n_rows = T + 9
        rows = gen.token_permutation(n_rows, seed=scatter_seed)[:T].astype(np.int32)       # not sorted: order of the call != order of the rows
        x_rows = np.zeros((n_rows,) + case.x.shape[1:], case.x.dtype)
        x_rows[rows] = case.x
        d_x = to_dev(x_rows)
    ws = torch.empty(tm.team_moe_workspace_size(case.cfg), dtype=torch.uint8, device=DEV)
    y = torch.full((n_rows or T, s.H), 7.0, dtype=out_dtype(s), device=DEV)
    e_a = torch.full((s.E,), 9, dtype=torch.uint8, device=DEV)
    n_a = torch.full((1,), -7, dtype=torch.int32, device=DEV)
    rep = torch.full((T,), -7, dtype=torch.int32, device=DEV)
    n_u = torch.full((1,), -7, dtype=torch.int32, device=DEV)
    w = case.d_w
    tm.team_moe_layer_forward_ex(case.cfg, d_x, y, T, w["router"], w["gate"], w["up"], w["down"], ws,
                                 row_index=None if rows is None else torch.from_numpy(rows).to(DEV), n_rows=n_rows,
                                 token_class=torch.from_numpy(token_class).to(DEV), activated_mask_out=e_a, n_activated_out=n_a,
                                 unique_rows=True, row_rep_out=rep, n_unique_out=n_u)
    torch.cuda.synchronize()
    o_rep = orc.row_representatives(case.x)
    assert np.array_equal(rep.cpu().numpy(), o_rep)
    n_unique = int((o_rep == np.arange(T)).sum())
    assert int(n_u.item()) == n_unique
    if rows is not None:
        live = torch.from_numpy(rows).long().to(DEV)
        other = torch.ones(n_rows, dtype=torch.bool, device=DEV)
        other[live] = False
        assert (y[other] == 7.0).all()
        y = y[live]
    assert torch.equal(y, y[torch.from_numpy(o_rep).long().to(DEV)])
    g_idx, g_gate, g_mask, g_n, _ = gpu_route_two_round(case, token_class)
    mask = e_a.cpu().numpy()
    assert np.array_equal(mask, g_mask) and int(n_a.item()) == g_n
    o_logits = oracle_logits(case)
    o_y, o_idx_m, _ = oracle_layer(case, mask, threads)
    set_safe_m, _ = safe_tokens(o_logits, mask, s.k)
    layer_err, n_band = check_layer(case, mask, y_to_host(y), g_idx, g_gate, o_y, o_idx_m, set_safe_m)
    return {"n_unique": n_unique, "n_activated": g_n, "layer_err": layer_err, "band_tokens": n_band}
