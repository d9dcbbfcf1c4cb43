"""GPU tests of the corners of the method and of the library's failure handling, each compared directly with the oracle:
exact ties between router scores, scores that are not numbers, the expert FFN called on its own and repeatedly, and a
wait inside the expert FFN kernel that gives up (forced from the host; every kernel still runs to its normal end).

Selection is compared without any tolerance band here: the oracle's rule (oracle_route_from_logits) is applied to the
scores the GPU itself produced, and indices must be equal element by element; the scores in turn are compared with the
oracle's.  A tie or a NaN is an exact property of the scores, so nothing needs to be waived.
"""
import numpy as np
import pytest
import torch

import paper_2602_08404_amd as tm
from oracle import c_oracle as orc
from paper_2602_08404_amd import inputs as gen

import harness as hz

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)


@pytest.fixture
def knobs():
    old = {}

    def set_knob(key, value):
        old.setdefault(key, tm.internal_get(key))
        tm.internal_set(key, value)

    yield set_knob
    for key, value in old.items():
        tm.internal_set(key, value)


def small_layer(T, E, k=8, H=2048, I=256, seed=11, renormalize=1):
    s = gen.MoEShape("corner", T=T, H=H, E=E, k=k, I=I, dtype="bf16", renormalize=renormalize)
    return s, gen.make_x(s, seed=seed), gen.make_weights(s, seed=seed)


def gates_match(g_gate, o_gate):
    """NaN where the oracle has NaN, otherwise within the gate bar."""
    assert np.array_equal(np.isnan(g_gate), np.isnan(o_gate))
    fin = ~np.isnan(o_gate)
    assert np.abs(g_gate[fin] - o_gate[fin]).max(initial=0.0) <= 2e-6


def check_selection_from_own_scores(case, mask, g_idx, g_gate, g_logits):
    s = case.shape
    o_idx, o_gate = orc.route_from_logits(g_logits, s.k, s.renormalize, mask)
    assert np.array_equal(g_idx, o_idx), np.nonzero((g_idx != o_idx).any(axis=1))[0][:8]
    gates_match(g_gate, o_gate)
    return o_idx, o_gate


def check_two_round_from_own_scores(case, token_class, g):
    s = case.shape
    g_idx, g_gate, g_mask, g_n, g_logits = g
    o_mask, o_idx, o_gate = orc.route_two_round(g_logits, s.k, token_class, s.renormalize)
    assert np.array_equal(g_mask, o_mask) and g_n == int(o_mask.sum())
    assert np.array_equal(g_idx, o_idx)
    gates_match(g_gate, o_gate)


def scores_match(g_logits, o_logits):
    assert np.array_equal(np.isnan(g_logits), np.isnan(o_logits))
    inf = np.isinf(o_logits)
    assert np.array_equal(g_logits[inf], o_logits[inf])
    fin = np.isfinite(o_logits)
    assert np.abs(g_logits[fin].astype(np.float64) - o_logits[fin]).max(initial=0.0) <= 2e-5 * max(1.0, np.abs(o_logits[fin]).max(initial=0.0))


def layer_rows_match(case, mask, o_idx, o_gate, y_gpu):
    """y against the oracle's expert FFN + combine on the given routing table (the oracle's rule applied to the GPU's scores):
    NaN rows where the oracle's are NaN, the layer's bar elsewhere."""
    o = orc.expert_rows(case.xf, case.wf["gate"], case.wf["up"], case.wf["down"], o_idx)
    ref = orc.combine(o, o_gate, o_idx)
    nan_rows = np.isnan(ref).any(axis=1)
    assert np.array_equal(np.isnan(y_gpu).any(axis=1), nan_rows)
    assert np.isnan(y_gpu[nan_rows]).all() == np.isnan(ref[nan_rows]).all()
    if (~nan_rows).any():
        assert hz.row_rel_err(y_gpu[~nan_rows], ref[~nan_rows]).max() <= hz.TOL[case.shape.dtype]


# ----------------------------------------------------------------------------- exact ties
@pytest.mark.parametrize("E,M", [(128, 128), (128, 32), (128, 5), (128, 1), (256, 256), (256, 40)])
def test_zero_router_picks_the_lowest_ids_of_the_set_with_uniform_gates(E, M):
    """W_r = 0: every score is exactly 0, so every token takes the k_eff lowest ids of the activated set, gates 1 / k_eff -
    through team_moe_route, both two-round kernels (32 and 300 tokens) and team_moe_layer_forward."""
    for T in (32, 300):
        s, x, w = small_layer(T, E)
        w["router"][:] = 0
        case = hz.Case.make(s, x, w)
        mask = None if M == E else gen.random_mask(E, M, seed=M)
        allowed = np.arange(E) if mask is None else np.nonzero(mask)[0]
        k_eff = min(s.k, len(allowed))
        expect = np.full((T, s.k), -1, np.int32)
        expect[:, :k_eff] = allowed[:k_eff]
        g_idx, g_gate, g_logits = hz.gpu_route(case, mask)
        assert not g_logits.any()
        assert np.array_equal(g_idx, expect)
        assert np.abs(g_gate[:, :k_eff] - 1.0 / k_eff).max() <= 1e-7 and not g_gate[:, k_eff:].any()
        o_idx, o_gate = check_selection_from_own_scores(case, mask, g_idx, g_gate, g_logits)
        y_gpu, _ = hz.gpu_layer(case, mask)
        layer_rows_match(case, mask, o_idx, o_gate, y_gpu)
        o_y, oo_idx, _ = hz.oracle_layer(case, mask)                    # and the oracle's whole layer, which sees the same ties
        assert np.array_equal(oo_idx, expect)
        assert hz.row_rel_err(y_gpu, o_y).max() <= hz.TOL["bf16"]
        # two-round routing: the first-round tokens take ids 0..k-1, which is then E_A for everybody
        cls = gen.token_classes(T, max(1, T // 8), seed=3)
        g2 = hz.gpu_route_two_round(case, cls)
        check_two_round_from_own_scores(case, cls, g2)
        assert np.array_equal(np.nonzero(g2[2])[0], np.arange(min(s.k, E)))
    say("zero router", E, M, "ok")


@pytest.mark.parametrize("E,renorm", [(128, 1), (256, 1), (128, 0)])
def test_duplicated_router_rows_tie_exactly(E, renorm):
    """Pairs of experts with the same router row, and a block of 12 (> k) experts sharing one row, so that ties occur inside
    the selection, across its boundary, and among more candidates than slots.  Equal rows give equal scores bit for bit on
    the GPU (same arithmetic in the same order for every expert), and the lower id must win everywhere."""
    for T in (32, 300):
        s, x, w = small_layer(T, E, renormalize=renorm)
        r = w["router"]
        for j in range(0, 40, 2):
            r[j + 1] = r[j]
        r[60:72] = r[60]
        r[E - 1] = r[3]                                       # a tie between a low and the highest id
        case = hz.Case.make(s, x, w)
        for mask in (None, gen.random_mask(E, E // 2, seed=9)):
            g_idx, g_gate, g_logits = hz.gpu_route(case, mask)
            assert np.array_equal(g_logits[:, 1:40:2], g_logits[:, 0:40:2]) and (g_logits[:, 60:72] == g_logits[:, 60:61]).all()
            scores_match(g_logits, hz.oracle_logits(case))
            o_idx, o_gate = check_selection_from_own_scores(case, mask, g_idx, g_gate, g_logits)
            # the ties really decide something: some token selects one expert of a tied pair but not the other
            allowed = np.ones(E, bool) if mask is None else mask != 0
            split = 0
            for t in range(T):
                sel = set(g_idx[t].tolist())
                split += sum(1 for j in range(0, 40, 2) if allowed[j] and allowed[j + 1] and (j in sel) != (j + 1 in sel))
                assert all(not (j + 1 in sel and j not in sel) for j in range(0, 40, 2) if allowed[j] and allowed[j + 1])
            assert split > 0
            y_gpu, _ = hz.gpu_layer(case, mask)
            layer_rows_match(case, mask, o_idx, o_gate, y_gpu)
        cls = gen.token_classes(T, max(2, T // 6), seed=5)
        check_two_round_from_own_scores(case, cls, hz.gpu_route_two_round(case, cls))
    say("duplicated rows", E, renorm, "ok")


# ----------------------------------------------------------------------------- scores that are not numbers
def _bf16(v):
    return gen.bf16_round(np.array([v], np.float32))[0]


@pytest.mark.parametrize("renorm", [1, 0])
def test_non_finite_scores_follow_the_oracle(renorm):
    """NaN and infinite router scores: a NaN router row (its expert's score is NaN for every token), a router row that
    overflows to +inf or -inf depending on the token, a token whose x holds a NaN (all of its scores are NaN) and tokens with
    -0 / +0 scores.  Selection, gates (NaN where the oracle's are NaN) and y (NaN rows where the oracle's are) must follow the
    oracle's reading, through the single-round router, both two-round kernels and the whole layer."""
    E = 128
    for T in (32, 300):
        s, x, w = small_layer(T, E, renormalize=renorm)
        r = w["router"]
        r[0] = _bf16(np.nan)                                  # first allowed expert: the case a running arg-max gets wrong
        r[17] = _bf16(np.nan)
        r[9] = 0
        r[9, 0] = _bf16(3.0e38)                               # score = 3e38 * x[t,0]: +inf or -inf once |x[t,0]| > 1.14
        r[30] = 0                                             # score exactly 0 for every token (+0 or -0 cannot differ)
        r[31] = 0
        x[:, 0] = _bf16(2.0)
        x[1::2, 0] = _bf16(-2.0)
        x[5, 100] = _bf16(np.nan)                             # token 5: every score NaN
        case = hz.Case.make(s, x, w)
        o_logits = hz.oracle_logits(case)
        assert np.isnan(o_logits[:, 0]).all() and np.isposinf(o_logits[0, 9]) and np.isneginf(o_logits[1, 9]) and np.isnan(o_logits[5]).all()
        for mask in (None, gen.random_mask(E, 9, seed=1) | np.eye(E, dtype=np.uint8)[0] | np.eye(E, dtype=np.uint8)[17],
                     np.eye(E, dtype=np.uint8)[[0, 17, 9, 30]].sum(0).astype(np.uint8)):      # the last: fewer numbers than k
            g_idx, g_gate, g_logits = hz.gpu_route(case, mask)
            scores_match(g_logits, o_logits)
            o_idx, o_gate = check_selection_from_own_scores(case, mask, g_idx, g_gate, g_logits)
            y_gpu, _ = hz.gpu_layer(case, mask)
            layer_rows_match(case, mask, o_idx, o_gate, y_gpu)
        few = np.eye(E, dtype=np.uint8)[[0, 17, 9, 30]].sum(0).astype(np.uint8)
        g_idx, _, _ = hz.gpu_route(case, few)
        assert g_idx[1].tolist() == [30, 9, 0, 17] + [-1] * 4  # 0 > -inf > NaN (id 0) > NaN (id 17)
        assert g_idx[0].tolist() == [9, 30, 0, 17] + [-1] * 4  # +inf first
        cls = gen.token_classes(T, max(2, T // 6), seed=7)
        cls[5] = 1                                            # the all-NaN token in the first round: it activates ids 0..k-1
        check_two_round_from_own_scores(case, cls, hz.gpu_route_two_round(case, cls))
        cls[5] = 0
        check_two_round_from_own_scores(case, cls, hz.gpu_route_two_round(case, cls))
    say("non-finite scores", renorm, "ok")


# ----------------------------------------------------------------------------- the expert FFN on its own
@pytest.mark.parametrize("T,E,M", [(32, 64, 20), (160, 64, 9)])
def test_expert_ffn_is_self_contained(T, E, M):
    """team_moe_expert_ffn twice in a row on one workspace, after a dispatch call that was given no workspace, and on a
    workspace full of arbitrary bytes: every call compared with the oracle's expert rows."""
    s, x, w = small_layer(T, E, I=384)
    case = hz.Case.make(s, x, w)
    mask = gen.random_mask(E, M, seed=2)
    _, o_idx, _ = hz.oracle_layer(case, mask)
    offsets, sorted_token, inv_pos, active, n_active = orc.dispatch(o_idx, E)
    o_rows = orc.expert_rows(case.xf, case.wf["gate"], case.wf["up"], case.wf["down"], o_idx)
    valid = inv_pos >= 0
    n_rows = int(offsets[E])
    ref = np.zeros((T * s.k, s.H))
    ref[inv_pos[valid]] = o_rows[valid]
    ws = torch.randint(0, 256, (tm.team_moe_workspace_size(case.cfg),), dtype=torch.uint8, device=hz.DEV)
    # tables from the library's own dispatch call, which gets no workspace
    d = [torch.full((n,), -7, dtype=torch.int32, device=hz.DEV) for n in (E + 1, T * s.k, T * s.k, E, 1)]
    tm.team_moe_build_dispatch(case.cfg, torch.from_numpy(o_idx).to(hz.DEV), T, *d, workspace=None)
    outs = []
    for call in range(3):
        out = torch.full((T * s.k, s.H), float("nan"), dtype=torch.float32, device=hz.DEV)
        tm.team_moe_expert_ffn(case.cfg, case.d_x, T, d[0], d[1], d[3], d[4], case.d_w["gate"], case.d_w["up"], case.d_w["down"], out, ws)
        outs.append(out)
    torch.cuda.synchronize()
    assert tm.team_moe_workspace_status(ws) == 0              # arbitrary bytes are not a failure mark
    for out in outs:
        got = out.cpu().numpy().astype(np.float64)
        assert hz.row_rel_err(got[:n_rows], ref[:n_rows]).max() <= hz.TOL["bf16"]
        assert np.isnan(got[n_rows:]).all()
        assert torch.equal(out[:n_rows], outs[0][:n_rows])
    say("expert FFN alone", (T, E, M), "ok")


# ----------------------------------------------------------------------------- a wait that gives up
@pytest.mark.parametrize("T,E,M", [(32, 64, 20), (160, 64, 9)])           # register-operand body / streaming body of the FFN kernel
def test_a_wait_that_gives_up_is_reported_and_leaves_nan(T, E, M, knobs):
    """The down projection of an expert waits for its gate/up projection, which other workgroups compute.  With the testing
    knob "ffn_skip_publish" those workgroups never announce their results and with "ffn_spin_limit" = 4 every such wait gives up
    after a few polls: all kernels run to their normal end, every row of the expert outputs and of y is NaN (not a product of
    incomplete data), team_moe_workspace_status reports the failure once, and the next ordinary call is correct again."""
    s, x, w = small_layer(T, E, I=384)
    case = hz.Case.make(s, x, w)
    mask = gen.random_mask(E, M, seed=2)
    ws = torch.zeros(tm.team_moe_workspace_size(case.cfg), dtype=torch.uint8, device=hz.DEV)
    assert tm.team_moe_workspace_status(ws) == 0
    knobs("ffn_skip_publish", 1)
    knobs("ffn_spin_limit", 4)
    y_bad, _ = hz.gpu_layer(case, mask, ws)
    assert np.isnan(y_bad).all()
    assert tm.team_moe_workspace_status(ws) == -5
    assert tm.status_string(-5)
    assert tm.team_moe_workspace_status(ws) == 0              # reported once
    # the mark survives later calls until it is asked for
    hz.gpu_layer(case, mask, ws)
    knobs("ffn_skip_publish", 0)
    knobs("ffn_spin_limit", 1 << 16)
    y_good, _ = hz.gpu_layer(case, mask, ws)
    assert tm.team_moe_workspace_status(ws) == -5
    assert tm.team_moe_workspace_status(ws) == 0
    o_y, o_idx, _ = hz.oracle_layer(case, mask)
    g_idx, g_gate, _ = hz.gpu_route(case, mask)
    set_safe, _ = hz.safe_tokens(hz.oracle_logits(case), mask, s.k)
    hz.check_layer(case, mask, y_good, g_idx, g_gate, o_y, o_idx, set_safe)
    say("forced give-up", (T, E, M), "ok")


def test_workspace_status_of_the_static_array_and_bad_arguments():
    assert tm.team_moe_workspace_status(None) in (0,)         # the static array of the current device: never failed
    t = torch.zeros(64, dtype=torch.uint8, device=hz.DEV)
    assert tm.team_moe_workspace_status(t) == -3              # smaller than a status area
