"""The entry point that allocates nothing (team_moe_layer_forward_static: the workspace is a static device array inside the
library) against team_moe_layer_forward with a caller-owned workspace: same kernels, so the outputs must be the same bits.
Two calls in a row on the shared array, the second with a smaller input; then a configuration that does not fit the array."""
import numpy as np
import pytest
import torch

import paper_2602_08404_amd as tm
from paper_2602_08404_amd import inputs as gen

import harness as hz

pytestmark = pytest.mark.gpu


def test_static_scratch_layer_matches_the_workspace_layer_on_two_calls_in_a_row():
    s = gen.scaled(gen.CFG2, E=32, I=256)                      # a small layer of the config-2 family: 32 tokens, top-8 of 32 experts
    big = hz.Case.make(s, gen.make_x(s, seed=3), gen.make_weights(s, seed=3))
    s_small = gen.scaled(s, T=11)
    small = big.with_x(s_small, gen.make_x(s_small, seed=4))
    mask = gen.random_mask(s.E, 13, seed=1)
    d_mask = torch.from_numpy(mask).to(hz.DEV)
    print("static scratch:", s, "then T =", s_small.T, flush=True)
    outs = []
    for case, m in ((big, d_mask), (small, None)):             # second call: fewer tokens, other routing, on the same array
        sh, w = case.shape, case.d_w
        y = torch.full((sh.T, sh.H), 7.0, dtype=torch.bfloat16, device=hz.DEV)
        tm.team_moe_layer_forward_static(case.cfg, case.d_x, sh.T, w["router"], w["gate"], w["up"], w["down"], m, y)
        outs.append(y)
    torch.cuda.synchronize()
    for (case, m), y in zip(((big, mask), (small, None)), outs):
        _, y_ref = hz.gpu_layer(case, m)
        assert torch.equal(y, y_ref)
        # and against the oracle, to the layer's bar
        o_y, _, _ = hz.oracle_layer(case, m)
        assert hz.row_rel_err(hz.y_to_host(y), o_y).max() <= hz.TOL["bf16"]


def test_static_scratch_rejects_configurations_that_do_not_fit():
    cfg = tm.make_config(2048, 512, 256, 8, "bf16", 1, 256)   # 256 tokens x top-8 x 2048 floats of expert outputs alone exceed the array
    assert tm.team_moe_workspace_size(cfg) > (16 << 20)
    t = torch.zeros(16, dtype=torch.bfloat16, device=hz.DEV)
    with pytest.raises(tm.TeamMoeError) as e:
        tm.team_moe_layer_forward_static(cfg, t, 256, t, t, t, t, None, t)
    assert e.value.status == -3
