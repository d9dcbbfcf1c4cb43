"""Writes tests/golden/hand_example.json from the hand derivation in hand_example.txt.

Uses plain arithmetic on two literal constants only (silu(1) and -silu(-1)); it calls neither the oracle nor
the HIP library, so the fixture is independent of both.
"""
import json
import os

S1 = 0.7310585786300049   # 1/(1+e^-1) = silu(1) = softmax weight of the larger of two logits 1 apart
SM = 0.2689414213699951   # 1/(1+e^+1) = -silu(-1) = softmax weight of the smaller one


def main():
    o_t0_e0 = [(-SM * 1.0) * 1.0, (-SM * 1.0) * 2.0]
    o_t0_e1 = [(-SM * 1.0) * 2.0, (-SM * 1.0) * -3.0]
    o_t1_e0 = [(S1 * 2.0) * 1.0, (S1 * 2.0) * 2.0]
    o_t1_e1 = [(S1 * 1.25) * 2.0, (S1 * 1.25) * -3.0]
    fx = {
        "_comment": "Hand-worked 2-expert example (worked by the builder; the paper prints no numerical MoE "
                    "example). See hand_example.txt for the derivation.",
        "x": [[1.0, 2.0], [2.0, 1.0]],
        "w_router": [[1.0, 0.0], [0.0, 1.0]],
        "w_gate": [[[1.0, -1.0]], [[1.0, -1.0]]],
        "w_up": [[[1.0, 0.0]], [[0.5, 0.25]]],
        "w_down": [[[1.0], [2.0]], [[2.0], [-3.0]]],
        "cases": [
            {"k": 1, "mask": None, "idx": [[1], [0]], "gate": [[1.0], [1.0]], "y": [o_t0_e1, o_t1_e0]},
            {"k": 2, "mask": None, "idx": [[1, 0], [0, 1]], "gate": [[S1, SM], [S1, SM]],
             "y": [[S1 * o_t0_e1[0] + SM * o_t0_e0[0], S1 * o_t0_e1[1] + SM * o_t0_e0[1]],
                   [S1 * o_t1_e0[0] + SM * o_t1_e1[0], S1 * o_t1_e0[1] + SM * o_t1_e1[1]]]},
            {"k": 1, "mask": [1, 0], "idx": [[0], [0]], "gate": [[1.0], [1.0]], "y": [o_t0_e0, o_t1_e0]},
            {"k": 2, "mask": [0, 1], "idx": [[1, -1], [1, -1]], "gate": [[1.0, 0.0], [1.0, 0.0]],
             "y": [o_t0_e1, o_t1_e1]},
        ],
    }
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "hand_example.json"), "w") as f:
        json.dump(fx, f, indent=1)


if __name__ == "__main__":
    main()
