"""Writes tests/golden/tiny_decode_trajectory.json from the CPU oracle alone.

The paper prints no numeric value for the denoise-step path (no worked example, no table of logits or
confidences), so this fixture cites no passage: it freezes what the oracle, as pinned by
tests/test_oracle_pins.py, produces on the tiny workload (2 layers, d_model 256, 4 heads x 64, MLP 688,
vocabulary 4096 with id 4095 = [MASK], float32 weights drawn N(0, 0.02) with the LM head scaled x8, seed 0;
64 random prompt tokens, one block of 32 [MASK]; threshold 0.9 with a floor of 1; and the entropy rule with
theta = 5.443 nats and a floor of 1).  tests/test_oracle_pins.py re-runs the oracle against it, so a change
of the oracle's arithmetic shows up as a diff of this file, to be justified in the commit that makes it.

Run from the repository root:  python tests/golden/make_golden.py
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from oracle import dllm_oracle as O                      # noqa: E402
from paper_2601_07568_amd import synth                   # noqa: E402  (seeded inputs only)


def trajectory(rule, tau, m):
    ms = synth.TINY
    w = synth.Weights(ms, 0)
    prompt = synth.random_tokens(ms, 0, 64)
    rec = []
    seq, steps = O.decode(w, prompt, 1, 32, tau, m, record=rec, rule=rule)
    out = []
    for r in rec:
        ch = r["chosen"]
        out.append({"chosen": [int(i) for i in ch], "tokens": [int(r["cand"][i]) for i in ch],
                    "conf": [round(float(r["conf"][i]), 6) for i in ch],
                    "entropy": [round(float(r["entropy"][i]), 5) for i in ch]})
    return {"rule": rule, "threshold": tau, "floor": m, "steps": steps, "final_block": [int(t) for t in seq[64:]],
            "trajectory": out}


def build():
    return {"workload": "tiny, seed 0, prompt 64, block 32", "runs": [trajectory("prob", 0.9, 1), trajectory("entropy", 5.443, 1)]}


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_decode_trajectory.json")
    with open(path, "w") as f:
        json.dump(build(), f, indent=1)
        f.write("\n")
    print("wrote", path)
