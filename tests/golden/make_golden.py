#!/usr/bin/env python3
"""Writes tests/golden/tiny_trajectory.json from the CPU oracle alone.

The paper prints no worked numeric example (its figures are images), so this fixture is not a pin of
the oracle against the paper: it freezes what the pinned oracle computes on the small fp32
configuration (2 layers, d 256, 4 heads x 64, FFN 688, vocab 1024; prompt 32, window 8, 64 new
tokens; the seeded synthetic weights, prompt and buffer), so that a later change of the oracle, of the
input generators or of the HIP path shows up as a diff against a stored trajectory (Sec. 4.1-4.4:
accepted ids, verified count K per step, step count, the approximate tail at the stop).

Run from the repository root:  python tests/golden/make_golden.py
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
import oracle          # noqa: E402
import synthgen        # noqa: E402


def trajectory():
    shape = synthgen.SHAPES["tiny"]
    om = oracle.model_from_synth(shape)
    P, W, N = 32, 8, 64
    prompt = synthgen.prompts(1, P, shape.vocab)[0]
    buf = synthgen.buffer_init(1, N + 2 * W, shape.vocab)[0]
    ref = om.jacobi_generate(prompt, buf, W, N)
    greedy = om.greedy_ar(prompt, N)
    assert (ref["ids"] == greedy).all()
    return {"config": {"shape": "tiny", "prompt": P, "window": W, "new_tokens": N,
                       "weight_seed": synthgen.WEIGHT_SEED, "prompt_seed": synthgen.PROMPT_SEED,
                       "buffer_seed": synthgen.BUFFER_SEED},
            "prompt": prompt.tolist(), "ids": ref["ids"].tolist(), "K": ref["K"].tolist(), "steps": int(ref["steps"]),
            "tail": ref["tail"].tolist()}


if __name__ == "__main__":
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_trajectory.json")
    with open(out, "w") as f:
        json.dump(trajectory(), f, indent=1)
        f.write("\n")
    print("wrote", out)
