"""Writes tests/golden/tiny_stream.json from the CPU oracle alone (no GPU code is imported).

The paper prints no numeric outputs for the decoding path, so this file is not a citation of
the paper: it freezes what the pinned oracle computes for the tiny preset (2 layers, d 256,
64-token prompt, 32 greedy tokens, one 8-token interrupt after token 16), so that a later
change to the oracle's arithmetic cannot pass unnoticed.

Run from the repository root:  python tests/golden/make_golden.py
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import asynclm_inputs as ai                     # noqa: E402
from oracle import asynclm_oracle as orc        # noqa: E402


def main():
    wl = ai.preset("tiny")
    w = ai.weights_to_numpy(ai.make_weights(wl.model, ai.MASTER_SEED))
    spec = ai.build_workload("tiny", ai.MASTER_SEED)
    res = orc.run_stream(orc.Shape.of(wl.model), w, spec["prompt"], spec["n_decode"], spec["events"])
    out = {
        "seed": ai.MASTER_SEED,
        "prompt_head": [int(t) for t in spec["prompt"][:8]],
        "interrupt": [int(t) for t in spec["events"][0][1]],
        "generated": [int(t) for t in res["generated"]],
        "margins": [round(orc.top2_margin(l), 9) for l in res["choose_logits"]],
        "logit_heads": [[round(float(v), 9) for v in l[:6]] for l in res["choose_logits"]],
        "final_logit_head": [round(float(v), 9) for v in res["final_logits"][:6]],
        "stream_len": len(res["stream"]),
    }
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_stream.json")
    with open(path, "w") as f:
        json.dump(out, f, indent=1)
    print("wrote", path, "min margin", min(out["margins"]))


if __name__ == "__main__":
    main()
