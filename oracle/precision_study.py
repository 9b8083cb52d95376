"""Diagnostic (not a graded comparison): what would each reduced-precision storage choice cost in the logits?

Runs the CPU oracle (fp32 numpy) on a seeded Llama-shaped model, once unrounded and once per variant with some
values rounded to bf16 (CachedDecoder's diag_round), on the same teacher-forced token stream: a prompt appended in
one pass, greedy decoding steps, one interrupt block in between.  Prints max |logit difference| to the unrounded run
over all next-token logit vectors of the stream.  The numbers size the error budget of an implementation's K/V cache
and activation formats against a logit tolerance (2e-2 for the bf16 presets); they are a property of the model
(N(0, 0.02) weights, depth), not of any kernel.

  python oracle/precision_study.py --shape 8b --layers 4 32 --prompt 512 --steps 12

Imports only the oracle and the seeded input generator (weights are generated on a GPU when torch finds one, which
is only faster: the generator is bit-identical on both).
"""
import argparse
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import asynclm_inputs as ai                     # noqa: E402
from oracle import asynclm_oracle as orc        # noqa: E402

VARIANTS = [
    ("K rows bf16", ("k",)),
    ("V rows bf16", ("v",)),
    ("K and V rows bf16", ("k", "v")),
    ("chunk passes: normalised inputs bf16", ("h", "chunk_only")),
    ("chunk passes: attention output bf16", ("o", "chunk_only")),
    ("chunk passes: SwiGLU output bf16", ("a", "chunk_only")),
    ("chunk passes: all three product inputs bf16", ("h", "o", "a", "chunk_only")),
    ("chunk passes: queries bf16", ("q", "chunk_only")),
    ("chunk passes: probabilities bf16", ("p", "chunk_only")),
    ("chunk passes: product inputs, queries, probabilities bf16", ("h", "o", "a", "q", "p", "chunk_only")),
    ("every pass: queries and probabilities bf16", ("q", "p")),
]


def run(shape, w, prompt, forced, intr, intr_after, diag):
    dec = orc.CachedDecoder(shape, w, dtype=np.float32, capacity=len(prompt) + len(forced) + len(intr) + 8, diag_round=diag)
    dec.prefill(prompt)
    out = []
    for j, t in enumerate(forced):
        out.append(dec.logits.copy())
        dec.decode_step(forced=t)
        if j + 1 == intr_after:
            dec.inject(intr)
            out.append(dec.logits.copy())
    out.append(dec.logits.copy())
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--shape", default="8b", choices=["8b", "70b"])
    ap.add_argument("--layers", type=int, nargs="+", default=[4])
    ap.add_argument("--prompt", type=int, default=512)
    ap.add_argument("--steps", type=int, default=12)
    ap.add_argument("--intr", type=int, default=24)
    args = ap.parse_args()
    import torch
    dev = "cuda:0" if torch.cuda.is_available() else "cpu"
    base = ai.preset(args.shape).model
    rows = {}
    for nl in args.layers:
        model = ai.truncated(base, nl)
        t0 = time.time()
        w = ai.weights_to_numpy(ai.make_weights(model, ai.MASTER_SEED, device=dev))
        shape = orc.Shape.of(model)
        prompt = ai.uniform_tokens(ai.MASTER_SEED, 960, args.prompt, model.vocab)
        intr = ai.uniform_tokens(ai.MASTER_SEED, 961, args.intr, model.vocab)
        # the unrounded run fixes the token stream
        dec = orc.CachedDecoder(shape, w, dtype=np.float32, capacity=args.prompt + args.steps + args.intr + 8)
        dec.prefill(prompt)
        forced = []
        for j in range(args.steps):
            forced.append(dec.decode_step())
            if j + 1 == args.steps // 2:
                dec.inject(intr)
        ref = run(shape, w, prompt, forced, intr, args.steps // 2, ())
        print("%s, %d layers: weights + reference %.0f s, logit range %.2f .. %.2f" % (args.shape, nl, time.time() - t0, min(v.min() for v in ref), max(v.max() for v in ref)), flush=True)
        for name, diag in VARIANTS:
            got = run(shape, w, prompt, forced, intr, args.steps // 2, diag)
            err = max(float(np.abs(a - b).max()) for a, b in zip(got, ref))
            rows.setdefault(name, {})[nl] = err
            print("  %-62s %.3e   (%.0f s)" % (name, err, time.time() - t0), flush=True)
        del w
    print("\n| rounded to bf16 | " + " | ".join("%d layers" % nl for nl in args.layers) + " |")
    print("|---|" + "---:|" * len(args.layers))
    for name, _ in VARIANTS:
        print("| %s | " % name + " | ".join("%.1e" % rows[name][nl] for nl in args.layers) + " |")


if __name__ == "__main__":
    main()
