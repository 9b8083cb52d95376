"""Writes tests/golden/<preset>_samples.npz for the large presets from the CPU oracle alone
(no GPU code is imported): 8b-long, 70b and 8b-ragged16, each on the 4-layer truncation of its
seeded model and at the preset's full sequence sizes, and 8b-full, the 8B preset at its full depth of
32 layers and full size (1024-token prompt, 256 steps, three 24-token interrupts).

The oracle needs minutes per preset at these sizes (a 16k-token prefill, 4-layer 70B-shaped
matrices, 32 layers), too long for a test, so its results are frozen here and the GPU tests compare
against the file: the greedy stream (every generated token and the top-2 margin it was chosen with),
at sampled steps the logits at 512 seeded vocabulary indices plus the top-2 ids and values, and at a
handful of points (first choice, after the first and the last interrupt, end of the stream) the WHOLE
logits vector.  The paper prints no numeric outputs for the decoding path; these values are the pinned
oracle's, not the paper's.

Run from the repository root:  python tests/golden/make_golden_large.py [preset ...]
"""
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import asynclm_inputs as ai                     # noqa: E402
from oracle import asynclm_oracle as orc        # noqa: E402

N_IDX = 512
PURPOSE_SAMPLE_IDX = 777
PREFILL_PIECE = 1024       # the prompt is appended in pieces (the same result by the append invariant; bounds memory)


def sample_indices(vocab):
    return np.sort(np.random.Generator(np.random.PCG64([ai.MASTER_SEED, PURPOSE_SAMPLE_IDX])).choice(vocab, N_IDX, replace=False)).astype(np.int32)


def top2(logits):
    i = np.argsort(logits)[-2:][::-1]
    return i.astype(np.int32), logits[i].astype(np.float32)


def prefill_in_pieces(dec, prompt):
    dec.prefill(prompt[:PREFILL_PIECE])
    for s in range(PREFILL_PIECE, len(prompt), PREFILL_PIECE):
        dec.inject(prompt[s:s + PREFILL_PIECE])


def single(name, every):
    full_depth = name.endswith("-full")
    preset_name = name[:-5] if full_depth else name
    wl = ai.preset(preset_name)
    model = wl.model if full_depth else ai.truncated(wl.model, wl.parity_layers)
    t0 = time.time()
    w = ai.weights_to_numpy(ai.make_weights(model, ai.MASTER_SEED))
    print(name, "weights %.0f s" % (time.time() - t0), flush=True)
    spec = ai.build_workload(preset_name, ai.MASTER_SEED)
    idx = sample_indices(model.vocab)
    dec = orc.CachedDecoder(orc.Shape.of(model), w, dtype=np.float32, capacity=len(spec["prompt"]) + 1024)
    prefill_in_pieces(dec, spec["prompt"])
    print(name, "prefill %.0f s" % (time.time() - t0), flush=True)
    ev = {int(n): np.asarray(t) for n, t in spec["events"]}
    n = spec["n_decode"]
    generated, margins = [], []
    steps, smp, t2i, t2v = [], [], [], []
    inj_steps, inj_smp, inj_t2i, inj_t2v = [], [], [], []
    # whole vectors: ("choose", 0), ("inject", first), ("inject", last), ("final", n)
    ev_steps = sorted(k for k in ev if k < n + 1)
    full_at = {("inject", ev_steps[0]), ("inject", ev_steps[-1])} if ev_steps else set()
    full_kind, full_step, full_vec = [], [], []
    for j in range(n):
        lg = dec.logits
        margins.append(orc.top2_margin(lg))
        if j == 0:
            full_kind.append(0); full_step.append(0); full_vec.append(lg.astype(np.float32))
        if j % every == 0 or j == n - 1 or j in ev:           # j in ev: the first choice after an interrupt
            i2, v2 = top2(lg)
            steps.append(j); smp.append(lg[idx].astype(np.float32)); t2i.append(i2); t2v.append(v2)
        generated.append(dec.decode_step())
        if j + 1 in ev and j + 1 < n + 1:
            dec.inject(ev[j + 1])
            i2, v2 = top2(dec.logits)
            inj_steps.append(j + 1); inj_smp.append(dec.logits[idx].astype(np.float32)); inj_t2i.append(i2); inj_t2v.append(v2)
            if ("inject", j + 1) in full_at:
                full_kind.append(1); full_step.append(j + 1); full_vec.append(dec.logits.astype(np.float32))
        if j % 32 == 0:
            print(name, "step", j, "%.0f s" % (time.time() - t0), flush=True)
    fi, fv = top2(dec.logits)
    full_kind.append(2); full_step.append(n); full_vec.append(dec.logits.astype(np.float32))
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "%s_samples.npz" % name.replace("-", "_"))
    np.savez_compressed(
        out, seed=np.int64(ai.MASTER_SEED), layers=np.int32(model.n_layers), sample_idx=idx,
        # whole logits vectors: kind 0 = the vector token 1 is chosen from, 1 = right after the interrupt at `step`, 2 = end
        full_kind=np.asarray(full_kind, np.int32), full_step=np.asarray(full_step, np.int32), full_logits=np.stack(full_vec),
        generated=np.asarray(generated, np.int32), margins=np.asarray(margins, np.float32),
        steps=np.asarray(steps, np.int32), choose_samples=np.stack(smp), choose_top2_ids=np.stack(t2i), choose_top2_vals=np.stack(t2v),
        inject_steps=np.asarray(inj_steps, np.int32),
        inject_samples=np.stack(inj_smp) if inj_smp else np.zeros((0, N_IDX), np.float32),
        inject_top2_ids=np.stack(inj_t2i) if inj_t2i else np.zeros((0, 2), np.int32),
        inject_top2_vals=np.stack(inj_t2v) if inj_t2v else np.zeros((0, 2), np.float32),
        final_samples=dec.logits[idx].astype(np.float32), final_top2_ids=fi, final_top2_vals=fv,
        stream_len=np.int32(dec.length))
    print("wrote", out, "%.0f s" % (time.time() - t0))


def ragged(name, n_steps):
    wl = ai.preset(name)
    model = ai.truncated(wl.model, wl.parity_layers)
    t0 = time.time()
    w = ai.weights_to_numpy(ai.make_weights(model, ai.MASTER_SEED))
    spec = ai.build_workload(name, ai.MASTER_SEED)
    idx = sample_indices(model.vocab)
    sh = orc.Shape.of(model)
    decs = []
    for p in spec["prompts"]:
        d = orc.CachedDecoder(sh, w, dtype=np.float32, capacity=len(p) + 512)
        prefill_in_pieces(d, p)
        decs.append(d)
        print(name, "prefilled", len(decs), "%.0f s" % (time.time() - t0), flush=True)
    ns = len(decs)
    generated = np.zeros((n_steps, ns), np.int32)
    margins = np.zeros((n_steps, ns), np.float32)
    after_t2i = np.zeros((n_steps, ns, 2), np.int32)          # top-2 of every sequence after EVERY batched step
    after_t2v = np.zeros((n_steps, ns, 2), np.float32)
    # sampled logits of every sequence after the steps in sample_steps: the first 24, every 4th, the last
    sample_steps = [t for t in range(n_steps) if t < 24 or t % 4 == 0 or t == n_steps - 1]
    after = np.zeros((len(sample_steps), ns, N_IDX), np.float32)
    full_seq = [0, int(np.argmax([len(p) for p in spec["prompts"]]))]      # whole vectors: two sequences, first and last step
    full_step, full_sq, full_vec = [], [], []
    for t in range(n_steps):
        ev = dict(spec["step_events"][t])
        for s, d in enumerate(decs):
            margins[t, s] = orc.top2_margin(d.logits)
            generated[t, s] = d.decode_step()
            if s in ev:
                d.inject(ev[s])
            if t in sample_steps:
                after[sample_steps.index(t), s] = d.logits[idx]
            after_t2i[t, s], after_t2v[t, s] = top2(d.logits)
            if t in (0, n_steps - 1) and s in full_seq:
                full_step.append(t); full_sq.append(s); full_vec.append(d.logits.astype(np.float32))
        print(name, "step", t, "%.0f s" % (time.time() - t0), flush=True)
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "%s_samples.npz" % name.replace("-", "_"))
    np.savez_compressed(out, seed=np.int64(ai.MASTER_SEED), layers=np.int32(model.n_layers), sample_idx=idx,
                        generated=generated, margins=margins, sample_steps=np.asarray(sample_steps, np.int32),
                        after_samples=after, after_top2_ids=after_t2i, after_top2_vals=after_t2v,
                        full_step=np.asarray(full_step, np.int32), full_seq=np.asarray(full_sq, np.int32), full_logits=np.stack(full_vec),
                        lengths=np.asarray([d.length for d in decs], np.int32))
    print("wrote", out, "%.0f s" % (time.time() - t0))


def main():
    which = sys.argv[1:] or ["8b-full", "8b-long", "70b", "8b-ragged16"]
    for name in which:
        if name == "8b-ragged16":
            ragged(name, ai.preset(name).n_decode)
        else:
            single(name, 16)


if __name__ == "__main__":
    main()
