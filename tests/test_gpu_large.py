"""GPU parity at the full sequence sizes of the large presets (8b-long, 8b-ragged16, 70b), each on the
4-layer truncation of its seeded model, and of the 8B preset at its full depth of 32 layers (8b-full), against
oracle results frozen in tests/golden/*_samples.npz.

The oracle needs minutes per preset at these sizes (16k-token prefill, 70B-shaped matrices, 16 sequences, 32
layers), so tests/golden/make_golden_large.py (which imports only the oracle and the input generator) wrote its
greedy streams, top-2 margins, at sampled steps the logits at 512 seeded vocabulary indices plus the top-2 ids
and values, and at a handful of points the whole logits vector.  Checked here, through the C ABI, in the
configuration bench.py times:
  * greedy ids at EVERY step where the oracle's top-2 margin exceeds 1e-2 (the runs are teacher-forced with
    the oracle's stream);
  * sampled logits within the bf16 tolerance 2e-2, and the sampled top-2 values;
  * every entry of the whole vectors (first choice, after the first and the last interrupt, end of the stream);
  * sequence lengths.
The last test runs the 8B preset at full depth and full size (the configuration bench.py times) and checks the
method's invariants, which hold at any size: in-flight inject == stateless re-prefill == token-by-token append,
merged pass == token then inject, K/V swap round trip bit-exact.
"""
import os

import numpy as np
import pytest
import torch

import asynclm_inputs as ai

pytestmark = pytest.mark.gpu

TOL = 2e-2
MARGIN = 1e-2
GOLD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _gold(name):
    path = os.path.join(GOLD, "%s_samples.npz" % name.replace("-", "_"))
    if not os.path.exists(path):
        pytest.skip("no frozen oracle samples for %s (run tests/golden/make_golden_large.py)" % name)
    z = np.load(path)
    assert int(z["seed"]) == ai.MASTER_SEED
    return z


def _model(name, gold):
    wl = ai.preset(name)
    model = ai.truncated(wl.model, int(gold["layers"]))
    w_dev = ai.make_weights(model, device=torch.device("cuda:0"))
    torch.cuda.synchronize()
    return wl, model, w_dev


def _check_samples(got, idx, want, t2i, t2v, what):
    err = float(np.abs(got[idx] - want).max())
    assert err <= TOL, (what, err)
    e2 = float(np.abs(got[t2i] - t2v).max())
    assert e2 <= TOL, (what, "top-2", e2)
    return max(err, e2)


def _check_full(got, want, what):
    assert got.shape == want.shape
    err = float(np.abs(got - want).max())
    assert err <= TOL, (what, "whole vector", err)
    return err


def _single_sequence(name):
    import paper_2412_07017_amd as pkg
    z = _gold(name)
    preset_name = name[:-5] if name.endswith("-full") else name
    wl, model, w_dev = _model(preset_name, z)
    if name.endswith("-full"):
        assert model.n_layers == wl.model.n_layers
    spec = ai.build_workload(preset_name)
    full = {(int(k), int(s)): v for k, s, v in zip(z["full_kind"], z["full_step"], z["full_logits"])}
    n_full = 0
    idx = z["sample_idx"]
    gen, margins = z["generated"], z["margins"]
    n = spec["n_decode"]
    assert len(gen) == n
    ev = {int(k): np.asarray(t) for k, t in spec["events"]}
    total = len(spec["prompt"]) + n + sum(len(t) for t in ev.values())
    lm = pkg.AsyncLM(model, w_dev, max_positions=total + 8, stream=torch.cuda.Stream())
    lm.prefill(0, spec["prompt"])
    samples = {int(s): k for k, s in enumerate(z["steps"])}
    inj = {int(s): k for k, s in enumerate(z["inject_steps"])}
    worst, gated = 0.0, 0
    for j in range(n):
        got = lm.logits(0)
        assert np.isfinite(got).all()
        if margins[j] > MARGIN:
            assert int(np.argmax(got)) == int(gen[j]), (j, float(margins[j]))
            gated += 1
        if j in samples:
            k = samples[j]
            worst = max(worst, _check_samples(got, idx, z["choose_samples"][k], z["choose_top2_ids"][k], z["choose_top2_vals"][k], ("step", j)))
        if (0, j) in full:
            worst = max(worst, _check_full(got, full[(0, j)], ("step", j))); n_full += 1
        assert lm.decode_step(0, forced_token=int(gen[j])) == int(gen[j])
        if j + 1 in ev:
            lm.inject_interrupt(0, ev[j + 1])
            k = inj[j + 1]
            got_i = lm.logits(0)
            worst = max(worst, _check_samples(got_i, idx, z["inject_samples"][k], z["inject_top2_ids"][k], z["inject_top2_vals"][k], ("inject", j + 1)))
            if (1, j + 1) in full:
                worst = max(worst, _check_full(got_i, full[(1, j + 1)], ("inject", j + 1))); n_full += 1
    last = lm.logits(0)
    worst = max(worst, _check_samples(last, idx, z["final_samples"], z["final_top2_ids"], z["final_top2_vals"], "final"))
    worst = max(worst, _check_full(last, full[(2, n)], "final")); n_full += 1
    assert n_full == len(full)
    assert lm.seq_len(0) == int(z["stream_len"]) == total
    lm.close()
    print("%s / %d layers: max |logit err| = %.3e over %d sampled and %d whole vectors, %d margin-gated ids identical over %d steps"
          % (name, model.n_layers, worst, len(samples) + len(inj) + 1, n_full, gated, n))


@pytest.mark.timeout(900)
def test_8b_long_context_workload_matches_frozen_oracle():
    """16384-token prompt, 512 tokens, 8 interrupts of 48 tokens: long-context decode attention (many splits
    merged by the last workgroup) and chunk attention over 17k keys."""
    _single_sequence("8b-long")


@pytest.mark.timeout(900)
def test_8b_workload_at_full_depth_matches_frozen_oracle():
    """The headline configuration at full depth and full size: 32 layers, 1024-token prompt, 256 tokens, 24-token
    interrupts after tokens 64, 128 and 192."""
    _single_sequence("8b-full")


@pytest.mark.timeout(900)
def test_70b_shape_workload_matches_frozen_oracle():
    """70B shape (d 8192, 64 query heads over 8 kv heads, ffn 28672): 4096-token prompt, 256 tokens, 32-token
    interrupts every 32 steps."""
    _single_sequence("70b")


@pytest.mark.timeout(900)
def test_8b_ragged16_batched_steps_match_frozen_oracle():
    """16 sequences with contexts between 512 and 4096 tokens, batched steps with the seeded interrupt
    arrivals (Sec. 5.3 merged form): every step is one asynclm_step_batch call."""
    import paper_2412_07017_amd as pkg
    name = "8b-ragged16"
    z = _gold(name)
    wl, model, w_dev = _model(name, z)
    spec = ai.build_workload(name)
    idx = z["sample_idx"]
    gen, margins = z["generated"], z["margins"]
    n_steps, ns = gen.shape
    grow = [n_steps + sum(len(t) for ev in spec["step_events"][:n_steps] for s, t in ev if s == q) for q in range(ns)]
    max_pos = max(len(p) + g for p, g in zip(spec["prompts"], grow)) + 8
    lm = pkg.AsyncLM(model, w_dev, max_positions=max_pos, max_seqs=ns, stream=torch.cuda.Stream())
    for q, p in enumerate(spec["prompts"]):
        lm.prefill(q, p)
    seqs = list(range(ns))
    assert n_steps == wl.n_decode                               # every batched step of the preset is frozen
    sampled = {int(t): k for k, t in enumerate(z["sample_steps"])}
    full = {(int(t), int(q)): v for t, q, v in zip(z["full_step"], z["full_seq"], z["full_logits"])}
    worst, gated, rows, n_full, biggest = 0.0, 0, 0, 0, 0
    for t in range(n_steps):
        ev = dict(spec["step_events"][t])
        intr = [ev.get(q, []) for q in seqs]
        rows += ns + sum(len(x) for x in intr)
        biggest = max(biggest, ns + sum(len(x) for x in intr))
        if (margins[t] > MARGIN).all():
            got = lm.step_batch(seqs, None, intr)               # greedy on the device
            assert list(got) == [int(v) for v in gen[t]], t
            gated += ns
        else:
            got = lm.step_batch(seqs, [int(v) for v in gen[t]], intr)
            assert list(got) == [int(v) for v in gen[t]]
        for q in seqs:
            got_q = lm.logits(q)
            assert np.isfinite(got_q).all()
            t2i, t2v = z["after_top2_ids"][t, q], z["after_top2_vals"][t, q]
            e2 = float(np.abs(got_q[t2i] - t2v).max())                      # top-2 values after every step
            assert e2 <= TOL, ("step", t, "seq", q, "top-2", e2)
            worst = max(worst, e2)
            if t in sampled:
                worst = max(worst, _check_samples(got_q, idx, z["after_samples"][sampled[t], q], t2i, t2v, ("step", t, "seq", q)))
            if (t, q) in full:
                worst = max(worst, _check_full(got_q, full[(t, q)], ("step", t, "seq", q))); n_full += 1
    assert n_full == len(full)
    assert [lm.seq_len(q) for q in seqs] == [int(v) for v in z["lengths"]]
    lm.close()
    print("%s / %d layers: max |logit err| = %.3e over %d batched steps (%.1f rows per step, at most %d), %d sampled steps, %d whole "
          "vectors, %d greedy ids identical" % (name, model.n_layers, worst, n_steps, rows / n_steps, biggest, len(sampled), n_full, gated))


@pytest.mark.timeout(900)
def test_8b_full_depth_full_size_invariants_of_the_method():
    """The 8B preset as bench.py runs it (32 layers, 1024-token prompt, greedy decoding steps, a 24-token interrupt
    injected in flight), checked through properties that hold at any size, because no oracle run fits a test here:
      * Sec. 3.2 / 5.5: the live context after the in-flight inject and a stateless re-prefill of the same token
        stream give the same next-token logits (two different kernel paths: single-row decode kernels + 24-row
        pass against 512-row prefill passes);
      * the same stream appended token by token through the decode kernels alone agrees as well;
      * Sec. 5.4: swapping the K/V cache out and in again reproduces the logits bit for bit, and decoding goes on
        identically from the restored sequence;
      * the merged form of Sec. 5.3 (chosen token + interrupt in one pass) equals token-then-inject.
    """
    import paper_2412_07017_amd as pkg
    wl = ai.preset("8b")
    model = wl.model
    w_dev = ai.make_weights(model, device=torch.device("cuda:0"))
    torch.cuda.synchronize()
    spec = ai.build_workload("8b")
    prompt = [int(t) for t in spec["prompt"]]
    intr = [int(t) for t in spec["events"][0][1]]
    assert len(prompt) == 1024 and len(intr) == 24
    lm = pkg.AsyncLM(model, w_dev, max_positions=1280, max_seqs=3, stream=torch.cuda.Stream())
    lm.prefill(0, prompt)
    history = list(prompt)
    for _ in range(64):
        history.append(lm.decode_step(0))
    # merged form on a copy of the sequence (slot 2): chosen token + interrupt in one pass
    lm.prefill(2, history)
    tok_merged = lm.step_batch([2], None, [intr])[0]
    tok = lm.decode_step(0)
    assert tok == tok_merged
    history.append(tok)
    lm.inject_interrupt(0, intr)
    history += intr
    live = lm.logits(0)
    assert np.isfinite(live).all() and lm.seq_len(0) == len(history) == 1024 + 65 + 24
    merged = lm.logits(2)
    top2 = np.sort(live)[-2:]
    margin = float(top2[1] - top2[0])

    def agree(other, what):
        err = float(np.abs(other - live).max())
        print("%s vs live context: max |logit diff| = %.3e (top-2 margin %.3e)" % (what, err, margin))
        assert err <= TOL, (what, err)
        if margin > MARGIN:
            assert int(np.argmax(other)) == int(np.argmax(live)), what

    agree(merged, "merged token + interrupt pass")
    lm.reset(2)
    lm.prefill(1, history)                                  # stateless variant: the whole stream again
    agree(lm.logits(1), "re-prefill in 512-row passes")
    lm.reset(1)
    lm.set_option("chunk", 1)                               # the whole stream through the single-row kernels
    lm.prefill(1, history)
    agree(lm.logits(1), "token-by-token append")
    lm.set_option("chunk", 512)
    lm.reset(1)
    # trap: swap out, drop, swap in on another slot
    nbytes = lm.kv_bytes(0)
    image = torch.empty(nbytes, dtype=torch.uint8).pin_memory()
    lm.kv_swap_out(0, image.data_ptr(), nbytes)
    lm.kv_swap_in(1, image.data_ptr(), nbytes)
    assert np.array_equal(lm.logits(1), live) and lm.seq_len(1) == lm.seq_len(0)
    a = [lm.decode_step(0) for _ in range(4)]
    b = [lm.decode_step(1) for _ in range(4)]
    assert a == b and np.array_equal(lm.logits(0), lm.logits(1))
    lm.close()
