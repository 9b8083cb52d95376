"""GPU parity on the tiny fp32 preset: every logit vector of the stream against the CPU oracle.

Tolerance (fp32 preset): max |logit error| <= 1e-4; greedy ids identical wherever the oracle's
top-2 margin exceeds 1e-2.  All calls go through the C ABI (ctypes binding).
"""
import numpy as np
import pytest
import torch

import asynclm_inputs as ai
from oracle import asynclm_oracle as orc
from cml_reference import ReferenceMonitor

pytestmark = pytest.mark.gpu

TOL = 1e-4
MARGIN = 1e-2


@pytest.fixture(scope="module")
def tiny():
    import paper_2412_07017_amd as pkg
    wl = ai.preset("tiny")
    spec = ai.build_workload("tiny")
    w_cpu = ai.weights_to_numpy(ai.make_weights(wl.model))
    ref = orc.run_stream(orc.Shape.of(wl.model), w_cpu, spec["prompt"], spec["n_decode"], spec["events"])
    dev = torch.device("cuda:0")
    w_dev = ai.make_weights(wl.model, device=dev)
    stream = torch.cuda.Stream(device=dev)
    return pkg, wl, spec, w_cpu, w_dev, stream, ref


def _new(t, **kw):
    pkg, wl, spec, w_cpu, w_dev, stream, ref = t
    return pkg.AsyncLM(wl.model, w_dev, max_positions=kw.pop("max_positions", 128), max_seqs=kw.pop("max_seqs", 1), stream=stream)


def test_weights_identical_on_device_and_host(tiny):
    pkg, wl, spec, w_cpu, w_dev, stream, ref = tiny
    for k in ("embed", "lm_head"):
        assert np.array_equal(w_dev[k].cpu().numpy(), w_cpu[k])
    for l in range(wl.model.n_layers):
        for k in ("wqkv", "wo", "wgate_up", "wdown"):
            assert np.array_equal(w_dev[k][l].cpu().numpy(), w_cpu[k][l])


@pytest.mark.parametrize("mode", ["fused", "graph", "plain", "two_streams", "two_streams_graph"])
def test_teacher_forced_stream_matches_oracle(tiny, mode):
    """The same stream through the single persistent kernel, the captured graph of per-operation kernels,
    plain launches of those kernels, and the step whose kernels alternate between two streams and hand over
    through counters in device memory (launched directly and as a captured graph)."""
    pkg, wl, spec, w_cpu, w_dev, stream, ref = tiny
    lm = _new(tiny)
    lm.set_option("fused", 1 if mode == "fused" else 0)
    lm.set_option("graph", 1 if mode in ("graph", "two_streams_graph") else 0)
    lm.set_option("pipeline", 1 if mode.startswith("two_streams") else 0)
    lm.prefill(0, spec["prompt"])
    ev = {n: t for n, t in spec["events"]}
    worst = 0.0
    for j in range(spec["n_decode"]):
        got = lm.logits(0)
        assert np.isfinite(got).all()
        worst = max(worst, float(np.abs(got - ref["choose_logits"][j]).max()))
        if orc.top2_margin(ref["choose_logits"][j]) > MARGIN:
            assert int(np.argmax(got)) == ref["generated"][j]
        tok = lm.decode_step(0, forced_token=ref["generated"][j])
        assert tok == ref["generated"][j]
        if j + 1 in ev:
            lm.inject_interrupt(0, ev[j + 1])
            worst = max(worst, float(np.abs(lm.logits(0) - ref["inject_logits"][j + 1]).max()))
    worst = max(worst, float(np.abs(lm.logits(0) - ref["final_logits"]).max()))
    assert lm.seq_len(0) == len(ref["stream"])
    if mode.startswith("two_streams"):
        # the last step did run on two streams: its kernels left their time stamps (5 per layer + the output head)
        stamps = lm.profile_trace()
        assert stamps.shape == (3 * (5 * wl.model.n_layers + 1), 2), stamps.shape
        assert (stamps[1::3] >= stamps[0::3]).all() and (stamps[2::3] >= stamps[1::3]).all()
    lm.close()
    assert worst <= TOL, worst


def test_free_running_greedy_matches_oracle(tiny):
    pkg, wl, spec, w_cpu, w_dev, stream, ref = tiny
    lm = _new(tiny)
    lm.prefill(0, spec["prompt"])
    ev = {n: t for n, t in spec["events"]}
    for j in range(spec["n_decode"]):
        margin = orc.top2_margin(ref["choose_logits"][j])
        tok = lm.decode_step(0)                      # device-side greedy argmax
        if margin > MARGIN:
            assert tok == ref["generated"][j], (j, margin)
        elif tok != ref["generated"][j]:
            top2 = np.argsort(ref["choose_logits"][j])[-2:]
            assert tok in top2
            break                                    # streams legitimately diverge after a near tie
        if j + 1 in ev:
            lm.inject_interrupt(0, ev[j + 1])
    lm.close()


def test_inject_equals_prefill_of_concatenation_on_device(tiny):
    pkg, wl, spec, w_cpu, w_dev, stream, ref = tiny
    s = ref["stream"]
    a = _new(tiny)
    a.prefill(0, s[:70]); a.inject_interrupt(0, s[70:81]); a.inject_interrupt(0, s[81:90])
    b = _new(tiny)
    b.prefill(0, s[:90])
    c = _new(tiny)
    c.prefill(0, s[:50])
    for t in s[50:90]:
        c.decode_step(0, forced_token=t, want_token=False)
    la, lb, lc = a.logits(0), b.logits(0), c.logits(0)
    want = orc.full_logits(orc.Shape.of(wl.model), w_cpu, s[:90])[-1]
    for got in (la, lb, lc):
        assert np.abs(got - want).max() <= TOL
    assert np.abs(la - lb).max() <= 2e-5 and np.abs(lc - lb).max() <= 2e-5
    for x in (a, b, c):
        x.close()


@pytest.mark.parametrize("nsplit", [1, 2, 4, 16, 33, 64])
def test_attention_split_count_does_not_change_logits(tiny, nsplit):
    pkg, wl, spec, w_cpu, w_dev, stream, ref = tiny
    s = ref["stream"]
    lm = _new(tiny)
    lm.set_option("fused", 0)                 # the split count is a knob of the per-operation attention kernel
    lm.set_option("attn_split", nsplit)
    lm.prefill(0, s[:97])
    want = orc.full_logits(orc.Shape.of(wl.model), w_cpu, s[:97])[-1]
    assert np.abs(lm.logits(0) - want).max() <= TOL
    lm.close()


@pytest.mark.timeout(300)
def test_long_context_single_row_attention_with_automatic_splits(tiny):
    """Contexts beyond 2048 tokens on the single-row attention kernel (fp32 models never take the matrix-core
    variant): one split per 256 positions, merged by the last workgroup of each kv head; below, up to 8 splits
    merged by the O projection.  Checked across both regimes against the incremental oracle."""
    pkg, wl, spec, w_cpu, w_dev, stream, ref = tiny
    toks = [int(t) for t in ai.uniform_tokens(ai.MASTER_SEED, 931, 2600, wl.model.vocab)]
    dec = orc.CachedDecoder(orc.Shape.of(wl.model), w_cpu)
    lm = _new(tiny, max_positions=2700)
    worst = 0.0
    done = 0
    for upto in (1000, 2040, 2049, 2300, 2600):      # prefill, then appends that cross the 2048 boundary
        part = toks[done:upto]
        if done == 0:
            lm.prefill(0, part); dec.prefill(part)
        else:
            lm.inject_interrupt(0, part); dec.inject(part)
        done = upto
        worst = max(worst, float(np.abs(lm.logits(0) - dec.logits).max()))
        tok = dec.decode_step()                       # one decoding step at each length (the stream grows by it)
        assert lm.decode_step(0, forced_token=tok) == tok
        worst = max(worst, float(np.abs(lm.logits(0) - dec.logits).max()))
        assert lm.seq_len(0) == dec.length
    lm.close()
    print("tiny fp32, contexts 1000..2600: max |logit err| = %.3e" % worst)
    assert worst <= TOL, worst


def test_two_sequences_are_independent(tiny):
    pkg, wl, spec, w_cpu, w_dev, stream, ref = tiny
    s = ref["stream"]
    lm = _new(tiny, max_seqs=2)
    lm.prefill(0, s[:40])
    lm.prefill(1, s[10:31])
    lm.decode_step(0, forced_token=s[40])
    lm.inject_interrupt(1, s[31:36])
    sh = orc.Shape.of(wl.model)
    assert np.abs(lm.logits(0) - orc.full_logits(sh, w_cpu, s[:41])[-1]).max() <= TOL
    assert np.abs(lm.logits(1) - orc.full_logits(sh, w_cpu, s[10:36])[-1]).max() <= TOL
    lm.reset(0)
    assert lm.seq_len(0) == 0 and lm.seq_len(1) == 26
    lm.prefill(0, s[5:9])
    assert np.abs(lm.logits(0) - orc.full_logits(sh, w_cpu, s[5:9])[-1]).max() <= TOL
    lm.close()


def test_error_paths_leave_state_unchanged(tiny):
    pkg, wl, spec, w_cpu, w_dev, stream, ref = tiny
    s = ref["stream"]
    lm = _new(tiny, max_positions=20)

    def code(fn, *a, **k):
        with pytest.raises(pkg.AsyncLMError) as ei:
            fn(*a, **k)
        return ei.value.code

    assert code(lm.decode_step, 0) == pkg.E_STATE
    assert code(lm.inject_interrupt, 0, [1, 2]) == pkg.E_STATE
    assert code(lm.logits, 0) == pkg.E_STATE
    assert code(lm.prefill, 1, [1]) == pkg.E_INVAL                  # bad sequence index
    assert code(lm.prefill, 0, [1, wl.model.vocab]) == pkg.E_INVAL  # token id out of range
    assert code(lm.prefill, 0, []) == pkg.E_INVAL
    assert code(lm.prefill, 0, list(range(21))) == pkg.E_CAPACITY
    assert lm.seq_len(0) == 0
    lm.prefill(0, s[:15])
    before = lm.logits(0)
    assert code(lm.prefill, 0, [1]) == pkg.E_STATE
    assert code(lm.inject_interrupt, 0, s[15:21]) == pkg.E_CAPACITY  # 15 + 6 > 20
    assert code(lm.inject_interrupt, 0, [-1]) == pkg.E_INVAL
    assert code(lm.decode_step, 0, wl.model.vocab) == pkg.E_INVAL
    assert code(lm.set_option, "nonsense", 1) == pkg.E_INVAL
    assert lm.seq_len(0) == 15 and np.array_equal(lm.logits(0), before)
    lm.inject_interrupt(0, s[15:20])
    assert code(lm.decode_step, 0) == pkg.E_CAPACITY
    assert lm.seq_len(0) == 20
    lm.close()


def test_results_are_deterministic(tiny):
    pkg, wl, spec, w_cpu, w_dev, stream, ref = tiny
    outs = []
    for _ in range(2):
        lm = _new(tiny)
        lm.prefill(0, spec["prompt"])
        for _ in range(5):
            lm.decode_step(0)
        outs.append(lm.logits(0))
        lm.close()
    assert np.array_equal(outs[0], outs[1])


def _batch_reference(sh, w_cpu, prompts, plan, dtype):
    """Oracle of a batched run: one cached decoder per sequence, stepped independently (Sec. 5.3: a step
    appends [chosen token] ++ [queued interrupt tokens] to the sequence).  plan[t] = {seq: tokens}."""
    decs = [orc.CachedDecoder(sh, w_cpu, dtype=dtype) for _ in prompts]
    for d, p in zip(decs, prompts):
        d.prefill(p)
    choose, chosen, after = [], [], []
    for ev in plan:
        choose.append([d.logits.copy() for d in decs])
        toks = []
        for s, d in enumerate(decs):
            toks.append(d.decode_step())
            if s in ev:
                d.inject(ev[s])
        chosen.append(toks)
        after.append([d.logits.copy() for d in decs])
    return choose, chosen, after


def test_step_batch_matches_independent_oracle_sequences(tiny):
    """asynclm_step_batch on the fp32 preset (sequence-by-sequence fallback of models outside the matrix-core
    append path): three sequences, interrupts riding with the chosen token, greedy and forced choices."""
    pkg, wl, spec, w_cpu, w_dev, stream, ref = tiny
    V = wl.model.vocab
    prompts = [ai.uniform_tokens(ai.MASTER_SEED, 901, n, V, sub=i) for i, n in enumerate((5, 17, 33))]
    plan = [{}, {1: ai.uniform_tokens(ai.MASTER_SEED, 902, 6, V)}, {0: ai.uniform_tokens(ai.MASTER_SEED, 902, 3, V, sub=1),
            2: ai.uniform_tokens(ai.MASTER_SEED, 902, 9, V, sub=2)}, {}, {}]
    choose, chosen, after = _batch_reference(orc.Shape.of(wl.model), w_cpu, prompts, plan, np.float64)
    lm = _new(tiny, max_seqs=3)
    for s, p in enumerate(prompts):
        lm.prefill(s, p)
    worst = 0.0
    for t, ev in enumerate(plan):
        intr = [ev.get(s, []) for s in range(3)]
        if t % 2 == 0:      # greedy on the device
            got = lm.step_batch([0, 1, 2], None, intr)
            for s in range(3):
                if orc.top2_margin(choose[t][s]) > MARGIN:
                    assert got[s] == chosen[t][s]
                assert got[s] == chosen[t][s], "near tie in the seeded reference stream: pick another seed"
        else:
            got = lm.step_batch([2, 0, 1], [chosen[t][2], chosen[t][0], chosen[t][1]], [intr[2], intr[0], intr[1]])
            assert list(got) == [chosen[t][2], chosen[t][0], chosen[t][1]]
        for s in range(3):
            worst = max(worst, float(np.abs(lm.logits(s) - after[t][s]).max()))
    assert [lm.seq_len(s) for s in range(3)] == [5 + 5 + 3, 17 + 5 + 6, 33 + 5 + 9]
    lm.close()
    assert worst <= TOL, worst


def test_step_batch_rejects_bad_arguments_without_changing_state(tiny):
    pkg, wl, spec, w_cpu, w_dev, stream, ref = tiny
    lm = _new(tiny, max_seqs=3, max_positions=40)
    lm.prefill(0, spec["prompt"][:30])
    lm.prefill(1, spec["prompt"][:10])
    before = lm.logits(0).copy()
    for args, code in ((([0, 0], None, None), pkg.E_INVAL), (([0, 3], None, None), pkg.E_INVAL),
                       (([0, 2], None, None), pkg.E_STATE), (([0, 1], [0, wl.model.vocab], None), pkg.E_INVAL),
                       (([1, 0], None, [[1], list(range(10))]), pkg.E_CAPACITY),
                       (([0, 1], None, [[], [wl.model.vocab]]), pkg.E_INVAL)):
        with pytest.raises(pkg.AsyncLMError) as ei:
            lm.step_batch(*args)
        assert ei.value.code == code, args
    assert lm.seq_len(0) == 30 and lm.seq_len(1) == 10
    assert np.array_equal(lm.logits(0), before)
    lm.close()


def test_banned_tokens_change_the_greedy_choice_only(tiny):
    """Device half of the token monitor (Sec. 5.1): banned ids are skipped by the greedy choice, starting with
    the very next token, and the logits stay unmasked."""
    pkg, wl, spec, w_cpu, w_dev, stream, ref = tiny
    sh = orc.Shape.of(wl.model)
    dec = orc.CachedDecoder(sh, w_cpu)
    dec.prefill(spec["prompt"])
    lm = _new(tiny)
    lm.prefill(0, spec["prompt"])
    order = list(np.argsort(-dec.logits, kind="stable"))
    for banned in ([order[0]], [order[0], order[1], order[2]], [], [order[1]]):
        lm.set_banned_tokens(0, banned)
        want = dec.decode_step(banned=banned)
        got = lm.decode_step(0)
        assert got == want, banned
        assert np.abs(lm.logits(0) - dec.logits).max() <= TOL
        order = list(np.argsort(-dec.logits, kind="stable"))
    # a list set before a forward pass applies to the token chosen after it, forced tokens ignore the list
    lm.set_banned_tokens(0, [order[0]])
    assert lm.decode_step(0, forced_token=int(order[0])) == order[0]
    dec.decode_step(forced=int(order[0]))
    top = int(np.argmax(dec.logits))
    lm.set_banned_tokens(0, [top])
    assert lm.decode_step(0) == dec.decode_step(banned=[top])
    with pytest.raises(pkg.AsyncLMError):
        lm.set_banned_tokens(0, [wl.model.vocab])
    with pytest.raises(pkg.AsyncLMError):
        lm.set_banned_tokens(0, list(range(32)))
    lm.close()


def test_kv_swap_out_and_in_restores_the_sequence_exactly(tiny):
    """Trap handling (Sec. 5.4): the K/V state swapped to host memory and back continues bit-identically, also
    into another sequence slot and after the slot was used for something else."""
    pkg, wl, spec, w_cpu, w_dev, stream, ref = tiny
    lm = _new(tiny, max_seqs=2)
    s = ref["stream"]
    lm.prefill(0, s[:50])
    for t in s[50:55]:
        lm.decode_step(0, forced_token=t)
    nbytes = lm.kv_bytes(0)
    buf = torch.empty(nbytes, dtype=torch.uint8).pin_memory()
    with pytest.raises(pkg.AsyncLMError) as ei:
        lm.kv_swap_out(0, buf.data_ptr(), nbytes - 1)
    assert ei.value.code == pkg.E_CAPACITY
    lm.kv_swap_out(0, buf.data_ptr(), nbytes)
    before = lm.logits(0).copy()
    # uninterrupted continuation, for reference
    want_tok = [lm.decode_step(0) for _ in range(4)]
    want = lm.logits(0).copy()
    lm.reset(0)
    lm.prefill(0, s[3:20])                       # the slot is reused while the sequence is paused
    lm.reset(0)
    with pytest.raises(pkg.AsyncLMError) as ei:
        lm.kv_swap_in(1, buf.data_ptr(), nbytes - 8)
    assert ei.value.code == pkg.E_INVAL and lm.seq_len(1) == 0
    for slot in (0, 1):
        lm.kv_swap_in(slot, buf.data_ptr(), nbytes)
        assert lm.seq_len(slot) == 55
        assert np.array_equal(lm.logits(slot), before)
        assert [lm.decode_step(slot) for _ in range(4)] == want_tok
        assert np.array_equal(lm.logits(slot), want)
    with pytest.raises(pkg.AsyncLMError) as ei:
        lm.kv_swap_in(0, buf.data_ptr(), nbytes)  # not empty
    assert ei.value.code == pkg.E_STATE
    # and the result is the oracle's
    assert np.abs(want - orc.full_logits(orc.Shape.of(wl.model), w_cpu, list(s[:55]) + want_tok)[-1]).max() <= TOL
    lm.close()


def test_interruptible_session_end_to_end_matches_oracle_replay(tiny):
    """The host control plane driving the library (token masks, peek, merged token + interrupt passes, forced
    trap END, pause / resume) against a replay with the CPU oracle under the same rules: identical token stream,
    logits within tolerance, the interrupt marker never generated, no interrupt inside a call block."""
    pkg, wl, spec, w_cpu, w_dev, stream, ref = tiny
    sh = orc.Shape.of(wl.model)
    prompt = spec["prompt"]
    # CML ids taken from tokens this random model likes to generate, so that a call block opens and closes, an
    # interrupt is deferred and a trap pauses the session within the run (checked below)
    cml = pkg.CML(call=65, intr=1001, trap=930, end=313, head=191)
    arrivals = {1: ([7], [8, 9]), 4: ([10], [11]), 12: ([12, 13], [14] * 5), 30: ([15], [16])}
    n_steps = 48

    def blocks_of(q):
        out = []
        for cid, val in q:
            out += [cml.intr] + cid + [cml.head] + val + [cml.end]
        return out

    # replay with the oracle
    dec = orc.CachedDecoder(sh, w_cpu)
    dec.prefill(prompt)
    mon = ReferenceMonitor(cml)
    queue, paused, want_stream, deferred, calls, traps = [], False, [], 0, 0, 0
    for t in range(n_steps):
        if t in arrivals:
            queue.append(arrivals[t])
        if paused:
            if queue:
                b = blocks_of(queue); queue = []
                dec.inject(b); want_stream += b; paused = False
            continue
        forced = mon.forced()
        tok = forced if forced is not None else orc.greedy(dec.logits, mon.banned())
        merge = forced is None and not mon.critical and queue and tok not in (cml.call, cml.trap)
        if queue and not merge:
            deferred += 1
        dec.decode_step(forced=tok)
        want_stream.append(tok)
        if merge:
            b = blocks_of(queue); queue = []
            dec.inject(b); want_stream += b
        evn = mon.observe(tok)
        if evn is not None and evn[0] == "call":
            calls += 1
        if evn is not None and evn[0] == "trap":
            paused = True
            traps += 1
    assert calls >= 1 and deferred >= 1 and traps >= 1, (calls, deferred, traps)    # the run exercises all three

    lm = _new(tiny, max_positions=400)
    lm.prefill(0, prompt)
    ses = pkg.InterruptibleSession(lm, 0, cml)
    got_calls = 0
    for t in range(n_steps):
        if t in arrivals:
            ses.submit_interrupt(*arrivals[t])
        r = ses.step()
        assert r.token != cml.intr
        got_calls += r.call is not None
    assert ses.stream == want_stream
    assert got_calls == calls
    assert lm.seq_len(0) == len(prompt) + len(want_stream) == dec.length
    assert np.abs(lm.logits(0) - dec.logits).max() <= TOL
    lm.close()


def test_session_group_end_to_end_matches_oracle_replays(tiny):
    """Three sessions of one context driven by SessionGroup: every iteration is one batched pass carrying each running
    session's chosen token and queued interrupts.  Each session is replayed alone with the CPU oracle under the same
    rules (mask per monitor state, interrupts only outside blocks, trap END forced, pause / resume): identical token
    streams and logits within tolerance for every session."""
    pkg, wl, spec, w_cpu, w_dev, stream, ref = tiny
    sh = orc.Shape.of(wl.model)
    cml = pkg.CML(call=65, intr=1001, trap=930, end=313, head=191)
    prompts = [spec["prompt"], spec["prompt"][5:50], [int(t) for t in ai.uniform_tokens(ai.MASTER_SEED, 941, 33, wl.model.vocab)]]
    arrivals = [{1: ([7], [8, 9]), 4: ([10], [11]), 12: ([12, 13], [14] * 5), 30: ([15], [16])},
                {0: ([20], [21]), 9: ([22], [23, 24, 25])},
                {3: ([30], [31] * 7), 17: ([32], [33]), 18: ([34], [35])}]
    n_steps = 40

    def blocks_of(q):
        out = []
        for cid, val in q:
            out += [cml.intr] + cid + [cml.head] + val + [cml.end]
        return out

    want, decs = [], []
    for prompt, arr in zip(prompts, arrivals):
        dec = orc.CachedDecoder(sh, w_cpu)
        dec.prefill(prompt)
        mon = ReferenceMonitor(cml)
        queue, paused, out = [], False, []
        for t in range(n_steps):
            if t in arr:
                queue.append(arr[t])
            if paused:
                if queue:
                    b = blocks_of(queue); queue = []
                    dec.inject(b); out += b; paused = False
                continue
            forced = mon.forced()
            tok = forced if forced is not None else orc.greedy(dec.logits, mon.banned())
            dec.decode_step(forced=tok)
            out.append(tok)
            evn = mon.observe(tok)
            trapped = evn is not None and evn[0] == "trap"
            if queue and not mon.critical and not trapped:
                b = blocks_of(queue); queue = []
                dec.inject(b); out += b
            if trapped:
                paused = True
        want.append(out); decs.append(dec)

    lm = _new(tiny, max_positions=400, max_seqs=3)
    for q, prompt in enumerate(prompts):
        lm.prefill(q, prompt)
    sessions = [pkg.InterruptibleSession(lm, q, cml) for q in range(3)]
    grp = pkg.SessionGroup(lm, sessions)
    for t in range(n_steps):
        for q, arr in enumerate(arrivals):
            if t in arr:
                sessions[q].submit_interrupt(*arr[t])
        for r in grp.step():
            assert r.token != cml.intr
    for q in range(3):
        assert sessions[q].stream == want[q], q
        assert lm.seq_len(q) == decs[q].length
        assert np.abs(lm.logits(q) - decs[q].logits).max() <= TOL
    lm.close()
