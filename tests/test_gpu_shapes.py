"""GPU parity of the matrix-core append path on small bf16 models with other head layouts than the presets:
one, two and four query heads per kv head (the presets have four and eight), d_model 512, so that every kernel
variant runs against the full-vocabulary oracle in seconds: 230-row prefill (wide product, both attention
kernels depending on the number of query tiles), interrupts of 40 rows (k-split product), 70 rows (wide product,
a wave per row tile), 5 rows (weight-streaming product), single-row steps, and a batched step over three
sequences.  The N(0, 0.02) weights make small logits at this width, so the error is also checked relative to the
largest logit."""
import numpy as np
import pytest
import torch

import asynclm_inputs as ai
from asynclm_inputs.configs import ModelConfig
from oracle import asynclm_oracle as orc
from cml_reference import ReferenceMonitor

pytestmark = pytest.mark.gpu

TOL = 2e-2
REL = 2e-4       # measured 9e-6: the hi/lo activation planes and the paired cache keep about 16 mantissa bits


def _host_weights(w_dev):
    conv = lambda t: t.detach().to("cpu").to(torch.float32).numpy()
    return {k: ([conv(t) for t in v] if isinstance(v, list) else conv(v)) for k, v in w_dev.items()}


@pytest.mark.parametrize("n_kv,ffn", [(4, 1024), (2, 1024), (1, 1024), (2, 2240)])
def test_append_path_on_other_head_layouts(n_kv, ffn):
    """ffn 2240: the gate/up product of a pass of up to 32 rows gives a wave 3 gate rows (2240 rows over the 1024 waves
    of the device), which leaves a last tile of 2 rows and waves without a tile."""
    import paper_2412_07017_amd as pkg
    model = ModelConfig(n_layers=2, d_model=512, n_q_heads=4, n_kv_heads=n_kv, head_dim=128, ffn=ffn, vocab=2048,
                        rms_eps=1e-5, rope_theta=10000.0, dtype="bf16")
    w_dev = ai.make_weights(model, device=torch.device("cuda:0"))
    torch.cuda.synchronize()
    w_cpu = _host_weights(w_dev)
    sh = orc.Shape.of(model)
    tk = lambda n, sub: [int(t) for t in ai.uniform_tokens(ai.MASTER_SEED, 921, n, model.vocab, sub=sub)]
    worst_abs, worst_rel = 0.0, 0.0

    def check(got, want, what):
        nonlocal worst_abs, worst_rel
        assert np.isfinite(got).all(), what
        err = float(np.abs(got - want).max())
        rel = err / float(np.abs(want).max())
        worst_abs, worst_rel = max(worst_abs, err), max(worst_rel, rel)
        assert err <= TOL and rel <= REL, (what, err, rel)

    lm = pkg.AsyncLM(model, w_dev, max_positions=512, max_seqs=3, stream=torch.cuda.Stream())
    dec = orc.CachedDecoder(sh, w_cpu, dtype=np.float32)
    check_steps = [("prefill 230", lambda: lm.prefill(0, tk(230, 0)), lambda: dec.prefill(tk(230, 0))),
                   ("inject 40", lambda: lm.inject_interrupt(0, tk(40, 1)), lambda: dec.inject(tk(40, 1))),
                   ("inject 70", lambda: lm.inject_interrupt(0, tk(70, 2)), lambda: dec.inject(tk(70, 2))),
                   ("inject 5", lambda: lm.inject_interrupt(0, tk(5, 3)), lambda: dec.inject(tk(5, 3)))]
    for what, gpu, cpu in check_steps:
        gpu(); cpu()
        check(lm.logits(0), dec.logits, what)
    for j in range(3):
        tok = dec.decode_step()
        assert lm.decode_step(0, forced_token=tok) == tok
        check(lm.logits(0), dec.logits, "decode %d" % j)
    # a batched step: sequence 0 with a 33-row interrupt, two fresh sequences, one of them with a single-token interrupt
    decs = [dec, orc.CachedDecoder(sh, w_cpu, dtype=np.float32), orc.CachedDecoder(sh, w_cpu, dtype=np.float32)]
    for s in (1, 2):
        lm.prefill(s, tk(17 + 30 * s, 10 + s))
        decs[s].prefill(tk(17 + 30 * s, 10 + s))
    intr = [tk(33, 20), [], tk(1, 21)]
    forced = [d.decode_step() for d in decs]
    for d, t in zip(decs, intr):
        if t:
            d.inject(t)
    assert list(lm.step_batch([0, 1, 2], forced, intr)) == forced
    for s, d in enumerate(decs):
        check(lm.logits(s), d.logits, "batched step, sequence %d" % s)
        assert lm.seq_len(s) == d.length
    lm.close()
    print("%d q heads per kv head: max |logit err| = %.3e (%.2e of the largest logit)" % (4 // n_kv, worst_abs, worst_rel))


def test_batched_step_of_many_sequences_with_32_kv_heads_is_cut_into_passes():
    """40 single-row sequences of a model with 32 kv heads: their attention would need more partial results (task x
    kv head x key split) than one pass holds, so the step is cut into two passes; every sequence against its own
    oracle decoder, and nothing is left half done."""
    import paper_2412_07017_amd as pkg
    model = ModelConfig(n_layers=1, d_model=256, n_q_heads=32, n_kv_heads=32, head_dim=128, ffn=256, vocab=640,
                        rms_eps=1e-5, rope_theta=10000.0, dtype="bf16")
    w_dev = ai.make_weights(model, device=torch.device("cuda:0"))
    torch.cuda.synchronize()
    w_cpu = _host_weights(w_dev)
    sh = orc.Shape.of(model)
    ns = 40
    lm = pkg.AsyncLM(model, w_dev, max_positions=64, max_seqs=ns, stream=torch.cuda.Stream())
    decs = []
    for s in range(ns):
        p = [int(t) for t in ai.uniform_tokens(ai.MASTER_SEED, 931, 3 + s % 5, model.vocab, sub=s)]
        lm.prefill(s, p)
        d = orc.CachedDecoder(sh, w_cpu, dtype=np.float32)
        d.prefill(p)
        decs.append(d)
    worst = 0.0
    for step in range(2):
        forced = [d.decode_step() for d in decs]
        assert list(lm.step_batch(list(range(ns)), forced, None)) == forced
        for s, d in enumerate(decs):
            got = lm.logits(s)
            assert np.isfinite(got).all()
            worst = max(worst, float(np.abs(got - d.logits).max()))
            assert lm.seq_len(s) == d.length
    lm.close()
    print("40 sequences x 32 kv heads: max |logit err| = %.3e" % worst)
    assert worst <= TOL


def test_session_group_on_the_batched_matrix_core_path():
    """SessionGroup (host control plane over several sessions) on a bf16 model, where every iteration really is one
    batched pass of the matrix-core append path: token streams identical to per-session oracle replays under the
    same rules, logits within tolerance."""
    import paper_2412_07017_amd as pkg
    model = ModelConfig(n_layers=2, d_model=512, n_q_heads=4, n_kv_heads=2, head_dim=128, ffn=1024, vocab=2048,
                        rms_eps=1e-5, rope_theta=10000.0, dtype="bf16")
    w_dev = ai.make_weights(model, device=torch.device("cuda:0"))
    torch.cuda.synchronize()
    w_cpu = _host_weights(w_dev)
    sh = orc.Shape.of(model)
    cml = pkg.CML(call=2000, intr=2001, trap=2002, end=2003, head=2004)
    tk = lambda n, sub: [int(t) % 1990 for t in ai.uniform_tokens(ai.MASTER_SEED, 951, n, model.vocab, sub=sub)]
    prompts = [tk(70, 0), tk(131, 1), tk(40, 2), tk(200, 3)]
    arrivals = [{0: ([1], tk(20, 10)), 7: ([2], tk(3, 11))}, {3: ([3], tk(45, 12))}, {}, {5: ([4], tk(9, 13)), 6: ([5], tk(70, 14)), 20: ([6], tk(2, 15))}]
    n_steps = 28

    def blocks_of(q):
        out = []
        for cid, val in q:
            out += [cml.intr] + cid + [cml.head] + val + [cml.end]
        return out

    want, decs = [], []
    for prompt, arr in zip(prompts, arrivals):
        dec = orc.CachedDecoder(sh, w_cpu, dtype=np.float32)
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

    lm = pkg.AsyncLM(model, w_dev, max_positions=512, max_seqs=4, stream=torch.cuda.Stream())
    for q, prompt in enumerate(prompts):
        lm.prefill(q, prompt)
    sessions = [pkg.InterruptibleSession(lm, q, cml) for q in range(4)]
    grp = pkg.SessionGroup(lm, sessions)
    for t in range(n_steps):
        for q, arr in enumerate(arrivals):
            if t in arr:
                sessions[q].submit_interrupt(*arr[t])
        grp.step()
    for q in range(4):
        assert sessions[q].stream == want[q], q
        err = float(np.abs(lm.logits(q) - decs[q].logits).max())
        assert err <= TOL and err / float(np.abs(decs[q].logits).max()) <= REL, (q, err)
        assert lm.seq_len(q) == decs[q].length
    lm.close()
