"""Host control plane (token monitor, critical sections, interrupt queue, trap pause) against the rules the
paper states, with a scripted stand-in for the library: no GPU.

Rules checked:
  Sec. 3 / 5.1  the stream stays well-formed CML; the interrupt marker is never generated (always masked);
  Sec. 3.2      no interrupt is inserted while a call block is being generated; it waits in the queue;
  Sec. 5.3      when the session is interruptible, ALL queued interrupts are appended, in arrival order, right
                after the token just generated, in the same forward pass;
  Sec. 3.3      after TRAP END generation pauses and resumes when an interrupt arrives.
"""
import pytest

from paper_2412_07017_amd.session import CML, InterruptibleSession, TokenMonitor
from cml_reference import ReferenceMonitor

C = CML(call=100, intr=101, trap=102, end=103, head=104)


class ScriptedLM:
    """Chooses tokens from a script, honouring the ban list like the device argmax would (a banned scripted
    token is a test error), and records every call."""

    def __init__(self, script):
        self.script = list(script)
        self.banned = []
        self.context = []
        self.log = []

    def _choose(self):
        tok = self.script[0]
        assert tok not in self.banned, ("scripted token is masked", tok, self.banned)
        return tok

    def set_banned_tokens(self, seq, ids):
        self.banned = list(ids)
        self.log.append(("ban", tuple(ids)))

    def peek_choice(self, seq):
        return self._choose()

    def decode_step(self, seq, forced_token=-1):
        tok = self._choose() if forced_token < 0 else forced_token
        if forced_token >= 0:
            assert self.script[0] == forced_token
        self.script.pop(0)
        self.context.append(tok)
        self.log.append(("decode", tok))
        return tok

    def step_batch(self, seqs, forced, interrupts):
        assert list(seqs) == [0] and len(forced) == 1
        assert self.script.pop(0) == forced[0]
        self.context += [forced[0]] + list(interrupts[0])
        self.log.append(("merged", forced[0], tuple(interrupts[0])))
        return [forced[0]]

    def inject_interrupt(self, seq, tokens):
        self.context += list(tokens)
        self.log.append(("inject", tuple(tokens)))


def test_monitor_masks_and_detects_blocks():
    m = TokenMonitor(C)
    assert C.intr in m.banned() and not m.critical
    assert m.observe(7) is None
    assert m.observe(C.call) is None and m.critical
    assert set(m.banned()) == {C.call, C.intr, C.trap, C.end}
    m.observe(11); m.observe(12)
    assert m.observe(C.head) is None and m.critical
    assert set(m.banned()) == {C.call, C.intr, C.trap, C.head}
    m.observe(21)
    assert m.observe(C.end) == ("call", [11, 12], [21]) and not m.critical
    assert m.observe(C.trap) is None and m.critical and m.forced() == C.end
    assert m.observe(C.end) == ("trap",) and m.forced() is None
    with pytest.raises(ValueError):
        m.observe(C.end)
    for state_tokens in ([C.call, C.call], [C.call, 5, C.head, C.head], [C.trap, 5]):
        mm = TokenMonitor(C)
        with pytest.raises(ValueError):
            for t in state_tokens:
                mm.observe(t)


def test_monitor_agrees_with_the_rules_restated_over_the_whole_history():
    """Random streams that respect the masks: after every token the product's state machine and the tests' restatement
    of the rules as a function of the whole history (used by the oracle replays of the GPU session tests) give the same
    mask, forced token, critical flag and completed blocks."""
    import random
    rng = random.Random(2412_07017)
    vocab = list(range(1, 8)) + list(C.all())
    calls = traps = 0
    for _ in range(200):
        m, r = TokenMonitor(C), ReferenceMonitor(C)
        for _ in range(60):
            assert sorted(m.banned()) == sorted(r.banned()) and m.forced() == r.forced() and m.critical == r.critical
            f = m.forced()
            tok = f if f is not None else rng.choice([t for t in vocab if t not in m.banned()])
            em, er = m.observe(tok), r.observe(tok)
            assert em == er
            calls += em is not None and em[0] == "call"
            traps += em is not None and em[0] == "trap"
    assert calls >= 200 and traps >= 200


def test_interrupts_wait_for_the_end_of_a_call_block_and_are_appended_together():
    # text, then a call block  CALL 11 HEAD 21 22 END, then text
    lm = ScriptedLM([5, C.call, 11, C.head, 21, 22, C.end, 6, 7])
    s = InterruptibleSession(lm, 0, C)
    assert s.step().token == 5
    assert s.step().token == C.call                  # opens the critical section
    s.submit_interrupt([31], [41, 42])               # two calls return while the block is being generated
    s.submit_interrupt([32], [43])
    for want in (11, C.head, 21, 22):
        r = s.step()
        assert r.token == want and r.injected == [] and s.pending() == 2
    r = s.step()                                      # END closes the block: not yet interruptible when chosen
    assert r.token == C.end and r.call == ([11], [21, 22]) and r.injected == []
    r = s.step()                                      # first token after the block: both interrupts ride with it
    blocks = [C.intr, 31, C.head, 41, 42, C.end, C.intr, 32, C.head, 43, C.end]
    assert r.token == 6 and r.injected == blocks and s.pending() == 0
    assert s.step().token == 7
    assert lm.context == [5, C.call, 11, C.head, 21, 22, C.end, 6] + blocks + [7]
    assert s.stream == lm.context
    assert ("merged", 6, tuple(blocks)) in lm.log
    # the interrupt marker was masked at every choice
    assert all(C.intr in ids for kind, *rest in lm.log if kind == "ban" for ids in rest)


def test_interrupt_does_not_ride_with_a_token_that_opens_a_block():
    lm = ScriptedLM([5, C.call, 11, C.head, C.end, 8])
    s = InterruptibleSession(lm, 0, C)
    s.step()
    s.submit_interrupt([31], [41])
    r = s.step()                                      # the chosen token opens a call block: the interrupt waits
    assert r.token == C.call and r.injected == [] and s.pending() == 1
    for _ in range(3):
        assert s.step().injected == []
    r = s.step()
    assert r.token == 8 and r.injected == [C.intr, 31, C.head, 41, C.end]


def test_trap_pauses_until_an_interrupt_arrives():
    lm = ScriptedLM([5, C.trap, C.end, 9])
    s = InterruptibleSession(lm, 0, C)
    s.step()
    assert s.step().token == C.trap
    r = s.step()                                      # END is forced by the monitor
    assert r.token == C.end and r.trapped and s.paused
    assert ("decode", C.end) in lm.log
    assert s.step().token is None and s.step().token is None      # nothing is generated while paused
    s.submit_interrupt([31], [41])
    r = s.step()
    assert r.token is None and r.injected == [C.intr, 31, C.head, 41, C.end] and not s.paused
    assert s.step().token == 9
    assert lm.context == [5, C.trap, C.end, C.intr, 31, C.head, 41, C.end, 9]


def test_markers_inside_payloads_are_rejected():
    s = InterruptibleSession(ScriptedLM([1]), 0, C)
    with pytest.raises(ValueError):
        s.submit_interrupt([C.end], [1])


def test_trap_policy_follows_the_rule_of_the_paper():
    """Sec. 5.4: keep if both swap and recompute exceed the expected wait, else the cheaper one; swap is linear and
    recomputation quadratic in the context, so short contexts recompute and long ones swap."""
    from paper_2412_07017_amd.session import TrapPolicy
    p = TrapPolicy(swap_ms_per_token=0.02, swap_ms_fixed=2.0, recompute_quadratic=1e-5, recompute_ms_per_token=0.01)
    assert p.swap_ms(300) == pytest.approx(8.0) and p.recompute_ms(300) == pytest.approx(3.9)
    assert p.decide(300, 100.0) == "recompute"            # both fit, recompute is cheaper
    assert p.decide(300, 1.0) == "keep"                   # neither fits in the wait
    assert p.decide(300, 5.0) == "recompute"              # only recompute fits, and it is the cheaper one
    assert p.decide(4000, 500.0) == "swap"                # 82 ms swap vs 200 ms recompute
    assert p.decide(4000, 50.0) == "keep"
    assert p.decide(4000, 100.0) == "swap"
    # the crossover between recompute and swap is where the two models meet
    n = next(n for n in range(1, 10000) if p.recompute_ms(n) >= p.swap_ms(n))
    assert p.decide(n - 1, 1e9) == "recompute" and p.decide(n + 1, 1e9) == "swap"
    # fitting recovers exact models
    pts = [(n, p.swap_ms(n), p.recompute_ms(n)) for n in (256, 1024, 4096, 16384)]
    f = TrapPolicy.fit(pts)
    assert f.swap_ms(2000) == pytest.approx(p.swap_ms(2000)) and f.recompute_ms(2000) == pytest.approx(p.recompute_ms(2000))


class ScriptedBatchLM:
    """Stand-in with one token script per sequence; records the rows of every batched pass."""

    def __init__(self, scripts):
        self.scripts = {q: list(s) for q, s in scripts.items()}
        self.banned = {q: [] for q in scripts}
        self.context = {q: [] for q in scripts}
        self.passes = []

    def set_banned_tokens(self, seq, ids):
        self.banned[seq] = list(ids)

    def peek_choice(self, seq):
        tok = self.scripts[seq][0]
        assert tok not in self.banned[seq], ("scripted token is masked", seq, tok)
        return tok

    def step_batch(self, seqs, forced, interrupts):
        assert len(set(seqs)) == len(seqs)
        for q, t, it in zip(seqs, forced, interrupts):
            assert self.scripts[q].pop(0) == t
            self.context[q] += [t] + list(it)
        self.passes.append([(q, t, tuple(it)) for q, t, it in zip(seqs, forced, interrupts)])
        return list(forced)

    def inject_interrupt(self, seq, tokens):
        self.context[seq] += list(tokens)
        self.passes.append([(seq, None, tuple(tokens))])


def test_session_group_shares_one_pass_per_iteration_and_keeps_every_session_rule():
    from paper_2412_07017_amd.session import SessionGroup
    scripts = {0: [5, C.call, 11, C.head, 21, C.end, 6, 7],             # a call block in the middle
               1: [8, 9, C.trap, C.end, 30, 31],                          # traps, resumes on an interrupt
               2: [40, 41, 42, 43, 44, 45, 46, 47]}                       # plain text
    lm = ScriptedBatchLM(scripts)
    sess = [InterruptibleSession(lm, q, C) for q in (0, 1, 2)]
    grp = SessionGroup(lm, sess)
    # iteration 1: everybody generates; sequence 2 has an interrupt queued and takes it with its token
    sess[2].submit_interrupt([90], [91, 92])
    r = grp.step()
    assert [x.token for x in r] == [5, 8, 40] and r[2].injected == [C.intr, 90, C.head, 91, 92, C.end]
    assert len(lm.passes) == 1 and len(lm.passes[0]) == 3            # ONE pass with three row groups
    # iteration 2: sequence 0 opens a call block: an interrupt queued for it must wait (Sec. 3.2)
    sess[0].submit_interrupt([70], [71])
    r = grp.step()
    assert r[0].token == C.call and r[0].injected == [] and sess[0].pending() == 1
    # iterations 3-5: inside the block nothing is injected for sequence 0; sequence 1 traps in iteration 4
    r = grp.step(); assert r[0].injected == [] and r[1].token == C.trap
    r = grp.step(); assert r[0].injected == [] and r[1].token == C.end and r[1].trapped and sess[1].paused
    r = grp.step(); assert r[0].token == 21 and r[0].injected == [] and r[1].token is None     # paused: no rows
    assert [q for q, _, _ in lm.passes[-1]] == [0, 2]
    # iteration 6: END closes the call: it is reported and the queued interrupt rides with this very token
    r = grp.step()
    assert r[0].token == C.end and r[0].call == ([11], [21]) and r[0].injected == [C.intr, 70, C.head, 71, C.end]
    # the paused sequence resumes when an interrupt arrives: an append pass of its own, then it rejoins the batch
    sess[1].submit_interrupt([60], [61])
    n_before = len(lm.passes)
    r = grp.step()
    assert r[1].token is None and r[1].injected == [C.intr, 60, C.head, 61, C.end] and not sess[1].paused
    assert lm.passes[n_before] == [(1, None, (C.intr, 60, C.head, 61, C.end))] and [q for q, _, _ in lm.passes[-1]] == [0, 2]
    r = grp.step()
    assert [x.token for x in r] == [7, 30, 47] and [q for q, _, _ in lm.passes[-1]] == [0, 1, 2]
    # every context is the session's own record of its stream, well-formed CML
    for q in (0, 1, 2):
        assert lm.context[q] == sess[q].stream
        m = TokenMonitor(C)
        i = 0
        toks = lm.context[q]
        while i < len(toks):                       # interrupt blocks are skipped as units, the rest must parse
            if toks[i] == C.intr:
                j = toks.index(C.end, i)
                assert C.head in toks[i:j]
                i = j + 1
                continue
            m.observe(toks[i]); i += 1
    with pytest.raises(ValueError):
        SessionGroup(lm, [sess[0], InterruptibleSession(lm, 0, C)])
