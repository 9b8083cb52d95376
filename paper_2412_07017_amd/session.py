"""Host control plane of one interruptible generation session, above the C ABI.

What the paper's inference process does around the model (Fig. 4, Sec. 3, Sec. 5), on token ids only:

* token monitor (Sec. 5.1): a finite-state machine over the CML tokens that keeps the generated stream
  well-formed by masking the next-token choice (the interrupt marker can never be generated; inside a call
  block only the block's own structure is allowed), detects completed calls and traps, and sets the
  critical-section flag;
* critical section (Sec. 3.2): while a call block is being generated, interrupts are not injected; they wait
  in the queue until the block is closed;
* interrupt manager (Sec. 5.3): interrupts handed in by executor threads are queued; when the session is
  interruptible, ALL queued interrupts are formatted as interrupt blocks, concatenated, and appended to the
  token that was just chosen, so the model processes them in the same forward pass (asynclm_step_batch on one
  sequence);
* trap (Sec. 3.3 / 5.4): after a trap block the session pauses; it resumes when an interrupt arrives;
* several sessions (SessionGroup): one batched pass per iteration carries every running session's chosen token
  and queued interrupts.

The CML text grammar, tokenisation and the executor itself are outside: this class sees integer ids.  A call
block is  CALL id.. HEAD body.. END,  an interrupt block  INTR id.. HEAD value.. END,  a trap  TRAP END.
"""
from __future__ import annotations

import threading
from collections import deque
from dataclasses import dataclass, field
from typing import Deque, List, Optional, Sequence, Tuple

TEXT, CALL_ID, CALL_BODY, TRAP_OPEN = "text", "call_id", "call_body", "trap_open"


@dataclass(frozen=True)
class CML:
    """Token ids of the five CML markers (Sec. 3)."""
    call: int
    intr: int
    trap: int
    end: int
    head: int

    def all(self) -> Tuple[int, ...]:
        return (self.call, self.intr, self.trap, self.end, self.head)


@dataclass
class StepResult:
    token: Optional[int]                       # None: the session is paused (trap) and nothing was generated
    injected: List[int] = field(default_factory=list)      # interrupt tokens appended with this token
    call: Optional[Tuple[List[int], List[int]]] = None     # (id tokens, body tokens) of a call completed by this token
    trapped: bool = False                      # this token completed a trap block: the session is now paused


class TokenMonitor:
    """The CML state machine.  `banned()` is the mask for the next choice, `forced()` a token that must come next
    (the END of a trap block), `observe(token)` advances the state and reports completed calls / traps."""

    def __init__(self, cml: CML):
        self.cml = cml
        self.state = TEXT
        self._id: List[int] = []
        self._body: List[int] = []

    @property
    def critical(self) -> bool:
        """True while a call or trap block is open: no interrupt may be inserted (Sec. 3.2)."""
        return self.state != TEXT

    def banned(self) -> List[int]:
        c = self.cml
        if self.state == TEXT:
            return [c.intr, c.head, c.end]             # blocks are opened with CALL or TRAP only
        if self.state == CALL_ID:
            return [c.call, c.intr, c.trap, c.end]     # the identifier ends with HEAD
        if self.state == CALL_BODY:
            return [c.call, c.intr, c.trap, c.head]    # the body ends with END
        return [c.intr]

    def forced(self) -> Optional[int]:
        return self.cml.end if self.state == TRAP_OPEN else None

    def observe(self, token: int):
        """Returns ("call", ids, body) / ("trap",) / None."""
        c = self.cml
        if self.state == TEXT:
            if token == c.call:
                self.state, self._id, self._body = CALL_ID, [], []
            elif token == c.trap:
                self.state = TRAP_OPEN
            elif token in (c.intr, c.head, c.end):
                raise ValueError("token %d is not allowed outside a block" % token)
            return None
        if self.state == CALL_ID:
            if token == c.head:
                self.state = CALL_BODY
            elif token in (c.call, c.intr, c.trap, c.end):
                raise ValueError("token %d is not allowed in a call identifier" % token)
            else:
                self._id.append(token)
            return None
        if self.state == CALL_BODY:
            if token == c.end:
                self.state = TEXT
                return ("call", list(self._id), list(self._body))
            if token in (c.call, c.intr, c.trap, c.head):
                raise ValueError("token %d is not allowed in a call body" % token)
            self._body.append(token)
            return None
        if token != c.end:
            raise ValueError("a trap block is TRAP END")
        self.state = TEXT
        return ("trap",)


class InterruptibleSession:
    """One sequence of an AsyncLM context driven as in Fig. 4.  `lm` needs decode_step, step_batch and
    set_banned_tokens (paper_2412_07017_amd.AsyncLM has them; tests use a scripted stand-in)."""

    def __init__(self, lm, seq: int, cml: CML):
        self.lm, self.seq, self.cml = lm, seq, cml
        self.monitor = TokenMonitor(cml)
        self._queue: Deque[Tuple[List[int], List[int]]] = deque()
        self._lock = threading.Lock()
        self.paused = False
        self.stream: List[int] = []            # tokens this session appended to the context (generated + injected)
        self._mask: Optional[List[int]] = None

    # -- executor side (any thread) ---------------------------------------------------------------
    def submit_interrupt(self, call_id: Sequence[int], value: Sequence[int]) -> None:
        """A call returned (Sec. 5.2): queue (identifier tokens, result tokens)."""
        for t in list(call_id) + list(value):
            if t in self.cml.all():
                raise ValueError("CML marker inside an interrupt payload")
        with self._lock:
            self._queue.append((list(call_id), list(value)))

    def pending(self) -> int:
        with self._lock:
            return len(self._queue)

    # -- generation side (one thread) ---------------------------------------------------------------
    def _drain(self) -> List[int]:
        """All queued interrupts as one run of interrupt blocks (Sec. 5.3)."""
        c, out = self.cml, []
        with self._lock:
            while self._queue:
                cid, val = self._queue.popleft()
                out += [c.intr] + cid + [c.head] + val + [c.end]
        return out

    def _set_mask(self) -> None:
        mask = self.monitor.banned()
        if mask != self._mask:
            self.lm.set_banned_tokens(self.seq, mask)
            self._mask = mask

    def step(self) -> StepResult:
        """One iteration: choose a token under the monitor's mask, and if the session is interruptible after
        it, append every queued interrupt in the same forward pass."""
        if self.paused:
            if self.pending() == 0:
                return StepResult(token=None)
            # resume: the interrupts become the next rows of the context on their own
            blocks = self._drain()
            self.lm.inject_interrupt(self.seq, blocks)
            self.stream += blocks
            self.paused = False
            return StepResult(token=None, injected=blocks)
        self._set_mask()
        forced = self.monitor.forced()
        # The choice is made on the device; whether interrupts may follow it depends on the token, which the host
        # only learns afterwards.  A token can open a block (CALL / TRAP) only from the text state, so: in the
        # text state with interrupts pending, choose first with the forward deferred to the merged pass.
        blocks: List[int] = []
        if forced is None and not self.monitor.critical and self.pending():
            token = int(self.lm.peek_choice(self.seq))
            opens = token in (self.cml.call, self.cml.trap)
            if not opens:
                blocks = self._drain()
            got = self.lm.step_batch([self.seq], [token], [blocks])
            assert int(got[0]) == token
        else:
            token = int(self.lm.decode_step(self.seq, -1 if forced is None else forced))
        event = self.monitor.observe(token)
        self.stream += [token] + blocks
        res = StepResult(token=token, injected=blocks)
        if event is not None and event[0] == "call":
            res.call = (event[1], event[2])
        elif event is not None:
            res.trapped = True
            self.paused = True
        return res


class SessionGroup:
    """Several sessions of one AsyncLM context generating together: every iteration is ONE batched forward pass
    (asynclm_step_batch) whose rows are, per running session, [token just chosen] ++ [its queued interrupts], as in
    the interrupt manager of Sec. 5.3 applied to a batch of requests.  Each session keeps its own token monitor,
    mask, critical section, queue and trap state; paused sessions take no rows (a paused session with queued
    interrupts is resumed by an append pass of its own before the batched pass)."""

    def __init__(self, lm, sessions: Sequence[InterruptibleSession]):
        seqs = [s.seq for s in sessions]
        if len(set(seqs)) != len(seqs) or any(s.lm is not lm for s in sessions):
            raise ValueError("sessions must use distinct sequences of the same context")
        self.lm, self.sessions = lm, list(sessions)

    def step(self) -> List[StepResult]:
        results: List[Optional[StepResult]] = [None] * len(self.sessions)
        rows = []                                   # (index, session, token, blocks, event)
        for i, s in enumerate(self.sessions):
            if s.paused:
                if s.pending() == 0:
                    results[i] = StepResult(token=None)
                    continue
                blocks = s._drain()                 # resume: the interrupts become the next rows on their own
                self.lm.inject_interrupt(s.seq, blocks)
                s.stream += blocks
                s.paused = False
                results[i] = StepResult(token=None, injected=blocks)
                continue
            s._set_mask()
            forced = s.monitor.forced()
            # the token is chosen on the device under the session's mask; the host reads it before the pass because
            # whether interrupts may follow it depends on the token (a token that opens a block starts a critical section)
            token = int(self.lm.peek_choice(s.seq)) if forced is None else int(forced)
            event = s.monitor.observe(token)
            trapped = event is not None and event[0] == "trap"
            blocks = s._drain() if (not s.monitor.critical and not trapped and s.pending()) else []
            rows.append((i, s, token, blocks, event))
        if rows:
            got = self.lm.step_batch([r[1].seq for r in rows], [r[2] for r in rows], [r[3] for r in rows])
            for (i, s, token, blocks, event), g in zip(rows, got):
                assert int(g) == token
                s.stream += [token] + blocks
                res = StepResult(token=token, injected=blocks)
                if event is not None and event[0] == "call":
                    res.call = (event[1], event[2])
                elif event is not None:
                    res.trapped = True
                    s.paused = True
                results[i] = res
        return results


class TrapPolicy:
    """What to do with the K/V cache of a paused session (Sec. 5.4): keep it if neither dropping-and-recomputing nor
    swapping to host memory and back can finish within the expected wait for the next interrupt; otherwise take
    the cheaper of the two.  Costs come from models fitted to measurements: swap time linear in the number of
    cached tokens, recomputation time quadratic (Sec. 5.4, Sec. 6.4)."""

    def __init__(self, swap_ms_per_token: float, swap_ms_fixed: float, recompute_quadratic: float,
                 recompute_ms_per_token: float, recompute_ms_fixed: float = 0.0):
        self.swap = (float(swap_ms_per_token), float(swap_ms_fixed))
        self.recompute = (float(recompute_quadratic), float(recompute_ms_per_token), float(recompute_ms_fixed))

    @classmethod
    def fit(cls, points: Sequence[Tuple[int, float, float]]) -> "TrapPolicy":
        """points: (tokens, swap round trip in ms, recompute in ms) measurements; least squares."""
        import numpy as np
        n = np.array([p[0] for p in points], dtype=np.float64)
        sw = np.array([p[1] for p in points], dtype=np.float64)
        rc = np.array([p[2] for p in points], dtype=np.float64)
        a, b = np.linalg.lstsq(np.stack([n, np.ones_like(n)], 1), sw, rcond=None)[0]
        q, l, c = np.linalg.lstsq(np.stack([n * n, n, np.ones_like(n)], 1), rc, rcond=None)[0]
        return cls(a, b, q, l, c)

    def swap_ms(self, tokens: int) -> float:
        return self.swap[0] * tokens + self.swap[1]

    def recompute_ms(self, tokens: int) -> float:
        q, l, c = self.recompute
        return q * tokens * tokens + l * tokens + c

    def decide(self, tokens: int, expected_wait_ms: float) -> str:
        s, r = self.swap_ms(tokens), self.recompute_ms(tokens)
        if s > expected_wait_ms and r > expected_wait_ms:
            return "keep"
        return "recompute" if r < s else "swap"
