"""Latency model of synchronous, synchronous-parallel and asynchronous function calling (Sec. 6.3, App. A.1),
and a small event simulator of the asynchronous schedule that the closed forms describe.

A function call f has a generation time G(f) (its call block's tokens times the time per output token) and an
execution time E(f).  Tokens are generated sequentially by one model; executions run concurrently.
  sync           every call is generated, then executed, then the next one:   sum G + sum E
  sync-parallel  all calls are generated, then executed together:               sum G + max E
  async          a call starts executing as soon as its block is generated; generation continues meanwhile;
                 with independent calls in LPT order (longest execution first):
                 max_f ( E(f) + sum of G(g) over the calls g generated up to and including f )
The simulator also handles dependencies (a call can only be generated once the results it needs have arrived)
and, optionally, the cost of processing each interrupt (extra decoding time when a result is injected), which
is where the measured decode and inject times of the GPU path plug in.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple


@dataclass(frozen=True)
class Call:
    name: str
    gen: float                     # G(f)
    exe: float                     # E(f)
    deps: Tuple[str, ...] = ()     # calls whose results this one needs before it can be generated


def latency_sync(calls: Sequence[Call]) -> float:
    return sum(c.gen for c in calls) + sum(c.exe for c in calls)


def latency_sync_parallel(calls: Sequence[Call]) -> float:
    return sum(c.gen for c in calls) + max(c.exe for c in calls)


def latency_async_lpt(calls: Sequence[Call]) -> float:
    """Closed form for independent calls under LPT: pred(f) = the calls with E >= E(f)."""
    return max(f.exe + sum(g.gen for g in calls if g.exe >= f.exe) for f in calls)


def lpt_order(calls: Sequence[Call]) -> List[Call]:
    return sorted(calls, key=lambda c: -c.exe)


def simulate_async(calls: Sequence[Call], order: Optional[Sequence[str]] = None, policy: str = "lpt",
                   interrupt_cost: float = 0.0) -> Tuple[float, List[str]]:
    """Event simulation of asynchronous calling.  The model generates one call block at a time; a call's
    execution starts when its block is complete and runs concurrently with everything else.  With `order`, the
    calls are generated in exactly that order (waiting for missing results when necessary); otherwise the next
    call is chosen among those whose dependencies have returned by `policy` ("lpt": longest execution first,
    "fifo": input order).  Every returned result costs the model `interrupt_cost` of decoding time when it is
    injected (at the next block boundary).  Returns (time when the last result is in the context, generation order).
    """
    by_name: Dict[str, Call] = {c.name: c for c in calls}
    done_at: Dict[str, float] = {}         # call -> time its result is available
    seen: set = set()                      # results already injected into the context
    t, generated = 0.0, []
    pending = list(order) if order is not None else None
    remaining = [c.name for c in calls]

    def absorb(now: float) -> float:
        """Inject every result that has returned by `now` (each costs interrupt_cost of model time)."""
        while True:
            ready = sorted((n for n, d in done_at.items() if d <= now and n not in seen), key=lambda n: done_at[n])
            if not ready:
                return now
            for n in ready:
                seen.add(n)
                now += interrupt_cost

    while remaining:
        t = absorb(t)
        if pending is not None:
            nxt = pending[0]
            missing = [d for d in by_name[nxt].deps if d not in seen]
            if missing:                     # trap: wait for the earliest missing result, then look again
                t = max(t, min(done_at[d] for d in missing if d in done_at))
                continue
            pending.pop(0)
        else:
            ready = [n for n in remaining if all(d in seen for d in by_name[n].deps)]
            if not ready:                   # trap: nothing can be generated until a result arrives
                t = max(t, min(d for n, d in done_at.items() if n not in seen))
                continue
            nxt = max(ready, key=lambda n: by_name[n].exe) if policy == "lpt" else ready[0]
        c = by_name[nxt]
        t += c.gen
        done_at[nxt] = t + c.exe
        generated.append(nxt)
        remaining.remove(nxt)
    # the task is complete when every result has been injected
    while len(seen) < len(calls):
        t = max(t, min(d for n, d in done_at.items() if n not in seen))
        t = absorb(t)
    return t, generated


def speedup_estimate(mean_exe: float, mean_gen: float) -> float:
    """Theorem 6.2: L_sync / L_async is about 1 + E/G for many calls (error O((E/G)^2))."""
    return 1.0 + mean_exe / mean_gen
