"""CPU oracle for interruptible decoding: a plain Llama-style causal decoder in numpy.

TEST INFRASTRUCTURE ONLY.  This file is the independent checker for the HIP library; it
shares no code with it and must never be imported by the product path.  It is slow on
purpose: every function is the textbook definition written out, with no blocking or
fusion, so that it can be checked against the paper by eye.

What the paper fixes (arXiv 2412.07017):
  * Sec. 3.2 "Triggering interrupts": an interrupt is a block of tokens inserted at the
    end of the token stream (the LLM context); generation resumes after the block.
  * Sec. 5.3 "Interrupt manager": queued interrupts are appended to the tokens generated
    so far and are processed by the model in the next decoding step.
  * Sec. 5.5: the stateless variant discards the session and recomputes the whole context
    on every interrupt.  Both routes see the same context, so in-flight injection must
    give exactly the logits of a from-scratch pass over the concatenated stream.
The model itself is "Llama 3" (Sec. 1, Sec. 6); the paper specifies none of its internals,
so the decoder below is the standard one: RMSNorm (eps inside the root), rotary position
embedding on half-split pairs (i, i+dh/2), grouped-query causal attention with 1/sqrt(dh)
scaling, SwiGLU feed-forward, no biases, untied output head.

Two forms are given:
  O1  `full_logits`      - from scratch, explicit T x T masked score matrix, no cache.
  O2  `CachedDecoder`    - incremental, with a K/V cache and an append-chunk entry.
O1 is the definition; O2 is what gets timed and used on large shapes; tests tie O2 to O1.

Parity status: the paper prints no numeric model outputs, so absolute logit values are
"parity unpinned" by the paper.  They are pinned instead by (tests/test_oracle_pins.py):
an independent library implementation of the same architecture (transformers' Llama),
library attention / norm / activation routines, closed forms (zero output projections),
and invariants (causality, rotary shift invariance, GQA = replicated MHA, softmax rows
sum to one, inject == re-prefill of the concatenation).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np


@dataclass
class Shape:
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    vocab: int
    rms_eps: float
    rope_theta: float

    @classmethod
    def of(cls, cfg) -> "Shape":
        return cls(cfg.n_layers, cfg.d_model, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim,
                   cfg.ffn, cfg.vocab, cfg.rms_eps, cfg.rope_theta)


# ----------------------------------------------------------------------------------------
# elementary definitions
# ----------------------------------------------------------------------------------------

def rmsnorm(x: np.ndarray, gain: np.ndarray, eps: float) -> np.ndarray:
    """h_i = x_i * g_i / sqrt(mean_j x_j^2 + eps), over the last axis."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x * gain / np.sqrt(ms + eps)


def rope_rotate(u: np.ndarray, positions: np.ndarray, theta: float) -> np.ndarray:
    """Rotary embedding of u[T, H, dh] at absolute positions[T].

    Pair i couples components i and i + dh/2 and turns them by phi = t * theta^(-2i/dh).
    Angles are formed in float64 whatever the dtype of u.
    """
    T, H, dh = u.shape
    half = dh // 2
    inv_freq = np.float64(theta) ** (-2.0 * np.arange(half, dtype=np.float64) / dh)
    phi = positions.astype(np.float64)[:, None] * inv_freq[None, :]        # [T, half]
    c = np.cos(phi).astype(u.dtype)[:, None, :]
    s = np.sin(phi).astype(u.dtype)[:, None, :]
    a, b = u[..., :half], u[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def silu(z: np.ndarray) -> np.ndarray:
    return z / (1.0 + np.exp(-z))


def softmax_rows(s: np.ndarray) -> np.ndarray:
    """Softmax over the last axis with max subtraction; -inf entries get weight 0."""
    m = np.max(s, axis=-1, keepdims=True)
    e = np.exp(s - m)
    return e / np.sum(e, axis=-1, keepdims=True)


def greedy(logits: np.ndarray, banned: Sequence[int] = ()) -> int:
    """Index of the maximum; the lowest index wins ties.  `banned` ids are not eligible (the token
    monitor of Sec. 5.1 removes tokens such as the interrupt marker from the next-token distribution)."""
    if len(banned) == 0:
        return int(np.argmax(logits))
    masked = np.array(logits, dtype=np.float64, copy=True)
    masked[np.asarray(list(banned), dtype=np.int64)] = -np.inf
    return int(np.argmax(masked))


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16 (ties to even), returned as fp32.  Diagnostic use."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((b >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((b + r) & np.uint32(0xFFFF0000)).view(np.float32)


def _split_qkv(shape: Shape, wqkv: np.ndarray) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    nq, nkv = shape.n_q_heads * shape.head_dim, shape.n_kv_heads * shape.head_dim
    return wqkv[:nq], wqkv[nq:nq + nkv], wqkv[nq + nkv:nq + 2 * nkv]


def _cast(w, dtype):
    return w if w.dtype == dtype else w.astype(dtype)


# ----------------------------------------------------------------------------------------
# O1: from-scratch definition
# ----------------------------------------------------------------------------------------

def full_logits(shape: Shape, w: Dict[str, object], tokens: Sequence[int],
                dtype=np.float64, return_probs: bool = False, pos0: int = 0):
    """Next-token logits at every position of `tokens`: array [T, V].

    Follows the definition directly: embeds all T tokens, and in every layer forms the full
    T x T score matrix per query head with future positions set to -inf.
    If return_probs, also returns the attention probabilities [layer][Hq, T, T].
    `pos0` is the absolute position given to the first token (0 in normal use).
    """
    tokens = np.asarray(tokens, dtype=np.int64)
    T = tokens.shape[0]
    Hq, Hkv, dh = shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    group = Hq // Hkv
    pos = pos0 + np.arange(T)
    x = _cast(w["embed"][tokens], dtype)                                    # [T, d]
    future = np.triu(np.ones((T, T), dtype=bool), k=1)                       # j > t
    all_probs = []
    for l in range(shape.n_layers):
        wq, wk, wv = _split_qkv(shape, w["wqkv"][l])
        h = rmsnorm(x, _cast(w["attn_norm"][l], dtype), shape.rms_eps)
        q = (h @ _cast(wq, dtype).T).reshape(T, Hq, dh)
        k = (h @ _cast(wk, dtype).T).reshape(T, Hkv, dh)
        v = (h @ _cast(wv, dtype).T).reshape(T, Hkv, dh)
        q = rope_rotate(q, pos, shape.rope_theta)
        k = rope_rotate(k, pos, shape.rope_theta)
        o = np.zeros((T, Hq, dh), dtype=dtype)
        probs = np.zeros((Hq, T, T), dtype=dtype)
        for hq in range(Hq):
            hk = hq // group
            s = (q[:, hq, :] @ k[:, hk, :].T) / np.sqrt(dtype(dh))          # [T, T]
            s = np.where(future, -np.inf, s)
            p = softmax_rows(s)
            probs[hq] = p
            o[:, hq, :] = p @ v[:, hk, :]
        all_probs.append(probs)
        x = x + o.reshape(T, Hq * dh) @ _cast(w["wo"][l], dtype).T
        h2 = rmsnorm(x, _cast(w["ffn_norm"][l], dtype), shape.rms_eps)
        F = shape.ffn
        wg, wu = w["wgate_up"][l][:F], w["wgate_up"][l][F:]
        a = silu(h2 @ _cast(wg, dtype).T) * (h2 @ _cast(wu, dtype).T)
        x = x + a @ _cast(w["wdown"][l], dtype).T
    logits = rmsnorm(x, _cast(w["final_norm"], dtype), shape.rms_eps) @ _cast(w["lm_head"], dtype).T
    if return_probs:
        return logits, all_probs
    return logits


# ----------------------------------------------------------------------------------------
# O2: incremental form with a K/V cache
# ----------------------------------------------------------------------------------------

class CachedDecoder:
    """One sequence with a live K/V cache.

    `prefill`, `inject` and the forward of `decode_step` are the same operation: append a
    chunk of tokens to the end of the context (Sec. 3.2) and leave the logits that predict
    the token after the chunk.  `kv_round` (diagnostic only) rounds K and V to bf16 when
    they are written, to separate cache quantisation from kernel errors.  `diag_round` (diagnostic
    only, never used by a graded comparison) names further values to round to bf16, to measure what
    each reduced-precision storage choice of an implementation would cost in the logits:
      "k", "v"   cache rows at write (kv_round = both)
      "h"        the normalised inputs of the QKV, gate/up products     } only in passes of more
      "o"        the attention output (input of the O projection)       } than one row when
      "a"        the SwiGLU output (input of the down projection)       } "chunk_only" is also
      "q", "p"   the rotated queries / the softmax probabilities        } named
    """

    def __init__(self, shape: Shape, w: Dict[str, object], dtype=np.float64, kv_round: bool = False,
                 capacity: int = 0, diag_round: Sequence[str] = ()):
        self.shape, self.w, self.dtype, self.kv_round = shape, w, dtype, kv_round
        self.diag_round = frozenset(diag_round)
        L, Hkv, dh = shape.n_layers, shape.n_kv_heads, shape.head_dim
        # storage grows by doubling; rows [0, length) are valid
        cap = max(int(capacity), 16)
        self._k: List[np.ndarray] = [np.zeros((cap, Hkv, dh), dtype=dtype) for _ in range(L)]
        self._v: List[np.ndarray] = [np.zeros((cap, Hkv, dh), dtype=dtype) for _ in range(L)]
        self.tokens: List[int] = []
        self.logits: Optional[np.ndarray] = None

    @property
    def length(self) -> int:
        return len(self.tokens)

    def _store(self, l: int, at: int, k: np.ndarray, v: np.ndarray) -> None:
        need = at + k.shape[0]
        if need > self._k[l].shape[0]:
            cap = max(need, 2 * self._k[l].shape[0])
            for buf in (self._k, self._v):
                grown = np.zeros((cap,) + buf[l].shape[1:], dtype=self.dtype)
                grown[:at] = buf[l][:at]
                buf[l] = grown
        self._k[l][at:need] = k
        self._v[l][at:need] = v

    def keys(self, l: int) -> np.ndarray:
        return self._k[l][:self.length]

    def values(self, l: int) -> np.ndarray:
        return self._v[l][:self.length]

    def append(self, chunk: Sequence[int]) -> np.ndarray:
        sh, w, dt = self.shape, self.w, self.dtype
        chunk = np.asarray(chunk, dtype=np.int64)
        M = chunk.shape[0]
        if M == 0:
            raise ValueError("empty chunk")
        L0 = self.length
        Hq, Hkv, dh = sh.n_q_heads, sh.n_kv_heads, sh.head_dim
        group = Hq // Hkv
        pos = np.arange(L0, L0 + M)
        x = _cast(w["embed"][chunk], dt)
        # row r (absolute position L0 + r) may look at keys 0 .. L0 + r
        key_pos = np.arange(L0 + M)[None, :]
        hidden = key_pos > pos[:, None]
        # diagnostic rounding (identity in every graded use): see the class comment
        diag = self.diag_round if (M > 1 or "chunk_only" not in self.diag_round) else frozenset(self.diag_round & {"k", "v"})
        rd = lambda name, val: round_to_bf16(val).astype(dt) if name in diag else val
        for l in range(sh.n_layers):
            wq, wk, wv = _split_qkv(sh, w["wqkv"][l])
            h = rd("h", rmsnorm(x, _cast(w["attn_norm"][l], dt), sh.rms_eps))
            q = rope_rotate((h @ _cast(wq, dt).T).reshape(M, Hq, dh), pos, sh.rope_theta)
            k = rope_rotate((h @ _cast(wk, dt).T).reshape(M, Hkv, dh), pos, sh.rope_theta)
            v = (h @ _cast(wv, dt).T).reshape(M, Hkv, dh)
            if self.kv_round or "k" in self.diag_round:
                k = round_to_bf16(k).astype(dt)
            if self.kv_round or "v" in self.diag_round:
                v = round_to_bf16(v).astype(dt)
            q = rd("q", q)
            self._store(l, L0, k, v)
            K, Vv = self._k[l][:L0 + M], self._v[l][:L0 + M]
            o = np.zeros((M, Hq, dh), dtype=dt)
            for hq in range(Hq):
                hk = hq // group
                s = (q[:, hq, :] @ K[:, hk, :].T) / np.sqrt(dt(dh))
                s = np.where(hidden, -np.inf, s)
                o[:, hq, :] = rd("p", softmax_rows(s)) @ Vv[:, hk, :]
            x = x + rd("o", o.reshape(M, Hq * dh)) @ _cast(w["wo"][l], dt).T
            h2 = rd("h", rmsnorm(x, _cast(w["ffn_norm"][l], dt), sh.rms_eps))
            F = sh.ffn
            a = rd("a", silu(h2 @ _cast(w["wgate_up"][l][:F], dt).T) * (h2 @ _cast(w["wgate_up"][l][F:], dt).T))
            x = x + a @ _cast(w["wdown"][l], dt).T
        last = rmsnorm(x[-1], _cast(w["final_norm"], dt), sh.rms_eps)
        self.logits = _cast(w["lm_head"], dt) @ last
        self.tokens.extend(int(t) for t in chunk)
        return self.logits

    def prefill(self, tokens: Sequence[int]) -> np.ndarray:
        if self.length != 0:
            raise RuntimeError("prefill on a non-empty sequence")
        return self.append(tokens)

    def inject(self, tokens: Sequence[int]) -> np.ndarray:
        if self.length == 0:
            raise RuntimeError("inject on an empty sequence")
        return self.append(tokens)

    def decode_step(self, forced: Optional[int] = None, banned: Sequence[int] = ()) -> int:
        """Choose the next token (greedy over the ids not in `banned`, unless forced), append it, run one forward."""
        if self.logits is None:
            raise RuntimeError("decode on an empty sequence")
        tok = greedy(self.logits, banned) if forced is None else int(forced)
        self.append([tok])
        return tok


# ----------------------------------------------------------------------------------------
# stream construction
# ----------------------------------------------------------------------------------------

def run_stream(shape: Shape, w: Dict[str, object], prompt: Sequence[int], n_decode: int,
               events: Sequence[Tuple[int, Sequence[int]]], dtype=np.float64,
               kv_round: bool = False, progress=None) -> Dict[str, object]:
    """Greedy generation with interrupts spliced in.

    An event (n, I) appends the tokens I once the n-th generated token is in the stream and
    before the (n+1)-th is chosen, so token n+1 is predicted from the last token of I.

    Returns
      generated : the n_decode greedy tokens g_1..g_n
      choose_logits[j] : the logits g_{j+1} was chosen from (j = 0..n_decode-1)
      final_logits : logits after the last generated token was processed
      inject_logits : {n: logits right after the event at step n}
      stream : the whole context in order
    """
    dec = CachedDecoder(shape, w, dtype=dtype, kv_round=kv_round)
    ev = {int(n): np.asarray(t) for n, t in events}
    dec.prefill(prompt)
    generated, choose_logits, inject_logits = [], [], {}
    for j in range(1, n_decode + 1):
        choose_logits.append(dec.logits.copy())
        generated.append(dec.decode_step())
        if j in ev and j < n_decode + 1:
            dec.inject(ev[j])
            inject_logits[j] = dec.logits.copy()
        if progress is not None:
            progress(j)
    return {"generated": generated, "choose_logits": choose_logits, "final_logits": dec.logits.copy(),
            "inject_logits": inject_logits, "stream": list(dec.tokens)}


def top2_margin(logits: np.ndarray) -> float:
    part = np.partition(logits, -2)
    return float(part[-1] - part[-2])
