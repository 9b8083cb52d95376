"""Stateless, seeded generators for weights and token streams.

Weights
-------
Element `i` of the tensor with id `t` is a function of (seed, t, i) only, so any slice
can be produced on any device, in any order, with bit-identical results:

  key   = mix64(seed * GAMMA + t)                      (one SplitMix64 finaliser)
  z_j   = mix64(key + (3 i + j + 1) * GAMMA), j=0,1,2   (draws 3i..3i+2 of SplitMix64(key))
  S     = sum of the twelve 16-bit lanes of z_0, z_1, z_2   (exact integer, 0..786420)
  w     = float32(S - 393210) * float32(std * 2^-16)   (one IEEE fp32 multiply)

S is an Irwin-Hall(12) variate with mean 393210 and standard deviation 65536 (to 1e-10
relative), so w approximates N(0, std^2) with tails cut at 6 std.  All steps are integer
operations plus one correctly rounded multiply, hence identical on CPU and GPU.  For
bf16 storage the fp32 value is rounded to nearest-even.

SplitMix64 is the generator of Steele, Lea and Flood, "Fast splittable pseudorandom number
generators" (OOPSLA 2014) with the usual constants.

Tokens
------
Token ids and schedules come from numpy's PCG64 streams seeded by (seed, purpose id).
"""
from __future__ import annotations

from typing import Dict, List

import numpy as np
import torch

from .configs import ModelConfig, Workload, PRESETS

MASTER_SEED = 241207017

_MASK64 = (1 << 64) - 1
_GAMMA = 0x9E3779B97F4A7C15
_M1 = 0xBF58476D1CE4E5B9
_M2 = 0x94D049BB133111EB
_IH_MEAN = 6 * 65535  # 393210

# tensor ids
TID_EMBED, TID_LM_HEAD = 1, 3
TID_LAYER_BASE, TID_LAYER_STRIDE = 16, 8
TID_WQKV, TID_WO, TID_WGATE_UP, TID_WDOWN = 1, 2, 4, 5

# purpose ids of the numpy streams
PURPOSE_PROMPT, PURPOSE_INTR_TOKENS, PURPOSE_INTR_SCHEDULE, PURPOSE_RAGGED = 101, 102, 103, 104


def _signed(u: int) -> int:
    u &= _MASK64
    return u - (1 << 64) if u >= (1 << 63) else u


def _mix64_py(z: int) -> int:
    z &= _MASK64
    z = ((z ^ (z >> 30)) * _M1) & _MASK64
    z = ((z ^ (z >> 27)) * _M2) & _MASK64
    return z ^ (z >> 31)


def splitmix64_draws_py(seed: int, n: int) -> List[int]:
    """First n outputs of SplitMix64 started at `seed` (pure Python, for tests)."""
    return [_mix64_py(seed + (k + 1) * _GAMMA) for k in range(n)]


def tensor_key(seed: int, tensor_id: int) -> int:
    return _mix64_py(seed * _GAMMA + tensor_id)


def _mix64_t(z: torch.Tensor) -> torch.Tensor:
    # int64 arithmetic wraps modulo 2^64; '>>' is arithmetic, so the sign fill is masked off.
    z = (z ^ ((z >> 30) & 0x3FFFFFFFF)) * _signed(_M1)
    z = (z ^ ((z >> 27) & 0x1FFFFFFFFF)) * _signed(_M2)
    return z ^ ((z >> 31) & 0x1FFFFFFFF)


def _lanes16_sum(z: torch.Tensor) -> torch.Tensor:
    return (z & 0xFFFF) + ((z >> 16) & 0xFFFF) + ((z >> 32) & 0xFFFF) + ((z >> 48) & 0xFFFF)


def gaussian_flat(seed: int, tensor_id: int, start: int, count: int, std: float,
                  device: torch.device | str = "cpu") -> torch.Tensor:
    """fp32 values of flat elements [start, start+count) of tensor `tensor_id`."""
    key = tensor_key(seed, tensor_id)
    i = torch.arange(start, start + count, dtype=torch.int64, device=device)
    base = i * _signed(3 * _GAMMA) + _signed(key + _GAMMA)
    s = _lanes16_sum(_mix64_t(base))
    s += _lanes16_sum(_mix64_t(base + _signed(_GAMMA)))
    s += _lanes16_sum(_mix64_t(base + _signed(2 * _GAMMA)))
    scale = float(np.float32(std) * np.float32(2.0 ** -16))
    return (s - _IH_MEAN).to(torch.float32) * scale


def gaussian_tensor(seed: int, tensor_id: int, shape, std: float = 0.02, dtype: str = "fp32",
                    device: torch.device | str = "cpu", chunk: int = 1 << 24) -> torch.Tensor:
    """Whole tensor, generated in chunks to bound temporary memory."""
    n = int(np.prod(shape))
    tdt = torch.float32 if dtype == "fp32" else torch.bfloat16
    out = torch.empty(n, dtype=tdt, device=device)
    for s in range(0, n, chunk):
        c = min(chunk, n - s)
        out[s:s + c] = gaussian_flat(seed, tensor_id, s, c, std, device).to(tdt)
    return out.view(*shape)


def make_weights(model: ModelConfig, seed: int = MASTER_SEED,
                 device: torch.device | str = "cpu") -> Dict[str, object]:
    """All tensors of a decoder: N(0, 0.02) matrices, unit norm gains, no biases.

    Layout (row-major [out, in]): embed [V, d]; lm_head [V, d]; per layer
    wqkv [(Hq + 2 Hkv) dh, d] (query rows, then key rows, then value rows),
    wo [d, Hq dh], wgate_up [2 F, d] (gate rows, then up rows), wdown [d, F].
    """
    m, dt = model, model.dtype
    g = lambda tid, shape: gaussian_tensor(seed, tid, shape, 0.02, dt, device)
    ones = lambda: torch.ones(m.d_model, dtype=torch.float32, device=device)
    w: Dict[str, object] = {
        "embed": g(TID_EMBED, (m.vocab, m.d_model)),
        "final_norm": ones(),
        "lm_head": g(TID_LM_HEAD, (m.vocab, m.d_model)),
        "attn_norm": [], "wqkv": [], "wo": [], "ffn_norm": [], "wgate_up": [], "wdown": [],
    }
    for l in range(m.n_layers):
        b = TID_LAYER_BASE + TID_LAYER_STRIDE * l
        w["attn_norm"].append(ones())
        w["wqkv"].append(g(b + TID_WQKV, (m.qkv_rows, m.d_model)))
        w["wo"].append(g(b + TID_WO, (m.d_model, m.q_dim)))
        w["ffn_norm"].append(ones())
        w["wgate_up"].append(g(b + TID_WGATE_UP, (2 * m.ffn, m.d_model)))
        w["wdown"].append(g(b + TID_WDOWN, (m.d_model, m.ffn)))
    return w


def weights_to_numpy(w: Dict[str, object]) -> Dict[str, object]:
    """Host copy as fp32 numpy arrays (bf16 values widen exactly)."""
    conv = lambda t: t.detach().to("cpu").to(torch.float32).numpy()
    return {k: ([conv(t) for t in v] if isinstance(v, list) else conv(v)) for k, v in w.items()}


def _rng(seed: int, purpose: int, sub: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64([seed, purpose, sub]))


def uniform_tokens(seed: int, purpose: int, n: int, vocab: int, sub: int = 0) -> np.ndarray:
    return _rng(seed, purpose, sub).integers(0, vocab, size=n, dtype=np.int64).astype(np.int32)


def build_workload(name: str, seed: int = MASTER_SEED) -> Dict[str, object]:
    """Token-level description of a preset.

    Single-sequence presets return
      {"prompt": int32[P], "n_decode": N, "events": [(after_step, int32[k]), ...]}
    where an event (n, I) means: once the n-th generated token is in the stream and
    before the (n+1)-th is chosen, append I.  Events with n == n_decode are not emitted
    (they would have no successor token).
    The 16-sequence preset returns per-sequence prompts and, per step, the list of
    (sequence, interrupt tokens) pairs that arrive after that step's token.
    """
    wl: Workload = PRESETS[name]
    V = wl.model.vocab
    if wl.schedule == "ragged16":
        r = _rng(seed, PURPOSE_RAGGED)
        lens = r.integers(512, 4097, size=wl.n_seqs)
        prompts = [uniform_tokens(seed, PURPOSE_PROMPT, int(L), V, sub=s) for s, L in enumerate(lens)]
        rs = _rng(seed, PURPOSE_INTR_SCHEDULE)
        arrive = rs.random((wl.n_decode, wl.n_seqs)) < 0.05
        klen = rs.integers(wl.intr_len, wl.intr_len_hi + 1, size=(wl.n_decode, wl.n_seqs))
        steps = []
        n_ev = 0
        for t in range(wl.n_decode - 1):
            ev = []
            for s in range(wl.n_seqs):
                if arrive[t, s]:
                    ev.append((s, uniform_tokens(seed, PURPOSE_INTR_TOKENS, int(klen[t, s]), V, sub=n_ev)))
                    n_ev += 1
            steps.append(ev)
        steps.append([])
        return {"prompts": prompts, "n_decode": wl.n_decode, "step_events": steps}

    prompt = uniform_tokens(seed, PURPOSE_PROMPT, wl.prompt_len, V)
    if wl.schedule.startswith("single@"):
        at = [int(wl.schedule.split("@")[1])]
    elif wl.schedule == "every":
        at = [n for n in range(wl.intr_every, wl.n_decode, wl.intr_every)]
    elif wl.schedule == "uniform8":
        # A Poisson process conditioned on 8 arrivals in the window: 8 iid uniform steps.
        at = sorted(int(v) for v in _rng(seed, PURPOSE_INTR_SCHEDULE).integers(1, wl.n_decode, size=8))
    else:
        raise ValueError(wl.schedule)
    events = []
    for j, n in enumerate(at):
        toks = uniform_tokens(seed, PURPOSE_INTR_TOKENS, wl.intr_len, V, sub=j)
        if events and events[-1][0] == n:  # simultaneous arrivals are appended together
            events[-1] = (n, np.concatenate([events[-1][1], toks]))
        else:
            events.append((n, toks))
    return {"prompt": prompt, "n_decode": wl.n_decode, "events": events}
