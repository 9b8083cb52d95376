"""ctypes binding with the same names as the C ABI in include/asynclm.h (argument marshalling only)."""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence

import numpy as np

E_INVAL, E_STATE, E_CAPACITY, E_NOMEM, E_DEVICE = -1, -2, -3, -4, -5
KV_AUTO, KV_BF16, KV_PAIR_ROWS = 0, 1, 2

API_SYMBOLS = [
    "asynclm_create", "asynclm_destroy", "asynclm_prefill", "asynclm_decode_step",
    "asynclm_inject_interrupt", "asynclm_step_batch", "asynclm_set_banned_tokens", "asynclm_peek_token", "asynclm_kv_bytes", "asynclm_kv_swap_out", "asynclm_kv_swap_in", "asynclm_logits", "asynclm_logits_device", "asynclm_seq_len",
    "asynclm_reset", "asynclm_synchronize", "asynclm_set_option", "asynclm_profile_step", "asynclm_profile_trace",
    "asynclm_strerror", "asynclm_version", "asynclm_greedy_token_static",
]


class _Config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim", "ffn", "vocab")] + \
               [("rms_eps", C.c_float), ("rope_theta", C.c_float)] + \
               [(n, C.c_int32) for n in ("dtype", "max_seqs", "max_positions", "kv_format")]


class _Weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("final_norm", C.c_void_p), ("lm_head", C.c_void_p)] + \
               [(n, C.POINTER(C.c_void_p)) for n in ("attn_norm", "wqkv", "wo", "ffn_norm", "wgate_up", "wdown")]


class AsyncLMError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"{what}: error {code} ({_strerror(code)})")
        self.code = code


_lib = None


def library_path() -> str:
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), "libasynclm.so")


def _share_hip_runtime_with_torch() -> None:
    """PyTorch wheels ship their own libamdhip64 (soname libamdhip64.so.7).  Callers allocate device
    memory and streams with PyTorch, so the library must bind to that same runtime copy, whichever
    of the two gets loaded first: load PyTorch's copy globally before libasynclm.so is opened."""
    import importlib.util
    spec = importlib.util.find_spec("torch")
    if spec is None or not spec.origin:
        return
    cand = os.path.join(os.path.dirname(spec.origin), "lib", "libamdhip64.so")
    if os.path.exists(cand):
        C.CDLL(cand, mode=C.RTLD_GLOBAL)


def load_library():
    """Loads the HIP library; there is no fallback path - a missing library is an error."""
    global _lib
    if _lib is not None:
        return _lib
    path = library_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: build it first (python -m paper_2412_07017_amd.build)")
    _share_hip_runtime_with_torch()
    lib = C.CDLL(path)
    i32, p = C.c_int32, C.c_void_p
    lib.asynclm_create.argtypes = [C.POINTER(p), C.POINTER(_Config), C.POINTER(_Weights), p]
    lib.asynclm_destroy.argtypes = [p]
    lib.asynclm_prefill.argtypes = [p, i32, C.POINTER(i32), i32]
    lib.asynclm_decode_step.argtypes = [p, i32, i32, C.POINTER(i32)]
    lib.asynclm_inject_interrupt.argtypes = [p, i32, C.POINTER(i32), i32]
    lib.asynclm_logits.argtypes = [p, i32, C.POINTER(C.c_float), i32]
    lib.asynclm_logits_device.argtypes = [p, i32, C.POINTER(p)]
    lib.asynclm_seq_len.argtypes = [p, i32, C.POINTER(i32)]
    lib.asynclm_reset.argtypes = [p, i32]
    lib.asynclm_synchronize.argtypes = [p]
    lib.asynclm_set_option.argtypes = [p, C.c_char_p, i32]
    lib.asynclm_profile_step.argtypes = [p, i32, i32, C.POINTER(C.POINTER(C.c_char_p)), C.POINTER(C.c_float), C.POINTER(i32), i32]
    lib.asynclm_profile_trace.argtypes = [p, C.POINTER(C.c_uint64), i32, C.POINTER(i32), C.POINTER(i32)]
    lib.asynclm_step_batch.argtypes = [p, i32, C.POINTER(i32), C.POINTER(i32), C.POINTER(i32), C.POINTER(i32), C.POINTER(i32)]
    lib.asynclm_set_banned_tokens.argtypes = [p, i32, C.POINTER(i32), i32]
    lib.asynclm_peek_token.argtypes = [p, i32, C.POINTER(i32)]
    lib.asynclm_kv_bytes.argtypes = [p, i32, C.POINTER(C.c_uint64)]
    lib.asynclm_kv_swap_out.argtypes = [p, i32, p, C.c_uint64]
    lib.asynclm_kv_swap_in.argtypes = [p, i32, p, C.c_uint64]
    lib.asynclm_seq_len.argtypes = [p, i32, C.POINTER(i32)]
    lib.asynclm_reset.argtypes = [p, i32]
    lib.asynclm_synchronize.argtypes = [p]
    lib.asynclm_set_option.argtypes = [p, C.c_char_p, i32]
    lib.asynclm_greedy_token_static.argtypes = [p, i32, p, i32, p, p]
    lib.asynclm_strerror.argtypes = [C.c_int]
    lib.asynclm_strerror.restype = C.c_char_p
    lib.asynclm_version.restype = C.c_char_p
    for name in API_SYMBOLS:
        if name not in ("asynclm_strerror", "asynclm_version"):
            getattr(lib, name).restype = C.c_int
    _lib = lib
    return lib


def greedy_token_static(logits_dev: int, n: int, banned_dev: int, n_banned: int, token_out_dev: int, stream: int) -> int:
    """asynclm_greedy_token_static: all pointers are device addresses (ints); returns the C return code."""
    return int(load_library().asynclm_greedy_token_static(logits_dev, int(n), banned_dev or None, int(n_banned), token_out_dev, stream or None))


def _strerror(code: int) -> str:
    try:
        return load_library().asynclm_strerror(code).decode()
    except Exception:
        return "?"


def _tok(tokens) -> "np.ndarray":
    return np.ascontiguousarray(np.asarray(tokens, dtype=np.int32).reshape(-1))


class AsyncLM:
    """One library context.  `weights` holds torch tensors on the GPU (kept alive here);
    `stream` is a torch.cuda.Stream (or None for the null stream)."""

    def __init__(self, model, weights: Dict[str, object], max_positions: int, max_seqs: int = 1, stream=None,
                 kv_format: int = 0):
        self._lib = load_library()
        self._h = C.c_void_p()
        self._keep = (weights, stream)
        self.vocab = model.vocab
        cfg = _Config(model.n_layers, model.d_model, model.n_q_heads, model.n_kv_heads, model.head_dim,
                      model.ffn, model.vocab, model.rms_eps, model.rope_theta,
                      0 if model.dtype == "fp32" else 1, max_seqs, max_positions, kv_format)
        L = model.n_layers
        arr = lambda ts: (C.c_void_p * L)(*[t.data_ptr() for t in ts])
        self._arrays = [arr(weights[k]) for k in ("attn_norm", "wqkv", "wo", "ffn_norm", "wgate_up", "wdown")]
        w = _Weights(weights["embed"].data_ptr(), weights["final_norm"].data_ptr(), weights["lm_head"].data_ptr(),
                     *[C.cast(a, C.POINTER(C.c_void_p)) for a in self._arrays])
        sh = C.c_void_p(stream.cuda_stream) if stream is not None else C.c_void_p(0)
        self._check(self._lib.asynclm_create(C.byref(self._h), C.byref(cfg), C.byref(w), sh), "asynclm_create")

    def _check(self, rc: int, what: str) -> int:
        if rc < 0:
            raise AsyncLMError(rc, what)
        return rc

    def close(self):
        if self._h:
            self._lib.asynclm_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- the C ABI, one method per entry point ------------------------------------------------
    def prefill(self, seq: int, tokens) -> None:
        t = _tok(tokens)
        self._check(self._lib.asynclm_prefill(self._h, seq, t.ctypes.data_as(C.POINTER(C.c_int32)), len(t)), "asynclm_prefill")

    def decode_step(self, seq: int, forced_token: int = -1, want_token: bool = True) -> Optional[int]:
        out = C.c_int32(-1)
        self._check(self._lib.asynclm_decode_step(self._h, seq, int(forced_token), C.byref(out) if want_token else None), "asynclm_decode_step")
        return out.value if want_token else None

    def inject_interrupt(self, seq: int, tokens) -> None:
        t = _tok(tokens)
        self._check(self._lib.asynclm_inject_interrupt(self._h, seq, t.ctypes.data_as(C.POINTER(C.c_int32)), len(t)), "asynclm_inject_interrupt")

    def step_batch(self, seqs, forced=None, interrupts=None, want_tokens: bool = True):
        """interrupts: None, or one token list (possibly empty) per sequence."""
        sq = _tok(seqs)
        n = len(sq)
        p32 = C.POINTER(C.c_int32)
        fo = _tok(forced) if forced is not None else None
        if fo is not None and len(fo) != n:
            raise ValueError("forced needs one entry per sequence")
        off = toks = None
        if interrupts is not None:
            if len(interrupts) != n:
                raise ValueError("interrupts needs one entry per sequence")
            lens = [len(x) for x in interrupts]
            off = np.ascontiguousarray(np.concatenate([[0], np.cumsum(lens)]).astype(np.int32))
            toks = _tok(np.concatenate([np.asarray(x, dtype=np.int32).reshape(-1) for x in interrupts]) if sum(lens) else [])
        out = np.full(n, -1, dtype=np.int32)
        self._check(self._lib.asynclm_step_batch(
            self._h, n, sq.ctypes.data_as(p32), fo.ctypes.data_as(p32) if fo is not None else None,
            toks.ctypes.data_as(p32) if toks is not None and len(toks) else None,
            off.ctypes.data_as(p32) if off is not None else None,
            out.ctypes.data_as(p32) if want_tokens else None), "asynclm_step_batch")
        return out if want_tokens else None

    def set_banned_tokens(self, seq: int, ids) -> None:
        t = _tok(ids)
        self._check(self._lib.asynclm_set_banned_tokens(self._h, seq, t.ctypes.data_as(C.POINTER(C.c_int32)) if len(t) else None,
                                                        len(t)), "asynclm_set_banned_tokens")

    def peek_choice(self, seq: int) -> int:
        out = C.c_int32(-1)
        self._check(self._lib.asynclm_peek_token(self._h, seq, C.byref(out)), "asynclm_peek_token")
        return out.value

    def kv_bytes(self, seq: int) -> int:
        n = C.c_uint64()
        self._check(self._lib.asynclm_kv_bytes(self._h, seq, C.byref(n)), "asynclm_kv_bytes")
        return n.value

    def kv_swap_out(self, seq: int, host_ptr: int, capacity: int) -> None:
        """host_ptr: address of a host buffer of `capacity` bytes (e.g. tensor.data_ptr() of a pinned uint8 tensor)."""
        self._check(self._lib.asynclm_kv_swap_out(self._h, seq, C.c_void_p(host_ptr), C.c_uint64(capacity)), "asynclm_kv_swap_out")

    def kv_swap_in(self, seq: int, host_ptr: int, nbytes: int) -> None:
        self._check(self._lib.asynclm_kv_swap_in(self._h, seq, C.c_void_p(host_ptr), C.c_uint64(nbytes)), "asynclm_kv_swap_in")

    def logits(self, seq: int) -> "np.ndarray":
        out = np.empty(self.vocab, dtype=np.float32)
        self._check(self._lib.asynclm_logits(self._h, seq, out.ctypes.data_as(C.POINTER(C.c_float)), self.vocab), "asynclm_logits")
        return out

    def logits_device(self, seq: int) -> int:
        p = C.c_void_p()
        self._check(self._lib.asynclm_logits_device(self._h, seq, C.byref(p)), "asynclm_logits_device")
        return p.value

    def seq_len(self, seq: int) -> int:
        n = C.c_int32()
        self._check(self._lib.asynclm_seq_len(self._h, seq, C.byref(n)), "asynclm_seq_len")
        return n.value

    def reset(self, seq: int) -> None:
        self._check(self._lib.asynclm_reset(self._h, seq), "asynclm_reset")

    def synchronize(self) -> None:
        self._check(self._lib.asynclm_synchronize(self._h), "asynclm_synchronize")

    def set_option(self, name: str, value: int) -> None:
        self._check(self._lib.asynclm_set_option(self._h, name.encode(), int(value)), "asynclm_set_option")

    def profile_trace(self) -> "np.ndarray":
        ns, nw = C.c_int32(), C.c_int32()
        self._check(self._lib.asynclm_profile_trace(self._h, None, 0, C.byref(ns), C.byref(nw)), "asynclm_profile_trace")
        out = np.zeros((ns.value, nw.value), dtype=np.uint64)
        if out.size:
            self._check(self._lib.asynclm_profile_trace(self._h, out.ctypes.data_as(C.POINTER(C.c_uint64)), out.size,
                                                        C.byref(ns), C.byref(nw)), "asynclm_profile_trace")
        return out

    def profile_step(self, seq: int, forced_token: int) -> Dict[str, Dict[str, float]]:
        cap = 64
        ms = (C.c_float * cap)()
        cnt = (C.c_int32 * cap)()
        names = C.POINTER(C.c_char_p)()
        n = self._check(self._lib.asynclm_profile_step(self._h, seq, int(forced_token), C.byref(names), ms, cnt, cap), "asynclm_profile_step")
        return {names[i].decode(): {"ms": float(ms[i]), "launches": int(cnt[i])} for i in range(n) if cnt[i] > 0}
