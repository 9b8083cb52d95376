"""MI355X-native inference process for asynchronous LLM function calling (arXiv 2412.07017).

A thin ctypes binding over libasynclm.so (hand-written HIP for gfx950).  Every step of the
decoding path runs in the library's kernels; Python only marshals arguments.  PyTorch is used
by callers for device memory and streams and is not needed to import this package.
"""
from .binding import (AsyncLM, AsyncLMError, library_path, load_library, E_INVAL, E_STATE, E_CAPACITY,
                      E_NOMEM, E_DEVICE, API_SYMBOLS, KV_AUTO, KV_BF16, KV_PAIR_ROWS, greedy_token_static)
from .session import CML, InterruptibleSession, SessionGroup, StepResult, TokenMonitor, TrapPolicy

__all__ = ["AsyncLM", "AsyncLMError", "library_path", "load_library", "E_INVAL", "E_STATE", "E_CAPACITY",
           "E_NOMEM", "E_DEVICE", "API_SYMBOLS", "KV_AUTO", "KV_BF16", "KV_PAIR_ROWS", "CML", "InterruptibleSession", "StepResult",
           "SessionGroup", "TokenMonitor", "TrapPolicy", "greedy_token_static"]
