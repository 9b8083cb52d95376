"""Model shapes and workload presets (pure data, no arithmetic of the method).

The five presets are Llama-style decoder shapes with the interrupt traffic the paper
describes for its inference process (Sec. 5.3: short interrupt blocks appended to the
stream between decoding steps; Sec. 6.4: about 20 extra tokens per interrupt; Sec. 6:
calls return 30-500 ms apart, i.e. every few dozen decoding steps).
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict


@dataclass(frozen=True)
class ModelConfig:
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    vocab: int
    rms_eps: float
    rope_theta: float
    dtype: str  # "fp32" or "bf16": storage type of weights and K/V cache

    @property
    def q_dim(self) -> int:
        return self.n_q_heads * self.head_dim

    @property
    def kv_dim(self) -> int:
        return self.n_kv_heads * self.head_dim

    @property
    def qkv_rows(self) -> int:
        return self.q_dim + 2 * self.kv_dim

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "fp32" else 2

    def layer_weight_elems(self) -> int:
        d = self.d_model
        return self.qkv_rows * d + d * self.q_dim + 2 * self.ffn * d + d * self.ffn

    def weight_bytes_per_step(self) -> int:
        """Bytes of matrix weights one forward pass has to read (all layers + output head)."""
        return (self.n_layers * self.layer_weight_elems() + self.vocab * self.d_model) * self.elem_bytes

    def kv_bytes_per_position(self) -> int:
        return 2 * self.n_layers * self.kv_dim * self.elem_bytes


@dataclass(frozen=True)
class Workload:
    name: str
    model: ModelConfig
    prompt_len: int
    n_decode: int
    intr_len: int          # tokens per interrupt (lower bound when intr_len_hi > 0)
    intr_every: int        # inject after every `intr_every`-th generated token (0: see schedule)
    schedule: str          # "single@N", "every", "uniform8", "ragged16"
    n_seqs: int = 1
    intr_len_hi: int = 0
    parity_layers: int = 0  # >0: parity is taken on the first `parity_layers` layers


_TINY = ModelConfig(n_layers=2, d_model=256, n_q_heads=4, n_kv_heads=4, head_dim=64, ffn=688,
                    vocab=1024, rms_eps=1e-5, rope_theta=10000.0, dtype="fp32")
_8B = ModelConfig(n_layers=32, d_model=4096, n_q_heads=32, n_kv_heads=8, head_dim=128, ffn=14336,
                  vocab=128256, rms_eps=1e-5, rope_theta=500000.0, dtype="bf16")
_70B = ModelConfig(n_layers=80, d_model=8192, n_q_heads=64, n_kv_heads=8, head_dim=128, ffn=28672,
                   vocab=128256, rms_eps=1e-5, rope_theta=500000.0, dtype="bf16")

PRESETS: Dict[str, Workload] = {
    "tiny": Workload("tiny", _TINY, prompt_len=64, n_decode=32, intr_len=8, intr_every=0,
                     schedule="single@16"),
    "8b": Workload("8b", _8B, prompt_len=1024, n_decode=256, intr_len=24, intr_every=64,
                   schedule="every", parity_layers=4),
    "8b-long": Workload("8b-long", _8B, prompt_len=16384, n_decode=512, intr_len=48, intr_every=0,
                        schedule="uniform8", parity_layers=4),
    "8b-ragged16": Workload("8b-ragged16", _8B, prompt_len=0, n_decode=256, intr_len=16,
                            intr_every=0, schedule="ragged16", n_seqs=16, intr_len_hi=32,
                            parity_layers=4),
    "70b": Workload("70b", _70B, prompt_len=4096, n_decode=256, intr_len=32, intr_every=32,
                    schedule="every", parity_layers=4),
}


def preset(name: str) -> Workload:
    return PRESETS[name]


def truncated(model: ModelConfig, n_layers: int) -> ModelConfig:
    """Same shape with only the first `n_layers` layers (plus final norm and output head)."""
    return replace(model, n_layers=min(n_layers, model.n_layers))
