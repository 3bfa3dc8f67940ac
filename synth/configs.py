"""Workload shapes: model geometry + batch / draft length / cache lengths.

Index = workload number.  0 is the tiny fp32 parity case; 1 is the verify-head
microbenchmark (no decoder layers); 2 is the 8B-shaped batch-1 case the
headline metric is quoted on; 3 is 8B-shaped batch 16 with ragged cache
lengths; 4 is the 70B-shaped case.  The 8B / 70B shapes are those of the
Llama-3.1 targets the paper evaluates (Sec. 4.1); gamma = 5 is the draft length
of its phase-timing experiment (Sec. 4.5).
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Tuple

import numpy as np


@dataclass(frozen=True)
class ModelShape:
    name: str
    dtype: str            # "fp32" | "bf16": storage type of weights and KV cache
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    rope_base: float
    rms_eps: float = 1e-5
    temperature: float = 1.0
    # workload
    batch: int = 1
    gamma: int = 4
    kv_len: Tuple[int, int] = (128, 128)   # inclusive range; equal ends = fixed length
    weight_std: float = 0.02

    @property
    def rows(self) -> int:
        return self.batch * (self.gamma + 1)

    @property
    def qkv_out(self) -> int:
        return (self.n_q_heads + 2 * self.n_kv_heads) * self.head_dim

    def params_streamed(self) -> int:
        """Weights every step must read once: all projections + LM head."""
        d, hd = self.d_model, self.head_dim
        per_layer = 2 * d * self.n_q_heads * hd + 2 * d * self.n_kv_heads * hd + 3 * d * self.d_ffn
        return self.n_layers * per_layer + self.vocab * d

    def elem_bytes(self) -> int:
        return 4 if self.dtype == "fp32" else 2

    def kv_lengths(self, seed: int = 0) -> np.ndarray:
        lo, hi = self.kv_len
        if lo == hi:
            return np.full(self.batch, lo, dtype=np.int32)
        rng = np.random.Generator(np.random.Philox(np.random.SeedSequence([seed, 0x6b766c656e])))
        return rng.integers(lo, hi + 1, size=self.batch, dtype=np.int32)

    def scaled(self, **kw) -> "ModelShape":
        return replace(self, **kw)


CONFIGS = {
    0: ModelShape("tiny_fp32", "fp32", 2, 256, 4, 4, 64, 768, 4096, 10000.0,
                  batch=1, gamma=4, kv_len=(128, 128)),
    1: ModelShape("verify_head_bf16", "bf16", 0, 4096, 32, 8, 128, 14336, 128256, 500000.0,
                  batch=64, gamma=8, kv_len=(0, 0)),
    2: ModelShape("llama8b_b1_g5", "bf16", 32, 4096, 32, 8, 128, 14336, 128256, 500000.0,
                  batch=1, gamma=5, kv_len=(1024, 1024)),
    3: ModelShape("llama8b_b16_g8", "bf16", 32, 4096, 32, 8, 128, 14336, 128256, 500000.0,
                  batch=16, gamma=8, kv_len=(512, 4096)),
    4: ModelShape("llama70b_b4_g5", "bf16", 80, 8192, 64, 8, 128, 28672, 128256, 500000.0,
                  batch=4, gamma=5, kv_len=(2048, 2048)),
}


# Draft model of the speculate -> verify cycle: Llama-3.2-1B-shaped (the paper pairs an 8B target with a 1B
# draft of the same family and vocabulary); workload fields follow the target they are paired with.
DRAFT_1B = ModelShape("llama1b_draft", "bf16", 16, 2048, 32, 8, 64, 8192, 128256, 500000.0,
                      batch=1, gamma=5, kv_len=(1024, 1024))


def shape_of(idx: int) -> ModelShape:
    return CONFIGS[idx]
