"""Seeded generators.  One integer seed -> independent Philox sub-streams keyed by
(purpose, layer, tensor, chunk), so any tensor (or any row range of it) can be
regenerated on its own and large models can be produced one layer at a time.

Storage types: fp32 tensors are numpy float32; bf16 tensors are numpy uint16 holding
the bf16 bit pattern (round-to-nearest-even of the float32 draw).
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from typing import Dict, Optional, Tuple

import numpy as np

from .configs import ModelShape

# ------------------------------------------------------------------ bf16 helpers


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit pattern (uint16), round to nearest even.  Finite inputs."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + r) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_bits_to_f64(b: np.ndarray) -> np.ndarray:
    return bf16_bits_to_f32(b).astype(np.float64)


def to_f64(a: np.ndarray) -> np.ndarray:
    """Storage array (float32, or uint16 bf16 bits) -> float64 values."""
    if a.dtype == np.uint16:
        return bf16_bits_to_f64(a)
    return a.astype(np.float64)


# ------------------------------------------------------------------ streams

_PURPOSE = {"weight": 1, "kv_k": 2, "kv_v": 3, "draft_logits": 4, "draft_pick": 5,
            "uniform": 6, "prompt": 7, "pending": 8, "hidden": 9, "norm_gain": 10}

TENSOR_NAMES = ("embed", "attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up",
                "w_down", "final_norm", "lm_head", "judge_w", "judge_b")
_TENSOR_ID = {n: i for i, n in enumerate(TENSOR_NAMES)}

_CHUNK_ELEMS = 1 << 22
_POOL: Optional[ThreadPoolExecutor] = None


def _pool() -> ThreadPoolExecutor:
    global _POOL
    if _POOL is None:
        _POOL = ThreadPoolExecutor(max_workers=max(1, min(16, os.cpu_count() or 1)))
    return _POOL


def _rng(seed: int, purpose: str, *key: int) -> np.random.Generator:
    ss = np.random.SeedSequence([int(seed), _PURPOSE[purpose], *[int(k) + 1 for k in key]])
    return np.random.Generator(np.random.Philox(ss))


def _normal_rows(seed: int, purpose: str, key: Tuple[int, ...], n_rows: int, n_cols: int,
                 std: float, dtype: str, rows: Optional[Tuple[int, int]] = None) -> np.ndarray:
    """[n_rows, n_cols] ~ N(0, std), generated in row chunks with one stream per chunk."""
    ch = max(1, _CHUNK_ELEMS // max(1, n_cols))
    r0, r1 = (0, n_rows) if rows is None else rows
    assert 0 <= r0 <= r1 <= n_rows
    out = np.empty((r1 - r0, n_cols), dtype=np.float32 if dtype == "fp32" else np.uint16)
    c0, c1 = r0 // ch, (r1 + ch - 1) // ch

    def work(c: int) -> None:
        lo, hi = c * ch, min(n_rows, (c + 1) * ch)
        g = _rng(seed, purpose, *key, c)
        blk = g.standard_normal((hi - lo, n_cols), dtype=np.float32)
        if std != 1.0:
            blk *= np.float32(std)
        a, b = max(lo, r0), min(hi, r1)
        sub = blk[a - lo:b - lo]
        out[a - r0:b - r0] = sub if dtype == "fp32" else f32_to_bf16_bits(sub)

    chunks = list(range(c0, c1))
    if len(chunks) <= 1:
        for c in chunks:
            work(c)
    else:
        list(_pool().map(work, chunks))
    return out


# ------------------------------------------------------------------ weights


class WeightSource:
    """Random-init decoder weights ~ N(0, weight_std); RMSNorm gains 1 (optionally
    jittered for tests that must notice a dropped gain); judge bias as given."""

    def __init__(self, shape: ModelShape, seed: int = 0, norm_jitter: float = 0.0,
                 judge_bias: float = 0.0):
        self.shape, self.seed = shape, seed
        self.norm_jitter, self.judge_bias = norm_jitter, judge_bias

    def dims(self, name: str) -> Tuple[int, int]:
        s = self.shape
        d, hd = s.d_model, s.head_dim
        return {
            "embed": (s.vocab, d), "lm_head": (s.vocab, d),
            "wq": (s.n_q_heads * hd, d), "wk": (s.n_kv_heads * hd, d), "wv": (s.n_kv_heads * hd, d),
            "wo": (d, s.n_q_heads * hd),
            "w_gate": (s.d_ffn, d), "w_up": (s.d_ffn, d), "w_down": (d, s.d_ffn),
            "attn_norm": (1, d), "ffn_norm": (1, d), "final_norm": (1, d),
            "judge_w": (1, d), "judge_b": (1, 1),
        }[name]

    def tensor(self, name: str, layer: int = -1, rows: Optional[Tuple[int, int]] = None) -> np.ndarray:
        """Storage-dtype array; matrices are [out, in] row-major, vectors are 1-D."""
        s = self.shape
        n_rows, n_cols = self.dims(name)
        if name in ("attn_norm", "ffn_norm", "final_norm"):
            g = np.ones(n_cols, dtype=np.float32)
            if self.norm_jitter:
                g += self.norm_jitter * _rng(self.seed, "norm_gain", _TENSOR_ID[name], layer + 1) \
                    .standard_normal(n_cols, dtype=np.float32)
            return g if s.dtype == "fp32" else f32_to_bf16_bits(g)
        if name == "judge_b":
            b = np.array([self.judge_bias], dtype=np.float32)
            return b if s.dtype == "fp32" else f32_to_bf16_bits(b)
        a = _normal_rows(self.seed, "weight", (_TENSOR_ID[name], layer + 1), n_rows, n_cols,
                         s.weight_std, s.dtype, rows)
        return a[0] if name == "judge_w" else a


# ------------------------------------------------------------------ caches, drafts


def make_kv_cache(shape: ModelShape, seed: int, seq: int, layer: int, length: int
                  ) -> Tuple[np.ndarray, np.ndarray]:
    """Synthetic cache of one (sequence, layer): K, V ~ N(0,1), each [n_kv_heads, length, head_dim]
    in the storage dtype.  Stands in for a real prefill where an fp64 prefill is infeasible."""
    n = shape.n_kv_heads * length
    k = _normal_rows(seed, "kv_k", (seq, layer), n, shape.head_dim, 1.0, shape.dtype)
    v = _normal_rows(seed, "kv_v", (seq, layer), n, shape.head_dim, 1.0, shape.dtype)
    return (k.reshape(shape.n_kv_heads, length, shape.head_dim),
            v.reshape(shape.n_kv_heads, length, shape.head_dim))


def make_pending(shape: ModelShape, seed: int) -> np.ndarray:
    return _rng(seed, "pending").integers(0, shape.vocab, size=shape.batch, dtype=np.int32)


def make_prompt(shape: ModelShape, seed: int, n: int, seq: int = 0) -> np.ndarray:
    return _rng(seed, "prompt", seq).integers(0, shape.vocab, size=n, dtype=np.int32)


def make_hidden(shape: ModelShape, seed: int) -> np.ndarray:
    """Final hidden states after RMSNorm for the head-only workload: [rows, d] ~ N(0,1)."""
    return _normal_rows(seed, "hidden", (0,), shape.rows, shape.d_model, 1.0, shape.dtype)


def make_draft(shape: ModelShape, seed: int, base_logits: Optional[np.ndarray] = None,
               noise: float = 2.0, greedy: bool = False) -> Dict[str, np.ndarray]:
    """Draft side of one cycle (Eq. 1): a draft distribution per (sequence, position), one token
    drawn from it, plus the uniforms the verifier will consume.

    Default: draft logits = noise * N(0,1), independent of the target (the benchmark recipe).
    With base_logits [B, gamma, V] the draft is base_logits + noise * N(0,1) (a draft that mostly
    agrees with the target - exercises high acceptance).  greedy=True picks argmax q.
    Returns tokens int32 [B,gamma], probs float32 [B,gamma,V], uniforms float32 [B,gamma+1]."""
    B, G, V = shape.batch, shape.gamma, shape.vocab
    probs = np.empty((B, G, V), dtype=np.float32)
    tokens = np.empty((B, G), dtype=np.int32)

    def work(b: int) -> None:
        g = _rng(seed, "draft_logits", b)
        pick = _rng(seed, "draft_pick", b)
        for j in range(G):
            z = noise * g.standard_normal(V)
            if base_logits is not None:
                z = z + np.asarray(base_logits[b, j], dtype=np.float64)
            z -= z.max()
            e = np.exp(z)
            q = e / e.sum()
            tokens[b, j] = int(np.argmax(q)) if greedy else int(pick.choice(V, p=q))
            probs[b, j] = q.astype(np.float32)

    list(_pool().map(work, range(B)))
    uniforms = _rng(seed, "uniform").random((B, G + 1), dtype=np.float32)
    return {"tokens": tokens, "probs": probs, "uniforms": uniforms}


def make_judge_dataset(seed: int, n: int, d: int, pos_rate: float = 0.61, shift: float = 1.0, n_dirs: int = 4,
                       task_seed: int = 0):
    """Synthetic (hidden state, label) pairs shaped like the verifier training set (paper Table
    "Data for training verifier": 69,432 samples, 61 % labelled acceptable, features = d-dimensional
    normed hidden states of unit scale).  Labels are Bernoulli(pos_rate); a feature row is standard
    normal noise plus a label-dependent offset spread over a few fixed random directions, with a
    per-sample random strength, so the classes overlap (ROC-AUC well below 1) as in the paper's ROC
    figure.  The directions depend on task_seed only, so sets drawn with different seeds (training,
    validation) come from the same population.  Returns (H float32 [n, d], y int32 [n])."""
    rng = np.random.default_rng([seed, 0x5E1F])
    y = (rng.random(n) < pos_rate).astype(np.int32)
    dirs = np.random.default_rng([task_seed, d, 0xD125]).standard_normal((n_dirs, d))
    dirs /= np.linalg.norm(dirs, axis=1, keepdims=True)
    strength = shift * rng.gamma(2.0, 0.5, size=(n, n_dirs))          # mean 1, sample-dependent
    sign = (2.0 * y - 1.0)[:, None]
    H = rng.standard_normal((n, d), dtype=np.float32)
    H += ((sign * strength) @ dirs / np.sqrt(n_dirs)).astype(np.float32)
    return H, y
