"""CPU fp64 oracle for one verification cycle of judge-assisted speculative decoding.

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain statement of what the
verification step computes.  It shares no code with the HIP library and must never be
imported by the product path: only tests/, the smoke check and the benchmark's
cpu_baseline leg may use it.  Everything is numpy float64; the only library primitives are
matmul / exp / cumsum.  No blocking, fusion or reordering beyond what the method states.

What is computed (paper section "Method", subsections "Conventional Speculative Decoding"
and "Judge Verification"):

  * target block forward (Eq. 2 / Eq. 4): the target model reads the prefix (held as a KV
    cache) plus the pending token and the gamma draft tokens, and returns gamma+1
    next-token distributions p and the hidden state h of every row.  The model family is
    the Llama-3 decoder the paper evaluates (Sec. 4.1): pre-norm, RMSNorm, rotary
    positions, grouped-query attention, SwiGLU feed-forward.
  * alignment test (Eq. 3): accept d_t iff u_t < min(1, p_t/q_t).
  * judge test (Eq. 5): accept d_t iff Verifier(h_t) > theta, Verifier = logistic regression.
  * a token is kept if either test approves it (Sec. 3.2, App. D.2); tokens are accepted in
    order until the first rejection (Sec. 3.1).
  * the draft proposal that feeds the cycle (Eq. 1): gamma sequential single-token decodes of the
    draft model, each drawing d from its own next-token law q (`draft_block`).
  * the training-label score (Sec. 3.3, Eq. 6 - 7): log-likelihood difference of the response with one
    token replaced, from two teacher-forced passes (`score_block`, `semantic_preservation`).
  * one more token is emitted: from the last distribution p_{t+gamma+1} if everything was
    accepted (Sec. 3.1, text after Eq. 2), otherwise from the residual distribution
    norm(max(0, p - q)) of "modified rejection sampling" (Sec. 2.2), which is the choice that
    makes the emitted-token law equal the target's.

Readings of points the paper leaves open (each is also listed in the design notes):
  R1  draft_probs is the full draft distribution per position; the test gathers q(d).
  R2  the test is evaluated as  u*q < p  (no division; q = 0 < p accepts, p = q = 0 rejects).
  R3  the judge's feature for d_j is the final, RMS-normed hidden state of the row whose
      *input* token is d_j; score = sigmoid(w.h + b); strict '>' against theta.        [parity unpinned]
  R4  when both tests reject at position j the emitted token comes from the residual at j,
      also after judge-accepted tokens.                                                [parity unpinned]
  R5  a token is drawn from weights w by inverse CDF in vocabulary order with the one
      supplied uniform: smallest k with  sum_{i<=k} w_i > u * sum(w).                 [parity unpinned]
  R6  temperature 0 means a one-hot p at the lowest-index arg-max.
  R7  rotary pairs dimension i with i + head_dim/2, angle = pos * base^(-2i/head_dim);
      no biases; untied embedding / LM head; eps inside the square root.              [parity unpinned]
  R8  the cache holds positions 0..L-1; the pending token (last emitted, not yet cached)
      is row 0 of the block; after the step L += 1 + n.
  R9  the cache is held in the model's storage type (bf16 or fp32), like the weights: the K/V
      of a new row are rounded to it (nearest even) when appended, and every read - also the
      block's own rows in the same step - sees the stored value.  This keeps "one block
      forward == gamma+1 single-token decodes" exact on what the cache holds.
  R12 top-k verification (the relaxed baseline of Sec. 4.1, k = 2 in the experiments): d_j is kept
      when fewer than k vocabulary entries precede it in the target's row j-1, ordered by
      decreasing logit and, for equal logits, increasing index; the emitted token after a
      rejection follows the same residual rule as every other mode.                    [parity unpinned]
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Callable, Dict, List, Optional, Sequence

import numpy as np

F64 = np.float64


@dataclass
class OracleConfig:
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    rope_base: float = 10000.0
    rms_eps: float = 1e-5
    temperature: float = 1.0


# get(name, layer, rows) -> float64 array.  Matrices are [out_features, in_features].
WeightFn = Callable[..., np.ndarray]


def round_to_storage(a: np.ndarray, storage: str) -> np.ndarray:
    """Round float64 values to the cache's storage type and return them as float64 (R9).
    "bf16": 8 significant bits, round to nearest, ties to even, done directly on the float64
    bit pattern (values are far inside bf16's exponent range); "fp32": IEEE single; "fp64": as is."""
    a = np.asarray(a, F64)
    if storage == "fp64":
        return a
    if storage == "fp32":
        return a.astype(np.float32).astype(F64)
    if storage == "bf16":
        u = np.ascontiguousarray(a).view(np.uint64)
        drop = np.uint64(52 - 7)                                   # mantissa bits beyond bf16's 7
        half = (np.uint64(1) << (drop - np.uint64(1))) - np.uint64(1)
        odd = (u >> drop) & np.uint64(1)
        r = (u + half + odd) & ~((np.uint64(1) << drop) - np.uint64(1))
        return r.view(F64)
    raise ValueError(storage)


class SeqCache:
    """KV cache of one sequence: k[l], v[l] are float64 [n_kv_heads, capacity, head_dim] holding
    values representable in `storage`; positions 0..length-1 are valid; `pending` is the last
    emitted, not yet cached token (R8)."""

    def __init__(self, cfg: OracleConfig, capacity: int, storage: str = "fp64"):
        self.storage = storage
        self.k = [np.zeros((cfg.n_kv_heads, capacity, cfg.head_dim), F64) for _ in range(cfg.n_layers)]
        self.v = [np.zeros((cfg.n_kv_heads, capacity, cfg.head_dim), F64) for _ in range(cfg.n_layers)]
        self.length = 0
        self.pending = 0
        self.capacity = capacity


# --------------------------------------------------------------------------- model pieces


def rmsnorm(x: np.ndarray, gain: np.ndarray, eps: float) -> np.ndarray:
    """x * gain / sqrt(mean(x^2) + eps), row-wise."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * gain


def rotary(x: np.ndarray, pos: int, base: float) -> np.ndarray:
    """Rotate one head vector x[head_dim] to position pos (R7)."""
    hd = x.shape[-1]
    half = hd // 2
    i = np.arange(half, dtype=F64)
    ang = float(pos) * base ** (-2.0 * i / hd)
    c, s = np.cos(ang), np.sin(ang)
    lo, hi = x[..., :half], x[..., half:]
    return np.concatenate([lo * c - hi * s, hi * c + lo * s], axis=-1)


def silu(x: np.ndarray) -> np.ndarray:
    return x / (1.0 + np.exp(-x))


def attention_row(q: np.ndarray, K: np.ndarray, V: np.ndarray) -> np.ndarray:
    """softmax(q.K^T / sqrt(hd)) V for one query vector over the keys it may see."""
    s = (K @ q) / np.sqrt(float(q.shape[0]))
    s = s - s.max()
    w = np.exp(s)
    w = w / w.sum()
    return w @ V


def block_forward(cfg: OracleConfig, W: WeightFn, caches: Sequence[SeqCache],
                  tokens: Sequence[Sequence[int]], lm_chunk: int = 16384,
                  want_logits: bool = True) -> List[Dict[str, np.ndarray]]:
    """Target forward (Eq. 2, Eq. 4) for a batch of independent sequences: sequence b feeds
    len(tokens[b]) new rows at positions L_b .. L_b+n_b-1.

    Row j of a sequence attends to its cached positions 0..L-1 and to its own block rows 0..j.
    K/V of the new rows are written into the cache at L..L+n-1; `length` is NOT advanced (the
    caller commits).  Sequences never interact: rows are only stacked so that each weight matrix
    is fetched once per layer.  Returns per sequence: logits [n, vocab], hn [n, d] (hidden after
    the final RMSNorm), h [n, d] (before it)."""
    Hq, Hkv, hd = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    group = Hq // Hkv
    counts = [len(t) for t in tokens]
    offs = np.concatenate([[0], np.cumsum(counts)]).astype(int)
    for c, t in zip(caches, tokens):
        if c.length + len(t) > c.capacity:
            raise ValueError("KV capacity exceeded")
    x = np.stack([W("embed", -1, (int(t), int(t) + 1))[0] for seq in tokens for t in seq])  # [rows, d]
    R = x.shape[0]
    for l in range(cfg.n_layers):
        a = rmsnorm(x, W("attn_norm", l), cfg.rms_eps)
        q = (a @ W("wq", l).T).reshape(R, Hq, hd)
        k = (a @ W("wk", l).T).reshape(R, Hkv, hd)
        v = (a @ W("wv", l).T).reshape(R, Hkv, hd)
        att = np.zeros((R, Hq, hd), F64)
        for b, cache in enumerate(caches):
            L = cache.length
            for j in range(counts[b]):
                r = offs[b] + j
                for h in range(Hq):
                    q[r, h] = rotary(q[r, h], L + j, cfg.rope_base)
                for h in range(Hkv):
                    k[r, h] = rotary(k[r, h], L + j, cfg.rope_base)
                cache.k[l][:, L + j, :] = round_to_storage(k[r], cache.storage)
                cache.v[l][:, L + j, :] = round_to_storage(v[r], cache.storage)
            for j in range(counts[b]):
                r = offs[b] + j
                for h in range(Hq):
                    g = h // group
                    att[r, h] = attention_row(q[r, h], cache.k[l][g, :L + j + 1],
                                              cache.v[l][g, :L + j + 1])
        x = x + att.reshape(R, Hq * hd) @ W("wo", l).T
        f = rmsnorm(x, W("ffn_norm", l), cfg.rms_eps)
        x = x + (silu(f @ W("w_gate", l).T) * (f @ W("w_up", l).T)) @ W("w_down", l).T
    hn = rmsnorm(x, W("final_norm"), cfg.rms_eps)
    logits = None
    if want_logits:
        logits = np.empty((R, cfg.vocab), F64)
        for r0 in range(0, cfg.vocab, lm_chunk):
            r1 = min(cfg.vocab, r0 + lm_chunk)
            logits[:, r0:r1] = hn @ W("lm_head", -1, (r0, r1)).T
    out = []
    for b in range(len(caches)):
        sl = slice(offs[b], offs[b + 1])
        o = {"h": x[sl], "hn": hn[sl]}
        if want_logits:
            o["logits"] = logits[sl]
        out.append(o)
    return out


# --------------------------------------------------------------------------- verification


def target_distribution(logits: np.ndarray, temperature: float) -> np.ndarray:
    """p = softmax(logits / T) via log-sum-exp; T = 0 -> one-hot at the lowest-index arg-max (R6)."""
    if temperature == 0.0:
        p = np.zeros_like(logits, dtype=F64)
        p[int(np.argmax(logits))] = 1.0
        return p
    z = np.asarray(logits, F64) / temperature
    z = z - z.max()
    e = np.exp(z)
    return e / e.sum()


def alignment_accepts(u: float, q_d: float, p_d: float) -> bool:
    """Eq. 3: accept iff u < min(1, p/q), evaluated without the division (R2)."""
    return bool(u * q_d < p_d)


def judge_score(w: np.ndarray, b: float, hn_row: np.ndarray) -> float:
    """Logistic-regression verifier on a target hidden state (Eq. 5, R3)."""
    z = float(np.dot(w, hn_row) + b)
    return 1.0 / (1.0 + np.exp(-z))


def accepted_length(ok: Sequence[bool]) -> int:
    """Tokens are accepted in order until the first rejection (Sec. 3.1)."""
    n = 0
    for bit in ok:
        if not bit:
            break
        n += 1
    return n


def draw(weights: np.ndarray, u: float) -> int:
    """Inverse CDF in index order with one uniform (R5)."""
    c = np.cumsum(weights)
    total = c[-1]
    hit = np.nonzero(c > u * total)[0]
    if hit.size:
        return int(hit[0])
    return int(np.nonzero(weights > 0)[0][-1])


def emitted_token(p_rows: np.ndarray, q_rows: np.ndarray, n: int, gamma: int, u: float) -> int:
    """The one extra token of the cycle.  All accepted -> draw from the last distribution;
    else draw from norm(max(0, p_n - q_{n+1})) at the first rejected position (R4); if that
    residual has no mass fall back to p_n."""
    if n == gamma:
        return draw(p_rows[gamma], u)
    w = np.maximum(0.0, p_rows[n] - q_rows[n])        # q_rows[n] is the draft law of d_{n+1}
    if w.sum() <= 0.0:
        w = p_rows[n]
    return draw(w, u)


def token_rank(logits_row: np.ndarray, token: int) -> int:
    """Position of `token` in the row ordered by decreasing logit, equal logits by increasing index
    (the order in which R6 picks the arg-max): 0 for the arg-max itself."""
    row = np.asarray(logits_row)
    ref = row[token]
    return int(np.count_nonzero(row > ref) + np.count_nonzero(row[:token] == ref))


def verify_tail(logits: np.ndarray, judge_scores: np.ndarray, draft_tokens: Sequence[int],
                draft_probs: np.ndarray, uniforms: Sequence[float], theta: float,
                temperature: float, mode: str = "two_stage", top_k: int = 2) -> Dict[str, object]:
    """Everything after the forward for one sequence.

    logits [gamma+1, V]: row j is the target's next-token logits after reading block row j, so
    row j-1 tests draft d_j (j = 1..gamma) and row gamma is the bonus distribution.
    judge_scores [gamma]: entry j-1 is Verifier(h) of the row whose input is d_j.
    draft_probs [gamma, V]; uniforms [gamma+1] (last one draws the emitted token).
    mode: "two_stage" (either test), "alignment" (Eq. 3 only), "judge" (Eq. 5 only), "topk" (the
    relaxed baseline of Sec. 4.1: d_j is kept when it is among the target's top_k tokens)."""
    gamma = len(draft_tokens)
    p = np.stack([target_distribution(logits[j], temperature) for j in range(gamma + 1)])
    q = np.asarray(draft_probs, F64)
    a_bits, g_bits, k_bits, p_at_d = [], [], [], []
    for j in range(1, gamma + 1):
        d = int(draft_tokens[j - 1])
        p_d, q_d = p[j - 1, d], q[j - 1, d]
        p_at_d.append(p_d)
        a_bits.append(alignment_accepts(float(uniforms[j - 1]), q_d, p_d))
        g_bits.append(bool(judge_scores[j - 1] > theta))
        k_bits.append(token_rank(logits[j - 1], d) < top_k)
    if mode == "alignment":
        ok = list(a_bits)
    elif mode == "judge":
        ok = list(g_bits)
    elif mode == "topk":
        ok = list(k_bits)
    else:
        ok = [a or g for a, g in zip(a_bits, g_bits)]
    n = accepted_length(ok)
    nxt = emitted_token(p, q, n, gamma, float(uniforms[gamma]))
    return {"accepted_len": n, "next_token": nxt, "align_bits": a_bits, "judge_bits": g_bits, "topk_bits": k_bits,
            "p_at_draft": np.array(p_at_d), "p": p}


def verify_step(cfg: OracleConfig, W: WeightFn, caches: Sequence[SeqCache],
                draft_tokens: np.ndarray, draft_probs: np.ndarray, uniforms: np.ndarray,
                theta: float, mode: str = "two_stage", top_k: int = 2) -> List[Dict[str, object]]:
    """One full cycle for a batch of sequences; commits every cache (R8).
    draft_tokens [B, gamma], draft_probs [B, gamma, V], uniforms [B, gamma+1]."""
    B, gamma = np.asarray(draft_tokens).shape
    toks = [[caches[b].pending] + [int(t) for t in draft_tokens[b]] for b in range(B)]
    fw = block_forward(cfg, W, caches, toks)
    w, bias = W("judge_w"), float(np.asarray(W("judge_b")).reshape(-1)[0])
    results = []
    for b, cache in enumerate(caches):
        scores = np.array([judge_score(w, bias, fw[b]["hn"][j]) for j in range(1, gamma + 1)])
        res = verify_tail(fw[b]["logits"], scores, draft_tokens[b], draft_probs[b], uniforms[b],
                          theta, cfg.temperature, mode, top_k)
        L0 = cache.length
        res.update(logits=fw[b]["logits"], hn=fw[b]["hn"], judge_scores=scores,
                   k_new=[cache.k[l][:, L0:L0 + gamma + 1].copy() for l in range(cfg.n_layers)],
                   v_new=[cache.v[l][:, L0:L0 + gamma + 1].copy() for l in range(cfg.n_layers)])
        cache.length = L0 + 1 + res["accepted_len"]
        cache.pending = res["next_token"]
        results.append(res)
    return results


def draft_block(cfg: OracleConfig, W: WeightFn, caches: Sequence[SeqCache], gamma: int,
                uniforms: np.ndarray, feed_last: bool = True):
    """Draft proposal (Sec. 2.2, Eq. 1): the draft model M_q generates gamma tokens one at a time,
    d_{t+i} ~ q(. | x_<=t, d_{t+1..t+i-1}).  cfg / W / caches are the DRAFT model's.  Step j reads the
    pending token (R8), takes q_j = softmax(logits / T) of that one row (R6 at T = 0), draws d_{j+1} by
    the inverse-CDF rule R5 with uniforms[j][b], and the drawn token becomes the pending one.
    feed_last: the last drafted token is also run through the layers, so the cache ends with a row for
    every drafted token.  Returns tokens [B, gamma] and probs [B, gamma, V]; commits every cache."""
    B = len(caches)
    tokens = np.zeros((B, gamma), dtype=np.int64)
    probs = np.zeros((B, gamma, cfg.vocab), F64)
    for j in range(gamma):
        fw = block_forward(cfg, W, caches, [[c.pending] for c in caches])
        for b, c in enumerate(caches):
            q = target_distribution(fw[b]["logits"][0], cfg.temperature)
            d = draw(q, float(uniforms[j][b]))
            probs[b, j] = q
            tokens[b, j] = d
            c.length += 1
            c.pending = d
    if feed_last:
        block_forward(cfg, W, caches, [[c.pending] for c in caches], want_logits=False)
        for c in caches:
            c.length += 1
    return tokens, probs


def score_block(cfg: OracleConfig, W: WeightFn, caches: Sequence[SeqCache], inputs: np.ndarray,
                targets: np.ndarray) -> List[Dict[str, np.ndarray]]:
    """Teacher forcing: feed inputs[b] on top of cache b and return, per row, the log-probability of
    targets[b][j] under softmax(logits_j / T) (the terms of Eq. 7), with the rows' hidden states.
    Does not commit the caches."""
    fw = block_forward(cfg, W, caches, [[int(t) for t in row] for row in inputs])
    out = []
    for b in range(len(caches)):
        lp = np.empty(len(inputs[b]), F64)
        for j, t in enumerate(targets[b]):
            if cfg.temperature == 0.0:
                lp[j] = 0.0 if int(np.argmax(fw[b]["logits"][j])) == int(t) else -np.inf
            else:
                z = fw[b]["logits"][j] / cfg.temperature
                m = z.max()
                lp[j] = z[int(t)] - (m + np.log(np.exp(z - m).sum()))
        out.append({"logprob": lp, "hn": fw[b]["hn"]})
    return out


def semantic_preservation(cfg: OracleConfig, W: WeightFn, cache: SeqCache, y_next: Sequence[int], z: int,
                          tau: float) -> Dict[str, object]:
    """Semantic preservation score of replacing y_i by z (Sec. 3.3, Eq. 6 in its autoregressive form Eq. 7).
    The cache holds the response up to y_{i-2} and y_{i-1} is its pending token (R8); y_next = [y_i,
    y_{i+1}, .., y_{i+N}] (N future tokens).  Two teacher-forced passes of N+1 rows:
        original:  inputs [y_{i-1}, y_i, y_{i+1}, .., y_{i+N-1}]  targets [y_i, y_{i+1}, .., y_{i+N}]
        replaced:  inputs [y_{i-1}, z,   y_{i+1}, .., y_{i+N-1}]  targets [z,   y_{i+1}, .., y_{i+N}]
    s_prefix = log P(z | y_<i) - log P(y_i | y_<i)  (row 0 of both),
    suffix   = log P(y_>i | y_<i, z) - log P(y_>i | y_<=i)  (rows 1..N),
    s = s_prefix + suffix, label = s > tau (Step 3), h_z = hidden state of the row that reads z (Eq. 4)."""
    y_next = [int(t) for t in y_next]
    ins_y = [cache.pending] + y_next[:-1]
    ins_z = [cache.pending, int(z)] + y_next[1:-1] if len(y_next) > 1 else [cache.pending]
    tg_y, tg_z = y_next, [int(z)] + y_next[1:]
    a = score_block(cfg, W, [cache], [ins_y], [tg_y])[0]
    b = score_block(cfg, W, [cache], [ins_z], [tg_z])[0]
    s_prefix = float(b["logprob"][0] - a["logprob"][0])
    suffix = float(b["logprob"][1:].sum() - a["logprob"][1:].sum())
    s = s_prefix + suffix
    h_z = b["hn"][1] if len(y_next) > 1 else None
    return {"s": s, "s_prefix": s_prefix, "suffix": suffix, "label": bool(s > tau), "h_z": h_z,
            "logprob_y": a["logprob"], "logprob_z": b["logprob"]}


def prefill(cfg: OracleConfig, W: WeightFn, cache: SeqCache, tokens: Sequence[int]) -> int:
    """Fill the cache from prompt tokens; the pending token becomes the arg-max continuation."""
    fw = block_forward(cfg, W, [cache], [list(tokens)])[0]
    cache.length += len(tokens)
    cache.pending = int(np.argmax(fw["logits"][-1]))
    return cache.pending
