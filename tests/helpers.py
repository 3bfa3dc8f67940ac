"""Glue shared by the tests: turns the seeded generators' storage arrays into what each
side consumes.  No method arithmetic lives here."""
from __future__ import annotations

from collections import OrderedDict

import numpy as np

import synth
from oracle import selfjudge_oracle as orc


def oracle_config(shape: synth.ModelShape) -> orc.OracleConfig:
    return orc.OracleConfig(shape.n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads,
                            shape.head_dim, shape.d_ffn, shape.vocab, shape.rope_base,
                            shape.rms_eps, shape.temperature)


def oracle_weights(src: synth.WeightSource, cache_items: int = 64):
    """float64 view of the generator's (dtype-rounded) tensors, with a small LRU so tiny models
    are not regenerated on every call."""
    lru: "OrderedDict[tuple, np.ndarray]" = OrderedDict()

    def get(name, layer=-1, rows=None):
        key = (name, layer, rows)
        if key in lru:
            lru.move_to_end(key)
            return lru[key]
        a = synth.to_f64(src.tensor(name, layer, rows))
        if cache_items and a.nbytes <= (64 << 20):
            lru[key] = a
            if len(lru) > cache_items:
                lru.popitem(last=False)
        return a

    return get


def dict_weights(tensors: dict):
    """WeightFn over an explicit {(name, layer): float64 array} dict (hand-built test models)."""
    def get(name, layer=-1, rows=None):
        a = tensors[(name, layer)]
        if rows is not None:
            a = a[rows[0]:rows[1]]
        return a
    return get


def random_model(shape: synth.ModelShape, seed: int, scale: float = 1.0, norm_jitter: float = 0.1,
                 judge_bias: float = 0.0) -> dict:
    """Small fp64 model with O(1) activations (weights ~ N(0, scale/sqrt(fan_in)))."""
    rng = np.random.default_rng(seed)
    src = synth.WeightSource(shape, seed)
    t = {}
    def mat(name, layer):
        r, c = src.dims(name)
        t[(name, layer)] = rng.standard_normal((r, c)) * scale / np.sqrt(c)
    t[("embed", -1)] = rng.standard_normal((shape.vocab, shape.d_model))
    mat("lm_head", -1)
    for l in range(shape.n_layers):
        for n in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down"):
            mat(n, l)
        for n in ("attn_norm", "ffn_norm"):
            t[(n, l)] = 1.0 + norm_jitter * rng.standard_normal(shape.d_model)
    t[("final_norm", -1)] = 1.0 + norm_jitter * rng.standard_normal(shape.d_model)
    t[("judge_w", -1)] = rng.standard_normal(shape.d_model) / np.sqrt(shape.d_model)
    t[("judge_b", -1)] = np.array([judge_bias])
    return t


def random_cache(cfg: orc.OracleConfig, length: int, capacity: int, seed: int) -> orc.SeqCache:
    rng = np.random.default_rng(seed)
    c = orc.SeqCache(cfg, capacity)
    for l in range(cfg.n_layers):
        c.k[l][:, :length] = rng.standard_normal((cfg.n_kv_heads, length, cfg.head_dim))
        c.v[l][:, :length] = rng.standard_normal((cfg.n_kv_heads, length, cfg.head_dim))
    c.length = length
    c.pending = int(rng.integers(0, cfg.vocab))
    return c
