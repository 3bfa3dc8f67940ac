"""Glue between the seeded generators and the device library: turns a ModelShape / WeightSource into the
library's configuration and tensor provider.  Argument plumbing only - no method arithmetic, and nothing here
touches the oracle.  (The library is imported when a function is called, so `import synth` works without it.)"""
from __future__ import annotations

from .configs import ModelShape
from .generate import WeightSource


def sj_config(shape: ModelShape, max_gamma: int | None = None):
    import paper_2510_02329_amd as sj
    return sj.SJConfig(n_layers=shape.n_layers, d_model=shape.d_model, n_q_heads=shape.n_q_heads,
                       n_kv_heads=shape.n_kv_heads, head_dim=shape.head_dim, d_ffn=shape.d_ffn, vocab=shape.vocab,
                       dtype=0 if shape.dtype == "fp32" else 1, rope_base=shape.rope_base, rms_eps=shape.rms_eps,
                       temperature=shape.temperature, max_gamma=max_gamma or shape.gamma)


def load_model(shape: ModelShape, src: WeightSource, max_gamma: int | None = None, log=print) -> int:
    """sj_model_load with the generator as the tensor provider (one layer at a time: a 70B-shaped model never sits
    in host memory).  `log` receives a progress line every few layers of a deep model."""
    import paper_2510_02329_amd as sj

    def provider(name, layer):
        if name == "wq" and layer % 8 == 0 and shape.n_layers > 40:
            log(f"  loading layer {layer}/{shape.n_layers}")             # long loads must show progress
        return src.tensor(name, layer)
    return sj.sj_model_load(sj_config(shape, max_gamma), provider)


def fill_cache(kv: int, shape: ModelShape, seed: int, lens, pending) -> None:
    """Uploads the seeded K / V rows of every (sequence, layer) and sets length and pending token."""
    import paper_2510_02329_amd as sj
    from .generate import make_kv_cache
    for b in range(shape.batch):
        for l in range(shape.n_layers):
            k, v = make_kv_cache(shape, seed, b, l, int(lens[b]))
            sj.sj_kv_set_layer(kv, b, l, k, v, int(lens[b]))
        sj.sj_kv_set_state(kv, b, int(lens[b]), int(pending[b]))
