"""The seeded generators: determinism, row-range regeneration, bf16 rounding, recipe shapes."""
import numpy as np
import torch

import synth


def test_bf16_rounding_matches_torch():
    rng = np.random.default_rng(0)
    a = (rng.standard_normal(20000) * 10 ** rng.uniform(-6, 6, 20000)).astype(np.float32)
    bits = synth.f32_to_bf16_bits(a)
    ref = torch.from_numpy(a).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bits, ref)
    back = synth.bf16_bits_to_f32(bits)
    assert np.array_equal(back, torch.from_numpy(a).to(torch.bfloat16).float().numpy())


def test_weights_deterministic_and_sliceable():
    shape = synth.CONFIGS[0]
    a = synth.WeightSource(shape, 3).tensor("w_gate", 1)
    b = synth.WeightSource(shape, 3).tensor("w_gate", 1)
    c = synth.WeightSource(shape, 4).tensor("w_gate", 1)
    assert a.shape == (768, 256) and a.dtype == np.float32
    assert np.array_equal(a, b) and not np.array_equal(a, c)
    assert not np.array_equal(a, synth.WeightSource(shape, 3).tensor("w_gate", 0))
    assert abs(float(a.std()) - 0.02) < 1e-3 and abs(float(a.mean())) < 1e-3
    big = synth.CONFIGS[2]
    src = synth.WeightSource(big, 0)
    rows = src.tensor("lm_head", -1, (1000, 1100))
    assert rows.dtype == np.uint16 and rows.shape == (100, 4096)
    one = src.tensor("lm_head", -1, (1050, 1051))
    assert np.array_equal(one[0], rows[50])
    span = src.tensor("lm_head", -1, (1020, 1030))       # crosses a generation chunk (1024 rows)
    assert np.array_equal(span, rows[20:30])


def test_draft_recipe():
    shape = synth.CONFIGS[0]
    d = synth.make_draft(shape, 1)
    assert d["tokens"].shape == (1, 4) and d["probs"].shape == (1, 4, 4096)
    assert d["uniforms"].shape == (1, 5) and d["uniforms"].dtype == np.float32
    assert (d["uniforms"] >= 0).all() and (d["uniforms"] < 1).all()
    assert np.allclose(d["probs"].sum(-1), 1, atol=1e-5)
    assert (d["tokens"] >= 0).all() and (d["tokens"] < 4096).all()
    assert all(d["probs"][0, j, d["tokens"][0, j]] > 0 for j in range(4))
    d2 = synth.make_draft(shape, 1)
    assert np.array_equal(d["tokens"], d2["tokens"]) and np.array_equal(d["probs"], d2["probs"])


def test_kv_lengths_ragged():
    lens = synth.CONFIGS[3].kv_lengths(0)
    assert lens.shape == (16,) and lens.min() >= 512 and lens.max() <= 4096
    assert len(set(lens.tolist())) > 8
    assert synth.CONFIGS[2].kv_lengths(0).tolist() == [1024]
