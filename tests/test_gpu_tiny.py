"""GPU parity on the tiny fp32 workload (2 layers, d=256, MHA 4x64, vocab 4096, cache 128, gamma 4):
prefill, one verification step, and a second step that reads what the first appended."""
import numpy as np
import pytest

import paper_2510_02329_amd as sj
import synth
from oracle import selfjudge_oracle as orc
from tests import gpu_common as G
from tests import helpers

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def tiny():
    shape = synth.CONFIGS[0]
    src = synth.WeightSource(shape, seed=0, norm_jitter=0.1, judge_bias=0.05)
    gpu = G.Gpu(shape, src, [192])
    cfg = helpers.oracle_config(shape)
    W = helpers.oracle_weights(src)
    cache = orc.SeqCache(cfg, 192, storage=shape.dtype)
    prompt = synth.make_prompt(shape, 0, 128)
    print("prefill gpu", flush=True)
    sj.sj_prefill(gpu.model, gpu.kv, 0, prompt.tolist())
    print("prefill oracle", flush=True)
    orc.prefill(cfg, W, cache, prompt.tolist())
    yield shape, gpu, cfg, W, cache
    gpu.close()


def test_prefill_and_two_steps(tiny):
    shape, gpu, cfg, W, cache = tiny
    ln, pend = sj.sj_kv_state(gpu.kv, 1)
    assert ln[0] == 128 == cache.length
    assert pend[0] == cache.pending
    for l in range(shape.n_layers):
        k, v = gpu.kv_rows(0, l, 0, 128)
        G.close_enough(k, cache.k[l][:, :128], "fp32", f"prefill K layer {l}")
        G.close_enough(v, cache.v[l][:, :128], "fp32", f"prefill V layer {l}")
    for step, theta in enumerate((0.5, 0.38)):
        draft = synth.make_draft(shape, seed=10 + step)
        L0 = cache.length
        print(f"step {step} gpu", flush=True)
        out = gpu.step(draft, theta)
        ref = orc.verify_step(cfg, W, [cache], draft["tokens"], draft["probs"], draft["uniforms"], theta)[0]
        G.close_enough(out["logits"][0], ref["logits"], "fp32", "logits")
        G.close_enough(out["hn"][0], ref["hn"], "fp32", "hidden")
        G.close_enough(out["judge_scores"][0], ref["judge_scores"], "fp32", "judge scores")
        G.close_enough(out["p_at_draft"][0], ref["p_at_draft"], "fp32", "p(d)")
        for l in range(shape.n_layers):
            k, v = gpu.kv_rows(0, l, L0, shape.gamma + 1)
            G.close_enough(k, ref["k_new"][l], "fp32", f"appended K layer {l}")
            G.close_enough(v, ref["v_new"][l], "fp32", f"appended V layer {l}")
        bad, excused = G.replay_matches(shape, out, draft, theta)
        assert not bad, bad
        bits = [(1 if a else 0) | (2 if g else 0) for a, g in zip(ref["align_bits"], ref["judge_bits"])]
        assert out["bits"][0].tolist() == bits
        assert int(out["accepted_len"][0]) == ref["accepted_len"]
        assert 0 <= int(out["accepted_len"][0]) <= shape.gamma
        assert int(out["next_token"][0]) == ref["next_token"]
        ln, pend = sj.sj_kv_state(gpu.kv, 1)
        assert ln[0] == cache.length and pend[0] == cache.pending
