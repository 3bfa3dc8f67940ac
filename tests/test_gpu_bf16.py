"""GPU parity in bf16: a scaled-down Llama-shaped decoder with grouped-query attention (several MFMA
tiles, ragged cache lengths, a batch) and the full 8B-shaped batch-1 workload the benchmark times."""
import numpy as np
import pytest
import torch

import paper_2510_02329_amd as sj
import synth
from oracle import selfjudge_oracle as orc
from tests import gpu_common as G
from tests import helpers
from tests.progress import say

pytestmark = pytest.mark.gpu


def _fill_caches(shape, gpu, cfg, lens, seed, capacity):
    caches = []
    pend = synth.make_pending(shape, seed)
    for b in range(shape.batch):
        c = orc.SeqCache(cfg, capacity[b], storage=shape.dtype)
        for l in range(shape.n_layers):
            k, v = synth.make_kv_cache(shape, seed, b, l, int(lens[b]))
            sj.sj_kv_set_layer(gpu.kv, b, l, k, v, int(lens[b]))
            c.k[l][:, :lens[b]] = synth.to_f64(k)
            c.v[l][:, :lens[b]] = synth.to_f64(v)
        if shape.n_layers > 40:
            say(f"  cache of sequence {b} filled")
        c.length, c.pending = int(lens[b]), int(pend[b])
        sj.sj_kv_set_state(gpu.kv, b, int(lens[b]), int(pend[b]))
        caches.append(c)
    return caches


def _compare_step(shape, gpu, cfg, W, caches, draft, theta, label, force_rounding=False, scale=1.0):
    B, gamma = draft["tokens"].shape
    L0 = [c.length for c in caches]
    out = gpu.step(draft, theta, gamma)
    flips = {"rows": 0, "flips": 0}
    if force_rounding:
        G.force_device_rounding(gpu, caches, gamma, flips)
    ref = orc.verify_step(cfg, W, caches, draft["tokens"], draft["probs"], draft["uniforms"], theta)
    if force_rounding:
        say(f"{label}: {flips['flips']} of {flips['rows']} stored K/V elements took the other bf16 neighbour")
        assert flips["flips"] < 0.10 * flips["rows"]
    stats = {}
    for b in range(B):
        lg = G.close_enough(out["logits"][b], ref[b]["logits"], shape.dtype, f"{label} logits seq {b}", scale=scale)
        stats["logits"] = max(stats.get("logits", (0.0, 0.0)), lg, key=lambda t: t[1])
        G.close_enough(out["hn"][b], ref[b]["hn"], shape.dtype, f"{label} hidden seq {b}")
        G.close_enough(out["judge_scores"][b], ref[b]["judge_scores"], shape.dtype, f"{label} judge seq {b}")
        for l in (0, shape.n_layers - 1):
            k, v = gpu.kv_rows(b, l, L0[b], gamma + 1)
            G.close_enough(k, ref[b]["k_new"][l], shape.dtype, f"{label} appended K seq {b} layer {l}")
            G.close_enough(v, ref[b]["v_new"][l], shape.dtype, f"{label} appended V seq {b} layer {l}")
    # decisions: exact on replay of the device's own logits (B); against the pure oracle (C) a mismatch is
    # excused only when the oracle's margin is inside the logit tolerance
    bad, excused = G.replay_matches(shape, out, draft, theta)
    assert not bad, bad
    cnt = G.decisions_vs_oracle(shape, out, ref, draft, theta)
    say(f"{label}: replay excused {excused}; vs pure oracle: tokens equal {cnt['tokens_equal']}/{cnt['tokens']}, "
          f"excused bits {cnt['bit_excused']} lengths {cnt['len_excused']} tokens {cnt['token_excused']}, "
          f"unexcused {cnt['unexcused']}")
    assert excused == 0 and cnt["unexcused"] == 0
    stats["decisions"] = cnt
    ln, pend = sj.sj_kv_state(gpu.kv, B)
    assert (0 <= out["accepted_len"]).all() and (out["accepted_len"] <= gamma).all()
    assert (ln == np.array(L0) + 1 + out["accepted_len"]).all()
    assert (pend == out["next_token"]).all()
    return out, ref, stats


SMALL = synth.ModelShape("small_bf16", "bf16", 3, 512, 8, 2, 128, 1408, 4992, 500000.0,
                         batch=3, gamma=5, weight_std=0.05)


@pytest.mark.parametrize("theta", [0.5])
def test_small_gqa_bf16_two_steps(theta):
    shape = SMALL
    src = synth.WeightSource(shape, seed=1, norm_jitter=0.1, judge_bias=-0.1)
    cap = [448, 448, 448]
    gpu = G.Gpu(shape, src, cap)
    try:
        cfg = helpers.oracle_config(shape)
        W = helpers.oracle_weights(src)
        lens = [70, 200, 333]
        caches = _fill_caches(shape, gpu, cfg, lens, seed=2, capacity=cap)
        for step in range(2):
            draft = synth.make_draft(shape, seed=20 + step)
            out, ref, _ = _compare_step(shape, gpu, cfg, W, caches, draft, theta, f"step {step}")
            # keep both sides on the same trajectory for the chained step even if a near-tie differed
            for b, c in enumerate(caches):
                c.length = c.length - 1 - ref[b]["accepted_len"] + 1 + int(out["accepted_len"][b])
                c.pending = int(out["next_token"][b])
    finally:
        gpu.close()


@pytest.mark.parametrize("batch,gamma,lens", [
    (3, 7, [70, 200, 333]),                                        # 24 rows: two row tiles
    (10, 15, [0, 33, 1500, 64, 129, 700, 31, 32, 255, 1024]),      # 160 rows: two launches of the many-row
])                                                                 # GEMM; empty, one-step and 12-range contexts
def test_small_gqa_bf16_many_rows(batch, gamma, lens):
    """More than 16 query rows (the LDS-staged projections), contexts from empty to many key ranges
    (several key steps per wave, the ticketed merge in more than one batch)."""
    import dataclasses
    shape = dataclasses.replace(SMALL, name=f"small_bf16_b{batch}_g{gamma}", batch=batch, gamma=gamma)
    src = synth.WeightSource(shape, seed=3, norm_jitter=0.1, judge_bias=0.2)
    cap = [max(64, l + gamma + 1 + 17) for l in lens]
    gpu = G.Gpu(shape, src, cap)
    try:
        cfg = helpers.oracle_config(shape)
        W = helpers.oracle_weights(src)
        caches = _fill_caches(shape, gpu, cfg, lens, seed=4, capacity=cap)
        draft = synth.make_draft(shape, seed=40)
        _compare_step(shape, gpu, cfg, W, caches, draft, 0.5, f"rows {batch * (gamma + 1)}")
    finally:
        gpu.close()


def test_llama8b_batch1_full_size():
    """The benchmark workload: 32 layers, d 4096, 32/8 heads of 128, FFN 14336, vocab 128256, cache 1024,
    gamma 5, in the launch configuration bench.py times.  The oracle runs the whole step in fp64."""
    shape = synth.CONFIGS[2]
    src = synth.WeightSource(shape, seed=0)
    cap = [1024 + 64]
    say("loading 8B-shaped model")
    gpu = G.Gpu(shape, src, cap)
    try:
        cfg = helpers.oracle_config(shape)
        W = helpers.oracle_weights(src, cache_items=0)
        caches = _fill_caches(shape, gpu, cfg, shape.kv_lengths(0), seed=0, capacity=cap)
        draft = synth.make_draft(shape, seed=0)
        gamma, dev = shape.gamma, gpu.dev
        len0, pend0 = sj.sj_kv_state(gpu.kv, 1)
        # teacher-forced scoring of the same rows (Eq. 6 - 7): the state stays put, so the step below sees it unchanged
        ins = np.concatenate([[caches[0].pending], draft["tokens"][0]]).astype(np.int32)[None]
        tgt = np.concatenate([draft["tokens"][0], [17]]).astype(np.int32)[None]
        lp = torch.zeros((1, gamma + 1), dtype=torch.float32, device=dev)
        sj.sj_score_block(gpu.model, gpu.kv, gamma + 1, torch.from_numpy(ins).to(dev), torch.from_numpy(tgt).to(dev), lp)
        torch.cuda.synchronize()
        assert (np.array(sj.sj_kv_state(gpu.kv, 1)) == np.array([len0, pend0])).all()
        say("step")
        out, ref, stats = _compare_step(shape, gpu, cfg, W, caches, draft, 0.5, "8B")
        say("8B logits max err %.3e worst err/bound %.2f" % stats["logits"])
        lg = ref[0]["logits"] / shape.temperature
        lse = np.log(np.exp(lg - lg.max(axis=1, keepdims=True)).sum(axis=1)) + lg.max(axis=1)
        lp_ref = lg[np.arange(gamma + 1), tgt[0]] - lse
        a_tol, r_tol = G.TOL["bf16"]
        lp_err = np.abs(lp.cpu().numpy()[0] - lp_ref).max()
        say("8B teacher-forced log-probabilities max err %.3e" % lp_err)
        assert lp_err <= 2 * (a_tol + r_tol * np.abs(ref[0]["logits"]).max())
        # top-k verification on the same state: decisions replayed by the oracle's tail on the device's logits
        sj.sj_kv_rewind(gpu.kv, len0.tolist(), pend0.tolist())
        sj.sj_set_mode(gpu.kv, sj.SJ_MODE_TOPK)
        out_k = gpu.step(draft, 0.5)
        tail = orc.verify_tail(out_k["logits"][0].astype(np.float64), out_k["judge_scores"][0], draft["tokens"][0],
                               draft["probs"][0], draft["uniforms"][0], 0.5, shape.temperature, "topk", 2)
        assert [(int(x) >> 2) & 1 for x in out_k["bits"][0]] == [int(t) for t in tail["topk_bits"]]
        assert int(out_k["accepted_len"][0]) == tail["accepted_len"] and int(out_k["next_token"][0]) == tail["next_token"]
        assert np.array_equal(out_k["logits"], out["logits"])               # the mode does not touch the forward
        sj.sj_set_mode(gpu.kv, sj.SJ_MODE_TWO_STAGE)
        # peaked and greedy target distributions (same forward, so the oracle's logits are reused): here the emitted
        # token is meaningful - on the flat T = 1 distribution almost any draw sits next to a cell boundary
        w_j, b_j = W("judge_w"), float(np.asarray(W("judge_b")).reshape(-1)[0])
        for T in (0.125, 0.0):
            sj.sj_set_temperature(gpu.model, T)
            sj.sj_kv_rewind(gpu.kv, len0.tolist(), pend0.tolist())
            shape_T = shape.scaled(temperature=T)
            out_T = gpu.step(draft, 0.5)
            ref_T = dict(ref[0])
            ref_T.update(orc.verify_tail(ref[0]["logits"], ref[0]["judge_scores"], draft["tokens"][0], draft["probs"][0],
                                         draft["uniforms"][0], 0.5, T))
            bad, excused = G.replay_matches(shape_T, out_T, draft, 0.5)
            assert not bad and excused == 0, (T, bad, excused)
            cnt = G.decisions_vs_oracle(shape_T, out_T, [ref_T], draft, 0.5)
            say(f"8B T={T}: accepted {int(out_T['accepted_len'][0])} (oracle {ref_T['accepted_len']}), token "
                  f"{int(out_T['next_token'][0])} (oracle {ref_T['next_token']}), {cnt}")
            assert cnt["unexcused"] == 0
            assert np.array_equal(out_T["logits"], out["logits"])           # temperature does not touch the forward
        sj.sj_set_temperature(gpu.model, shape.temperature)
        # three operand planes on this shape with the start-up measurement on: the launch shapes are re-derived for
        # the new plane count; the logits move closer to the oracle
        sj.sj_set_operand_planes(gpu.kv, 3)
        sj.sj_kv_rewind(gpu.kv, len0.tolist(), pend0.tolist())
        out3 = gpu.step(draft, 0.5)
        err3, worst3 = G.close_enough(out3["logits"][0], ref[0]["logits"], shape.dtype, "8B logits, three planes")
        say("8B logits with three operand planes: max err %.3e worst err/bound %.3f (two planes: %.3f)" % (err3, worst3, stats["logits"][1]))
        assert worst3 <= stats["logits"][1]
        sj.sj_set_operand_planes(gpu.kv, 2)
    finally:
        gpu.close()
