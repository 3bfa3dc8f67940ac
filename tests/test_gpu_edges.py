"""GPU edge cases on small models: draft lengths 1 and max, temperature 0, verifier modes, judge
thresholds outside (0,1), capacity errors, out-of-range draft tokens, bitwise-repeatable reruns."""
import numpy as np
import pytest
import torch

import paper_2510_02329_amd as sj
import synth
from oracle import selfjudge_oracle as orc
from paper_2510_02329_amd import binding
from tests import gpu_common as G
from tests import helpers
from tests.test_gpu_bf16 import _fill_caches

pytestmark = pytest.mark.gpu

BASE = synth.ModelShape("edge_bf16", "bf16", 2, 256, 4, 2, 64, 512, 1024, 10000.0, batch=2, gamma=4, weight_std=0.08)


def _setup(shape, lens, seed=5, max_gamma=None, cap=None):
    src = synth.WeightSource(shape, seed=seed, norm_jitter=0.1, judge_bias=0.3)
    cap = cap or [l + 64 for l in lens]
    gpu = G.Gpu(shape, src, cap, max_gamma=max_gamma)
    cfg = helpers.oracle_config(shape)
    W = helpers.oracle_weights(src)
    caches = _fill_caches(shape, gpu, cfg, lens, seed=seed + 1, capacity=cap)
    return gpu, cfg, W, caches


def _oracle(cfg, W, caches, draft, theta, mode="two_stage"):
    return orc.verify_step(cfg, W, caches, draft["tokens"], draft["probs"], draft["uniforms"], theta, mode)


def _same_decisions(out, ref, B):
    for b in range(B):
        bits = [(1 if a else 0) | (2 if g else 0) for a, g in zip(ref[b]["align_bits"], ref[b]["judge_bits"])]
        assert out["bits"][b].tolist() == bits
        assert int(out["accepted_len"][b]) == ref[b]["accepted_len"]
        assert int(out["next_token"][b]) == ref[b]["next_token"]


@pytest.mark.parametrize("gamma", [1, 2, 7])
def test_draft_lengths(gamma):
    shape = BASE.scaled(gamma=gamma)
    gpu, cfg, W, caches = _setup(shape, [37, 64], max_gamma=7)
    try:
        draft = synth.make_draft(shape, seed=gamma)
        out = gpu.step(draft, 0.5, gamma)
        ref = _oracle(cfg, W, caches, draft, 0.5)
        for b in range(2):
            G.close_enough(out["logits"][b], ref[b]["logits"], "bf16", "logits")
        _same_decisions(out, ref, 2)
    finally:
        gpu.close()


def test_temperature_zero_is_greedy_match():
    """T = 0, judge off: accepted prefix = longest prefix of drafts equal to the target arg-max, and the
    emitted token is the arg-max at the first mismatch (strict speculative sampling, Sec. 3.1)."""
    shape = BASE.scaled(temperature=0.0, batch=2, gamma=4)
    gpu, cfg, W, caches = _setup(shape, [20, 45])
    try:
        # a draft that copies the target's own greedy continuation for 2 tokens, then diverges
        probe = synth.make_draft(shape, seed=1)
        import copy
        c2 = copy.deepcopy(caches)
        ref0 = _oracle(cfg, W, c2, probe, 1.0)
        greedy = [np.argmax(r["logits"], axis=1) for r in ref0]
        draft = synth.make_draft(shape, seed=2)
        for b in range(2):
            draft["tokens"][b, 0] = greedy[b][0]
        out = gpu.step(draft, 1.0)
        ref = _oracle(cfg, W, caches, draft, 1.0)
        _same_decisions(out, ref, 2)
        for b in range(2):
            n = int(out["accepted_len"][b])
            assert n >= 1
            am = np.argmax(ref[b]["logits"], axis=1)
            assert all(draft["tokens"][b, j] == am[j] for j in range(n))
            assert int(out["next_token"][b]) == am[n]
    finally:
        gpu.close()


@pytest.mark.parametrize("mode,name", [(sj.SJ_MODE_ALIGNMENT, "alignment"), (sj.SJ_MODE_JUDGE, "judge"),
                                       (sj.SJ_MODE_TWO_STAGE, "two_stage")])
def test_verifier_modes(mode, name):
    shape = BASE
    gpu, cfg, W, caches = _setup(shape, [50, 31])
    try:
        sj.sj_set_mode(gpu.kv, mode)
        draft = synth.make_draft(shape, seed=9)
        out = gpu.step(draft, 0.45)
        ref = _oracle(cfg, W, caches, draft, 0.45, name)
        for b in range(2):
            assert int(out["accepted_len"][b]) == ref[b]["accepted_len"]
            assert int(out["next_token"][b]) == ref[b]["next_token"]
    finally:
        gpu.close()


@pytest.mark.parametrize("k", [1, 2, 3])
def test_topk_mode(k):
    """Top-k verification (the relaxed baseline of Sec. 4.1): drafts placed at the target's first, second,
    third ... ranked token; decisions replayed exactly by the oracle's tail on the device's own logits."""
    import copy
    shape = BASE.scaled(batch=2, gamma=4)
    gpu, cfg, W, caches = _setup(shape, [50, 31])
    try:
        probe = synth.make_draft(shape, seed=3)
        ref0 = _oracle(cfg, W, copy.deepcopy(caches), probe, 0.5)
        draft = synth.make_draft(shape, seed=4)
        # sequence 0: ranks 0, 1, 2, 0 of row 0's ordering (later rows follow other tokens: any rank);
        # sequence 1: rank 1 first
        draft["tokens"][0, 0] = np.argsort(-ref0[0]["logits"][0], kind="stable")[0]
        draft["tokens"][1, 0] = np.argsort(-ref0[1]["logits"][0], kind="stable")[1]
        sj.sj_set_mode(gpu.kv, sj.SJ_MODE_TOPK)
        sj.sj_set_topk(gpu.kv, k)
        out = gpu.step(draft, 0.5)
        ref = orc.verify_step(cfg, W, caches, draft["tokens"], draft["probs"], draft["uniforms"], 0.5, "topk", k)
        for b in range(2):
            G.close_enough(out["logits"][b], ref[b]["logits"], "bf16", "logits")
            tail = orc.verify_tail(out["logits"][b].astype(np.float64), out["judge_scores"][b], draft["tokens"][b],
                                   draft["probs"][b], draft["uniforms"][b], 0.5, shape.temperature, "topk", k)
            assert [(int(x) >> 2) & 1 for x in out["bits"][b]] == [int(t) for t in tail["topk_bits"]]
            assert int(out["accepted_len"][b]) == tail["accepted_len"]
            assert int(out["next_token"][b]) == tail["next_token"]
        assert int(out["accepted_len"][0]) >= 1                      # the arg-max token passes every k
        assert (int(out["accepted_len"][1]) >= 1) == (k >= 2)        # the runner-up needs k >= 2
        with pytest.raises(sj.SJError):
            sj.sj_set_topk(gpu.kv, 0)
        with pytest.raises(sj.SJError):
            sj.sj_set_mode(gpu.kv, 4)
    finally:
        gpu.close()


def test_threshold_extremes_and_rerun_is_bit_identical():
    shape = BASE
    gpu, cfg, W, caches = _setup(shape, [50, 31])
    try:
        draft = synth.make_draft(shape, seed=11)
        lens0, pend0 = sj.sj_kv_state(gpu.kv, 2)
        off = gpu.step(draft, 1.0)                       # judge disabled: standard speculative decoding
        sj.sj_kv_rewind(gpu.kv, lens0.tolist(), pend0.tolist())
        allok = gpu.step(draft, -1.0)                    # judge accepts everything
        assert (allok["accepted_len"] == shape.gamma).all()
        assert (off["bits"] & 2 == 0).all() and (allok["bits"] & 2 == 2).all()
        assert (off["accepted_len"] <= allok["accepted_len"]).all()
        sj.sj_kv_rewind(gpu.kv, lens0.tolist(), pend0.tolist())
        a = gpu.step(draft, 0.5)
        sj.sj_kv_rewind(gpu.kv, lens0.tolist(), pend0.tolist())
        b = gpu.step(draft, 0.5)
        for k in ("logits", "hn", "judge_scores", "p_at_draft", "bits", "accepted_len", "next_token"):
            assert np.array_equal(a[k], b[k]), k         # deterministic reductions: reruns are bit-identical
        ref = _oracle(cfg, W, caches, draft, 0.5)
        _same_decisions(a, ref, 2)
    finally:
        gpu.close()


def test_two_cache_objects_on_one_model_are_bit_identical():
    """The launch shapes measured when the first cache object is created are kept with the model: a second object
    runs the same kernels in the same summation order (and a changed temperature only changes the tail)."""
    shape = BASE
    gpu, cfg, W, caches = _setup(shape, [50, 31])
    try:
        draft = synth.make_draft(shape, seed=12)
        a = gpu.step(draft, 0.5)
        kv2 = sj.sj_kv_create(gpu.model, shape.batch, [50 + 64, 31 + 64])
        first = gpu.kv
        try:
            gpu.kv = kv2
            cfg2 = helpers.oracle_config(shape)
            _fill_caches(shape, gpu, cfg2, [50, 31], seed=6, capacity=[50 + 64, 31 + 64])
            b = gpu.step(draft, 0.5)
            for k in ("logits", "hn", "judge_scores", "p_at_draft", "bits", "accepted_len", "next_token"):
                assert np.array_equal(a[k], b[k]), k
            sj.sj_set_temperature(gpu.model, 0.5)
            sj.sj_kv_rewind(kv2, [50, 31], [int(c.pending) for c in caches])
            c2 = gpu.step(draft, 0.5)
            assert np.array_equal(c2["logits"], a["logits"])
            tail = [orc.verify_tail(c2["logits"][i].astype(np.float64), c2["judge_scores"][i], draft["tokens"][i], draft["probs"][i],
                                    draft["uniforms"][i], 0.5, 0.5) for i in range(2)]
            assert [int(x) for x in c2["accepted_len"]] == [t["accepted_len"] for t in tail]
            assert [int(x) for x in c2["next_token"]] == [t["next_token"] for t in tail]
            sj.sj_set_temperature(gpu.model, shape.temperature)
        finally:
            gpu.kv = first
            sj.sj_kv_free(kv2)
    finally:
        gpu.close()


def test_capacity_and_argument_errors():
    shape = BASE
    gpu, cfg, W, caches = _setup(shape, [60, 10], cap=[64, 64])
    try:
        draft = synth.make_draft(shape, seed=3)
        dev = gpu.dev
        dt = torch.from_numpy(draft["tokens"]).to(dev); dp = torch.from_numpy(draft["probs"]).to(dev)
        un = torch.from_numpy(draft["uniforms"]).to(dev)
        acc = torch.zeros(2, dtype=torch.int32, device=dev); nxt = torch.zeros(2, dtype=torch.int32, device=dev)
        lens0, pend0 = sj.sj_kv_state(gpu.kv, 2)
        with pytest.raises(sj.SJError) as e:             # 60 + 4 + 1 > 64
            sj.sj_verify_step(gpu.model, gpu.kv, 4, dt, dp, un, 0.5, acc, nxt)
        assert e.value.code == binding.SJ_ECAPACITY
        lens1, pend1 = sj.sj_kv_state(gpu.kv, 2)
        assert (lens0 == lens1).all() and (pend0 == pend1).all()          # nothing was modified
        for bad_gamma in (0, 5):
            with pytest.raises(sj.SJError) as e:
                sj.sj_verify_step(gpu.model, gpu.kv, bad_gamma, dt, dp, un, 0.5, acc, nxt)
            assert e.value.code == binding.SJ_EINVAL
        with pytest.raises(sj.SJError) as e:
            sj.sj_verify_step(gpu.model, gpu.kv, 4, dt, None, un, 0.5, acc, nxt)
        assert e.value.code == binding.SJ_EINVAL
        with pytest.raises(sj.SJError):
            sj.sj_kv_set_state(gpu.kv, 0, 65, 0)
        with pytest.raises(sj.SJError):
            sj.sj_kv_set_state(gpu.kv, 2, 1, 0)
        # an out-of-range draft token is clamped on the device, never read out of bounds
        sj.sj_kv_set_state(gpu.kv, 0, 10, int(pend0[0]))
        dt_bad = dt.clone(); dt_bad[0, 1] = 10 ** 6; dt_bad[1, 0] = -5
        sj.sj_verify_step(gpu.model, gpu.kv, 4, dt_bad, dp, un, 0.5, acc, nxt)
        torch.cuda.synchronize()
        assert ((acc >= 0) & (acc <= 4)).all() and ((nxt >= 0) & (nxt < shape.vocab)).all()
    finally:
        gpu.close()


def test_three_plane_operand_is_closer_than_one():
    """The operand-plane setting trades nothing in HBM traffic: 1 plane rounds activations to bf16 at every
    product, 3 planes carry them exactly.  The logit error against the oracle must shrink accordingly."""
    shape = BASE.scaled(batch=1)
    errs = {}
    for planes in (1, 2, 3):
        gpu, cfg, W, caches = _setup(shape, [40])
        try:
            sj.sj_set_operand_planes(gpu.kv, planes)
            draft = synth.make_draft(shape, seed=4)
            out = gpu.step(draft, 0.5)
            ref = _oracle(cfg, W, caches, draft, 0.5)
            errs[planes] = float(np.abs(out["logits"][0] - ref[0]["logits"]).max())
        finally:
            gpu.close()
    assert errs[3] < errs[2] < errs[1], errs
    assert errs[3] < 1e-4 and errs[1] > 10 * errs[2], errs


RING = synth.ModelShape("ring_bf16", "bf16", 2, 512, 8, 2, 128, 1536, 4992, 10000.0, batch=1, gamma=3, weight_std=0.06)


@pytest.mark.parametrize("gamma,planes", [(3, 2), (7, 2), (8, 2), (15, 2), (5, 1)])
def test_lds_ring_projections(gamma, planes, monkeypatch):
    """Every projection of this shape fits the LDS-ring kernel.  Up to 8 rows both operand planes ride in one product,
    from 9 rows on (and with a single plane) there is one product per plane: both layouts against the oracle and
    against the register-ring kernel on the same inputs.  SJ_TUNE=0 pins the rule's launch shapes; SJ_RING_ROWS moves
    the row limit of the rule (16: ring everywhere, 0: never)."""
    shape = RING.scaled(gamma=gamma)
    draft = synth.make_draft(shape, seed=gamma)
    logits = {}
    for ring_rows in (16, 0):
        monkeypatch.setenv("SJ_TUNE", "0")
        monkeypatch.setenv("SJ_RING_ROWS", str(ring_rows))
        gpu, cfg, W, caches = _setup(shape, [150], max_gamma=15)
        try:
            if planes != 2:
                sj.sj_set_operand_planes(gpu.kv, planes)
            names = [sj.sj_kernel_class_shape(gpu.kv, c, gamma + 1) for c in (1, 2, 3, 4, 5)]
            assert all(n.startswith("gemm_ring" if ring_rows else "gemm_skinny") for n in names), names
            out = gpu.step(draft, 0.5, gamma)
            logits[ring_rows] = out["logits"][0].copy()
            if planes == 2:
                ref = _oracle(cfg, W, caches, draft, 0.5)
                G.close_enough(out["logits"][0], ref[0]["logits"], "bf16", f"logits, ring rows {ring_rows}")
                _same_decisions(out, ref, 1)
        finally:
            gpu.close()
    # the two kernels add in different orders; with a single plane every product input is then rounded to bf16 (2^-9),
    # so last-bit differences of an fp32 sum surface as whole bf16 ulps further on
    diff = np.abs(logits[16] - logits[0])
    abs_tol, rel_tol = (5e-3, 1e-2) if planes == 2 else (5e-2, 5e-2)
    print(f"ring vs register-ring kernel, {planes} plane(s), {gamma + 1} rows: max |diff| {float(diff.max()):.3e}")
    assert (diff <= abs_tol + rel_tol * np.abs(logits[0])).all(), float(diff.max())
