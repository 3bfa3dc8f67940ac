"""GPU parity of the draft proposal (Sec. 2.2, Eq. 1): gamma sequential single-token decodes producing the
draft tokens and their distributions, and one whole speculate -> verify cycle on the device."""
import dataclasses

import numpy as np
import pytest
import torch

import paper_2510_02329_amd as sj
import synth
from oracle import selfjudge_oracle as orc
from tests import gpu_common as G
from tests import helpers
from tests.test_gpu_bf16 import SMALL, _fill_caches

pytestmark = pytest.mark.gpu


def _device_draft(gpu, gamma, uniforms, feed_last=True):
    B, V = gpu.shape.batch, gpu.shape.vocab
    un = torch.from_numpy(np.ascontiguousarray(uniforms.astype(np.float32))).to(gpu.dev)
    toks = torch.full((B, gamma), -7, dtype=torch.int32, device=gpu.dev)
    probs = torch.full((B, gamma, V), -1.0, dtype=torch.float32, device=gpu.dev)
    sj.sj_draft_block(gpu.model, gpu.kv, gamma, un, feed_last, toks, probs, torch.cuda.current_stream())
    torch.cuda.synchronize()
    return toks.cpu().numpy(), probs.cpu().numpy()


@pytest.mark.parametrize("dtype,batch,gamma,temperature", [("bf16", 3, 4, 1.0), ("bf16", 1, 6, 0.7), ("fp32", 2, 3, 1.0),
                                                           ("bf16", 2, 3, 0.0)])
def test_draft_block_matches_oracle(dtype, batch, gamma, temperature):
    shape = dataclasses.replace(SMALL, name=f"draft_{dtype}", dtype=dtype, batch=batch, gamma=gamma, temperature=temperature)
    src = synth.WeightSource(shape, seed=5, norm_jitter=0.1)
    _draft_case(shape, src, [40, 133, 7][:batch], own_draws=True)


def test_draft_block_1b_shaped_full_size():
    """The draft model of the paper's Llama pairing at its real shape (16 layers, d 2048, 32/8 heads of 64, vocab
    128256), cache 1024, gamma 5: the configuration `bench.py --cycle` times."""
    shape = dataclasses.replace(synth.DRAFT_1B, batch=1, gamma=5)
    src = synth.WeightSource(shape, seed=0)
    print("loading the 1B-shaped draft model", flush=True)
    _draft_case(shape, src, [1024], own_draws=False, cache_items=0)


def _draft_case(shape, src, lens, own_draws, cache_items=None):
    dtype, batch, gamma = shape.dtype, shape.batch, shape.gamma
    cap = [l + gamma + 20 for l in lens]
    gpu = G.Gpu(shape, src, cap)
    try:
        cfg = helpers.oracle_config(shape)
        W = helpers.oracle_weights(src) if cache_items is None else helpers.oracle_weights(src, cache_items=cache_items)
        caches = _fill_caches(shape, gpu, cfg, lens, seed=6, capacity=cap)
        pend0 = [c.pending for c in caches]
        uniforms = np.random.default_rng(8).random((gamma, batch)).astype(np.float32)
        toks, probs = _device_draft(gpu, gamma, uniforms)
        assert ((0 <= toks) & (toks < shape.vocab)).all()
        a_tol, r_tol = G.TOL[dtype]
        # 1. every q row against the oracle's forward over the tokens the DEVICE fed (teacher forcing keeps
        #    the comparison meaningful even if a draw at a near-tie went the other way)
        fw = orc.block_forward(cfg, W, caches, [[pend0[b]] + [int(t) for t in toks[b]] for b in range(batch)])
        for b in range(batch):
            for j in range(gamma):
                q_ref = orc.target_distribution(fw[b]["logits"][j], shape.temperature)
                assert abs(float(probs[b, j].sum()) - 1.0) < 1e-4
                if shape.temperature == 0.0:
                    top2 = np.sort(fw[b]["logits"][j])[-2:]
                    if top2[1] - top2[0] > 2 * (a_tol + r_tol * abs(top2[1])):
                        assert (probs[b, j] == q_ref).all()
                    continue
                tau = a_tol + r_tol * np.abs(fw[b]["logits"][j]).max()          # logit tolerance -> relative on q
                err = np.abs(probs[b, j] - q_ref)
                assert (err <= q_ref * (np.exp(2 * tau) - 1) + 1e-7).all(), f"q row {b},{j}: max err {err.max():.3e}"
                # 2. the token is the inverse-CDF draw from the device's own row (exact up to fp32 rounding of q)
                c = np.cumsum(probs[b, j].astype(np.float64))
                t = float(uniforms[j, b]) * c[-1]
                k = int(toks[b, j])
                lo = c[k - 1] if k > 0 else 0.0
                assert lo - 1e-6 <= t < c[k] + 1e-6, f"token {b},{j} is not the draw for u = {uniforms[j, b]}"
        # 3. state and cache rows: one row per fed token (pending, d_1 .. d_gamma with feed_last)
        ln, pend = sj.sj_kv_state(gpu.kv, batch)
        assert (ln == np.array(lens) + gamma + 1).all() and (pend == toks[:, -1]).all()
        for b in range(batch):
            for l in (0, shape.n_layers - 1):
                k, v = gpu.kv_rows(b, l, lens[b], gamma + 1)
                G.close_enough(k, caches[b].k[l][:, lens[b]:lens[b] + gamma + 1], dtype, f"draft K seq {b} layer {l}")
                G.close_enough(v, caches[b].v[l][:, lens[b]:lens[b] + gamma + 1], dtype, f"draft V seq {b} layer {l}")
        if not own_draws:
            return
        # 4. the oracle's own draft (drawing for itself) agrees on the tokens, except at near-ties of the CDF
        caches2 = _fill_caches(shape, gpu, cfg, lens, seed=6, capacity=cap)     # also resets the device state
        toks_ref, probs_ref = orc.draft_block(cfg, W, caches2, gamma, uniforms.astype(np.float64))
        for b in range(batch):
            for j in range(gamma):
                if toks_ref[b, j] != toks[b, j]:
                    c = np.cumsum(probs_ref[b, j])
                    t = float(uniforms[j, b])
                    edge = np.abs(c - t).min()
                    tau = a_tol + r_tol * 8.0
                    assert edge < np.exp(2 * tau) - 1, f"draft token {b},{j} differs away from a CDF edge ({edge:.3e})"
                    break                                                          # later tokens follow a different prefix
    finally:
        gpu.close()


def test_speculate_then_verify_cycle_with_identical_models():
    """Draft model = target model: q equals p up to kernel-shape rounding, so with uniforms kept below 0.9 the
    ratio test alone accepts all gamma tokens; afterwards both caches hold the same accepted prefix."""
    gamma, batch = 5, 2
    shape = dataclasses.replace(SMALL, name="cycle", batch=batch, gamma=gamma)
    src = synth.WeightSource(shape, seed=9, norm_jitter=0.1)
    lens = [50, 91]
    cap = [l + gamma + 20 for l in lens]
    target = G.Gpu(shape, src, cap)
    draft_kv = sj.sj_kv_create(target.model, batch, cap)            # the same weights with a cache of their own
    try:
        cfg = helpers.oracle_config(shape)
        caches = _fill_caches(shape, target, cfg, lens, seed=12, capacity=cap)
        for b in range(batch):
            for l in range(shape.n_layers):
                k, v = synth.make_kv_cache(shape, 12, b, l, lens[b])
                sj.sj_kv_set_layer(draft_kv, b, l, k, v, lens[b])
            sj.sj_kv_set_state(draft_kv, b, lens[b], caches[b].pending)
        dev = target.dev
        rng = np.random.default_rng(3)
        un_d = torch.from_numpy((0.9 * rng.random((gamma, batch))).astype(np.float32)).to(dev)
        un_v = torch.from_numpy((0.9 * rng.random((batch, gamma + 1))).astype(np.float32)).to(dev)
        toks = torch.zeros((batch, gamma), dtype=torch.int32, device=dev)
        probs = torch.zeros((batch, gamma, shape.vocab), dtype=torch.float32, device=dev)
        acc = torch.zeros((batch,), dtype=torch.int32, device=dev)
        nxt = torch.zeros((batch,), dtype=torch.int32, device=dev)
        st = torch.cuda.current_stream()
        sj.sj_set_mode(target.kv, 1)                                  # alignment test only (Eq. 3)
        sj.sj_draft_block(target.model, draft_kv, gamma, un_d, True, toks, probs, st)
        sj.sj_verify_step(target.model, target.kv, gamma, toks, probs, un_v, 0.5, acc, nxt, st)
        torch.cuda.synchronize()
        assert (acc.cpu().numpy() == gamma).all()
        ln_t, pend_t = sj.sj_kv_state(target.kv, batch)
        assert (ln_t == np.array(lens) + 1 + gamma).all()
        for b in range(batch):
            sj.sj_kv_set_state(draft_kv, b, int(ln_t[b]), int(pend_t[b]))      # keep the accepted prefix
        ln_d, pend_d = sj.sj_kv_state(draft_kv, batch)
        assert (ln_d == ln_t).all() and (pend_d == pend_t).all()
        dt = np.uint16
        for b in range(batch):
            n = gamma + 1
            kt = np.empty((shape.n_kv_heads, n, shape.head_dim), dt); vt = np.empty_like(kt)
            kd = np.empty_like(kt); vd = np.empty_like(kt)
            sj.sj_kv_read(target.kv, b, shape.n_layers - 1, lens[b], n, kt, vt)
            sj.sj_kv_read(draft_kv, b, shape.n_layers - 1, lens[b], n, kd, vd)
            G.close_enough(synth.to_f64(kd), synth.to_f64(kt), "bf16", f"accepted K rows seq {b}")
            G.close_enough(synth.to_f64(vd), synth.to_f64(vt), "bf16", f"accepted V rows seq {b}")
    finally:
        sj.sj_kv_free(draft_kv)
        target.close()


def test_draft_block_argument_errors():
    shape = dataclasses.replace(SMALL, name="draft_err", batch=1, gamma=2, n_layers=1)
    src = synth.WeightSource(shape, seed=1)
    gpu = G.Gpu(shape, src, [64])
    try:
        dev = gpu.dev
        un = torch.zeros((70, 1), dtype=torch.float32, device=dev)
        toks = torch.zeros((1, 70), dtype=torch.int32, device=dev)
        probs = torch.zeros((1, 2, shape.vocab), dtype=torch.float32, device=dev)
        with pytest.raises(sj.SJError):
            sj.sj_draft_block(gpu.model, gpu.kv, 0, un, True, toks, probs)
        with pytest.raises(sj.SJError):
            sj.sj_draft_block(gpu.model, gpu.kv, 2, None, True, toks, probs)
        sj.sj_kv_set_state(gpu.kv, 0, 62, 3)                          # 62 + 2 + 1 rows do not fit 64
        with pytest.raises(sj.SJError):
            sj.sj_draft_block(gpu.model, gpu.kv, 2, un, True, toks, probs)
    finally:
        gpu.close()
