"""GPU parity of teacher-forced scoring and the semantic preservation score built from it (Sec. 3.3,
Eq. 6 - 7): two passes of N + 1 rows on the same cache, log-probabilities gathered at the given targets."""
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


def _score(gpu, inputs, targets, hidden_row=None):
    B, n = inputs.shape
    dev = gpu.dev
    it = torch.from_numpy(np.ascontiguousarray(inputs.astype(np.int32))).to(dev)
    tt = torch.from_numpy(np.ascontiguousarray(targets.astype(np.int32))).to(dev)
    lp = torch.full((B, n), 7.0, dtype=torch.float32, device=dev)
    hz = torch.zeros((B, gpu.shape.d_model), dtype=torch.float32, device=dev) if hidden_row is not None else None
    sj.sj_score_block(gpu.model, gpu.kv, n, it, tt, lp, hidden_row or 0, hz, torch.cuda.current_stream())
    torch.cuda.synchronize()
    return lp.cpu().numpy().astype(np.float64), (hz.cpu().numpy() if hz is not None else None)


@pytest.mark.parametrize("dtype,N", [("bf16", 20), ("fp32", 7)])
def test_semantic_preservation_score_matches_oracle(dtype, N):
    """A batch of mismatch positions of one response: every sequence of the batch is the same response cut at a
    different position i (its own cache length), scored with N future tokens (the paper uses N = 20)."""
    batch = 3
    shape = dataclasses.replace(SMALL, name=f"score_{dtype}", dtype=dtype, batch=batch, gamma=N)      # rows per pass: N + 1
    src = synth.WeightSource(shape, seed=13, norm_jitter=0.1)
    lens = [30, 75, 131]
    cap = [l + N + 8 for l in lens]
    gpu = G.Gpu(shape, src, cap)
    try:
        cfg = helpers.oracle_config(shape)
        W = helpers.oracle_weights(src)
        caches = _fill_caches(shape, gpu, cfg, lens, seed=14, capacity=cap)
        rng = np.random.default_rng(15)
        y_next = rng.integers(0, shape.vocab, (batch, N + 1))
        z = (y_next[:, 0] + 1 + rng.integers(0, shape.vocab - 1, batch)) % shape.vocab
        pend = np.array([c.pending for c in caches])
        ins_y = np.concatenate([pend[:, None], y_next[:, :-1]], axis=1)
        ins_z = ins_y.copy(); ins_z[:, 1] = z
        tg_y = y_next.copy()
        tg_z = y_next.copy(); tg_z[:, 0] = z
        lp_y, _ = _score(gpu, ins_y, tg_y)
        lp_z, hz = _score(gpu, ins_z, tg_z, hidden_row=1)
        ln, pd = sj.sj_kv_state(gpu.kv, batch)
        assert (ln == np.array(lens)).all() and (pd == pend).all()              # scoring leaves the state alone
        a_tol, r_tol = G.TOL[dtype]
        tau = 0.0
        for b in range(batch):
            ref = orc.semantic_preservation(cfg, W, caches[b], y_next[b], int(z[b]), tau)
            # a log-probability is a logit minus a log-sum-exp of logits: twice the logit tolerance
            bound_row = 2 * (a_tol + r_tol * 8.0)
            assert np.abs(lp_y[b] - ref["logprob_y"]).max() <= bound_row, np.abs(lp_y[b] - ref["logprob_y"]).max()
            assert np.abs(lp_z[b] - ref["logprob_z"]).max() <= bound_row
            s_dev = float(lp_z[b].sum() - lp_y[b].sum())
            assert abs(s_dev - ref["s"]) <= 2 * (N + 1) * bound_row
            print(f"{dtype} seq {b}: s = {s_dev:.5f} (oracle {ref['s']:.5f}), max row err "
                  f"{max(np.abs(lp_y[b] - ref['logprob_y']).max(), np.abs(lp_z[b] - ref['logprob_z']).max()):.2e}", flush=True)
            if abs(ref["s"] - tau) > 2 * (N + 1) * bound_row:
                assert (s_dev > tau) == ref["label"]
            G.close_enough(hz[b], ref["h_z"], dtype, f"h_z seq {b}")
    finally:
        gpu.close()


def test_score_block_argument_errors_and_one_row():
    shape = dataclasses.replace(SMALL, name="score_err", batch=1, gamma=3, n_layers=1)
    src = synth.WeightSource(shape, seed=1)
    gpu = G.Gpu(shape, src, [64])
    try:
        cfg = helpers.oracle_config(shape)
        W = helpers.oracle_weights(src)
        caches = _fill_caches(shape, gpu, cfg, [10], seed=2, capacity=[64])
        dev = gpu.dev
        it = torch.zeros((1, 8), dtype=torch.int32, device=dev)
        lp = torch.zeros((1, 8), dtype=torch.float32, device=dev)
        with pytest.raises(sj.SJError):
            sj.sj_score_block(gpu.model, gpu.kv, 0, it, it, lp)
        with pytest.raises(sj.SJError):
            sj.sj_score_block(gpu.model, gpu.kv, 5, it, it, lp)                  # more rows than max_gamma + 1
        with pytest.raises(sj.SJError):
            sj.sj_score_block(gpu.model, gpu.kv, 2, it, None, lp)
        with pytest.raises(sj.SJError):
            sj.sj_score_block(gpu.model, gpu.kv, 2, it, it, lp, 2, torch.zeros((1, shape.d_model), device=dev))
        # one row = the prefix-only score: log p(target) of the pending token's row
        ins = np.array([[caches[0].pending]]); tg = np.array([[123]])
        got, _ = _score(gpu, ins, tg)
        ref = orc.score_block(cfg, W, caches, ins, tg)[0]["logprob"]
        assert abs(got[0, 0] - ref[0]) < 2 * (1e-2 + 2e-2 * 8.0)
    finally:
        gpu.close()
