"""The allocation-free variant of the verification tail (static device workspace) against the ordinary entry
point on the same inputs: two calls in a row, the second smaller, then a shape that does not fit."""
import dataclasses

import numpy as np
import pytest
import torch

import paper_2510_02329_amd as sj
import synth
from tests import gpu_common as G

pytestmark = pytest.mark.gpu


def _inputs(shape, seed, dev):
    hidden = synth.make_hidden(shape, seed=seed)                       # [R, d] storage-type bits
    draft = synth.make_draft(shape, seed=seed)
    return (torch.from_numpy(hidden.view(np.int16)).to(dev), draft,
            torch.from_numpy(np.ascontiguousarray(draft["tokens"])).to(dev),
            torch.from_numpy(np.ascontiguousarray(draft["probs"])).to(dev),
            torch.from_numpy(np.ascontiguousarray(draft["uniforms"])).to(dev))


def test_static_workspace_head_matches_the_allocating_entry_point():
    base = dataclasses.replace(synth.CONFIGS[1], name="head_small", d_model=1024, vocab=32768)
    src = synth.WeightSource(base, seed=5, judge_bias=0.1)
    model = G.load_model(dataclasses.replace(base, batch=2, gamma=7), src, max_gamma=7)
    dev = torch.device("cuda:0")
    stream = torch.cuda.current_stream()
    try:
        for batch, gamma, seed, theta in ((2, 7, 11, 0.5), (1, 3, 12, 0.38)):     # the second call is smaller
            shape = dataclasses.replace(base, batch=batch, gamma=gamma)
            hid, draft, dt, dp, un = _inputs(shape, seed, dev)
            kv = sj.sj_kv_create(model, batch, None)
            ref_acc = torch.full((batch,), -7, dtype=torch.int32, device=dev)
            ref_nxt = torch.full((batch,), -7, dtype=torch.int32, device=dev)
            sj.sj_verify_head(model, kv, gamma, hid, dt, dp, un, theta, ref_acc, ref_nxt, stream)
            acc = torch.full((batch,), -9, dtype=torch.int32, device=dev)
            nxt = torch.full((batch,), -9, dtype=torch.int32, device=dev)
            sj.sj_verify_head_static(model, batch, gamma, hid, dt, dp, un, theta, acc, nxt, stream)
            torch.cuda.synchronize()
            sj.sj_kv_free(kv)
            print("static head", batch, gamma, acc.tolist(), nxt.tolist(), flush=True)
            assert acc.tolist() == ref_acc.tolist()                 # decisions and tokens: bit-exact
            assert nxt.tolist() == ref_nxt.tolist()
            assert all(0 <= a <= gamma for a in acc.tolist()) and all(0 <= t < base.vocab for t in nxt.tolist())
        # a request beyond the static workspace is refused before anything is launched
        big = dataclasses.replace(base, batch=5, gamma=7)
        hid, draft, dt, dp, un = _inputs(big, 13, dev)
        acc = torch.zeros(5, dtype=torch.int32, device=dev)
        with pytest.raises(sj.SJError):
            sj.sj_verify_head_static(model, 5, 7, hid, dt, dp, un, 0.5, acc, acc.clone(), stream)     # 40 rows > 32
    finally:
        sj.sj_model_free(model)
