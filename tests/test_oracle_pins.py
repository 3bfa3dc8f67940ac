"""Pins for the CPU oracle: each test checks it against something the paper or the
mathematics fixes, not against itself.  The paper prints no worked numeric example, so there are
no golden values from it; pins are closed forms, invariants, exhaustive enumeration and library
cross-checks.  CPU only."""
from fractions import Fraction

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import synth
from oracle import selfjudge_oracle as orc
from tests import helpers

TINY = synth.ModelShape("pin", "fp32", 2, 32, 4, 2, 8, 48, 64, 10000.0, batch=1, gamma=4)


def _tiny(seed=0, **kw):
    cfg = helpers.oracle_config(TINY.scaled(**kw) if kw else TINY)
    shape = TINY.scaled(**kw) if kw else TINY
    return shape, cfg, helpers.random_model(shape, seed)


# ------------------------------------------------------------------ P1: greedy reduction
# Target temperature 0 (the paper's setting, Sec. 4.1 "Implementation Details") with the judge
# off must reduce to strict speculative sampling (Sec. 3.1): accept while draft == target arg-max.


@pytest.mark.parametrize("seed", range(20))
def test_greedy_reduction(seed):
    rng = np.random.default_rng(seed)
    gamma, V = 6, 17
    logits = rng.standard_normal((gamma + 1, V))
    greedy = logits.argmax(axis=1)
    drafts = greedy[:gamma].copy()
    n_match = int(rng.integers(0, gamma + 1))
    if n_match < gamma:
        drafts[n_match] = (drafts[n_match] + 1 + rng.integers(0, V - 1)) % V
        for j in range(n_match + 1, gamma):          # whatever follows must not matter
            drafts[j] = rng.integers(0, V)
    q = rng.dirichlet(np.ones(V), size=gamma)
    u = rng.random(gamma + 1)
    res = orc.verify_tail(logits, np.zeros(gamma), drafts, q, u, theta=1.0, temperature=0.0)
    assert res["accepted_len"] == n_match
    assert res["next_token"] == greedy[n_match]


def test_temperature_zero_lowest_index_tie():
    p = orc.target_distribution(np.array([0.5, 2.0, 2.0, -1.0]), 0.0)
    assert p.tolist() == [0.0, 1.0, 0.0, 0.0]


# ------------------------------------------------------------------ P3: exact law of the emitted token
# Standard speculative sampling reproduces the target distribution (Sec. 1, Sec. 2.2, Sec. 3.1).
# gamma = 1, judge off: the token at the first new position is d if accepted, else the resampled
# one.  Enumerate every d (weight q(d)) and a midpoint grid of the uniforms whose size is a
# multiple of every denominator involved: the counts are then exact integers.


def _law_of_first_token(p8, q8, p2_8):
    V = len(p8)
    p = np.array(p8, float) / 8
    q = np.array(q8, float) / 8
    p2 = np.array(p2_8, float) / 8
    with np.errstate(divide="ignore"):
        logits = np.log(np.stack([p, p2]))            # softmax(log p) = p; -inf -> probability 0
    N = 840 * 8                                       # multiple of every integer <= 8
    grid = (np.arange(N) + 0.5) / N
    law = [Fraction(0)] * V
    bonus_law = [Fraction(0)] * V
    for d in range(V):
        if q8[d] == 0:
            continue
        wd = Fraction(q8[d], 8)
        acc = 0
        for u1 in grid:
            r = orc.verify_tail(logits, np.zeros(1), [d], q[None], [u1, 0.3], 1.0, 1.0)
            acc += r["accepted_len"]
        p_acc = Fraction(acc, N)
        law[d] += wd * p_acc
        # outcome of the second uniform; accept depends on u1 only, the draw on u2 only
        u_rej = None if acc == N else grid[-1]
        u_acc = None if acc == 0 else grid[0]
        if u_rej is not None:
            cnt = [0] * V
            for u2 in grid:
                r = orc.verify_tail(logits, np.zeros(1), [d], q[None], [u_rej, u2], 1.0, 1.0)
                assert r["accepted_len"] == 0
                cnt[r["next_token"]] += 1
            for k in range(V):
                law[k] += wd * (1 - p_acc) * Fraction(cnt[k], N)
        if u_acc is not None:
            cnt = [0] * V
            for u2 in grid:
                r = orc.verify_tail(logits, np.zeros(1), [d], q[None], [u_acc, u2], 1.0, 1.0)
                assert r["accepted_len"] == 1
                cnt[r["next_token"]] += 1
            for k in range(V):
                bonus_law[k] += wd * p_acc * Fraction(cnt[k], N)
    return law, bonus_law


@pytest.mark.parametrize("p8,q8", [
    ([1, 3, 0, 4], [2, 1, 4, 1]),        # p has a zero where q has mass
    ([2, 2, 2, 2], [0, 5, 3, 0]),        # q has zeros; non-dyadic ratios 2/5, 2/3
    ([0, 0, 7, 1], [1, 1, 3, 3]),
    ([3, 1, 3, 1], [3, 1, 3, 1]),        # p == q: always accepted
])
def test_emitted_token_law_equals_target(p8, q8):
    p2_8 = [1, 2, 5, 0]
    law, bonus = _law_of_first_token(p8, q8, p2_8)
    assert law == [Fraction(x, 8) for x in p8]
    # closed form: acceptance mass beta = sum_k min(p_k, q_k); the bonus token follows p_{t+2}
    beta = sum(Fraction(min(a, b), 8) for a, b in zip(p8, q8))
    assert sum(bonus) == beta
    assert bonus == [beta * Fraction(x, 8) for x in p2_8]


def test_ratio_rule_edge_cases():
    # Eq. 3 with u in [0,1): q = 0 < p accepts for every u; p = 0 rejects for every u.
    for u in (0.0, 0.5, 0.999999):
        assert orc.alignment_accepts(u, 0.0, 0.25)
        assert not orc.alignment_accepts(u, 0.25, 0.0)
        assert not orc.alignment_accepts(u, 0.0, 0.0)
        assert orc.alignment_accepts(u, 0.25, 0.25) == (u < 1.0)
        assert orc.alignment_accepts(u, 0.5, 0.25) == (u < 0.5)


# ------------------------------------------------------------------ P4: range / monotonicity / modes


@pytest.mark.parametrize("seed", range(30))
def test_accept_invariants(seed):
    rng = np.random.default_rng(100 + seed)
    gamma, V = int(rng.integers(1, 9)), 23
    logits = 2 * rng.standard_normal((gamma + 1, V))
    q = rng.dirichlet(np.ones(V) * 0.3, size=gamma)
    drafts = [int(rng.choice(V, p=q[j])) for j in range(gamma)]
    u = rng.random(gamma + 1)
    scores = rng.random(gamma)

    def run(theta, mode="two_stage"):
        return orc.verify_tail(logits, scores, drafts, q, u, theta, 1.0, mode)

    sd = run(1.0)
    assert sd["accepted_len"] == run(0.3, "alignment")["accepted_len"]      # judge off == standard SD
    assert run(-1.0)["accepted_len"] == gamma                                  # judge accepts everything
    prev = gamma
    for theta in np.linspace(-0.1, 1.0, 23):
        r = run(float(theta))
        assert 0 <= r["accepted_len"] <= gamma
        assert 0 <= r["next_token"] < V
        assert r["accepted_len"] <= prev                                       # non-increasing in theta
        prev = r["accepted_len"]
        two, ali, jud = r, run(float(theta), "alignment"), run(float(theta), "judge")
        assert two["accepted_len"] >= max(ali["accepted_len"], jud["accepted_len"])
        # a token is kept iff either verifier approves (App. D.2)
        ok = [a or g for a, g in zip(two["align_bits"], two["judge_bits"])]
        assert two["accepted_len"] == (ok + [False]).index(False)
        assert two["judge_bits"] == [bool(s > theta) for s in scores]


# ------------------------------------------------------------------ P6: softmax / residual / sigmoid identities


@pytest.mark.parametrize("T", [0.5, 1.0, 2.0])
def test_softmax_and_residual_identities(T):
    rng = np.random.default_rng(7)
    V = 101
    logits = 3 * rng.standard_normal(V)
    p = orc.target_distribution(logits, T)
    assert abs(p.sum() - 1) < 1e-14 and (p > 0).all()
    # shift invariance and the closed form exp(l/T)/sum
    assert np.allclose(p, orc.target_distribution(logits + 5.0, T), rtol=1e-13)
    assert np.allclose(p, np.exp(logits / T) / np.exp(logits / T).sum(), rtol=1e-12)
    q = rng.dirichlet(np.ones(V))
    beta = np.minimum(p, q).sum()
    assert abs(np.maximum(0, p - q).sum() - (1 - beta)) < 1e-14
    assert abs(np.maximum(0, q - p).sum() - (1 - beta)) < 1e-14


def test_draw_is_inverse_cdf():
    w = np.array([0.0, 2.0, 0.0, 1.0, 1.0, 0.0])
    # cells: token 1 on [0, .5), token 3 on [.5, .75), token 4 on [.75, 1)
    assert [orc.draw(w, u) for u in (0.0, 0.49, 0.5, 0.74, 0.75, 0.999)] == [1, 1, 3, 3, 4, 4]
    # zero-weight tokens are never drawn, whatever u
    assert all(orc.draw(w, u) in (1, 3, 4) for u in np.linspace(0, 0.999999, 97))
    # unnormalised weights give the same draw
    assert all(orc.draw(w, u) == orc.draw(7 * w, u) for u in np.linspace(0, 0.99, 50))


def test_residual_used_on_rejection_and_bonus_on_full_accept():
    V, gamma = 5, 2
    p = np.array([[.1, .2, .3, .4, 0], [.2, .2, .2, .2, .2], [0, 0, 0, 0, 1.0]])
    with np.errstate(divide="ignore"):
        logits = np.log(p)
    q = np.array([[.4, .1, .1, .4, 0], [.6, .1, .1, .1, .1]])
    # reject d_1 = 0 (p/q = .25 < u): residual of row 0 = norm([0,.1,.2,0,0]) -> tokens 1 | 2
    r = orc.verify_tail(logits, np.zeros(2), [0, 1], q, [0.9, 0.0, 0.30], 1.0, 1.0)
    assert (r["accepted_len"], r["next_token"]) == (0, 1)
    r = orc.verify_tail(logits, np.zeros(2), [0, 1], q, [0.9, 0.0, 0.34], 1.0, 1.0)
    assert (r["accepted_len"], r["next_token"]) == (0, 2)
    # accept d_1 = 3 (p = q), reject d_2 = 0 (p/q = 1/3): residual of row 1 = [0,.1,.1,.1,.1]
    r = orc.verify_tail(logits, np.zeros(2), [3, 0], q, [0.5, 0.5, 0.6], 1.0, 1.0)
    assert (r["accepted_len"], r["next_token"]) == (1, 3)
    # accept both -> bonus from row gamma (one-hot at 4)
    r = orc.verify_tail(logits, np.zeros(2), [3, 0], q, [0.5, 0.1, 0.6], 1.0, 1.0)
    assert (r["accepted_len"], r["next_token"]) == (2, 4)
    # judge rescues the rejected d_2; judge index j-1 belongs to d_j
    r = orc.verify_tail(logits, np.array([0.0, 0.9]), [3, 0], q, [0.5, 0.5, 0.6], 0.5, 1.0)
    assert r["accepted_len"] == 2
    r = orc.verify_tail(logits, np.array([0.9, 0.0]), [3, 0], q, [0.5, 0.5, 0.6], 0.5, 1.0)
    assert r["accepted_len"] == 1


def test_judge_sigmoid_threshold_equivalence():
    rng = np.random.default_rng(3)
    w, h = rng.standard_normal(16), rng.standard_normal(16)
    for b in (-1.0, 0.0, 2.0):
        z = float(w @ h + b)
        s = orc.judge_score(w, b, h)
        assert 0 < s < 1 and abs(np.log(s / (1 - s)) - z) < 1e-12
        for theta in (0.28, 0.38, 0.5):                         # thresholds of Table 2
            assert (s > theta) == (z > np.log(theta / (1 - theta)))
    assert orc.judge_score(w, 0.0, np.zeros(16)) == 0.5


# ------------------------------------------------------------------ P7: special cases of the model pieces


def test_rotary_special_cases():
    rng = np.random.default_rng(0)
    x = rng.standard_normal(16)
    assert np.array_equal(orc.rotary(x, 0, 10000.0), x)                      # position 0: identity
    y = orc.rotary(x, 37, 10000.0)
    assert abs(np.linalg.norm(y) - np.linalg.norm(x)) < 1e-13               # a rotation
    # head_dim 2: one plane, frequency base^0 = 1 -> plain rotation by `pos` radians
    v = orc.rotary(np.array([1.0, 0.0]), 1, 500000.0)
    assert np.allclose(v, [np.cos(1.0), np.sin(1.0)], atol=1e-15)
    # pairing is (i, i + hd/2) with frequency base^(-2i/hd): complex form
    hd, pos, base = 16, 11, 500000.0
    z = x[:hd // 2] + 1j * x[hd // 2:]
    zr = z * np.exp(1j * pos * base ** (-np.arange(hd // 2) / (hd // 2)))
    assert np.allclose(orc.rotary(x, pos, base), np.concatenate([zr.real, zr.imag]), atol=1e-13)
    # relative-position property: <R_m q, R_n k> depends on m - n only
    q, k = rng.standard_normal(16), rng.standard_normal(16)
    a = orc.rotary(q, 9, base) @ orc.rotary(k, 4, base)
    b = orc.rotary(q, 105, base) @ orc.rotary(k, 100, base)
    assert abs(a - b) < 1e-12


def test_rmsnorm_special_cases():
    x = np.array([[3.0, -3.0, 3.0, -3.0]])
    assert np.allclose(orc.rmsnorm(x / 3, np.ones(4), 0.0), x / 3)          # unit RMS, gain 1: identity
    assert np.allclose(orc.rmsnorm(x, np.array([1, 2, 3, 4.0]), 0.0), [[1, -2, 3, -4]])
    assert np.allclose(orc.rmsnorm(x, np.ones(4), 7.0), x / 4.0)            # eps inside the root: sqrt(9+7)


def test_zero_output_projections_reduce_to_embedding_readout():
    shape, cfg, t = _tiny(1)
    for l in range(cfg.n_layers):
        t[("wo", l)] = np.zeros_like(t[("wo", l)])
        t[("w_down", l)] = np.zeros_like(t[("w_down", l)])
    W = helpers.dict_weights(t)
    cache = helpers.random_cache(cfg, 5, 16, seed=2)
    toks = [3, 9, 27]
    out = orc.block_forward(cfg, W, [cache], [toks])[0]
    for j, tok in enumerate(toks):
        e = t[("embed", -1)][tok]
        hn = e / np.sqrt((e * e).mean() + cfg.rms_eps) * t[("final_norm", -1)]
        assert np.allclose(out["logits"][j], t[("lm_head", -1)] @ hn, atol=1e-12)


# ------------------------------------------------------------------ P2: block verify == sequential decode


@pytest.mark.parametrize("seed", [0, 1])
def test_block_equals_sequential(seed):
    shape, cfg, t = _tiny(seed)
    W = helpers.dict_weights(t)
    L, n = 7, 5
    toks = [int(x) for x in np.random.default_rng(seed).integers(0, cfg.vocab, n)]
    blk_cache = helpers.random_cache(cfg, L, 16, seed=5)
    seq_cache = helpers.random_cache(cfg, L, 16, seed=5)
    blk = orc.block_forward(cfg, W, [blk_cache], [toks])[0]
    for j, tok in enumerate(toks):
        one = orc.block_forward(cfg, W, [seq_cache], [[tok]])[0]
        seq_cache.length += 1
        assert np.allclose(one["logits"][0], blk["logits"][j], atol=1e-11, rtol=1e-11)
        assert np.allclose(one["hn"][0], blk["hn"][j], atol=1e-11, rtol=1e-11)
    for l in range(cfg.n_layers):
        assert np.allclose(seq_cache.k[l][:, :L + n], blk_cache.k[l][:, :L + n], atol=1e-12)
        assert np.allclose(seq_cache.v[l][:, :L + n], blk_cache.v[l][:, :L + n], atol=1e-12)
    assert blk_cache.length == L                                             # forward does not commit


def test_batch_rows_are_independent():
    shape, cfg, t = _tiny(3)
    W = helpers.dict_weights(t)
    ca, cb = helpers.random_cache(cfg, 4, 16, 11), helpers.random_cache(cfg, 9, 16, 12)
    both = orc.block_forward(cfg, W, [ca, cb], [[1, 2, 3], [4, 5]])
    ca2, cb2 = helpers.random_cache(cfg, 4, 16, 11), helpers.random_cache(cfg, 9, 16, 12)
    a = orc.block_forward(cfg, W, [ca2], [[1, 2, 3]])[0]
    b = orc.block_forward(cfg, W, [cb2], [[4, 5]])[0]
    assert np.allclose(both[0]["logits"], a["logits"], atol=1e-12)
    assert np.allclose(both[1]["logits"], b["logits"], atol=1e-12)


def test_storage_rounding_matches_library_and_ties_to_even():
    rng = np.random.default_rng(1)
    a32 = (rng.standard_normal(50000) * 10 ** rng.uniform(-4, 4, 50000)).astype(np.float32)
    got = orc.round_to_storage(a32.astype(np.float64), "bf16")
    ref = torch.from_numpy(a32).to(torch.bfloat16).double().numpy()       # fp32 inputs: no double rounding
    assert np.array_equal(got, ref)
    assert orc.round_to_storage(np.array([1 + 2.0 ** -8]), "bf16")[0] == 1.0              # tie -> even
    assert orc.round_to_storage(np.array([1 + 3 * 2.0 ** -8]), "bf16")[0] == 1 + 2.0 ** -6
    assert orc.round_to_storage(np.array([1 + 2.0 ** -8 + 2.0 ** -40]), "bf16")[0] == 1 + 2.0 ** -7
    assert orc.round_to_storage(np.array([-0.3]), "bf16")[0] == -0.30078125
    x = rng.standard_normal(1000)
    assert np.array_equal(orc.round_to_storage(x, "fp32"), x.astype(np.float32).astype(np.float64))
    assert np.array_equal(orc.round_to_storage(x, "fp64"), x)


@pytest.mark.parametrize("storage", ["bf16", "fp32"])
def test_block_equals_sequential_on_stored_cache(storage):
    """With a bf16 / fp32 cache the block's own rows are read back as stored, so the block forward
    still equals token-by-token decoding exactly (no tolerance beyond fp64 summation order)."""
    shape, cfg, t = _tiny(2)
    W = helpers.dict_weights(t)
    L, toks = 9, [3, 1, 4, 1, 5]
    def mk():
        c = helpers.random_cache(cfg, L, 24, seed=7)
        c.storage = storage
        for l in range(cfg.n_layers):
            c.k[l][:] = orc.round_to_storage(c.k[l], storage)
            c.v[l][:] = orc.round_to_storage(c.v[l], storage)
        return c
    cb, cs = mk(), mk()
    blk = orc.block_forward(cfg, W, [cb], [toks])[0]
    for j, tok in enumerate(toks):
        one = orc.block_forward(cfg, W, [cs], [[tok]])[0]
        cs.length += 1
        assert np.allclose(one["logits"][0], blk["logits"][j], atol=1e-11, rtol=1e-11)
    for l in range(cfg.n_layers):
        assert np.array_equal(cs.k[l][:, :L + 5], cb.k[l][:, :L + 5])
        assert np.array_equal(cb.k[l][:, L:L + 5], orc.round_to_storage(cb.k[l][:, L:L + 5], storage))
    # and the stored rows differ from what an unrounded cache would hold
    cu = helpers.random_cache(cfg, L, 24, seed=7)
    for l in range(cfg.n_layers):
        cu.k[l][:] = orc.round_to_storage(cu.k[l], storage); cu.v[l][:] = orc.round_to_storage(cu.v[l], storage)
    orc.block_forward(cfg, W, [cu], [toks])
    assert not np.array_equal(cu.k[0][:, L:L + 5], cb.k[0][:, L:L + 5])


# ------------------------------------------------------------------ P5: library cross-check of the decoder


def _torch_forward(cfg, t, cache, toks):
    """The same decoder block written with torch library ops (float64): embedding, rms_norm,
    linear, complex-multiply rotary, scaled_dot_product_attention with an explicit mask, silu."""
    dd = torch.float64
    T = lambda a: torch.tensor(np.asarray(a), dtype=dd)
    L, n = cache.length, len(toks)
    Hq, Hkv, hd = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    x = F.embedding(torch.tensor(toks), T(t[("embed", -1)]))
    pos = torch.arange(L, L + n, dtype=dd)
    freqs = cfg.rope_base ** (-torch.arange(0, hd, 2, dtype=dd) / hd)
    rot = torch.polar(torch.ones(n, hd // 2, dtype=dd), pos[:, None] * freqs[None, :])   # e^{i pos f}

    def rope(v):                                   # v [n, H, hd]; pairs (i, i+hd/2) as complex numbers
        z = torch.complex(v[..., :hd // 2], v[..., hd // 2:]) * rot[:, None, :]
        return torch.cat([z.real, z.imag], dim=-1)

    mask = torch.zeros(n, L + n, dtype=torch.bool)
    for j in range(n):
        mask[j, :L + j + 1] = True
    for l in range(cfg.n_layers):
        a = F.rms_norm(x, (cfg.d_model,), T(t[("attn_norm", l)]), cfg.rms_eps)
        q = rope(F.linear(a, T(t[("wq", l)])).view(n, Hq, hd))
        k = rope(F.linear(a, T(t[("wk", l)])).view(n, Hkv, hd))
        v = F.linear(a, T(t[("wv", l)])).view(n, Hkv, hd)
        K = torch.cat([T(cache.k[l][:, :L]), k.transpose(0, 1)], dim=1)     # [Hkv, L+n, hd]
        Vv = torch.cat([T(cache.v[l][:, :L]), v.transpose(0, 1)], dim=1)
        K = K.repeat_interleave(Hq // Hkv, dim=0)
        Vv = Vv.repeat_interleave(Hq // Hkv, dim=0)
        o = F.scaled_dot_product_attention(q.transpose(0, 1)[None], K[None], Vv[None],
                                           attn_mask=mask[None, None])[0]   # [Hq, n, hd]
        x = x + F.linear(o.transpose(0, 1).reshape(n, Hq * hd), T(t[("wo", l)]))
        f = F.rms_norm(x, (cfg.d_model,), T(t[("ffn_norm", l)]), cfg.rms_eps)
        x = x + F.linear(F.silu(F.linear(f, T(t[("w_gate", l)]))) * F.linear(f, T(t[("w_up", l)])),
                         T(t[("w_down", l)]))
    hn = F.rms_norm(x, (cfg.d_model,), T(t[("final_norm", -1)]), cfg.rms_eps)
    return F.linear(hn, T(t[("lm_head", -1)])).numpy(), hn.numpy()


@pytest.mark.parametrize("seed,base", [(0, 10000.0), (1, 500000.0)])
def test_forward_matches_torch_library_ops(seed, base):
    shape, cfg, t = _tiny(seed, rope_base=base)
    W = helpers.dict_weights(t)
    cache = helpers.random_cache(cfg, 11, 24, seed=seed + 40)
    toks = [5, 0, 63, 17, 17, 2]
    logits_t, hn_t = _torch_forward(cfg, t, cache, toks)
    out = orc.block_forward(cfg, W, [cache], [toks])[0]
    assert np.allclose(out["logits"], logits_t, atol=1e-10, rtol=1e-10)
    assert np.allclose(out["hn"], hn_t, atol=1e-10, rtol=1e-10)


# ------------------------------------------------------------------ whole step: state update (R8)


def test_verify_step_commits_length_and_pending():
    shape, cfg, t = _tiny(4)
    W = helpers.dict_weights(t)
    cache = helpers.random_cache(cfg, 6, 32, seed=9)
    rng = np.random.default_rng(0)
    gamma = 4
    q = rng.dirichlet(np.ones(cfg.vocab), size=(1, gamma))
    d = np.array([[int(rng.choice(cfg.vocab, p=q[0, j])) for j in range(gamma)]])
    u = rng.random((1, gamma + 1))
    pend0 = cache.pending
    res = orc.verify_step(cfg, W, [cache], d, q, u, theta=0.5)[0]
    n = res["accepted_len"]
    assert cache.length == 6 + 1 + n and cache.pending == res["next_token"]
    # the block fed [pending, d_1..d_gamma]: its K rows are now cache rows 6..6+gamma
    c2 = helpers.random_cache(cfg, 6, 32, seed=9)
    fw = orc.block_forward(cfg, W, [c2], [[pend0] + d[0].tolist()])[0]
    assert np.allclose(fw["logits"], res["logits"])
    assert np.allclose(c2.k[0][:, 6:6 + gamma + 1], res["k_new"][0])
    # the judge reads rows 1..gamma (inputs d_1..d_gamma), not row 0
    w = t[("judge_w", -1)]
    expect = 1 / (1 + np.exp(-(fw["hn"][1:] @ w)))
    assert np.allclose(res["judge_scores"], expect, atol=1e-12)


# ------------------------------------------------------------------ prefill (R6, R8)
# Pinned against token-by-token decoding on a cache of its own (the prompt's K / V rows and the last row's logits
# must be those of n sequential single-token steps) and against the tie rule: with two equal largest logits the
# pending token is the lower index.


@pytest.mark.parametrize("seed", [0, 1])
def test_prefill_equals_sequential_decode_and_breaks_ties_low(seed):
    shape, cfg, t = _tiny(seed)
    W = helpers.dict_weights(t)
    rng = np.random.default_rng(seed)
    prompt = [int(x) for x in rng.integers(0, cfg.vocab, size=7)]
    cache = orc.SeqCache(cfg, 16)
    pend = orc.prefill(cfg, W, cache, prompt)
    seq = orc.SeqCache(cfg, 16)
    last = None
    for tok in prompt:                                   # one token at a time, each on top of the rows before it
        last = orc.block_forward(cfg, W, [seq], [[tok]])[0]["logits"][0]
        seq.length += 1
    assert cache.length == len(prompt) == seq.length
    for l in range(cfg.n_layers):
        assert np.allclose(cache.k[l][:, :7], seq.k[l][:, :7], atol=1e-12)
        assert np.allclose(cache.v[l][:, :7], seq.v[l][:, :7], atol=1e-12)
    k = int(np.argmax(last))
    assert pend == k == cache.pending
    # tie: give a lower-index vocabulary entry the same LM-head row as the winner (or a higher one when k = 0)
    t2 = dict(t)
    lm = t[("lm_head", -1)].copy()
    other = k - 1 if k > 0 else k + 1
    lm[other] = lm[k]
    t2[("lm_head", -1)] = lm
    c2 = orc.SeqCache(cfg, 16)
    assert orc.prefill(cfg, helpers.dict_weights(t2), c2, prompt) == min(k, other)
    # all logits equal: index 0
    t3 = dict(t)
    t3[("lm_head", -1)] = np.zeros_like(lm)
    assert orc.prefill(cfg, helpers.dict_weights(t3), orc.SeqCache(cfg, 16), prompt) == 0


# ------------------------------------------------------------------ P8: draft proposal (Eq. 1)
# The draft block is gamma single-token decodes.  Pinned against things it does not compute itself:
# a from-scratch forward of the whole sequence (positions, caching, which token is fed), the verification
# step of an identical target (p = q makes the ratio test of Eq. 3 accept everything), the greedy
# continuation at temperature 0, and the exact law of the first draw.


def _from_scratch_logits(cfg, W, prefix_cache_seed, L, fed):
    """Logits of every fed token when the whole run is one block on a fresh copy of the cache."""
    c = helpers.random_cache(cfg, L, 64, seed=prefix_cache_seed)
    return orc.block_forward(cfg, W, [c], [list(fed)])[0]["logits"]


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_draft_block_rows_equal_from_scratch_forward(seed):
    shape, cfg, t = _tiny(seed)
    W = helpers.dict_weights(t)
    L, gamma = 5, 4
    cache = helpers.random_cache(cfg, L, 64, seed=11)
    pend0 = cache.pending
    u = np.random.default_rng(seed).random((gamma, 1))
    toks, probs = orc.draft_block(cfg, W, [cache], gamma, u, feed_last=True)
    fed = [pend0] + [int(x) for x in toks[0]]                     # the tokens that entered the model, in order
    logits = _from_scratch_logits(cfg, W, 11, L, fed)
    for j in range(gamma):
        z = logits[j] / cfg.temperature
        e = np.exp(z - z.max())
        assert np.allclose(probs[0, j], e / e.sum(), atol=1e-12)   # q_j is the law after j drafted tokens
        assert abs(probs[0, j].sum() - 1.0) < 1e-12
        c = np.cumsum(probs[0, j])                                  # R5: smallest k with cdf > u
        assert c[toks[0, j]] > u[j, 0] * c[-1] and (toks[0, j] == 0 or c[toks[0, j] - 1] <= u[j, 0] * c[-1])
    assert cache.length == L + gamma + 1 and cache.pending == int(toks[0, -1])
    # the cache rows are those of the from-scratch block (all gamma + 1 fed tokens with feed_last)
    c2 = helpers.random_cache(cfg, L, 64, seed=11)
    orc.block_forward(cfg, W, [c2], [fed])
    for l in range(cfg.n_layers):
        assert np.allclose(cache.k[l][:, :L + gamma + 1], c2.k[l][:, :L + gamma + 1], atol=1e-12)
        assert np.allclose(cache.v[l][:, :L + gamma + 1], c2.v[l][:, :L + gamma + 1], atol=1e-12)
    # without feed_last the last drafted token has no row yet
    cache3 = helpers.random_cache(cfg, L, 64, seed=11)
    toks3, _ = orc.draft_block(cfg, W, [cache3], gamma, u, feed_last=False)
    assert (toks3 == toks).all() and cache3.length == L + gamma


@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_identical_draft_and_target_accept_every_token(seed):
    """p = q: u * q < p holds for every u in [0, 1) wherever q > 0, so the alignment test alone keeps all
    gamma tokens, whatever the uniforms (Sec. 2.2: the acceptance rate is sum min(p, q) = 1)."""
    shape, cfg, t = _tiny(seed)
    W = helpers.dict_weights(t)
    L, gamma, B = 6, 5, 2
    rng = np.random.default_rng(100 + seed)
    draft_caches = [helpers.random_cache(cfg, L + b, 64, seed=20 + b) for b in range(B)]
    target_caches = [helpers.random_cache(cfg, L + b, 64, seed=20 + b) for b in range(B)]
    toks, probs = orc.draft_block(cfg, W, draft_caches, gamma, rng.random((gamma, B)), feed_last=True)
    res = orc.verify_step(cfg, W, target_caches, toks, probs, rng.random((B, gamma + 1)), theta=0.5, mode="alignment")
    for b in range(B):
        assert res[b]["accepted_len"] == gamma
        # both caches now describe the same accepted prefix once the draft's is cut to len0 + 1 + n
        assert target_caches[b].length == L + b + 1 + gamma == draft_caches[b].length
        for l in range(cfg.n_layers):
            n = target_caches[b].length
            assert np.allclose(draft_caches[b].k[l][:, :n], target_caches[b].k[l][:, :n], atol=1e-11)


def test_draft_block_is_greedy_at_temperature_zero():
    shape, cfg, t = _tiny(5, temperature=0.0)
    W = helpers.dict_weights(t)
    L, gamma = 4, 5
    cache = helpers.random_cache(cfg, L, 64, seed=31)
    pend0 = cache.pending
    toks, probs = orc.draft_block(cfg, W, [cache], gamma, np.random.default_rng(0).random((gamma, 1)))
    logits = _from_scratch_logits(cfg, W, 31, L, [pend0] + [int(x) for x in toks[0]])
    assert [int(np.argmax(logits[j])) for j in range(gamma)] == [int(x) for x in toks[0]]
    assert all(probs[0, j, toks[0, j]] == 1.0 and probs[0, j].sum() == 1.0 for j in range(gamma))


def test_first_draft_token_follows_q_exactly():
    """Exhaustive over a grid of uniforms (midpoints of N equal cells): the share of the grid that draws token
    k is q_k up to one cell per token."""
    shape, cfg, t = _tiny(7)
    W = helpers.dict_weights(t)
    N = 4000
    counts = np.zeros(cfg.vocab)
    q = None
    for i in range(N):
        cache = helpers.random_cache(cfg, 3, 16, seed=41)
        toks, probs = orc.draft_block(cfg, W, [cache], 1, np.array([[(i + 0.5) / N]]), feed_last=False)
        counts[toks[0, 0]] += 1
        q = probs[0, 0]
    assert np.abs(counts / N - q).max() <= 1.0 / N + 1e-12


# ------------------------------------------------------------------ P9: semantic preservation score (Eq. 6 - 7)
# The score is a difference of joint log-likelihoods of two continuations of the same prefix; the oracle gets
# it from two teacher-forced blocks.  Pinned against the definition evaluated by single-token decodes, the
# trivial replacement, the prefix-only special case and the normalisation of the scored distributions.


def _joint_loglik_sequential(cfg, W, cache_seed, L, pending, tokens):
    """log P(tokens | prefix) by feeding one token at a time and committing the cache (no block forward)."""
    c = helpers.random_cache(cfg, L, 64, seed=cache_seed)
    c.pending = pending
    total = 0.0
    for t in tokens:
        logits = orc.block_forward(cfg, W, [c], [[c.pending]])[0]["logits"][0] / cfg.temperature
        total += logits[t] - (logits.max() + np.log(np.exp(logits - logits.max()).sum()))
        c.length += 1
        c.pending = int(t)
    return float(total)


@pytest.mark.parametrize("seed,N", [(0, 0), (1, 1), (2, 5), (3, 9)])
def test_semantic_preservation_score_is_the_joint_likelihood_difference(seed, N):
    shape, cfg, t = _tiny(seed)
    W = helpers.dict_weights(t)
    rng = np.random.default_rng(50 + seed)
    L = 6
    cache = helpers.random_cache(cfg, L, 64, seed=60)
    y_next = [int(x) for x in rng.integers(0, cfg.vocab, N + 1)]
    z = int((y_next[0] + 1 + rng.integers(0, cfg.vocab - 1)) % cfg.vocab)
    res = orc.semantic_preservation(cfg, W, cache, y_next, z, tau=0.0)
    ll_z = _joint_loglik_sequential(cfg, W, 60, L, cache.pending, [z] + y_next[1:])
    ll_y = _joint_loglik_sequential(cfg, W, 60, L, cache.pending, y_next)
    assert abs(res["s"] - (ll_z - ll_y)) < 1e-9                       # Eq. 6 == Eq. 7
    assert abs(res["s"] - (res["s_prefix"] + res["suffix"])) < 1e-12
    assert res["label"] == (res["s"] > 0.0)
    assert cache.length == L                                          # scoring does not commit
    if N == 0:                                                        # prefix-only score: one softmax
        logits = orc.block_forward(cfg, W, [helpers.random_cache(cfg, L, 64, seed=60)], [[cache.pending]])[0]["logits"][0]
        p = np.exp(logits - logits.max()); p /= p.sum()
        assert abs(res["s"] - (np.log(p[z]) - np.log(p[y_next[0]]))) < 1e-10 and res["suffix"] == 0.0


def test_replacing_a_token_by_itself_scores_zero_and_swapping_negates():
    shape, cfg, t = _tiny(4)
    W = helpers.dict_weights(t)
    cache = helpers.random_cache(cfg, 5, 64, seed=61)
    y_next = [3, 17, 40, 8]
    same = orc.semantic_preservation(cfg, W, cache, y_next, y_next[0], tau=0.0)
    assert same["s"] == 0.0 and same["label"] is False
    fwd = orc.semantic_preservation(cfg, W, cache, y_next, 29, tau=-1e9)
    back = orc.semantic_preservation(cfg, W, cache, [29] + y_next[1:], y_next[0], tau=-1e9)
    assert abs(fwd["s"] + back["s"]) < 1e-10 and fwd["label"] and back["label"]
    # h_z is the hidden state of the row that READS z: it changes with z, row 0 (reads y_{i-1}) does not
    other = orc.semantic_preservation(cfg, W, cache, y_next, 30, tau=0.0)
    assert not np.allclose(fwd["h_z"], other["h_z"])


def test_scored_rows_are_normalised_distributions():
    shape, cfg, t = _tiny(6)
    W = helpers.dict_weights(t)
    cache = helpers.random_cache(cfg, 4, 64, seed=62)
    ins = [[cache.pending, 5, 9]]
    tot = np.zeros(3)
    for v in range(cfg.vocab):                                        # every token as the target of every row
        tot += np.exp(orc.score_block(cfg, W, [cache], ins, [[v, v, v]])[0]["logprob"])
    assert np.allclose(tot, 1.0, atol=1e-10)


# ------------------------------------------------------------------ P10: top-k verification (Sec. 4.1 baseline, R12)
def test_token_rank_against_a_stable_sort_with_ties():
    rng = np.random.default_rng(0)
    for trial in range(20):
        row = rng.integers(0, 6, 40).astype(np.float64)            # many equal logits
        order = np.argsort(-row, kind="stable")                    # library routine: decreasing, ties by index
        for tok in range(40):
            assert orc.token_rank(row, tok) == int(np.nonzero(order == tok)[0][0])


def test_topk_mode_special_cases():
    rng = np.random.default_rng(1)
    V, gamma = 50, 6
    logits = rng.normal(size=(gamma + 1, V))
    toks = rng.integers(0, V, gamma)
    toks[0] = int(np.argmax(logits[0]))                             # the target's own token
    toks[1] = int(np.argsort(-logits[1])[1])                        # its runner-up
    toks[2] = int(np.argsort(-logits[2])[2])                        # third: fails k = 2
    q = rng.dirichlet(np.ones(V), gamma)
    u = rng.random(gamma + 1)
    scores = np.zeros(gamma)
    r2 = orc.verify_tail(logits, scores, toks, q, u, 0.5, 1.0, "topk", 2)
    assert r2["topk_bits"][:3] == [True, True, False] and r2["accepted_len"] == 2
    # k = V keeps everything, k = 1 keeps exactly the arg-max tokens, acceptance is monotone in k
    assert orc.verify_tail(logits, scores, toks, q, u, 0.5, 1.0, "topk", V)["accepted_len"] == gamma
    r1 = orc.verify_tail(logits, scores, toks, q, u, 0.5, 1.0, "topk", 1)
    assert r1["topk_bits"] == [int(t) == int(np.argmax(logits[j])) for j, t in enumerate(toks)]
    lens = [orc.verify_tail(logits, scores, toks, q, u, 0.5, 1.0, "topk", k)["accepted_len"] for k in range(1, V + 1)]
    assert all(a <= b for a, b in zip(lens, lens[1:]))
    # k = 1 at temperature 0 with a greedy (one-hot) draft is the alignment test of Eq. 3
    onehot = np.zeros((gamma, V)); onehot[np.arange(gamma), toks] = 1.0
    a = orc.verify_tail(logits, scores, toks, onehot, u, 0.5, 0.0, "alignment")
    k1 = orc.verify_tail(logits, scores, toks, onehot, u, 0.5, 0.0, "topk", 1)
    assert a["align_bits"] == k1["topk_bits"] and a["accepted_len"] == k1["accepted_len"] and a["next_token"] == k1["next_token"]
