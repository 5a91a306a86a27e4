"""Pins for the CPU oracle: things the mathematics fixes, independent of oracle/ itself."""
import math

import numpy as np
import pytest

from oracle import paging, sampling
from oracle import transformer as otf
from paper_2601_05475_amd import synth

import bruteforce
from golden_io import paper_values
from helpers import oracle_config, small_shape


# ---------------------------------------------------------------- whole forward pass
@pytest.mark.parametrize("shape_kw", [
    dict(L=1, d=8, Hq=2, Hkv=1, hd=4, F=12, V=16),
    dict(L=2, d=16, Hq=4, Hkv=2, hd=4, F=12, V=32),
    dict(L=2, d=12, Hq=6, Hkv=2, hd=2, F=10, V=20, base=500.0),
])
def test_forward_matches_bruteforce(shape_kw):
    s = small_shape(**shape_kw)
    w = synth.make_weights(s, seed=7)
    # larger-than-init weights so that softmax and SiLU are far from their linear regime
    for lw in w["layers"]:
        for k in lw:
            if not k.endswith("norm"):
                lw[k] = lw[k] * 25.0
    w["embed"] = w["embed"] * 50.0
    toks = synth.tokens(11, 1, (11,), s.vocab)
    got = otf.forward(oracle_config(s), w, toks)[0]
    cfgd = dict(n_layers=s.n_layers, d_model=s.d_model, n_q_heads=s.n_q_heads,
                n_kv_heads=s.n_kv_heads, head_dim=s.head_dim, rms_eps=s.rms_eps,
                rope_base=s.rope_base)
    want = np.array(bruteforce.forward(cfgd, w, list(toks)))
    assert got.shape == want.shape
    # non-trivial attention: some softmax row must be far from uniform
    assert np.abs(want).max() > 1e-2
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-9 * max(1.0, np.abs(want).max()))


def test_shared_prefix_equals_unshared():
    s = small_shape(L=2, d=32, Hq=4, Hkv=2, hd=8, F=40, V=64)
    cfg = oracle_config(s)
    w = synth.make_weights(s, seed=3)
    prefix = synth.tokens(5, 1, (9,), s.vocab)
    suf = synth.tokens(5, 2, (3, 5), s.vocab)
    plast, shared = otf.forward_shared(cfg, w, prefix, suf)
    for b in range(3):
        full = otf.forward_unshared(cfg, w, prefix, suf[b])
        np.testing.assert_allclose(shared[b], full[len(prefix):], rtol=0, atol=1e-12)
        np.testing.assert_allclose(plast, full[len(prefix) - 1], rtol=0, atol=1e-12)


def test_decode_equals_prefill_and_causality():
    s = small_shape(L=2, d=32, Hq=4, Hkv=2, hd=8, F=40, V=64)
    cfg = oracle_config(s)
    w = synth.make_weights(s, seed=4)
    toks = synth.tokens(6, 1, (10,), s.vocab)
    full = otf.forward(cfg, w, toks)[0]
    cache = None
    for t in range(10):                       # token by token
        lg, cache = otf.forward(cfg, w, toks[t:t + 1], cache)
        np.testing.assert_allclose(lg[0], full[t], rtol=0, atol=1e-12)
    toks2 = toks.copy()
    toks2[7:] = (toks2[7:] + 1) % s.vocab     # later tokens do not influence earlier logits
    full2 = otf.forward(cfg, w, toks2)[0]
    np.testing.assert_array_equal(full[:7], full2[:7])
    assert np.abs(full[7:] - full2[7:]).max() > 0


def test_identical_candidates_give_identical_rows():
    s = small_shape()
    cfg = oracle_config(s)
    w = synth.make_weights(s, seed=5)
    prefix = synth.tokens(1, 1, (6,), s.vocab)
    suf = np.tile(synth.tokens(1, 2, (1, 4), s.vocab), (3, 1))
    _, out = otf.forward_shared(cfg, w, prefix, suf)
    np.testing.assert_array_equal(out[0], out[1])
    np.testing.assert_array_equal(out[0], out[2])


# ---------------------------------------------------------------- RMSNorm closed forms
def test_rmsnorm_closed_forms():
    d, eps = 16, 1e-6
    g = np.linspace(0.5, 1.5, d)
    c = 3.0
    np.testing.assert_allclose(otf.rmsnorm(np.full((1, d), c), g, eps)[0],
                               g * c / math.sqrt(c * c + eps), rtol=1e-15)
    a, j = -2.0, 5
    x = np.zeros((1, d)); x[0, j] = a
    y = otf.rmsnorm(x, g, eps)[0]
    assert y[j] == pytest.approx(g[j] * a / math.sqrt(a * a / d + eps), rel=1e-15)
    assert np.all(np.delete(y, j) == 0)
    x = np.random.default_rng(0).normal(size=(3, d))
    np.testing.assert_allclose(otf.rmsnorm(7.0 * x, g, 0.0), otf.rmsnorm(x, g, 0.0), rtol=1e-14)
    # eps matters where it should: zero input stays zero, finite
    assert np.all(otf.rmsnorm(np.zeros((1, d)), g, eps) == 0)


# ---------------------------------------------------------------- RoPE closed forms
def test_rope_closed_forms():
    rng = np.random.default_rng(1)
    hd, base = 8, 10000.0
    z = rng.normal(size=(5, 3, hd))
    np.testing.assert_array_equal(otf.rope(z, np.zeros(5, int), base), z)       # pos 0 identity
    pos = np.array([0, 1, 7, 100, 4095])
    r = otf.rope(z, pos, base)
    np.testing.assert_allclose(np.linalg.norm(r, axis=-1), np.linalg.norm(z, axis=-1), rtol=1e-13)
    # hd = 2: (1, 0) -> (cos pos, sin pos)
    e = otf.rope(np.array([[[1.0, 0.0]]]).repeat(3, 0), np.array([1, 2, 3]), base)
    np.testing.assert_allclose(e[:, 0, 0], np.cos([1, 2, 3]), atol=1e-15)
    np.testing.assert_allclose(e[:, 0, 1], np.sin([1, 2, 3]), atol=1e-15)
    # relative-position property
    q, k = rng.normal(size=(1, 1, hd)), rng.normal(size=(1, 1, hd))
    def dot(m, n):
        return float(np.sum(otf.rope(q, [m], base) * otf.rope(k, [n], base)))
    assert dot(9, 4) == pytest.approx(dot(105, 100), rel=1e-11)
    assert abs(dot(9, 4) - dot(9, 5)) > 1e-3
    # pairing: perturbing coordinate i changes only outputs i and i + hd/2
    z1 = rng.normal(size=(1, 1, hd)); z2 = z1.copy(); z2[0, 0, 1] += 1.0
    diff = np.abs(otf.rope(z1, [3], base) - otf.rope(z2, [3], base))[0, 0]
    assert set(np.flatnonzero(diff > 0)) == {1, 1 + hd // 2}
    # frequency of pair i is base^(-2i/hd): pair 1 of hd=8 at pos 1 rotates by base^-0.25
    one = np.zeros((1, 1, hd)); one[0, 0, 1] = 1.0
    out = otf.rope(one, [1], base)[0, 0]
    assert out[1] == pytest.approx(math.cos(base ** -0.25), rel=1e-14)
    assert out[1 + hd // 2] == pytest.approx(math.sin(base ** -0.25), rel=1e-14)


# ---------------------------------------------------------------- attention invariants
def test_attention_invariants():
    rng = np.random.default_rng(2)
    T, S, Hq, Hkv, hd = 3, 7, 4, 2, 8
    q = rng.normal(size=(T, Hq, hd)); k = rng.normal(size=(S, Hkv, hd)); v = rng.normal(size=(S, Hkv, hd))
    qpos = np.array([6, 6, 6]); kpos = np.arange(S)
    p = otf.softmax_rows(rng.normal(size=(5, 9)) * 10)
    assert np.abs(p.sum(-1) - 1).max() < 1e-12
    # one visible key -> that value exactly
    o = otf.attention(q, k, v, np.array([0, 0, 0]), kpos)
    for a in range(Hq):
        np.testing.assert_allclose(o[:, a], np.tile(v[0, a // 2], (T, 1)), rtol=1e-15)
    # zero queries -> equal scores -> mean of the visible values
    o = otf.attention(np.zeros_like(q), k, v, qpos, kpos)
    np.testing.assert_allclose(o[0, 3], v[:, 1].mean(0), rtol=1e-13)
    # GQA mapping: head a reads kv head a // G
    v2 = v.copy(); v2[:, 1] += 1.0
    d = otf.attention(q, k, v2, qpos, kpos) - otf.attention(q, k, v, qpos, kpos)
    assert np.abs(d[:, :2]).max() == 0 and np.allclose(d[:, 2:], 1.0)
    # scale 1/sqrt(hd): one query, two keys, closed form
    q1 = np.zeros((1, 1, 4)); q1[0, 0, 0] = 2.0
    k2 = np.zeros((2, 1, 4)); k2[0, 0, 0] = 1.0
    v2 = np.array([[[1.0, 0, 0, 0]], [[0, 1.0, 0, 0]]])
    o = otf.attention(q1, k2, v2, [1], [0, 1])[0, 0]
    w0 = 1.0 / (1.0 + math.exp(-(2.0 * 1.0) / math.sqrt(4)))
    np.testing.assert_allclose(o[:2], [w0, 1 - w0], rtol=1e-14)
    # attention_one equals the batched routine
    one = otf.attention_one(q[0, 1], k[:, 0], v[:, 0])
    np.testing.assert_allclose(one, otf.attention(q, k, v, qpos, kpos)[0, 1], rtol=1e-13)


def test_split_softmax_merge_identity():
    """Any partition of the keys, merged by (max, sum, weighted value), is the full softmax."""
    rng = np.random.default_rng(3)
    S, hd = 37, 8
    q = rng.normal(size=hd) * 3; k = rng.normal(size=(S, hd)); v = rng.normal(size=(S, hd))
    want = otf.attention_one(q, k, v)
    parts = [(0, 5), (5, 6), (6, 30), (30, 37)]
    ms, ls, os_ = [], [], []
    for a, b in parts:
        s = k[a:b] @ q / math.sqrt(hd)
        m = s.max(); e = np.exp(s - m)
        ms.append(m); ls.append(e.sum()); os_.append(e @ v[a:b])
    M = max(ms)
    num = sum(np.exp(m - M) * o for m, o in zip(ms, os_))
    den = sum(np.exp(m - M) * l for m, l in zip(ms, ls))
    np.testing.assert_allclose(num / den, want, rtol=1e-13)


def test_silu_and_linear():
    assert otf.silu(np.array([0.0]))[0] == 0
    assert otf.silu(np.array([40.0]))[0] == pytest.approx(40.0, rel=1e-15)
    assert abs(otf.silu(np.array([-40.0]))[0]) < 1e-15
    assert otf.silu(np.array([1.0]))[0] == pytest.approx(1 / (1 + math.exp(-1)), rel=1e-15)
    x = np.array([[1.0, 2.0, 3.0]]); w = np.array([[1.0, 0, 0], [0, 0, 2.0]])   # [out][in]
    np.testing.assert_array_equal(otf.linear(x, w), [[1.0, 6.0]])


# ---------------------------------------------------------------- sampler
def test_sampler_special_cases():
    rng = np.random.default_rng(4)
    lg = rng.normal(size=200).astype(np.float32)
    top = int(np.argmax(lg))
    assert sampling.sample(lg, 0.0, 50, 0.3)[0] == top
    assert sampling.sample(lg, 0.8, 1, 0.9)[0] == top
    assert sampling.sample(lg, 0.8, 50, 0.0)[0] == top                       # u = 0 -> top token
    tok, ids, _ = sampling.sample(lg, 0.8, 50, np.float32(1 - 2 ** -24))
    assert tok == ids[-1] and len(ids) == 50                                 # u -> 1: k-th token
    assert list(ids) == sorted(range(200), key=lambda i: (-lg[i], i))[:50]
    # ties: all equal -> floor(u k)-th lowest id
    eq = np.zeros(64, np.float32)
    for u in (0.0, 0.26, 0.5, 0.99):
        assert sampling.sample(eq, 0.7, 10, u)[0] == int(u * 10)
    assert sampling.sample(eq, 0.0, 10, 0.5)[0] == 0                          # argmax tie: lowest id
    # full vocabulary when k <= 0 or k >= V
    assert len(sampling.sample(lg, 1.0, 0, 0.5)[1]) == 200
    assert len(sampling.sample(lg, 1.0, 500, 0.5)[1]) == 200
    # determinism
    assert sampling.sample(lg, 0.7, 50, 0.4321)[0] == sampling.sample(lg, 0.7, 50, 0.4321)[0]


def test_sampler_two_logit_closed_form_and_frequencies():
    pv = paper_values()
    T = pv["temperature_reward_model"]
    a, b = 1.3, 0.2
    lg = np.array([b, a], np.float32)
    p_top = 1.0 / (1.0 + math.exp(-(a - b) / T))
    us = synth.uniforms(99, 1, (100000,))
    picks = np.array([sampling.sample(lg, T, 2, u)[0] for u in us[:20000]])
    frac = np.mean(picks == 1)
    assert abs(frac - p_top) < 4 * math.sqrt(p_top * (1 - p_top) / 20000)
    # threshold sits at the closed-form probability
    assert sampling.sample(lg, T, 2, np.float32(p_top - 1e-4))[0] == 1
    assert sampling.sample(lg, T, 2, np.float32(p_top + 1e-4))[0] == 0
    # temperature really divides: at the generation temperature the top token is likelier
    Tg = pv["temperature_generation"]
    assert sampling.sample(lg, Tg, 2, np.float32(p_top + 1e-3))[0] == 1


def test_sampler_top_k_restricts_support():
    lg = np.arange(100, dtype=np.float32) * 0.01
    us = synth.uniforms(5, 1, (2000,))
    picks = {sampling.sample(lg, 1.0, 7, u)[0] for u in us}
    assert picks == set(range(93, 100))


# ---------------------------------------------------------------- scoring
def test_reward_logprobs_and_score():
    pv = paper_values()
    labels = np.array(pv["reward_labels"])
    rng = np.random.default_rng(5)
    lg = rng.normal(size=50) * 3
    lp_all = sampling.reward_logprobs(lg, np.arange(50))
    assert abs(np.exp(lp_all).sum() - 1) < 1e-12
    ids = np.array([3, 17, 4, 40, 9])
    lp = sampling.reward_logprobs(lg, ids)
    np.testing.assert_allclose(lp, lp_all[ids], rtol=0, atol=0)
    # shifting all logits changes nothing
    np.testing.assert_allclose(sampling.reward_logprobs(lg + 11.0, ids), lp, atol=1e-12)
    # equal reward logits -> expectation of labels 0..4 is 2
    lg2 = lg.copy(); lg2[ids] = 0.7
    assert sampling.expected_value(sampling.reward_logprobs(lg2, ids), labels, 1.0) == pytest.approx(2.0, abs=1e-14)
    # one dominant label -> its value
    lg3 = lg.copy(); lg3[ids[3]] = 60.0
    assert sampling.expected_value(sampling.reward_logprobs(lg3, ids), labels, 1.0) == pytest.approx(3.0, abs=1e-12)
    # two labels, closed form with temperature
    Ts = pv["temperature_reward_model"]
    got = sampling.expected_value(np.array([math.log(0.2), math.log(0.1)]), np.array([1.0, 4.0]), Ts)
    p1 = 0.2 ** (1 / Ts) / (0.2 ** (1 / Ts) + 0.1 ** (1 / Ts))
    assert got == pytest.approx(p1 * 1 + (1 - p1) * 4, rel=1e-13)


def test_rank_with_ties():
    assert list(sampling.rank(np.array([0.5, 2.0, 0.5, 3.0, 2.0]))) == [3, 1, 4, 0, 2]
    assert list(sampling.rank(np.array([1.0]))) == [0]


# ---------------------------------------------------------------- paging
def test_page_table_reference_small_example():
    # 3 candidates, page of 2 tokens, 5 steps: pages handed out in candidate order per boundary
    t = paging.page_tables(3, 5, 2, range(100))
    assert t.tolist() == [[0, 3, 6], [1, 4, 7], [2, 5, 8]]
    perm = [9, 8, 7, 6, 5, 4, 3, 2, 1, 0]
    t = paging.page_tables(2, 3, 2, perm)
    assert t.tolist() == [[9, 7], [8, 6]]
    assert paging.slot_of(t, 1, 2, 2) == (6, 0)
    assert paging.page_tables(2, 0, 4, range(4)).shape == (2, 0)
    # exactly one page when n_steps == page size; two when one more
    assert paging.page_tables(1, 4, 4, range(4)).tolist() == [[0]]
    assert paging.page_tables(1, 5, 4, range(4)).tolist() == [[0, 1]]


def test_page_pool_with_drops_worked_example():
    # worked by hand: 3 candidates, pages of 2 tokens, a pool of 7 pages in the order 10..16.
    # t=0: cands 0,1,2 take 10,11,12.  After 2 tokens candidate 1 leaves: queue 13,14,15,16,11.
    # t=2: cands 0,2 take 13,14.  t=4: 15,16.  t=6: 11 (reused) and then nothing is left.
    pool = paging.PagePool(3, 2, range(10, 17))
    pool.append(2)
    assert [pool.table(b) for b in range(3)] == [[10], [11], [12]]
    pool.drop([1])
    assert pool.free == [13, 14, 15, 16, 11] and pool.table(1) == []
    pool.append(4)
    assert pool.table(0) == [10, 13, 15] and pool.table(2) == [12, 14, 16]
    with pytest.raises(MemoryError):
        pool.append(1)
    assert pool.length == 6 and pool.free == [11] and pool.table(0) == [10, 13, 15]   # untouched
    pool.drop([0])
    assert pool.free == [11, 10, 13, 15]
    pool.append(3)
    assert pool.table(2) == [12, 14, 16, 11, 10] and pool.length == 9 and pool.alive == [2]
    # without drops it is the lock-step table
    pool = paging.PagePool(3, 2, range(100))
    pool.append(5)
    assert [pool.table(b) for b in range(3)] == paging.page_tables(3, 5, 2, range(100)).tolist()
    # several leave at once: pages return in ascending candidate order, whatever order is given
    pool = paging.PagePool(4, 1, range(8))
    pool.append(2)
    pool.drop([3, 0])
    assert pool.free == [0, 4, 3, 7]


def test_page_pool_candidates_of_different_lengths_worked_example():
    # worked by hand: pages of 2 tokens, pool 20, 21, ...; three candidates get 3, 1 and 4 tokens.
    # index 0: all three open their first page (20, 21, 22).  index 1: nobody is at a boundary.
    # index 2: candidate 0 (length 2) takes 23, candidate 1 has no token left, candidate 2 takes 24.
    pool = paging.PagePool(3, 2, range(20, 40))
    pool.append_each([3, 1, 4])
    assert [pool.table(b) for b in range(3)] == [[20, 23], [21], [22, 24]]
    assert pool.lens == {0: 3, 1: 1, 2: 4} and pool.length == 4
    pool.append(1)                 # lengths 3, 1, 4: only candidate 2 is at a boundary
    assert [pool.table(b) for b in range(3)] == [[20, 23], [21], [22, 24, 25]]
    pool.append(1)                 # lengths 4, 2, 5: candidates 0 and 1 are
    assert [pool.table(b) for b in range(3)] == [[20, 23, 26], [21, 27], [22, 24, 25]]
    # a call the queue cannot serve as a whole changes nothing
    pool = paging.PagePool(2, 2, [7, 8, 9])
    pool.append_each([2, 1])
    with pytest.raises(MemoryError):
        pool.append_each([1, 3])   # candidate 0 needs one page, candidate 1 needs one: only one is left
    assert pool.free == [9] and pool.lens == {0: 2, 1: 1}
    pool.append_each([1, 1])       # candidate 0 opens its second page, candidate 1 fills its first
    assert pool.table(0) == [7, 9] and pool.table(1) == [8] and pool.free == []


# ---------------------------------------------------------------- bf16 activation mode
def test_round_bf16_against_closed_forms_and_library():
    import torch
    r = otf.round_bf16
    # 8 significand bits: spacing 2^-7 in [1, 2); ties go to the even neighbour
    assert r(np.array([1.0 + 2.0 ** -8]))[0] == 1.0
    assert r(np.array([1.0 + 3 * 2.0 ** -8]))[0] == 1.0 + 2.0 ** -6
    assert r(np.array([1.0 + 2.0 ** -8 + 2.0 ** -20]))[0] == 1.0 + 2.0 ** -7
    assert r(np.array([-0.3]))[0] == -0.30078125
    assert np.array_equal(r(np.array([0.0, 1.0, -2.5, 2.0 ** -100])), [0.0, 1.0, -2.5, 2.0 ** -100])
    x = synth.normal(8, 1, (20000,), 0.0, 3.0, "f32")
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(r(x), want)
    assert np.abs(r(x) - x).max() <= np.abs(x).max() * 2.0 ** -8


def test_bf16_activation_mode_rounds_only_activation_tensors():
    s = small_shape(L=2, d=32, Hq=4, Hkv=2, hd=8, F=40, V=64, dtype="bf16")
    w = synth.weights_as_f32(synth.make_weights(s, 9))
    toks = synth.tokens(9, 1, (12,), s.vocab)
    exact = otf.forward(oracle_config(s, exact=True), w, toks)[0]
    rounded, cache = otf.forward(oracle_config(s), w, toks)
    rel = np.linalg.norm(rounded - exact) / np.linalg.norm(exact)
    assert 1e-5 < rel < 2e-2            # it does round, and only at the bf16 level
    for l in range(s.n_layers):         # the cache holds bf16 values
        assert np.array_equal(cache.k[l], otf.round_bf16(cache.k[l]))
        assert np.array_equal(cache.v[l], otf.round_bf16(cache.v[l]))
    assert oracle_config(small_shape()).act_dtype == "f64"
    # shared == unshared and decode == prefill hold in this mode too (same values are rounded)
    cfg = oracle_config(s)
    plast, shared = otf.forward_shared(cfg, w, toks[:7], toks[7:][None])
    np.testing.assert_allclose(shared[0], rounded[7:], rtol=0, atol=1e-12)


def test_layerwise_driver_of_the_fullsize_golden_script_equals_forward_shared():
    """tests/golden/make_fullsize_golden.py walks the layers in the outer loop and the sequences in
    the inner one (weights are generated once per layer).  Same arithmetic as forward_shared: the
    logits agree to float64 rounding (the matrix library sums a one-row product in another order
    than a many-row one), in both activation precisions, for suffixes of different lengths."""
    import importlib.util
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "make_fullsize_golden.py")
    spec = importlib.util.spec_from_file_location("make_fullsize_golden", path)
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    s = small_shape(L=3, d=32, Hq=4, Hkv=2, hd=8, F=40, V=64, dtype="bf16")
    seed = 21
    w = synth.weights_as_f32(synth.make_weights(s, seed))
    prefix = synth.tokens(5, 1, (9,), s.vocab)
    suf = synth.tokens(5, 2, (3, 5), s.vocab)
    suffixes = {0: suf[0, :5], 2: suf[2, :2]}
    cfgs = [oracle_config(s, exact=True), oracle_config(s, exact=False)]
    res = mod.forward_many(cfgs, s, seed, prefix, suffixes, log=lambda *a, **k: None)
    for cfg, (plast, xs, head) in zip(cfgs, res):
        want_p, want = otf.forward_shared(cfg, w, prefix, suf)
        np.testing.assert_allclose(plast, want_p, rtol=0, atol=1e-13)
        for b, toks in suffixes.items():
            got = otf.lm_logits(cfg, head, xs[b])
            np.testing.assert_allclose(got, want[b, :len(toks)], rtol=0, atol=1e-13)


def test_attention_parity_bound_sees_a_lost_key_block():
    """The bound the GPU attention tests use (relative L2 per row and head) against planted
    mistakes, on the oracle itself at the headline shape's key count (4096 prefix + 512 suffix keys
    of dimension 128, N(0, 1)): an output computed without one 32-key block, without one 64-key
    page, or with one split's partial state weighted twice fails it; bf16 rounding of the output
    passes.  (The absolute bound of 1.5e-2 used before passed all four.)"""
    from gpu_common import ATT_REL, rel_l2
    rng = np.random.default_rng(5)
    S, hd = 4608, 128
    q, k, v = rng.standard_normal(hd), rng.standard_normal((S, hd)), rng.standard_normal((S, hd))
    want = otf.attention_one(q, k, v)
    keep = np.ones(S, bool); keep[2048:2080] = False
    lost_block = otf.attention_one(q, k[keep], v[keep])
    keep = np.ones(S, bool); keep[4544:4608] = False
    lost_page = otf.attention_one(q, k[keep], v[keep])
    twice = otf.attention_one(q, np.concatenate([k, k[512:1024]]), np.concatenate([v, v[512:1024]]))
    rounded = otf.round_bf16(want)
    assert rel_l2(rounded, want) < ATT_REL["bf16"] / 3
    for wrong in (lost_block, lost_page, twice):
        assert rel_l2(wrong, want) > 2 * ATT_REL["bf16"]
        assert np.abs(wrong - want).max() < 1.5e-2          # what the old bound could not see


def test_logits_parity_statistics_see_mistakes_the_widened_bound_accepts(monkeypatch):
    """gpu_common.assert_logits_close on planted mistakes, CPU only.  The 'device' is the oracle's
    bf16-tensor mode with a fault planted in the oracle: (a) bf16 conversion by truncation instead
    of round-to-nearest, (b) a constant 1e-3 added to every logit.  Both stay inside the max-abs /
    relative bounds (stated tolerance or 1.5 x noise floor); the first is caught by the RMS ratio,
    the second by the mean signed error.  The unfaulted mode passes against itself."""
    import gpu_common
    s = small_shape(L=6, d=256, Hq=4, Hkv=2, hd=64, F=512, V=1024, dtype="bf16")
    w = synth.weights_as_f32(synth.make_weights(s, 31))
    prefix, suf = synth.tokens(8, 1, (40,), s.vocab), synth.tokens(8, 2, (2, 3), s.vocab)
    exact = otf.forward_shared(oracle_config(s, exact=True), w, prefix, suf)[1]
    floor = otf.forward_shared(oracle_config(s, exact=False), w, prefix, suf)[1]
    gpu_common.assert_logits_close(floor, exact, "bf16", "floor against itself", floor=floor)

    def truncate(x):
        f = np.ascontiguousarray(x, np.float32)
        return (f.view(np.uint32) & np.uint32(0xFFFF0000)).view(np.float32).reshape(f.shape).astype(np.float64)

    real_lm_logits = otf.lm_logits
    faults = {"truncation": lambda m: m.setattr(otf, "round_bf16", truncate),
              "logit offset": lambda m: m.setattr(otf, "lm_logits", lambda cfg, w_, x: real_lm_logits(cfg, w_, x) + 1e-3)}
    for name, plant in faults.items():
        with monkeypatch.context() as m:
            plant(m)
            wrong = otf.forward_shared(oracle_config(s, exact=False), w, prefix, suf)[1]
        err, rel = gpu_common._errs(wrong, exact)
        ferr, frel = gpu_common._errs(floor, exact)
        a_bound = max(gpu_common.TOL["bf16"][0], gpu_common.FLOOR_SLACK * ferr)
        r_bound = max(gpu_common.TOL["bf16"][1], gpu_common.FLOOR_SLACK * frel)
        assert err <= a_bound and rel <= r_bound, (name, err, a_bound, rel, r_bound)     # the old rule accepts it
        with pytest.raises(AssertionError):
            gpu_common.assert_logits_close(wrong, exact, "bf16", name, floor=floor)
    del gpu_common.PARITY_RECORDS[:]


def test_page_pool_pause_and_resume_by_hand():
    """Three candidates, pages of 2, free queue 10, 11, 12, ...: worked by hand.  Step 1: all take
    a page (10, 11, 12).  Candidate 1 pauses.  Steps 2-3: at step 3 candidates 0 and 2 reach a page
    boundary and take 13, 14; candidate 1 keeps page 11 and length 1.  Candidate 1 resumes; step 4:
    it fills its first page (no new page), 0 and 2 fill their second.  Step 5: candidate 0 takes 15,
    candidate 1 (length 2) takes 16, candidate 2 takes 17: ascending order, the resumed one in its
    place.  Dropping the paused candidate 2 later returns its pages in the order it took them."""
    pool = paging.PagePool(3, 2, range(10, 30))
    pool.append(1)
    pool.pause([1])
    pool.append(2)
    assert pool.table(0) == [10, 13] and pool.table(1) == [11] and pool.table(2) == [12, 14]
    assert pool.lens == {0: 3, 1: 1, 2: 3}
    pool.resume([1])
    pool.append(1)
    assert pool.table(1) == [11] and pool.lens[1] == 2
    pool.append(1)
    assert pool.table(0) == [10, 13, 15] and pool.table(1) == [11, 16] and pool.table(2) == [12, 14, 17]
    pool.pause([2])
    pool.resume([2])
    pool.drop([2])
    assert pool.free[-3:] == [12, 14, 17] and pool.alive == [0, 1]
