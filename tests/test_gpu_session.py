"""End-to-end parity of the four calls against the CPU oracle (through the C ABI)."""
import numpy as np
import pytest

from oracle import paging as opaging
from oracle import sampling as osamp
from paper_2601_05475_amd import binding, synth

from gpu_common import (SAMPLE_MARGIN, assert_logits_close, check_against_oracle,
                        check_sampler_on_logits, oracle_shared, teacher_forced_gpu)
from helpers import oracle_config, small_shape
from oracle import transformer as otf

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def tiny():
    wl = synth.WORKLOADS["tiny"]
    w = synth.make_weights(wl.shape, wl.seed_weights)
    return wl, w


def test_tiny_config_teacher_forced_logits_pages_and_sampler(tiny):
    """The tiny fp32 workload as specified: 128-token prefix, 4 candidates, 16 steps, pages of 4."""
    wl, w = tiny
    s = wl.shape
    prefix, suffix, us = synth.prefix_tokens(wl), synth.suffix_tokens(wl), synth.step_uniforms(wl)
    B, N = suffix.shape
    print("case: tiny teacher-forced", s, flush=True)
    pl, steps, sess, model = teacher_forced_gpu(s, w, prefix, suffix, wl.page_tokens)
    want_pl, want = oracle_shared(s, w, prefix, suffix)
    assert_logits_close(pl[None], want_pl[None], "f32", "prefix logits")
    assert_logits_close(steps, want, "f32", "decode logits")
    tab, n = sess.page_table()
    ref = opaging.page_tables(B, N, wl.page_tokens, range(sess.pool_pages()))
    assert list(n) == [ref.shape[1]] * B
    np.testing.assert_array_equal(tab[:, :ref.shape[1]], ref)


def test_tiny_sampler_on_device_logits(tiny):
    wl, w = tiny
    s = wl.shape
    prefix, suffix, us = synth.prefix_tokens(wl, 40), synth.suffix_tokens(wl, 4, 6), synth.step_uniforms(wl, 4, 7)
    model = binding.Model(s, w)
    sess = binding.Session(model, 64, 4, 8, 4)
    sess.prefill_shared(prefix)
    row = sess.logits(1)[0]
    toks, topk = sess.sample(4, wl.temperature, wl.top_k, us[0], want_topk=True)
    for b in range(4):
        check_sampler_on_logits(row, wl.temperature, wl.top_k, us[0][b], toks[b], topk[b])
    exact = 0
    for t in range(6):
        sess.decode_step(suffix[:, t])
        lg = sess.logits(4)
        toks, topk = sess.sample(4, wl.temperature, wl.top_k, us[t + 1], want_topk=True)
        for b in range(4):
            exact += check_sampler_on_logits(lg[b], wl.temperature, wl.top_k, us[t + 1][b], toks[b], topk[b])
    assert exact >= 22          # excuses must stay rare
    # greedy and full-vocabulary modes
    g = sess.sample(4, 0.0, 50, us[0])
    assert list(g) == [int(np.argmax(lg[b])) for b in range(4)]
    toks, topk = sess.sample(4, 1.0, 0, us[1], want_topk=True)
    assert topk.shape == (4, s.vocab)
    for b in range(4):
        check_sampler_on_logits(lg[b], 1.0, 0, us[1][b], toks[b], topk[b])


def test_free_running_matches_oracle(tiny):
    """Sample, feed back, repeat: the sequences equal the oracle's, apart from steps the oracle
    marks ambiguous (after such a step nothing more is compared for that candidate)."""
    from oracle import transformer as otf
    from helpers import oracle_config
    wl, w = tiny
    s = wl.shape
    cfg = oracle_config(s)
    P, B, N = 32, 4, 8
    prefix, us = synth.prefix_tokens(wl, P), synth.step_uniforms(wl, B, N)
    model = binding.Model(s, w)
    sess = binding.Session(model, P, B, N, 4)
    sess.prefill_shared(prefix)
    got = []
    for t in range(N):
        toks = sess.sample(B, wl.temperature, wl.top_k, us[t])
        got.append(toks.copy())
        sess.decode_step(None if t % 2 else toks, B)      # alternate host / device hand-over
    got = np.stack(got, 1)                                  # [B, N]
    plog, pcache = otf.forward(cfg, w, prefix)
    compared = 0
    for b in range(B):
        cache, lg = pcache.copy(), plog[-1]
        for t in range(N):
            tok, _, margin = osamp.sample(lg.astype(np.float32), wl.temperature, wl.top_k, us[t][b])
            if margin < 20 * SAMPLE_MARGIN:     # fp32 logits differ in the last bits too
                break
            assert tok == got[b, t], (b, t)
            compared += 1
            lg = otf.forward(cfg, w, np.array([tok]), cache)[0][0]
    assert compared >= B * N // 2


def test_physical_page_order_and_candidate_order_do_not_matter(tiny):
    wl, w = tiny
    s = wl.shape
    prefix, suffix = synth.prefix_tokens(wl, 50), synth.suffix_tokens(wl, 4, 10)
    _, base, sess, _ = teacher_forced_gpu(s, w, prefix, suffix, 4)
    n = sess.pool_pages()
    perm = np.random.default_rng(0).permutation(n).astype(np.int32)
    _, shuffled, sess2, _ = teacher_forced_gpu(s, w, prefix, suffix, 4, free_list=perm)
    np.testing.assert_array_equal(base, shuffled)                 # bit-identical
    tab, cnt = sess2.page_table()
    ref = opaging.page_tables(4, 10, 4, perm)
    np.testing.assert_array_equal(tab[:, :ref.shape[1]], ref)
    order = np.array([2, 0, 3, 1])
    _, permuted, _, _ = teacher_forced_gpu(s, w, prefix, suffix[order], 4)
    np.testing.assert_array_equal(permuted, base[:, order])


def test_reset_keeps_prefix_and_state_errors(tiny):
    wl, w = tiny
    s = wl.shape
    prefix, suffix = synth.prefix_tokens(wl, 20), synth.suffix_tokens(wl, 3, 5)
    model = binding.Model(s, w)
    sess = binding.Session(model, 32, 4, 5, 4)
    with pytest.raises(binding.McError) as e:
        sess.decode_step(suffix[:, 0])
    assert e.value.code == -2
    with pytest.raises(binding.McError) as e:
        sess.sample(3, 0.8, 50, np.zeros(3, np.float32))
    assert e.value.code == -2
    sess.prefill_shared(prefix)
    first = sess.logits(1).copy()
    runs = []
    for rep in range(2):
        out = []
        for t in range(5):
            sess.decode_step(suffix[:, t])
            out.append(sess.logits(3))
        runs.append(np.stack(out))
        with pytest.raises(binding.McError) as e:      # suffix capacity reached
            sess.decode_step(suffix[:, 0])
        assert e.value.code == -3
        sess.reset_candidates()
        np.testing.assert_array_equal(sess.logits(1), first)
    np.testing.assert_array_equal(runs[0], runs[1])
    # argument errors leave the session usable
    bad = suffix[:, 0].copy(); bad[1] = s.vocab
    for call in (lambda: sess.decode_step(bad), lambda: sess.decode_step(suffix[:, 0][:2].repeat(3)[:5]),
                 lambda: sess.sample(3, 0.8, 50, np.array([0.1, 1.0, 0.2], np.float32)),
                 lambda: sess.prefill_shared(np.zeros(33, np.int32))):
        with pytest.raises(binding.McError) as e:
            call()
        assert e.value.code == -1
    sess.decode_step(suffix[:, 0])
    np.testing.assert_array_equal(sess.logits(3), runs[0][0])


def test_score_candidates_tiny(tiny):
    """Reranking on the tiny shape with ragged suffixes; the paper's five labels 0..4."""
    wl, w = tiny
    s = wl.shape
    B, Ls = 6, 11
    prefix, suffix = synth.prefix_tokens(wl, 45), synth.suffix_tokens(wl, B, Ls)
    lens = np.array([11, 3, 7, 1, 11, 4], np.int32)
    ids = synth.reward_token_ids(wl, 5)
    vals = np.arange(5, dtype=np.float32)
    model = binding.Model(s, w)
    sess = binding.Session(model, 64, B, 12, 4, chunk_rows=16)     # forces several chunks
    sess.prefill_shared(prefix)
    lp, sc, rk = sess.score_candidates(suffix, lens, ids, vals, 0.7)
    _, ref = oracle_shared(s, w, prefix, suffix)                  # [Ls, B, V]
    want_lp = np.stack([osamp.reward_logprobs(ref[lens[b] - 1, b], ids) for b in range(B)])
    np.testing.assert_allclose(lp, want_lp, rtol=0, atol=1e-4)
    want_sc = np.array([osamp.expected_value(want_lp[b], vals, 0.7) for b in range(B)])
    np.testing.assert_allclose(sc, want_sc, rtol=0, atol=1e-4)
    # ranking: exact on the device's own scores; equals the oracle's where gaps are clear
    assert list(rk) == list(osamp.rank(sc))
    gaps = np.abs(np.diff(np.sort(want_sc)))
    if gaps.min() > 1e-3:
        assert list(rk) == list(osamp.rank(want_sc))
    got_logits = sess.logits(B)
    assert_logits_close(got_logits, np.stack([ref[lens[b] - 1, b] for b in range(B)]), "f32", "score logits")
    # scoring leaves the decode state alone: decoding afterwards equals decoding without it
    sess.decode_step(suffix[:4, 0])
    a = sess.logits(4)
    assert_logits_close(a, ref[0, :4], "f32", "decode after score")
    with pytest.raises(binding.McError):
        sess.score_candidates(suffix, lens, np.array([1, 1, 2, 3, 4]), vals)


@pytest.mark.parametrize("kw", [
    dict(L=2, d=128, Hq=4, Hkv=2, hd=32, F=200, V=1000, P=70, B=3, N=9, pg=8),
    dict(L=1, d=192, Hq=6, Hkv=1, hd=64, F=96, V=777, P=1, B=5, N=5, pg=4),
    dict(L=2, d=256, Hq=4, Hkv=4, hd=128, F=300, V=512, P=130, B=1, N=3, pg=16),
    # every matrix fits the tiled MFMA kernels (bf16): few-row streaming at decode, GEMM at prefill
    dict(L=2, d=256, Hq=4, Hkv=2, hd=64, F=512, V=1024, P=170, B=3, N=9, pg=8),
    dict(L=3, d=512, Hq=8, Hkv=2, hd=64, F=768, V=2048, P=33, B=40, N=3, pg=64),
])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_odd_shapes_both_dtypes(kw, dtype):
    s = small_shape("odd", kw["L"], kw["d"], kw["Hq"], kw["Hkv"], kw["hd"], kw["F"], kw["V"], dtype=dtype)
    w = synth.make_weights(s, 77)
    prefix = synth.tokens(5, 1, (kw["P"],), s.vocab)
    suffix = synth.tokens(5, 2, (kw["B"], kw["N"]), s.vocab)
    print("case: odd shape", kw, dtype, flush=True)
    pl, steps, _, _ = teacher_forced_gpu(s, w, prefix, suffix, kw["pg"], chunk_rows=32)
    check_against_oracle(s, w, prefix, suffix, pl, steps)


def test_1b_shape_two_layer_twin():
    """The 1B shape at full width (2048 wide, 32/8 heads of 64, FFN 8192, vocabulary 32000) with
    2 of its 16 layers: 16 candidates, 64-token pages crossed by a 70-step suffix is too slow for
    the oracle, so the suffix is 5 steps and the prefix 200 tokens (ragged against the page)."""
    wl = synth.WORKLOADS["1b"]
    s = wl.shape.with_layers(2)
    w = synth.make_weights(s, wl.seed_weights)
    prefix, suffix = synth.prefix_tokens(wl, 200), synth.suffix_tokens(wl, 16, 5)
    print("case: 1b twin", s, flush=True)
    pl, steps, sess, _ = teacher_forced_gpu(s, w, prefix, suffix, wl.page_tokens, chunk_rows=128)
    check_against_oracle(s, w, prefix, suffix, pl, steps)
    us = synth.step_uniforms(wl, 16, 1)[0]
    toks, topk = sess.sample(16, wl.temperature, wl.top_k, us, want_topk=True)
    for b in range(16):
        check_sampler_on_logits(steps[-1][b], wl.temperature, wl.top_k, us[b], toks[b], topk[b])


def test_two_runs_give_identical_bits():
    """No kernel on the path adds floating-point numbers in an order that depends on scheduling
    (partial sums meet in a fixed order, no floating-point atomics): two sessions on the same
    inputs (1B width, 2 layers, bf16 MFMA path with key splits, prefix of 1000 tokens, 70 steps
    crossing a page) leave bit-identical logits at every step and sample identical tokens."""
    wl = synth.WORKLOADS["1b"]
    s = wl.shape.with_layers(2)
    w = synth.make_weights(s, wl.seed_weights)
    prefix, suffix = synth.prefix_tokens(wl, 1000), synth.suffix_tokens(wl, 16, 70)
    us = synth.step_uniforms(wl, 16, 1)[0]
    runs = []
    for _ in range(2):
        pl, steps, sess, _ = teacher_forced_gpu(s, w, prefix, suffix, wl.page_tokens, chunk_rows=256)
        toks, topk = sess.sample(16, wl.temperature, wl.top_k, us, want_topk=True)
        runs.append((pl, steps, toks, topk))
        sess.close()
    for x, y in zip(runs[0], runs[1]):
        np.testing.assert_array_equal(x, y)
    # the scoring pass (many-row GEMMs with their fused epilogues, causal attention over
    # prefix + own suffix, reward read-out), twice on one session and once on a fresh one
    model = binding.Model(s, w)
    lens = np.array([2300, 2048, 1, 777], np.int32)
    sfx = synth.suffix_tokens(wl, 4, 2300)
    ids, vals = synth.reward_token_ids(wl, 5), np.arange(5, dtype=np.float32)
    outs = []
    for rep in range(2):
        sess = binding.Session(model, len(prefix), 4, 2300, wl.page_tokens, chunk_rows=4096)
        sess.prefill_shared(prefix)
        outs.append(sess.score_candidates(sfx, lens, ids, vals, 1.0))
        if rep == 0:
            outs.append(sess.score_candidates(sfx, lens, ids, vals, 1.0))
        sess.close()
    for o in outs[1:]:
        for x, y in zip(outs[0], o):
            np.testing.assert_array_equal(x, y)


def test_profiling_events_do_not_change_results():
    """Timing a kernel class (events attached to the launches for the few-row gate/up layer and
    decode attention, recorded around the launch for the others) reports one duration per
    sampled launch and leaves the logits bit-identical."""
    wl = synth.WORKLOADS["1b"]
    s = wl.shape.with_layers(2)
    w = synth.make_weights(s, wl.seed_weights)
    prefix, suffix = synth.prefix_tokens(wl, 300), synth.suffix_tokens(wl, 16, 6)
    model = binding.Model(s, w)
    ref = None
    for cls, per_step in [(None, 0), ("linear_gate_up", 2), ("attn_decode", 2), ("linear_down", 2), ("add_rmsnorm", 5)]:
        sess = binding.Session(model, len(prefix), 16, 8, wl.page_tokens, chunk_rows=128)
        sess.prefill_shared(prefix)
        if cls:
            sess.profile_begin(cls, 1)
        steps = _decode_all(sess, suffix)
        if cls:
            n, ms = sess.profile_end()
            assert n == per_step * suffix.shape[1], (cls, n)
            assert 0.0 < ms / n < 1.0, (cls, ms / n)          # a few microseconds each, not garbage
            np.testing.assert_array_equal(steps, ref)
        else:
            ref = steps
        sess.close()


def _as_f64(w):
    if isinstance(w, dict):
        return {k: _as_f64(v) for k, v in w.items()}
    if isinstance(w, (list, tuple)):
        return [_as_f64(v) for v in w]
    return np.asarray(w, np.float64)


@pytest.mark.timeout(1500)
def test_8b_shape_layer_at_the_benchmark_launch_configuration():
    """One layer of the 8B shape at full width (4096 wide, 32/8 heads of 128, FFN 14336) in the
    configuration the benchmark times: 4096-token shared prefix, 32 candidates, 64-token pages,
    automatic key splits.  The vocabulary is cut to 32000 to keep the oracle's float64 copies
    small (the LM-head shape itself is covered by an operation test).  Decode steps 1 and 2 for
    all candidates against the oracle.  One session prefills in 2048-row chunks; a second one in a
    single 4096-row chunk, as the benchmark does, which is large enough for the O and down
    projections to add to the residual stream in their own epilogue."""
    wl = synth.WORKLOADS["8b"]
    base = wl.shape
    s = synth.Shape("8b-L1-V32000", 1, base.d_model, base.n_q_heads, base.n_kv_heads, base.head_dim,
                    base.d_ffn, 32000, base.rope_base, base.dtype, base.rms_eps)
    w = synth.make_weights(s, wl.seed_weights)
    prefix = synth.tokens(9, 1, (wl.prefix_len,), s.vocab)
    suffix = synth.tokens(9, 2, (wl.n_cands, 2), s.vocab)
    print("case: 8b layer twin", s, flush=True)
    pl, steps, sess, _ = teacher_forced_gpu(s, w, prefix, suffix, wl.page_tokens, chunk_rows=2048,
                                            max_suffix=wl.n_steps)
    sess.close()
    print("case: 8b layer twin, one 4096-row chunk", flush=True)
    pl2, steps2, sess2, _ = teacher_forced_gpu(s, w, prefix, suffix, wl.page_tokens, chunk_rows=4096,
                                               max_suffix=wl.n_steps)
    sess2.close()
    w64 = _as_f64(synth.weights_as_f32(w))          # converted once: the oracle would redo it per call
    print("oracle: exact", flush=True)
    want_pl, want = otf.forward_shared(oracle_config(s, exact=True), w64, prefix, suffix)
    print("oracle: bf16 tensors", flush=True)
    fl_pl, fl = otf.forward_shared(oracle_config(s, exact=False), w64, prefix, suffix)
    assert_logits_close(pl[None], want_pl[None], "bf16", "prefix logits", fl_pl[None])
    assert_logits_close(steps, want.transpose(1, 0, 2), "bf16", "decode logits", fl.transpose(1, 0, 2))
    assert_logits_close(pl2[None], want_pl[None], "bf16", "prefix logits (4096-row chunk)", fl_pl[None])
    assert_logits_close(steps2, want.transpose(1, 0, 2), "bf16", "decode logits (4096-row chunk)", fl.transpose(1, 0, 2))


@pytest.mark.timeout(1500)
def test_32b_shape_layer_twin():
    """One layer of the 32B shape at full width (5120 wide, 40/8 heads of 128: five query heads
    per KV head; FFN 27648; vocabulary cut to 32000) with 64 candidates, i.e. two 32-row
    activation tiles in every weight-streaming layer and 320 query rows per KV head in decode
    attention.  Prefix of 1000 tokens (ragged against pages and blocks), decode steps 1..3."""
    wl = synth.WORKLOADS["32b"]
    base = wl.shape
    s = synth.Shape("32b-L1-V32000", 1, base.d_model, base.n_q_heads, base.n_kv_heads, base.head_dim,
                    base.d_ffn, 32000, base.rope_base, base.dtype, base.rms_eps)
    w = synth.make_weights(s, wl.seed_weights)
    prefix = synth.tokens(12, 1, (1000,), s.vocab)
    suffix = synth.tokens(12, 2, (wl.n_cands, 3), s.vocab)
    print("case: 32b layer twin", s, flush=True)
    pl, steps, sess, _ = teacher_forced_gpu(s, w, prefix, suffix, wl.page_tokens, chunk_rows=1024, max_suffix=64)
    us = synth.step_uniforms(wl, wl.n_cands, 1)[0]
    toks, topk = sess.sample(wl.n_cands, wl.temperature, wl.top_k, us, want_topk=True)
    sess.close()
    for b in range(0, wl.n_cands, 7):
        check_sampler_on_logits(steps[-1][b], wl.temperature, wl.top_k, us[b], toks[b], topk[b])
    w64 = _as_f64(synth.weights_as_f32(w))
    print("oracle: exact", flush=True)
    want_pl, want = otf.forward_shared(oracle_config(s, exact=True), w64, prefix, suffix)
    print("oracle: bf16 tensors", flush=True)
    fl_pl, fl = otf.forward_shared(oracle_config(s, exact=False), w64, prefix, suffix)
    assert_logits_close(pl[None], want_pl[None], "bf16", "prefix logits", fl_pl[None])
    assert_logits_close(steps, want.transpose(1, 0, 2), "bf16", "decode logits", fl.transpose(1, 0, 2))


@pytest.mark.timeout(1500)
def test_8b_shape_layer_scoring_in_one_large_chunk():
    """mc_score_candidates on one layer of the 8B shape at full width (vocabulary cut to 32000),
    4096-token shared prefix, four ragged suffixes (1024, 1024, 700 and 1 tokens) scored as one
    chunk of 2749 rows: large enough for the QKV rotation and the residual updates to run in the
    GEMM epilogues, as in the reranking benchmark.  Last-position logits against the oracle; the
    reward log-probs, scores and ranks against the oracle's rules applied to the device logits."""
    wl = synth.WORKLOADS["8b"]
    base = wl.shape
    s = synth.Shape("8b-L1-V32000", 1, base.d_model, base.n_q_heads, base.n_kv_heads, base.head_dim,
                    base.d_ffn, 32000, base.rope_base, base.dtype, base.rms_eps)
    w = synth.make_weights(s, wl.seed_weights)
    prefix = synth.tokens(11, 1, (wl.prefix_len,), s.vocab)
    lens = np.array([1024, 1024, 700, 1], np.int32)
    suffix = synth.tokens(11, 2, (4, 1024), s.vocab)
    ids = synth.tokens(11, 3, (64,), s.vocab)
    ids = np.unique(ids)[:8].astype(np.int32)
    vals = np.arange(8, dtype=np.float32)
    print("case: 8b layer scoring twin", s, flush=True)
    model = binding.Model(s, w)
    sess = binding.Session(model, wl.prefix_len, 4, 1024, wl.page_tokens, chunk_rows=8192)
    sess.prefill_shared(prefix)
    lp, sc, rk = sess.score_candidates(suffix, lens, ids, vals, 1.0)
    got = sess.logits(4)
    sess.close()
    want_lp = np.stack([osamp.reward_logprobs(got[b], ids) for b in range(4)])
    np.testing.assert_allclose(lp, want_lp, rtol=0, atol=1e-4)
    want_sc = np.array([osamp.expected_value(want_lp[b], vals, 1.0) for b in range(4)])
    np.testing.assert_allclose(sc, want_sc, rtol=0, atol=1e-4)
    assert list(rk) == list(osamp.rank(sc))
    w64 = _as_f64(synth.weights_as_f32(w))
    last = lambda out: np.stack([out[b, lens[b] - 1] for b in range(4)])
    print("oracle: exact", flush=True)
    _, want = otf.forward_shared(oracle_config(s, exact=True), w64, prefix, suffix)
    want = last(want)
    print("oracle: bf16 tensors", flush=True)
    _, fl = otf.forward_shared(oracle_config(s, exact=False), w64, prefix, suffix)
    assert_logits_close(got, want, "bf16", "scoring logits", last(fl))


# ---------------------------------------------------------------- growing the shared prefix
def _decode_all(sess, suffix):
    out = []
    for t in range(suffix.shape[1]):
        sess.decode_step(suffix[:, t])
        out.append(sess.logits(suffix.shape[0]))
    return np.stack(out)


@pytest.mark.parametrize("kw,dtype", [
    (dict(L=2, d=128, Hq=4, Hkv=2, hd=32, F=200, V=1000, pg=4, cut=101, chunk=32), "f32"),
    (dict(L=2, d=128, Hq=4, Hkv=2, hd=32, F=200, V=1000, pg=8, cut=1, chunk=0), "bf16"),
    # tiled bf16 path: MFMA prefill attention over prefix pages written by two calls, 64-token pages
    (dict(L=2, d=256, Hq=4, Hkv=2, hd=64, F=512, V=1024, pg=64, cut=70, chunk=64), "bf16"),
    (dict(L=2, d=256, Hq=8, Hkv=2, hd=128, F=512, V=1024, pg=64, cut=128, chunk=0), "bf16"),
])
def test_extend_shared_equals_one_prefill(kw, dtype):
    """Prefix written by prefill + two extensions: the logits after it and the decode steps on
    top of it are those of the oracle on the whole sequence (and of a single prefill)."""
    s = small_shape("ext", kw["L"], kw["d"], kw["Hq"], kw["Hkv"], kw["hd"], kw["F"], kw["V"], dtype=dtype)
    w = synth.make_weights(s, 78)
    P, B, N = 170, 3, 4
    prefix = synth.tokens(6, 1, (P,), s.vocab)
    suffix = synth.tokens(6, 2, (B, N), s.vocab)
    print("case: extend shared", kw, dtype, flush=True)
    model = binding.Model(s, w)
    sess = binding.Session(model, P, B, N, kw["pg"], kw["chunk"])
    cut = kw["cut"]
    sess.prefill_shared(prefix[:cut])
    sess.decode_step(suffix[:, 0])                  # candidates that the extension must drop
    sess.extend_shared(prefix[cut:cut + 37])
    sess.extend_shared(prefix[cut + 37:])
    pl = sess.logits(1)[0]
    steps = _decode_all(sess, suffix)
    check_against_oracle(s, w, prefix, suffix, pl, steps)
    one = binding.Session(model, P, B, N, kw["pg"], kw["chunk"])
    one.prefill_shared(prefix)
    tol = 1e-5 if dtype == "f32" else 3e-2          # chunk boundaries differ: not bit-identical
    np.testing.assert_allclose(one.logits(1)[0], pl, rtol=0, atol=tol * np.abs(pl).max())
    with pytest.raises(binding.McError) as e:       # the prefix is full
        sess.extend_shared(prefix[:1])
    assert e.value.code == -1


@pytest.mark.parametrize("kw,dtype", [
    (dict(L=2, d=128, Hq=4, Hkv=2, hd=32, F=200, V=1000, pg=4, P=50), "f32"),
    (dict(L=2, d=256, Hq=4, Hkv=2, hd=64, F=512, V=1024, pg=64, P=100), "bf16"),
    (dict(L=2, d=256, Hq=4, Hkv=2, hd=64, F=512, V=1024, pg=64, P=64), "f32"),
])
def test_promote_candidate_then_extend(kw, dtype):
    """Decode, promote one candidate's suffix into the prefix (a copy of its KV), extend with more
    tokens, decode again: everything equals the oracle on the concatenated sequence."""
    s = small_shape("pro", kw["L"], kw["d"], kw["Hq"], kw["Hkv"], kw["hd"], kw["F"], kw["V"], dtype=dtype)
    w = synth.make_weights(s, 79)
    P, B, N1, E, N2, keep = kw["P"], 4, 70, 9, 3, 2
    prefix = synth.tokens(7, 1, (P,), s.vocab)
    suf1 = synth.tokens(7, 2, (B, N1), s.vocab)
    extra = synth.tokens(7, 3, (E,), s.vocab)
    suf2 = synth.tokens(7, 4, (B, N2), s.vocab)
    print("case: promote", kw, dtype, flush=True)
    model = binding.Model(s, w)
    sess = binding.Session(model, P + N1 + E, B, N1, kw["pg"], 64)
    with pytest.raises(binding.McError) as e:
        sess.extend_shared(extra)
    assert e.value.code == -2
    sess.prefill_shared(prefix)
    with pytest.raises(binding.McError) as e:
        sess.promote_candidate(0)
    assert e.value.code == -2
    steps1 = _decode_all(sess, suf1)
    sess.promote_candidate(keep)
    np.testing.assert_array_equal(sess.logits(1)[0], steps1[-1][keep])
    grown = np.concatenate([prefix, suf1[keep]])
    # decoding straight on the promoted prefix (no extension)
    d0 = _decode_all(sess, suf2[:, :1])
    want_pl, want = oracle_shared(s, w, grown, suf2[:, :1])
    fl = oracle_shared(s, w, grown, suf2[:, :1], exact=False)[1] if dtype == "bf16" else None
    assert_logits_close(d0, want, dtype, "decode on the promoted prefix", fl)
    # then the feedback / critique tokens, and a new round of candidates
    sess.extend_shared(extra)
    pl = sess.logits(1)[0]
    steps2 = _decode_all(sess, suf2)
    check_against_oracle(s, w, np.concatenate([grown, extra]), suf2, pl, steps2)


# ---------------------------------------------------------------- critic workload: suffix prefill
@pytest.mark.parametrize("kw,dtype", [
    (dict(L=2, d=128, Hq=4, Hkv=2, hd=32, F=200, V=1000, pg=4, P=50, B=3, chunk=0), "f32"),
    (dict(L=2, d=128, Hq=4, Hkv=2, hd=32, F=200, V=1000, pg=8, P=9, B=5, chunk=32), "bf16"),
    # tiled bf16: MFMA attention over prefix pages + the candidate's own pages, chunks of 2 candidates
    (dict(L=2, d=256, Hq=4, Hkv=2, hd=64, F=512, V=1024, pg=64, P=100, B=5, chunk=160), "bf16"),
    (dict(L=2, d=256, Hq=8, Hkv=2, hd=128, F=512, V=1024, pg=64, P=64, B=2, chunk=0), "bf16"),
])
def test_prefill_suffix_then_decode(kw, dtype):
    """Per-candidate suffix written in bulk (after two ordinary decode steps, then 70 tokens at
    once, crossing page boundaries), then token-by-token decoding on top: every logit row equals
    the oracle's for the same sequences."""
    s = small_shape("crit", kw["L"], kw["d"], kw["Hq"], kw["Hkv"], kw["hd"], kw["F"], kw["V"], dtype=dtype)
    w = synth.make_weights(s, 80)
    P, B = kw["P"], kw["B"]
    n0, n1, n2 = 2, 70, 3
    prefix = synth.tokens(8, 1, (P,), s.vocab)
    suffix = synth.tokens(8, 2, (B, n0 + n1 + n2), s.vocab)
    print("case: prefill suffix", kw, dtype, flush=True)
    model = binding.Model(s, w)
    sess = binding.Session(model, P, B, n0 + n1 + n2, kw["pg"], kw["chunk"])
    with pytest.raises(binding.McError) as e:
        sess.prefill_suffix(suffix[:, :4])
    assert e.value.code == -2
    sess.prefill_shared(prefix)
    pl = sess.logits(1)[0]
    got = [None] * (n0 + n1 + n2)
    for t in range(n0):
        sess.decode_step(suffix[:, t])
        got[t] = sess.logits(B)
    sess.prefill_suffix(suffix[:, n0:n0 + n1])
    got[n0 + n1 - 1] = sess.logits(B)
    for t in range(n0 + n1, n0 + n1 + n2):
        sess.decode_step(suffix[:, t])
        got[t] = sess.logits(B)
    with pytest.raises(binding.McError) as e:       # the candidates' pages are full
        sess.prefill_suffix(suffix[:, :1])
    assert e.value.code == -3
    want_pl, want = oracle_shared(s, w, prefix, suffix)
    fl = oracle_shared(s, w, prefix, suffix, exact=False)[1] if dtype == "bf16" else None
    idx = [t for t in range(len(got)) if got[t] is not None]
    assert_logits_close(np.stack([got[t] for t in idx]), want[idx], dtype, "suffix prefill + decode",
                        None if fl is None else fl[idx])
    tab, n = sess.page_table()
    ref = opaging.page_tables(B, n0 + n1 + n2, kw["pg"], range(sess.pool_pages()))
    np.testing.assert_array_equal(tab[:, :ref.shape[1]], ref)


# ---------------------------------------------------------------- candidates that stop early
@pytest.mark.parametrize("kw,dtype", [
    (dict(L=2, d=128, Hq=4, Hkv=2, hd=32, F=200, V=1000, pg=4), "f32"),
    (dict(L=2, d=256, Hq=4, Hkv=2, hd=64, F=512, V=1024, pg=64), "bf16"),
    (dict(L=2, d=256, Hq=8, Hkv=2, hd=128, F=512, V=1024, pg=64), "bf16"),
])
def test_drop_candidates_midway(kw, dtype):
    """Candidates are independent sequences: dropping some leaves the others' logits what they
    were (the oracle's), while rows, page bookkeeping and pending sampled tokens follow the
    survivors.  70 steps cross a 64-token page boundary after the first drop."""
    s = small_shape("drop", kw["L"], kw["d"], kw["Hq"], kw["Hkv"], kw["hd"], kw["F"], kw["V"], dtype=dtype)
    w = synth.make_weights(s, 82)
    P, B, N = 90, 6, 70
    prefix = synth.tokens(11, 1, (P,), s.vocab)
    suffix = synth.tokens(11, 2, (B, N), s.vocab)
    print("case: drop candidates", kw, dtype, flush=True)
    model = binding.Model(s, w)
    ref = binding.Session(model, P + N, B, N, kw["pg"])
    ref.prefill_shared(prefix)
    full = _decode_all(ref, suffix)                                  # [N, B, V]
    sess = binding.Session(model, P + N, B, N, kw["pg"])
    sess.prefill_shared(prefix)
    alive = list(range(B))
    drops = {3: [1, 4], 66: [0]}
    tol = 0 if dtype == "f32" else 3e-2
    rows_of = {b: [] for b in range(B)}                              # every logits row a candidate produced
    for t in range(N):
        if t in drops:
            before = sess.logits(len(alive))
            sess.drop_candidates(drops[t])
            keep = [i for i, b in enumerate(alive) if b not in drops[t]]
            alive = [b for b in alive if b not in drops[t]]
            np.testing.assert_array_equal(sess.logits(len(alive)), before[keep])   # pending rows moved up
            with pytest.raises(binding.McError):
                sess.decode_step(suffix[:, t])                      # the old count is refused
            with pytest.raises(binding.McError):
                sess.drop_candidates(drops[t][:1])                  # already gone
        sess.decode_step(suffix[alive, t])
        got = sess.logits(len(alive))
        for i, b in enumerate(alive):
            rows_of[b].append(got[i])
        # an extra: the undisturbed run (its key splits are planned for six candidates, so bf16 rounds differently)
        np.testing.assert_allclose(got, full[t][alive], rtol=0, atol=tol * np.abs(full[t]).max() + 0.0)
    # the main evidence: every row of every candidate, up to its drop, against the oracle on that
    # candidate's own sequence
    want_pl, want = oracle_shared(s, w, prefix, suffix)              # [N, B, V]
    fl = oracle_shared(s, w, prefix, suffix, exact=False)[1] if dtype == "bf16" else None
    for b in range(B):
        n_b = len(rows_of[b])
        assert n_b == (N if b in alive else min(t for t, ds in drops.items() if b in ds))
        assert_logits_close(np.stack(rows_of[b]), want[:n_b, b], dtype, f"dropping candidates, candidate {b}: {n_b} steps",
                            None if fl is None else fl[:n_b, b])
    tab, n = sess.page_table()
    held = -(-N // kw["pg"])
    assert [int(x) for x in n[:B]] == [held if b in alive else 0 for b in range(B)]
    pool = opaging.PagePool(B, kw["pg"], range(sess.pool_pages()))   # the same calls on the reference pool
    for t in range(N):
        if t in drops:
            pool.drop(drops[t])
        pool.append(1)
    for b in alive:
        assert tab[b, :held].tolist() == pool.table(b)
    # a survivor can be promoted, a dropped candidate cannot
    with pytest.raises(binding.McError):
        sess.promote_candidate(1)
    sess.promote_candidate(alive[-1])
    np.testing.assert_array_equal(sess.logits(1)[0], got[-1])


@pytest.mark.parametrize("kw,dtype", [
    (dict(L=2, d=128, Hq=4, Hkv=2, hd=32, F=200, V=1000, pg=4, N=26, n0=7, n1=9, bulk=6), "f32"),
    (dict(L=2, d=256, Hq=4, Hkv=2, hd=64, F=512, V=1024, pg=64, N=330, n0=70, n1=130, bulk=100), "bf16"),
])
def test_small_page_pool_reuses_the_pages_of_dropped_candidates(kw, dtype):
    """Start many candidates, keep few: a pool far smaller than candidates x longest suffix is
    enough, because the pages of dropped candidates go back to the queue and are handed out
    again.  The survivors' logits are the oracle's although their later tokens sit in pages that
    held other candidates' keys before; the page table is the reference pool's, bit for bit; a
    step that would need more pages than are free is refused and changes nothing."""
    s = small_shape("pool", kw["L"], kw["d"], kw["Hq"], kw["Hkv"], kw["hd"], kw["F"], kw["V"], dtype=dtype)
    w = synth.make_weights(s, 83)
    pg, N, n0, n1, bulk = kw["pg"], kw["N"], kw["n0"], kw["n1"], kw["bulk"]
    P, B = 70, 6
    pages_full = B * -(-N // pg)
    # the smallest pool that carries 6 candidates to n0, 3 to n1 and 2 to N
    keep1, keep2 = [0, 2, 5], [2, 5]
    ref_pool = None
    for n_pool in range(1, pages_full):
        trial = opaging.PagePool(B, pg, range(n_pool))
        try:
            trial.append(n0); trial.drop([1, 3, 4]); trial.append(n1 - n0); trial.drop([0]); trial.append(N - n1)
        except MemoryError:
            continue
        ref_pool = n_pool
        break
    assert ref_pool is not None and ref_pool < pages_full // 2
    prefix = synth.tokens(12, 1, (P,), s.vocab)
    suffix = synth.tokens(12, 2, (B, N), s.vocab)
    print("case: small page pool", kw, dtype, "pool", ref_pool, "of", pages_full, flush=True)
    model = binding.Model(s, w)
    perm = np.random.default_rng(5).permutation(ref_pool).astype(np.int32)
    sess = binding.Session(model, P, B, N, pg, pool_pages=ref_pool)
    assert sess.pool_pages() == ref_pool
    sess.set_free_list(perm)
    pool = opaging.PagePool(B, pg, perm.tolist())
    sess.prefill_shared(prefix)
    alive = list(range(B))
    got = None
    t = 0
    while t < N:
        if t == n0:
            sess.drop_candidates([1, 3, 4]); pool.drop([1, 3, 4]); alive = keep1
        if t == n1:
            sess.drop_candidates([0]); pool.drop([0]); alive = keep2
        if t == n1 + 3:
            # a stretch written in bulk takes its pages off the same queue
            sess.prefill_suffix(suffix[alive, t:t + bulk]); pool.append(bulk)
            t += bulk
            continue
        sess.decode_step(suffix[alive, t]); pool.append(1)
        t += 1
    got = sess.logits(len(alive))
    tab, n = sess.page_table()
    held = -(-N // pg)
    assert [int(x) for x in n[:B]] == [held if b in alive else 0 for b in range(B)]
    for b in alive:
        assert tab[b, :held].tolist() == pool.table(b)
    reused = set(pool.table(2)) | set(pool.table(5))
    assert len(reused) == 2 * held and max(reused) < ref_pool
    want_pl, want = oracle_shared(s, w, prefix, suffix[alive])
    fl = oracle_shared(s, w, prefix, suffix[alive], exact=False)[1] if dtype == "bf16" else None
    assert_logits_close(got[None], want[-1:], dtype, "survivors after page reuse", None if fl is None else fl[-1:])
    # the pool is used up to within what one more boundary needs: a fresh set of 6 candidates
    # cannot start beyond it, and the refusal leaves the session as it was
    sess.reset_candidates()
    many = ref_pool // B * pg                                         # tokens all 6 can hold
    for t in range(min(many, N)):
        sess.decode_step(suffix[:, t])
    if many < N:
        before = sess.logits(B)
        with pytest.raises(binding.McError) as ei:
            sess.decode_step(suffix[:, many])
        assert ei.value.code == -3
        np.testing.assert_array_equal(sess.logits(B), before)
        sess.drop_candidates([0, 1, 2, 3])
        sess.decode_step(suffix[[4, 5], many])                        # goes on once pages are free
        want2 = oracle_shared(s, w, prefix, suffix[[4, 5], :many + 1])[1]
        fl2 = oracle_shared(s, w, prefix, suffix[[4, 5], :many + 1], exact=False)[1] if dtype == "bf16" else None
        assert_logits_close(sess.logits(2)[None], want2[-1:], dtype, "after a refused step",
                            None if fl2 is None else fl2[-1:])


@pytest.mark.parametrize("kw,dtype", [
    (dict(L=2, d=128, Hq=4, Hkv=2, hd=32, F=200, V=1000, pg=4, lens=[5, 1, 9, 4, 8], steps=9, drop_at=4, chunk=0), "f32"),
    (dict(L=2, d=256, Hq=4, Hkv=2, hd=64, F=512, V=1024, pg=64, lens=[70, 3, 130, 63, 65], steps=66, drop_at=40, chunk=160), "bf16"),
    (dict(L=2, d=256, Hq=8, Hkv=2, hd=128, F=512, V=1024, pg=64, lens=[1, 127, 64, 33], steps=4, drop_at=2, chunk=0), "bf16"),
])
def test_candidates_of_different_lengths(kw, dtype):
    """The critic's inputs differ in length per candidate (Sec. 3.3: each candidate's own code
    and execution feedback).  After one lock-step step every candidate gets a stretch of its own
    length in one pass, then all decode on from their own positions; one is dropped on the way and
    one is promoted with its own length.  Every logits row equals the oracle's for that
    candidate's own sequence; the page table is the reference pool's."""
    s = small_shape("rag", kw["L"], kw["d"], kw["Hq"], kw["Hkv"], kw["hd"], kw["F"], kw["V"], dtype=dtype)
    w = synth.make_weights(s, 84)
    pg, lens, steps = kw["pg"], kw["lens"], kw["steps"]
    P, B, E = 50, len(lens), 6
    N = 1 + max(lens) + steps + 2
    prefix = synth.tokens(13, 1, (P,), s.vocab)
    suffix = synth.tokens(13, 2, (B, N), s.vocab)
    extra = synth.tokens(13, 3, (E,), s.vocab)
    print("case: ragged candidates", kw, dtype, flush=True)
    want = oracle_shared(s, w, prefix, suffix)[1]                         # [N, B, V]: row j of b = after j + 1 tokens
    fl = oracle_shared(s, w, prefix, suffix, exact=False)[1] if dtype == "bf16" else None

    def check(sess, alive, cur, what):
        got = sess.logits(len(alive))
        ref = np.stack([want[cur[b] - 1, b] for b in alive])
        flo = None if fl is None else np.stack([fl[cur[b] - 1, b] for b in alive])[None]
        assert_logits_close(got[None], ref[None], dtype, what, flo)
        return got

    model = binding.Model(s, w)
    sess = binding.Session(model, P + N + E, B, N, pg, kw["chunk"])
    pool = opaging.PagePool(B, pg, range(sess.pool_pages()))
    sess.prefill_shared(prefix)
    sess.decode_step(suffix[:, 0]); pool.append(1)
    cur = {b: 1 for b in range(B)}
    alive = list(range(B))
    bulk = np.zeros((B, max(lens)), np.int32)
    for b in range(B):
        bulk[b, :lens[b]] = suffix[b, 1:1 + lens[b]]
    with pytest.raises(binding.McError):
        sess.prefill_suffix_ragged(bulk, [0] + lens[1:])                  # a length of 0 is refused
    sess.prefill_suffix_ragged(bulk, lens); pool.append_each(lens)
    for b in range(B):
        cur[b] += lens[b]
    check(sess, alive, cur, "after the ragged stretch")
    gone = 1
    for t in range(steps):
        if t == kw["drop_at"]:
            sess.drop_candidates([gone]); pool.drop([gone]); alive.remove(gone)
        sess.decode_step(np.array([suffix[b, cur[b]] for b in alive])); pool.append(1)
        for b in alive:
            cur[b] += 1
        if dtype == "f32" or t in (0, kw["drop_at"], steps - 1) or t % 16 == 0:
            check(sess, alive, cur, f"step {t}")
    got = sess.logits(len(alive))
    tab, n = sess.page_table()
    for b in range(B):
        held = -(-cur[b] // pg) if b in alive else 0
        assert int(n[b]) == held and tab[b, :held].tolist() == pool.table(b), (b, n[b], held)
    # a lock-step stretch after the ragged one keeps everybody at their own positions
    more = np.stack([suffix[b, cur[b]:cur[b] + 2] for b in alive])
    if all(cur[b] + 2 <= N for b in alive):
        sess.prefill_suffix(more); pool.append(2)
        for b in alive:
            cur[b] += 2
        got = check(sess, alive, cur, "lock-step stretch on ragged candidates")
    # promote a candidate that is not the longest: its own length moves into the prefix
    keep = min(alive, key=lambda b: cur[b])
    sess.promote_candidate(keep)
    np.testing.assert_array_equal(sess.logits(1)[0], got[alive.index(keep)])
    sess.extend_shared(extra)
    grown = np.concatenate([prefix, suffix[keep, :cur[keep]], extra])
    nxt = synth.tokens(13, 4, (2, 3), s.vocab)
    pl = sess.logits(1)[0]
    steps2 = _decode_all(sess, nxt)
    check_against_oracle(s, w, grown, nxt, pl, steps2)


def test_ragged_candidates_sample_on_the_device_and_score(tiny):
    """Candidates of different lengths: tokens drawn on the device feed the next step exactly as
    tokens passed from the host do, and scoring leaves the ragged decode state alone."""
    wl, w = tiny
    s = wl.shape
    prefix = synth.prefix_tokens(wl, 40)
    model = binding.Model(s, w)
    B = 4
    lens = [3, 1, 6, 4]
    bulk = synth.tokens(14, 1, (B, max(lens)), s.vocab)
    us = synth.step_uniforms(wl, B, 3)
    a = binding.Session(model, 40, B, 16, wl.page_tokens)
    b = binding.Session(model, 40, B, 16, wl.page_tokens)
    for sess in (a, b):
        sess.prefill_shared(prefix)
        sess.prefill_suffix_ragged(bulk, lens)
    for t in range(3):
        toks = a.sample(B, wl.temperature, wl.top_k, us[t])
        b.sample(B, wl.temperature, wl.top_k, us[t], want_tokens=False)     # ids stay on the device
        if t == 1:                                                          # scoring in between changes nothing
            lp, sc, rk = b.score_candidates(synth.tokens(14, 2, (B, 5), s.vocab), np.array([5, 2, 4, 1], np.int32),
                                            np.array([3, 7, 11], np.int32), np.array([0.0, 1.0, 2.0], np.float32), 1.0)
            assert np.all(np.isfinite(lp)) and sorted(rk.tolist()) == list(range(B))
            b.decode_step(toks)                                             # scoring consumed the pending logits' sample
        else:
            b.decode_step(None, B)
        a.decode_step(toks)
        np.testing.assert_array_equal(a.logits(B), b.logits(B))
    ta, na = a.page_table()
    tb, nb = b.page_table()
    np.testing.assert_array_equal(ta, tb)
    assert [int(x) for x in na[:B]] == [-(-(l + 3) // wl.page_tokens) for l in lens]


def test_drop_candidates_with_tokens_pending_on_the_device(tiny):
    wl, w = tiny
    s = wl.shape
    prefix = synth.prefix_tokens(wl, 40)
    model = binding.Model(s, w)
    B = 4
    us = synth.step_uniforms(wl, B, 2)
    a = binding.Session(model, 40, B, 8, wl.page_tokens)
    b = binding.Session(model, 40, B, 8, wl.page_tokens)
    for sess in (a, b):
        sess.prefill_shared(prefix)
    toks = a.sample(B, wl.temperature, wl.top_k, us[0])
    b.sample(B, wl.temperature, wl.top_k, us[0], want_tokens=False)   # ids stay on the device
    a.decode_step(toks)
    b.decode_step(None, B)
    toks = a.sample(B, wl.temperature, wl.top_k, us[1])
    b.sample(B, wl.temperature, wl.top_k, us[1], want_tokens=False)
    a.drop_candidates([0, 2])
    b.drop_candidates([0, 2])
    a.decode_step(toks[[1, 3]])
    b.decode_step(None, 2)
    np.testing.assert_array_equal(a.logits(2), b.logits(2))
    with pytest.raises(binding.McError):
        a.drop_candidates([1, 3])                                     # one candidate must stay



# ---------------------------------------------------------------- candidates that sit out and come back
@pytest.mark.parametrize("kw,dtype", [
    (dict(L=2, d=128, Hq=4, Hkv=2, hd=32, F=200, V=1000, pg=4), "f32"),
    (dict(L=2, d=256, Hq=4, Hkv=2, hd=64, F=512, V=1024, pg=64), "bf16"),
])
def test_pause_and_resume_candidates(kw, dtype):
    """Candidates sit out some steps (keeping pages and tokens) and come back at their own length.
    Every logits row of every candidate equals the oracle's for that candidate's own sequence; the
    page table equals the reference pool's after the same events; pending results of the others
    survive a pause; state errors are refused."""
    s = small_shape("pause", kw["L"], kw["d"], kw["Hq"], kw["Hkv"], kw["hd"], kw["F"], kw["V"], dtype=dtype)
    w = synth.make_weights(s, 84)
    pg = kw["pg"]
    P, B, N = 50, 5, 2 * pg + 9
    prefix = synth.tokens(12, 1, (P,), s.vocab)
    suffix = synth.tokens(12, 2, (B, N), s.vocab)
    print("case: pause / resume", kw, dtype, flush=True)
    model = binding.Model(s, w)
    sess = binding.Session(model, P, B, N, pg)
    sess.prefill_shared(prefix)
    pool = opaging.PagePool(B, pg, range(sess.pool_pages()))
    alive, fed = list(range(B)), [0] * B            # tokens each candidate has consumed
    rows_of = {b: [] for b in range(B)}

    def step():
        sess.decode_step(np.array([suffix[b, fed[b]] for b in alive], np.int32))
        pool.append(1)
        lg = sess.logits(len(alive))
        for i, b in enumerate(alive):
            fed[b] += 1
            rows_of[b].append(lg[i])
        return lg

    # events: (steps to run first, "pause" / "resume", ids)
    events = [(3, "pause", [1, 3]), (pg, "resume", [3]), (2, "pause", [0]), (pg - 1, "resume", [0, 1]), (4, None, None)]
    for n_steps, what, ids in events:
        for _ in range(n_steps):
            lg = step()
        if what == "pause":
            before = sess.logits(len(alive))
            sess.pause_candidates(ids); pool.pause(ids)
            keep = [i for i, b in enumerate(alive) if b not in ids]
            alive = [b for b in alive if b not in ids]
            np.testing.assert_array_equal(sess.logits(len(alive)), before[keep])     # the others' pending rows moved up
            for call in (lambda: sess.pause_candidates(ids[:1]), lambda: sess.drop_candidates(ids[:1]),
                         lambda: sess.promote_candidate(ids[0]), lambda: sess.resume_candidates([alive[0]])):
                with pytest.raises(binding.McError):
                    call()
        elif what == "resume":
            sess.resume_candidates(ids); pool.resume(ids)
            alive = sorted(alive + ids)
            with pytest.raises(binding.McError) as e:      # nothing is pending after a resume
                sess.sample(len(alive), 0.8, 50, np.zeros(len(alive), np.float32))
            assert e.value.code == -2
            with pytest.raises(binding.McError):
                sess.decode_step(None, len(alive))
    assert sorted(alive) == list(range(B)) and len(set(fed)) > 1
    want_pl, want = oracle_shared(s, w, prefix, suffix)              # [N, B, V]
    fl = oracle_shared(s, w, prefix, suffix, exact=False)[1] if dtype == "bf16" else None
    for b in range(B):
        assert len(rows_of[b]) == fed[b]
        assert_logits_close(np.stack(rows_of[b]), want[:fed[b], b], dtype, f"pause / resume, candidate {b}: {fed[b]} steps",
                            None if fl is None else fl[:fed[b], b])
    tab, n = sess.page_table()
    for b in range(B):
        held = -(-fed[b] // pg)
        assert int(n[b]) == held and tab[b, :held].tolist() == pool.table(b)
    # a reset forgets the paused ones as well
    sess.pause_candidates([2])
    sess.reset_candidates()
    with pytest.raises(binding.McError):
        sess.resume_candidates([2])


def test_oversample_then_filter_by_reward_score():
    """The search loop's call sequence on one session (Sec. 3.3, value-guided search: expand many,
    keep the promising): start 8 candidates, decode a stretch free-running, score what each has
    written so far with mc_score_candidates, drop the four lowest-ranked, decode on, promote the
    best survivor into the shared prefix and start a new round.  Scoring must leave the decode
    state alone, the ranks must be the oracle's ranking of the device scores, and every logits row
    must equal the oracle's on that candidate's own (sampled) sequence."""
    wl = synth.WORKLOADS["tiny"]
    s = wl.shape
    w = synth.make_weights(s, wl.seed_weights)
    P, B, N1, N2 = 40, 8, 6, 5
    prefix = synth.prefix_tokens(wl, P)
    us = synth.step_uniforms(wl, B, N1 + N2 + 1)
    model = binding.Model(s, w)
    sess = binding.Session(model, P + N1 + N2, B, N1 + N2, 4)
    sess.prefill_shared(prefix)
    seqs = [[] for _ in range(B)]
    rows = [[] for _ in range(B)]
    alive = list(range(B))

    def run(n, t0):
        for t in range(n):
            toks = sess.sample(len(alive), wl.temperature, wl.top_k, us[t0 + t][:len(alive)])
            sess.decode_step(None, len(alive))
            lg = sess.logits(len(alive))
            for i, b in enumerate(alive):
                seqs[b].append(int(toks[i]))
                rows[b].append(lg[i])

    run(N1, 0)
    ids = synth.reward_token_ids(wl, 5)
    vals = np.arange(5, dtype=np.float32)
    so_far = np.array([seqs[b] for b in alive], np.int32)
    pending = sess.logits(len(alive))
    lp, sc, rk = sess.score_candidates(so_far, [N1] * B, ids, vals, 0.7)
    assert list(rk) == list(osamp.rank(sc))
    worst = [alive[i] for i in rk[B // 2:]]
    # scoring overwrote the pending logits buffer: the next sample needs a decode step first; the
    # decode state itself is untouched, so feeding the last sampled tokens again is not needed:
    # drop the losers, then go on from host tokens
    sess.drop_candidates(sorted(worst))
    alive = [b for b in alive if b not in worst]
    nxt = np.array([osamp.sample(pending[list(range(B)).index(b)], wl.temperature, wl.top_k, float(us[N1][i]))[0]
                    for i, b in enumerate(alive)], np.int32)
    sess.decode_step(nxt)
    lg = sess.logits(len(alive))
    for i, b in enumerate(alive):
        seqs[b].append(int(nxt[i])); rows[b].append(lg[i])
    run(N2 - 1, N1 + 1)
    # every row against the oracle on the candidate's own sequence
    cfg = oracle_config(s)
    plog, pcache = otf.forward(cfg, w, prefix)
    for b in range(B):
        want = otf.forward(cfg, w, np.array(seqs[b]), pcache.copy())[0]
        assert_logits_close(np.stack(rows[b]), want, "f32", f"oversample / filter, candidate {b}")
    # the reward read-out of the scored stretch against the oracle
    for i in range(B):
        want_lp = osamp.reward_logprobs(otf.forward(cfg, w, so_far[i], pcache.copy())[0][-1], ids)
        np.testing.assert_allclose(lp[i], want_lp, rtol=0, atol=1e-4)
    best = alive[0]
    sess.promote_candidate(best)
    grown = np.concatenate([prefix, np.array(seqs[best], np.int32)])
    sess.decode_step(np.array([1, 2, 3], np.int32))
    want = otf.forward(cfg, w, grown)[1]
    got = sess.logits(3)
    for i, tok in enumerate([1, 2, 3]):
        ref = otf.forward(cfg, w, np.array([tok]), want.copy())[0][0]
        assert_logits_close(got[i][None], ref[None], "f32", "new round on the promoted prefix")
