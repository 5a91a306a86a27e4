"""Shared pieces of the GPU parity tests."""
import numpy as np

from oracle import sampling as osamp
from oracle import transformer as otf
from paper_2601_05475_amd import binding, synth
from helpers import oracle_config

# Logit tolerances: fp32 path 1e-4 (absolute and per-row relative L2); bf16 path max-abs 2e-2
# and per-row relative L2 1e-2.
#
# bf16 models hold every activation tensor in bf16.  That arithmetic alone moves the logits away
# from the exact ones, by an amount that grows with depth and that no implementation can avoid;
# the oracle measures it by rounding the same tensors in float64 ("noise floor").  Two bf16
# computations that differ only in the last bits of fp32 decorrelate to that same level within a
# few layers (a difference d before a rounding becomes sqrt(d * ulp) after it), so the floor is
# also the best possible agreement with the rounding oracle.  The bar for a bf16 path is
# therefore: within the stated tolerance, or within FLOOR_SLACK times the floor where the floor
# itself is beyond it.
TOL = {"f32": (1e-4, 1e-4), "bf16": (2e-2, 1e-2)}
FLOOR_SLACK = 1.5
SAMPLE_MARGIN = 1e-5      # |u - c_i| below this: device expf vs libm may flip the pick


def _errs(got, want):
    got = np.asarray(got, np.float64).reshape(-1, got.shape[-1])
    want = np.asarray(want, np.float64).reshape(-1, want.shape[-1])
    return np.abs(got - want).max(), (np.linalg.norm(got - want, axis=1) / np.linalg.norm(want, axis=1)).max()


def assert_logits_close(got, want, dtype, what="", floor=None):
    """got vs the exact oracle `want`; `floor`: the bf16-tensor oracle's logits (bf16 paths)."""
    atol, rtol = TOL[dtype]
    err, rel = _errs(got, want)
    if floor is not None:
        ferr, frel = _errs(floor, want)
        atol, rtol = max(atol, FLOOR_SLACK * ferr), max(rtol, FLOOR_SLACK * frel)
    assert err <= atol and rel <= rtol, f"{what}: max abs {err:.3e} (bound {atol:.3e}), rel L2 {rel:.3e} (bound {rtol:.3e})"
    return err, rel


def check_sampler_on_logits(logits_row, temperature, top_k, u, got_tok, got_topk=None):
    """The oracle sampler on the very logits the device sampled from: ids must be equal, except
    where the uniform sits within SAMPLE_MARGIN of a cumulative-probability boundary."""
    tok, ids, margin = osamp.sample(logits_row, temperature, top_k, float(u))
    if got_topk is not None:
        assert list(got_topk) == list(ids), "top-k id list differs"
    if tok != got_tok:
        assert margin < SAMPLE_MARGIN, f"token {got_tok} != oracle {tok}, margin {margin:.2e}"
        return False
    return True


def teacher_forced_gpu(shape, weights, prefix, suffix, page_tokens, chunk_rows=0, max_prefix=None,
                       max_suffix=None, free_list=None, prefix_splits=0):
    """Prefill + N decode steps with given suffix tokens [B, N]; returns (prefix_logits [V],
    step_logits [N, B, V], session, model)."""
    B, N = suffix.shape
    model = binding.Model(shape, weights)
    sess = binding.Session(model, max_prefix or len(prefix), B, max_suffix or max(N, 1), page_tokens, chunk_rows)
    if free_list is not None:
        sess.set_free_list(free_list)
    if prefix_splits:
        sess.set_prefix_splits(prefix_splits)
    sess.prefill_shared(prefix)
    pl = sess.logits(1)[0]
    steps = []
    for t in range(N):
        sess.decode_step(suffix[:, t])
        steps.append(sess.logits(B))
    return pl, np.stack(steps) if steps else np.zeros((0, B, shape.vocab), np.float32), sess, model


def oracle_shared(shape, weights, prefix, suffix, exact=True):
    """Oracle logits: (prefix last row [V], steps [N, B, V]).  exact=False: bf16 activation tensors."""
    cfg = oracle_config(shape, exact=exact)
    w = synth.weights_as_f32(weights)
    plast, out = otf.forward_shared(cfg, w, prefix, suffix)      # out [B, N, V]
    return plast, out.transpose(1, 0, 2)


def check_against_oracle(shape, weights, prefix, suffix, pl, steps):
    """Prefix and decode logits of the device against the oracle, to the bar of assert_logits_close."""
    want_pl, want = oracle_shared(shape, weights, prefix, suffix)
    if shape.dtype == "bf16":
        fl_pl, fl = oracle_shared(shape, weights, prefix, suffix, exact=False)
    else:
        fl_pl = fl = None
    assert_logits_close(pl[None], want_pl[None], shape.dtype, "prefix logits",
                        None if fl_pl is None else fl_pl[None])
    if steps.shape[0]:
        assert_logits_close(steps, want, shape.dtype, "decode logits", fl)
    return want_pl, want
