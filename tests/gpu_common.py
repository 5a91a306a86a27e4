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
#
# A maximum that grows with depth loses its power to discriminate, so three statistics with power
# stand beside it wherever a floor is given, all against the exact oracle:
#   * RMS error of the device / RMS error of the floor, over all rows <= RMS_RATIO, per row <=
#     RMS_RATIO_ROW (a row's error is one realisation of the hidden state's rounding noise, so single
#     rows scatter more than the aggregate);
#   * |mean signed error| <= BIAS_FRAC * RMS error (rounding noise has no sign; a dropped term,
#     a wrong scale or a truncating conversion has);
#   * the fraction of logits beyond the stated max-abs bound <= FRAC_SLACK * the fraction of the
#     floor's errors beyond that bound / RMS_RATIO (+ FRAC_EPS): a tail no heavier than the
#     floor's once the allowed ratio of the RMS errors is taken out (a tail fraction at a fixed
#     threshold of ~2.5 sigma triples when sigma grows by 13 %, so the raw fractions cannot be
#     compared).
TOL = {"f32": (1e-4, 1e-4), "bf16": (2e-2, 1e-2)}
FLOOR_SLACK = 1.5
RMS_RATIO, RMS_RATIO_ROW = 1.25, 1.6
BIAS_FRAC = 0.1
FRAC_SLACK, FRAC_EPS = 1.5, 1e-3
SAMPLE_MARGIN = 1e-5      # |u - c_i| below this: device expf vs libm may flip the pick

# one record per bf16 comparison of this test run; tests/conftest.py writes them out as a table
PARITY_RECORDS = []


def _rows(a):
    a = np.asarray(a, np.float64)
    return a.reshape(-1, a.shape[-1])


def error_stats(x, want, atol):
    """Distance of logits x from the exact ones: max-abs, worst per-row relative L2, RMS per row,
    mean signed error, fraction of elements beyond atol."""
    x, want = _rows(x), _rows(want)
    d = x - want
    return dict(err=float(np.abs(d).max()),
                rel=float((np.linalg.norm(d, axis=1) / np.linalg.norm(want, axis=1)).max()),
                rms_rows=np.sqrt(np.mean(d * d, axis=1)), rms=float(np.sqrt(np.mean(d * d))),
                mean=float(d.mean()), frac=float(np.mean(np.abs(d) > atol)))


def _errs(got, want):
    st = error_stats(got, want, 0.0)
    return st["err"], st["rel"]


def assert_logits_close(got, want, dtype, what="", floor=None):
    """got vs the exact oracle `want`; `floor`: the bf16-tensor oracle's logits (bf16 paths)."""
    atol, rtol = TOL[dtype]
    g = error_stats(got, want, atol)
    err, rel = g["err"], g["rel"]
    if floor is None:
        assert err <= atol and rel <= rtol, f"{what}: max abs {err:.3e} (bound {atol:.3e}), rel L2 {rel:.3e} (bound {rtol:.3e})"
        return err, rel
    f = error_stats(floor, want, atol)
    f_tail = error_stats(floor, want, atol / RMS_RATIO)["frac"]
    a_bound, r_bound = max(atol, FLOOR_SLACK * f["err"]), max(rtol, FLOOR_SLACK * f["rel"])
    ratio = g["rms"] / f["rms"]
    ratio_row = float((g["rms_rows"] / f["rms_rows"]).max())
    bias = abs(g["mean"]) / g["rms"]
    which = "stated" if (f["err"] * FLOOR_SLACK <= atol and f["rel"] * FLOOR_SLACK <= rtol) else "floor"
    rec = dict(what=what, rows=_rows(got).shape[0], cols=_rows(got).shape[1], err=err, rel=rel, floor_err=f["err"],
               floor_rel=f["rel"], bound_err=a_bound, bound_rel=r_bound, which=which, rms_ratio=ratio,
               rms_ratio_row=ratio_row, bias=bias, frac=g["frac"], floor_frac=f["frac"], floor_frac_scaled=f_tail)
    PARITY_RECORDS.append(rec)
    print("PARITY " + " ".join(f"{k}={v:.3e}" if isinstance(v, float) else f"{k}={v}" for k, v in rec.items()), flush=True)
    assert err <= a_bound and rel <= r_bound, \
        f"{what}: max abs {err:.3e} (bound {a_bound:.3e}), rel L2 {rel:.3e} (bound {r_bound:.3e}) [{which} bound]"
    assert ratio <= RMS_RATIO, f"{what}: RMS error {g['rms']:.3e} is {ratio:.2f} x the bf16 noise floor's {f['rms']:.3e}"
    assert ratio_row <= RMS_RATIO_ROW, f"{what}: a row's RMS error is {ratio_row:.2f} x the floor's"
    assert bias <= BIAS_FRAC, f"{what}: mean signed error {g['mean']:.3e} is {bias:.2f} of the RMS error"
    assert g["frac"] <= FRAC_SLACK * f_tail + FRAC_EPS, \
        f"{what}: {g['frac']:.2e} of the logits beyond {atol:g}, the floor has {f_tail:.2e} beyond {atol / RMS_RATIO:g}"
    return err, rel


# Attention outputs are compared per (row, head) by relative L2 error: with N(0, 1) keys and values
# a long softmax is nearly uniform and its output small (rms ~ 1/sqrt(keys)), so an absolute bound
# wide enough for bf16 rounding would not see a lost 32-key block; a relative one does (one block
# of 4608 keys carries ~8 % of the output's norm).  bf16 outputs are rounded to 8 bits (2^-9
# relative per element) and so are the probabilities that meet the values.
ATT_REL = {"f32": 2e-5, "bf16": 1e-2}


def rel_l2(got, want):
    got, want = np.asarray(got, np.float64), np.asarray(want, np.float64)
    return float(np.linalg.norm(got - want) / np.linalg.norm(want))


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
