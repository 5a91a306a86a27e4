"""Writes tests/golden/fullsize_<workload>.npz: oracle logits of the full-size workloads.

The 8B, 8B-reranking and 32B workloads at full depth, width, vocabulary and prefix length cost
the float64 oracle 0.1 to 1.4 PFLOP each, minutes to hours of CPU time: too slow to run inside
the GPU test suite.  This script runs the oracle once, here, on a seeded subset of (candidate,
step) pairs (teacher-forced suffixes, so any subset is legal) and stores what the GPU tests
compare against.  It calls only `oracle/` and the seeded input generator; nothing stored comes
from the GPU path.

Per workload it computes the logits twice: exact (nothing rounded) and with bf16 activation
tensors (the oracle's own reading of "bf16 activations": its distance from the exact logits is
the noise floor of bf16 arithmetic at that depth).  Stored per row (one row = the logits of one
candidate after one step, or of the last prefix position):
  * exact and bf16-mode logits at a seeded sample of vocabulary columns (float32);
  * over the whole vocabulary: the exact top-64 (ids, values), the exact log-sum-exp, and the
    bf16-mode row's max-abs / relative-L2 distance from the exact row.

Weights are generated layer by layer and widened to float64 once per layer; all sequences go
through a layer before the next layer is generated (`forward_many`), which is
`oracle.transformer.forward_shared` with the loops over layers and candidates exchanged
(tests/test_oracle_pins.py checks that the two agree to float64 rounding on a small shape).

Usage: python tests/golden/make_fullsize_golden.py <variant> ...   (variants: see VARIANTS; the
matrix library's thread count comes from OMP_NUM_THREADS / OPENBLAS_NUM_THREADS)
"""
from __future__ import annotations

import json
import os
import sys
import time

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from oracle import sampling as osamp  # noqa: E402
from oracle import transformer as otf  # noqa: E402
from paper_2601_05475_amd import synth  # noqa: E402

N_TOP = 64

# name -> (workload, layers or None = all, prefix length or None = the workload's, sampled columns)
VARIANTS = {
    "1b": ("1b", None, None, 2048),
    "8b": ("8b", None, None, 2048),
    "8b-twin": ("8b", 2, None, 1024),
    "8b-rerank": ("8b-rerank", None, None, 2048),
    "8b-rerank-twin": ("8b-rerank", 2, None, 2048),
    # full depth costs the float64 oracle 2.4 PFLOP and 1.4e12 softmax elements at the workload's
    # 16384-token prefix (more than a day on the 8-core host that writes these files): the
    # full-depth file is cut to a 4096-token prefix (2.6 hours), 8 candidates at steps 1 and 2 and
    # two that cross a page; the two-layer twin keeps all 16384 prefix tokens, 64 candidates, 1024 steps
    "32b": ("32b", None, 4096, 2048),
    "32b-twin": ("32b", 2, None, 1024),
}


def plan(name: str):
    """(workload, shape, prefix length, rows, sampled columns) with rows = list of (candidate,
    step); candidate -1 = last prefix position.  Step t (1-based) = the logits after the
    candidate's t-th suffix token."""
    wl_name, layers, prefix_len, n_cols = VARIANTS[name]
    wl = synth.WORKLOADS[wl_name]
    s = wl.shape if layers is None else wl.shape.with_layers(layers)
    B, N = wl.n_cands, wl.n_steps
    pg = wl.page_tokens
    if name == "1b":
        rows = [(b, t) for b in range(B) for t in (1, 2, pg, pg + 1)] + [(b, t) for b in (0, 7, 15) for t in (N - 1, N)]
    elif name == "8b":
        rows = [(b, t) for b in range(B) for t in (1, 2)] + [(b, t) for b in (0, 9, 18, 31) for t in (pg, pg + 1, N - 1, N)]
    elif name == "8b-twin":
        rows = [(b, t) for b in range(B) for t in (1, 2, pg - 1, pg, pg + 1, 2 * pg, 2 * pg + 1, N // 2, N // 2 + 1, N - 1, N)]
    elif name == "8b-rerank":
        # eight of the 64 suffixes at full depth (each costs the oracle 14 TFLOP and 1.7e10 softmax
        # elements per precision); the two-layer twin covers all 64
        rows = [(b, N) for b in (0, 9, 22, 31, 40, 47, 54, 63)]
    elif name == "8b-rerank-twin":
        rows = [(b, N) for b in range(B)]
    elif name == "32b":
        rows = [(b, t) for b in range(0, B, 8) for t in (1, 2)] + [(b, t) for b in (5, 63) for t in (pg, pg + 1)]
    elif name == "32b-twin":
        deep = (0, 9, 18, 27, 36, 45, 54, 63)
        rows = [(b, t) for b in range(B) for t in (1, 2, pg - 1, pg, pg + 1)] + \
               [(b, t) for b in deep for t in (2 * pg, 2 * pg + 1, N // 2, N // 2 + 1, N - 1, N)]
    else:
        raise ValueError(name)
    return wl, s, (prefix_len or wl.prefix_len), [(-1, 0)] + rows, n_cols


def lazy_f64(a: np.ndarray) -> np.ndarray:
    return (synth.bf16_bits_to_f32(a) if a.dtype == np.uint16 else a).astype(np.float64)


def forward_many(cfgs, shape, seed, prefix, suffixes, log=print):
    """For every oracle configuration in `cfgs` (same shape, different activation precision):
    logits of the last prefix position and of every position of every suffix (a dict
    candidate -> token array).  Returns [per cfg: (prefix_last [V], {cand: [n, V]})].

    Exactly forward_shared's arithmetic: each sequence is [prefix ; suffix], the prefix's keys
    and values are computed once per layer and every candidate continues from them."""
    P = len(prefix)
    embed = synth.normal(seed, synth._ST_EMBED, (shape.vocab, shape.d_model), 0.0, 0.02, shape.dtype)
    xs_p = [lazy_f64(embed[prefix]) for _ in cfgs]
    xs_s = [{b: lazy_f64(embed[t]) for b, t in suffixes.items()} for _ in cfgs]
    del embed
    pos_p = np.arange(P)
    t0 = time.time()
    for l in range(shape.n_layers):
        lw = {k: lazy_f64(v) for k, v in synth.make_layer(shape, seed, l).items()}
        for ci, cfg in enumerate(cfgs):
            xs_p[ci], kP, vP = otf.layer_forward(cfg, lw, xs_p[ci], pos_p, None, None)
            for b, toks in suffixes.items():
                xs_s[ci][b], _, _ = otf.layer_forward(cfg, lw, xs_s[ci][b], P + np.arange(len(toks)), kP, vP)
            del kP, vP
        log(f"  layer {l + 1}/{shape.n_layers} done, {time.time() - t0:.0f} s", flush=True)
    head = {"final_norm": lazy_f64(synth.normal(seed, synth._ST_FINAL_NORM, (shape.d_model,), 1.0, 0.02, shape.dtype)),
            "lm_head": lazy_f64(synth.normal(seed, synth._ST_LM_HEAD, (shape.vocab, shape.d_model), 0.0, 0.02, shape.dtype))}
    return [(otf.lm_logits(cfg, head, xs_p[ci][-1:])[0], {b: xs_s[ci][b] for b in suffixes}, head) for ci, cfg in enumerate(cfgs)]


def make(name: str, out_dir: str = HERE):
    wl, s, P, rows, n_cols = plan(name)
    prefix = synth.prefix_tokens(wl)[:P]
    suffix_all = synth.suffix_tokens(wl)
    need = {}
    for b, t in rows:
        if b >= 0:
            need[b] = max(need.get(b, 0), t)
    suffixes = {b: suffix_all[b, :n] for b, n in sorted(need.items())}
    mk = lambda act: otf.Config(s.n_layers, s.d_model, s.n_q_heads, s.n_kv_heads, s.head_dim, s.d_ffn, s.vocab,
                                s.rope_base, s.rms_eps, act)
    cfgs = [mk("f64"), mk("bf16")]
    print(f"{name}: {s.n_layers} layers, prefix {len(prefix)}, {len(suffixes)} suffixes of up to "
          f"{max(need.values())} tokens ({sum(need.values())} suffix rows), {len(rows)} stored rows", flush=True)
    res = forward_many(cfgs, s, wl.seed_weights, prefix, suffixes)
    cols = np.sort(np.random.default_rng(wl.seed_tokens).choice(s.vocab, n_cols, replace=False)).astype(np.int32)
    R = len(rows)
    exact = np.empty((R, n_cols), np.float32)
    floor = np.empty((R, n_cols), np.float32)
    top_ids = np.empty((R, N_TOP), np.int32)
    top_vals = np.empty((R, N_TOP), np.float32)
    lse = np.empty(R)
    floor_err = np.empty(R)
    floor_rel = np.empty(R)
    reward_ids = synth.reward_token_ids(wl, 8)
    lp_exact = np.empty((R, 8))
    lp_floor = np.empty((R, 8))
    for ri, (b, t) in enumerate(rows):
        full = []
        for ci, cfg in enumerate(cfgs):
            plast, xs, head = res[ci]
            full.append(plast if b < 0 else otf.lm_logits(cfg, head, xs[b][t - 1:t])[0])
        e, f = full
        exact[ri], floor[ri] = e[cols], f[cols]
        order = np.lexsort((np.arange(s.vocab), -e))[:N_TOP]
        top_ids[ri], top_vals[ri] = order, e[order]
        lse[ri] = e.max() + np.log(np.sum(np.exp(e - e.max())))
        floor_err[ri] = np.abs(f - e).max()
        floor_rel[ri] = np.linalg.norm(f - e) / np.linalg.norm(e)
        lp_exact[ri] = osamp.reward_logprobs(e, reward_ids)
        lp_floor[ri] = osamp.reward_logprobs(f, reward_ids)
    meta = dict(variant=name, workload=VARIANTS[name][0], n_layers=s.n_layers, prefix_len=int(P), rows=rows,
                n_cols=n_cols, n_top=N_TOP, reward_ids=reward_ids.tolist(),
                note="exact = float64 oracle, nothing rounded; floor = the oracle with bf16 activation tensors")
    path = os.path.join(out_dir, f"fullsize_{name}.npz")
    np.savez_compressed(path, meta=json.dumps(meta), cols=cols, exact=exact, floor=floor, top_ids=top_ids,
                        top_vals=top_vals, lse=lse, floor_err=floor_err, floor_rel=floor_rel,
                        lp_exact=lp_exact, lp_floor=lp_floor)
    print(f"wrote {path} ({os.path.getsize(path) / 1e6:.1f} MB); floor max-abs {floor_err.max():.3e}, rel {floor_rel.max():.3e}",
          flush=True)


if __name__ == "__main__":
    for nm in sys.argv[1:] or list(VARIANTS):
        make(nm)
