"""Benchmark of the shared-prefix decode hot path on one MI355X.

A "step" is one pass of the whole hot path for one batch: draw the next token of every
candidate (temperature / top-k sampling from the pending logits) and run one decode step for
all B candidates (embedding, 32 x {norm, QKV, RoPE + KV write, shared-prefix attention, O,
norm, SwiGLU FFN}, final norm, LM head).  The workload is the 8B-shape headline configuration:
B = 32 candidates on a 4096-token shared prefix, free-running sampling at T = 0.7 / top-k 50,
seeded synthetic weights and token ids.  The prefix prefill is done before the timed region and
reported separately.  Everything is resident in HBM when the clock starts; nothing crosses to
the host inside the timed region (sampled ids stay on the device).

Prints ONE JSON line: the metric and its value, the per-step time, the roofline figures of the
dominant kernel and of decode attention, and the oracle's rate on the host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published
MFMA_PEAK_TFLOPS = 2500.0    # MI355X dense bf16 MFMA, published


# HBM traffic of one gate/up launch from the FETCH_SIZE / WRITE_SIZE counter runs (KiB per
# dispatch, scaled by what the same counters read for a plain copy of known size; see
# profiles/decode_8b_traffic_counters.md).  Valid for the kernel source with this hash only.
TRAFFIC_GATE_UP = {"fetch_kib": 115760.5, "fetch_scale": 2.0, "write_kib": 896.0, "write_scale": 1.0,
                   "source": "paper_2601_05475_amd/csrc/kernels_mfma.hip",
                   "sha256": "195b3cd0cc63be24d006182355f7596e3582871f57e80ab923bcf591f9c5ba36"}


# Decode attention + merge at suffix lengths 255..258 (the same two counter runs: four timed steps
# sit at the middle of the 512-step workload, whose average suffix length is 256.5).
TRAFFIC_ATTN = {"fetch_kib": 26427.5, "merge_fetch_kib": 2922.0, "write_kib": 4680.0, "merge_write_kib": 256.0,
                "fetch_scale": 2.0, "write_scale": 1.0, "suffix_len": 256.5,
                "source": "paper_2601_05475_amd/csrc/kernels_attn.hip",
                "sha256": "0ab99c8fa2d8bfba6214bf19266d40b3861557b3f9ebbff542f3b9bf4a2434f7"}


def measured_attention_traffic_bytes(workload, mean_suffix_len):
    """HBM bytes of one layer-step's decode attention (both kernels) from the counter runs; None
    off the headline workload, once the kernel source has changed since the counters were taken,
    or when this run's mean suffix length is not the one they were taken at."""
    import hashlib
    if workload != "8b" or abs(mean_suffix_len - TRAFFIC_ATTN["suffix_len"]) > 2.0:
        return None
    t = TRAFFIC_ATTN
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), t["source"])
    try:
        with open(path, "rb") as f:
            if hashlib.sha256(f.read()).hexdigest() != t["sha256"]:
                return None
    except OSError:
        return None
    return ((t["fetch_kib"] + t["merge_fetch_kib"]) * t["fetch_scale"] +
            (t["write_kib"] + t["merge_write_kib"]) * t["write_scale"]) * 1024.0


def measured_traffic_bytes(workload):
    """Counter-derived HBM bytes per gate/up launch, or None if the kernel source has changed
    since the counters were taken (or the workload is not the one they were taken on)."""
    import hashlib
    if workload != "8b":
        return None
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), TRAFFIC_GATE_UP["source"])
    try:
        with open(path, "rb") as f:
            if hashlib.sha256(f.read()).hexdigest() != TRAFFIC_GATE_UP["sha256"]:
                return None
    except OSError:
        return None
    t = TRAFFIC_GATE_UP
    return (t["fetch_kib"] * t["fetch_scale"] + t["write_kib"] * t["write_scale"]) * 1024.0


def gate_up_kernel_name(s, n_cands):
    """Which form of the weight-streaming layer the library picks for gate/up at this shape (the
    rules of csrc/kernels_mfma.hip, restated for the record's label only)."""
    if n_cands > 32:
        return "skinny_shared_kernel" if (s.d_ffn // 32 + 3) // 4 >= 160 else "skinny_linear_kernel"
    rows = s.d_ffn // 256
    if s.d_ffn % 2048 == 0 and (s.d_ffn // 32) % 256 != 0 and rows <= 64:
        return "skinny_rows_kernel"
    return "skinny_linear_kernel"


def gate_up_bytes(s, n_cands):
    """Algorithmic bytes of one gate/up launch: both weight matrices once, the activations in
    and the SwiGLU product out (bf16)."""
    return 2 * s.d_ffn * s.d_model * 2 + n_cands * s.d_model * 2 + n_cands * s.d_ffn * 2


def attention_bytes(s, n_cands, prefix_len, suffix_len):
    """Algorithmic bytes of one decode-attention launch: prefix K and V once, every candidate's
    suffix K and V once, q in and o out (bf16)."""
    kv_tok = 2 * s.n_kv_heads * s.head_dim * 2
    return prefix_len * kv_tok + n_cands * suffix_len * kv_tok + 2 * n_cands * s.n_q_heads * s.head_dim * 2


def step_bytes(s, n_cands, prefix_len, mean_suffix_len):
    """Algorithmic HBM bytes of one decode step: every weight matrix once (bf16), the shared
    prefix's keys and values once per layer, every candidate's suffix keys and values once."""
    qd, kd = s.n_q_heads * s.head_dim, s.n_kv_heads * s.head_dim
    weights = 2 * (s.n_layers * ((qd + 2 * kd) * s.d_model + s.d_model * qd + 3 * s.d_ffn * s.d_model) + s.vocab * s.d_model)
    kv = s.n_layers * (prefix_len + n_cands * mean_suffix_len) * 2 * kd * 2
    return weights + kv


def matmul_yardstick_tflops(torch):
    """An independent yardstick for the matrix-core figures: the vendor library's bf16 GEMM behind
    torch.matmul on the gate/up shape of one 8B-shape scoring chunk (8192 x 28672 x 4096), N(0, 1)
    operands.  Reported only; the library never calls it."""
    M, N, K = 8192, 28672, 4096
    a = torch.randn(M, K, device="cuda").to(torch.bfloat16)
    b = torch.randn(N, K, device="cuda").to(torch.bfloat16)
    for _ in range(3):
        torch.matmul(a, b.t())
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(10):
        torch.matmul(a, b.t())
    e1.record()
    torch.cuda.synchronize()
    return 2.0 * M * N * K * 10 / (e0.elapsed_time(e1) * 1e-3) / 1e12


def cpu_baseline(wl, weights, n_layers_sample=4, n_cands_sample=16):
    """The oracle, as it stands, on a bounded sample of the same workload: one decode step at
    suffix length 1 for `n_cands_sample` of the B candidates through `n_layers_sample` layers
    (random bf16 prefix keys/values of the real shape) plus the final norm and LM head; times are
    scaled linearly to all candidates and the full depth."""
    from oracle import transformer as otf
    from paper_2601_05475_amd import synth
    s = wl.shape
    cfg = otf.Config(s.n_layers, s.d_model, s.n_q_heads, s.n_kv_heads, s.head_dim, s.d_ffn, s.vocab,
                     s.rope_base, s.rms_eps, "bf16")
    B, P = wl.n_cands, wl.prefix_len
    n_cands_sample, n_layers_sample = min(n_cands_sample, B), min(n_layers_sample, s.n_layers)
    layers = [{k: synth.bf16_bits_to_f32(v) for k, v in weights["layers"][l].items()} for l in range(n_layers_sample)]
    head = {"final_norm": synth.bf16_bits_to_f32(weights["final_norm"]),
            "lm_head": synth.bf16_bits_to_f32(weights["lm_head"])}
    kv = [(synth.bf16_bits_to_f32(synth.normal(7, 50 + l, (P, s.n_kv_heads, s.head_dim), 0.0, 1.0, "bf16")).astype(np.float64),
           synth.bf16_bits_to_f32(synth.normal(7, 80 + l, (P, s.n_kv_heads, s.head_dim), 0.0, 1.0, "bf16")).astype(np.float64))
          for l in range(n_layers_sample)]
    x0 = synth.bf16_bits_to_f32(weights["embed"][synth.suffix_tokens(wl, B, 1)[:, 0]]).astype(np.float64)
    t0 = time.perf_counter()
    outs = []
    for b in range(n_cands_sample):            # candidates are independent sequences
        x = x0[b:b + 1]
        for l in range(n_layers_sample):
            x, _, _ = otf.layer_forward(cfg, layers[l], x, np.array([P]), kv[l][0], kv[l][1])
        outs.append(x)
    t_layers = time.perf_counter() - t0
    t0 = time.perf_counter()
    otf.lm_logits(cfg, head, np.concatenate(outs))
    t_head = time.perf_counter() - t0
    step_s = (t_layers / n_layers_sample * s.n_layers + t_head) * B / n_cands_sample
    try:
        from threadpoolctl import threadpool_info
        cores = max([i.get("num_threads", 1) for i in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    return {"value": B / step_s, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"one decode step (suffix length 1, prefix {P}) for {n_cands_sample} of {B} candidates "
                      f"through {n_layers_sample} of {s.n_layers} layers + final norm + LM head, scaled "
                      f"linearly to {B} candidates and {s.n_layers} layers ({t_layers:.1f} s layers, "
                      f"{t_head:.1f} s head measured)"}


def measured_mfma_tflops(torch, binding):
    """bf16 MFMA rate with nothing else running (every wave issues MFMAs on operands it holds),
    operands ~ N(0, 1) like the activations of the run: the practical ceiling of a GEMM here."""
    n_wg, iters = 1024, 4096
    ops = torch.randn(n_wg * 256 * 48, device="cuda").to(torch.bfloat16)
    binding.op_mfma_probe(ops, n_wg, 256)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    fl = binding.op_mfma_probe(ops, n_wg, iters)
    e1.record()
    torch.cuda.synchronize()
    return fl / (e0.elapsed_time(e1) * 1e-3) / 1e12


def measured_read_gbs(torch, binding):
    """HBM read rate of a kernel that only streams (2 GiB, 16-byte non-temporal loads), GB/s."""
    buf = torch.zeros(2 << 30, dtype=torch.uint8, device="cuda")
    word = torch.zeros(1, dtype=torch.int32, device="cuda")
    binding.op_read_probe(buf, word)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(5):
        binding.op_read_probe(buf, word)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / 5
    del buf
    return (2 << 30) / (ms * 1e-3) / 1e9


def measured_copy_gbs(torch):
    """Read + write rate of a plain device copy of 1 GiB (an elementwise kernel), GB/s."""
    src = torch.zeros(256 << 20, dtype=torch.int32, device="cuda")
    dst = torch.empty_like(src)
    for _ in range(2):
        torch.add(src, 1, out=dst)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(5):
        torch.add(src, 1, out=dst)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / 5
    del src, dst
    return 2 * (1 << 30) / (ms * 1e-3) / 1e9


def cpu_baseline_rerank(wl, weights, n_layers_sample=1, rows_sample=64):
    """The oracle on a bounded sample of the scoring workload: the last `rows_sample` positions of
    ONE candidate suffix (attending to random prefix + suffix keys of the real length) through
    `n_layers_sample` layers; scaled linearly to all rows, candidates and layers.  The LM head is
    needed for one row per candidate only and is left out."""
    from oracle import transformer as otf
    from paper_2601_05475_amd import synth
    s = wl.shape
    cfg = otf.Config(s.n_layers, s.d_model, s.n_q_heads, s.n_kv_heads, s.head_dim, s.d_ffn, s.vocab,
                     s.rope_base, s.rms_eps, "bf16")
    P, Ls, B = wl.prefix_len, wl.n_steps, wl.n_cands
    n_keys = P + Ls - rows_sample
    layers = [{k: synth.bf16_bits_to_f32(v) for k, v in weights["layers"][l].items()} for l in range(n_layers_sample)]
    kv = [(synth.bf16_bits_to_f32(synth.normal(7, 50 + l, (n_keys, s.n_kv_heads, s.head_dim), 0.0, 1.0, "bf16")).astype(np.float64),
           synth.bf16_bits_to_f32(synth.normal(7, 80 + l, (n_keys, s.n_kv_heads, s.head_dim), 0.0, 1.0, "bf16")).astype(np.float64))
          for l in range(n_layers_sample)]
    x = synth.bf16_bits_to_f32(weights["embed"][synth.suffix_tokens(wl, 1, rows_sample)[0]]).astype(np.float64)
    t0 = time.perf_counter()
    for l in range(n_layers_sample):
        x, _, _ = otf.layer_forward(cfg, layers[l], x, np.arange(n_keys, n_keys + rows_sample), kv[l][0], kv[l][1])
    t = time.perf_counter() - t0
    total = t / n_layers_sample * s.n_layers * (Ls / rows_sample) * B
    try:
        from threadpoolctl import threadpool_info
        cores = max([i.get("num_threads", 1) for i in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    return {"value": B / total, "unit": "scored candidates/s", "cores": int(cores), "kind": "oracle",
            "sample": f"the last {rows_sample} of {Ls} suffix positions of one of {B} candidates through "
                      f"{n_layers_sample} of {s.n_layers} layers ({t:.1f} s measured), scaled linearly to all "
                      f"positions, candidates and layers; LM head (one row per candidate) left out"}


def bench_rerank(args, torch, binding, synth):
    """Scoring workload: B candidate suffixes of Ls tokens on the shared prefix, expected value of
    the categorical reward read at each suffix end.  A step = one mc_score_candidates call."""
    wl = synth.WORKLOADS[args.workload]
    s = wl.shape if not args.layers else wl.shape.with_layers(args.layers)
    B, P, Ls = wl.n_cands, wl.prefix_len, wl.n_steps
    K = args.steps if args.steps_given else 3
    W = args.warmup if args.warmup_given else 1
    chunk = args.chunk_rows or 8192
    t0 = time.perf_counter()
    weights = synth.make_weights(s, wl.seed_weights)
    t_gen = time.perf_counter() - t0
    model = binding.Model(s, weights)
    sess = binding.Session(model, P, B, Ls, wl.page_tokens, chunk_rows=chunk)
    torch.cuda.synchronize()
    prefix = synth.prefix_tokens(wl)
    suffix = synth.suffix_tokens(wl)
    lens = np.full(B, Ls, np.int32)
    R = 8
    ids = synth.reward_token_ids(wl, R)
    vals = np.arange(R, dtype=np.float32)
    t0 = time.perf_counter()
    sess.prefill_shared(prefix)
    sess.sync()
    t_prefill = time.perf_counter() - t0
    for _ in range(W):
        sess.score_candidates(suffix, lens, ids, vals, 1.0)
    sess.profile_begin("linear_gate_up", 1)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(K):
        sess.score_candidates(suffix, lens, ids, vals, 1.0)     # returns after the scores are on the host
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    n_gu, ms_gu = sess.profile_end()
    sess.profile_begin("attn_prefill", 1)
    sess.score_candidates(suffix, lens, ids, vals, 1.0)
    n_at, ms_at = sess.profile_end()
    mfma_meas = measured_mfma_tflops(torch, binding)
    rows = B * Ls
    n_chunks = -(-rows // (chunk // Ls * Ls))
    m_chunk = rows / n_chunks
    gu_flops = 2.0 * m_chunk * (2 * s.d_ffn) * s.d_model
    gu_us = ms_gu * 1e3 / max(n_gu, 1)
    layer_flops = 2.0 * rows * s.d_model * ((s.n_q_heads + 2 * s.n_kv_heads) * s.head_dim + s.n_q_heads * s.head_dim + 3 * s.d_ffn)
    attn_flops = 4.0 * s.n_q_heads * s.head_dim * B * Ls * (P + Ls / 2.0)          # per layer, causal
    out = {
        "metric": "scored candidates/s (8B-shape reranking: expected categorical reward at each suffix end)",
        "value": B * K / elapsed, "unit": "candidates/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": elapsed / K * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{args.workload}: {s.n_layers} layers of the 8B shape; {B} suffixes of {Ls} tokens on a "
                               f"shared prefix of {P}; {R} reward tokens; chunks of {chunk} rows",
                   "n_cands": B, "prefix_len": P, "suffix_len": Ls, "page_tokens": wl.page_tokens},
        "roofline": {"bound": "mfma", "kernel": "gemm256_kernel<GEMM_SWIGLU> (gate/up + SwiGLU)",
                     "achieved": gu_flops / gu_us / 1e6, "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": gu_flops / gu_us / 1e6 / MFMA_PEAK_TFLOPS, "traffic": None,
                     "launches_timed": n_gu, "avg_us": gu_us, "rows_per_launch": m_chunk,
                     "peak_measured": mfma_meas, "frac_of_measured": gu_flops / gu_us / 1e6 / mfma_meas},
        "whole_pass": {"linear_flops": layer_flops * s.n_layers, "attention_flops": attn_flops * s.n_layers,
                       "achieved_tflops": (layer_flops + attn_flops) * s.n_layers / (elapsed / K) / 1e12,
                       "attention_ms_per_pass": ms_at, "attention_tflops": attn_flops * s.n_layers / (ms_at * 1e-3) / 1e12},
        "prefill_s": t_prefill, "setup_s": {"generate_weights": t_gen},
        "yardsticks": {"hbm_copy_gbs": measured_copy_gbs(torch), "mfma_matmul_tflops": matmul_yardstick_tflops(torch),
                       "mfma_probe_tflops": mfma_meas,
                       "note": "torch.matmul bf16 8192x28672x4096 (the vendor library's GEMM on the gate/up shape of "
                               "one chunk) and the library's own MFMA-only probe: reported only"},
    }
    if args.layers:
        out["invalid"] = "layer count overridden"
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline_rerank(wl, weights)
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="8b", choices=["8b", "1b", "32b", "8b-rerank"],
                    help="8b (default): the headline decode workload; 1b, 32b: the same loop on the other "
                         "decode configurations; 8b-rerank: the scoring workload")
    ap.add_argument("--layers", type=int, default=0, help="override the layer count (diagnosis only; marks the line invalid)")
    ap.add_argument("--chunk-rows", type=int, default=0, help="rows per prefill / scoring chunk")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--suffix-start", type=int, default=None,
                    help="decode workloads: write this many tokens per candidate in one untimed pass before the "
                         "steps (default: (workload steps - timed steps) / 2, which centres the timed steps on "
                         "the workload's mean suffix length)")
    ap.add_argument("--prefix-splits", type=int, default=0,
                    help="decode attention: key-axis splits of the shared prefix (0 = the library's plan; "
                         "diagnosis only, marks the line invalid)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain elementwise copy of 256 MiB (a kernel of known traffic "
                         "that hardware-counter readings are scaled by)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: the library runs on one GPU; --gpus N with N > 1 is not supported", file=sys.stderr)
        sys.exit(2)
    args.steps_given, args.warmup_given = args.steps is not None, args.warmup is not None

    import torch
    from paper_2601_05475_amd import binding, synth
    binding.load_library()                      # raises if the HIP library is not built
    if args.workload == "8b-rerank":
        return bench_rerank(args, torch, binding, synth)
    wl = synth.WORKLOADS[args.workload]
    N = wl.n_steps
    if args.steps is None:
        args.steps = N
    if args.warmup is None:
        args.warmup = 8
    s = wl.shape if not args.layers else wl.shape.with_layers(args.layers)
    B, P = wl.n_cands, wl.prefix_len
    K, W = args.steps, args.warmup
    # Fewer timed steps than the workload has: they sit in the middle of the workload, at suffix
    # lengths S0 + 1 .. S0 + K, so that their mean length (and hence the per-step cost, which is
    # linear in the suffix length) is the whole workload's.  The S0 tokens before them are written
    # in one untimed pass.
    S0 = args.suffix_start if args.suffix_start is not None else (N - K) // 2
    if K < 1 or K > N or W < 0 or S0 < 0 or K + S0 > N or W + S0 > N:
        print(f"bench.py: steps (+ suffix start) must be in [1, {N}] and warmup in [0, {N}]", file=sys.stderr)
        sys.exit(2)
    mean_len = S0 + (K + 1) / 2.0

    t0 = time.perf_counter()
    weights = synth.make_weights(s, wl.seed_weights)
    t_gen = time.perf_counter() - t0
    t0 = time.perf_counter()
    model = binding.Model(s, weights)
    sess = binding.Session(model, P, B, N, wl.page_tokens, chunk_rows=args.chunk_rows or 4096)
    if args.prefix_splits:
        sess.set_prefix_splits(args.prefix_splits)
    torch.cuda.synchronize()
    t_upload = time.perf_counter() - t0

    prefix = synth.prefix_tokens(wl)
    us = synth.step_uniforms(wl, B, N)
    t0 = time.perf_counter()
    sess.prefill_shared(prefix)
    sess.sync()
    t_prefill = time.perf_counter() - t0

    head = synth.suffix_tokens(wl, B, S0) if S0 else None

    def start_candidates():
        if S0:
            sess.prefill_suffix(head)

    def run_steps(n):
        for t in range(n):
            sess.sample(B, wl.temperature, wl.top_k, us[S0 + t], want_tokens=False)
            sess.decode_step(None, B)

    start_candidates()
    run_steps(W)
    sess.sync()
    sess.reset_candidates()
    start_candidates()
    if args.calibration_copy:
        src = torch.zeros(64 << 20, dtype=torch.int32, device="cuda")      # 256 MiB read, 256 MiB written
        dst = torch.empty_like(src)
        torch.add(src, 1, out=dst)
        torch.cuda.synchronize()
        del src, dst

    # timed region; a sample of the gate/up launches carries HIP events of its own (attached to the
    # launch: begin and end of that dispatch on the session stream): about 256 launches of a long
    # run, and never more than one per step (a bracketed launch costs the stream about 5 us: two
    # per layer-pair of a 20-step run took 2 % off the rate), in a different layer each time
    stride = max(s.n_layers + 1, (s.n_layers * K) // 256)
    sess.profile_begin("linear_gate_up", stride)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run_steps(K)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    n_gu, ms_gu = sess.profile_end()

    # second pass (untimed): the decode-attention kernels over the same K steps
    sess.reset_candidates()
    start_candidates()
    sess.profile_begin("attn_decode", stride)
    step_ms = {}
    marks = sorted({1, K // 2, K} - {0})
    for t in range(K):
        if t + 1 in marks:                       # wall time of this one step, bracketed by syncs
            torch.cuda.synchronize()
            t1 = time.perf_counter()
        sess.sample(B, wl.temperature, wl.top_k, us[S0 + t], want_tokens=False)
        sess.decode_step(None, B)
        if t + 1 in marks:
            torch.cuda.synchronize()
            step_ms[str(S0 + t + 1)] = (time.perf_counter() - t1) * 1e3
    n_at, ms_at = sess.profile_end()
    at_bytes = float(np.mean([attention_bytes(s, B, P, S0 + t + 1) for t in range(K)]))

    read_gbs = measured_read_gbs(torch, binding)
    gu_us = ms_gu * 1e3 / max(n_gu, 1)
    at_us = ms_at * 1e3 / max(n_at, 1)
    gu_gbs = gate_up_bytes(s, B) / gu_us / 1e3
    at_gbs = at_bytes / at_us / 1e3
    ms_step = elapsed / K * 1e3
    sb = step_bytes(s, B, P, mean_len)
    out = {
        "metric": f"generated tokens/s at B candidates ({args.workload.upper()}-shape decode); % HBM roofline attn",
        "value": B * K / elapsed, "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{args.workload}-shape decode: {s.n_layers} layers, d {s.d_model}, "
                               f"{s.n_q_heads}/{s.n_kv_heads} heads of {s.head_dim}, FFN {s.d_ffn}, vocab {s.vocab}; "
                               f"B={B} candidates, shared prefix {P}, {N}-step workload, timed steps at suffix lengths "
                               f"{S0 + 1}..{S0 + K} (mean {mean_len:g}; the workload's mean is {(N + 1) / 2:g}), "
                               f"T={wl.temperature}, top-k {wl.top_k}",
                   "n_cands": B, "prefix_len": P, "page_tokens": wl.page_tokens, "suffix_start": S0},
        "roofline": {"bound": "hbm", "kernel": gate_up_kernel_name(s, B) + " (gate/up + SwiGLU)",
                     "achieved": gu_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gu_gbs / HBM_PEAK_GBS,
                     "peak_measured": read_gbs, "frac_of_measured": gu_gbs / read_gbs,
                     "traffic": measured_traffic_bytes(args.workload), "algorithmic_bytes": gate_up_bytes(s, B),
                     "launches_timed": n_gu, "avg_us": gu_us,
                     # decode attention, the kernel the metric's second half names: both launches of one layer-step
                     "attn": {"bound": "hbm", "kernel": "decode_attention_kernel + decode_attention_merge_kernel",
                              "achieved": at_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": at_gbs / HBM_PEAK_GBS,
                              "traffic": measured_attention_traffic_bytes(args.workload, mean_len),
                              "algorithmic_bytes": at_bytes, "mean_suffix_len": mean_len,
                              "launches_timed": n_at, "avg_us": at_us},
                     # the whole step against the HBM roofline: algorithmic bytes of one step / its time / peak
                     "step": {"algorithmic_bytes": sb, "achieved": sb / ms_step / 1e6, "unit": "GB/s",
                              "frac": sb / ms_step / 1e6 / HBM_PEAK_GBS}},
        "step_frac": sb / ms_step / 1e6 / HBM_PEAK_GBS,
        "step_ms_at_suffix_len": step_ms,
        "prefill_s": t_prefill, "setup_s": {"generate_weights": t_gen, "upload_and_pack": t_upload},
        "yardsticks": {"hbm_copy_gbs": measured_copy_gbs(torch), "hbm_read_probe_gbs": read_gbs,
                       "mfma_matmul_tflops": matmul_yardstick_tflops(torch),
                       "note": "torch device copy (read + write) and torch.matmul bf16 8192x28672x4096: "
                               "independent of the library, reported only"},
    }
    if args.layers:
        out["invalid"] = "layer count overridden"
    if args.prefix_splits:
        out["invalid"] = "prefix splits overridden"
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, weights)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
