"""Host-side checks of the C ABI: the library loads, exports every declared symbol, and its
sizing / validation code behaves (no GPU work is launched here)."""
import ctypes as C
import os
import re

import pytest

from paper_2601_05475_amd import binding, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        import __graft_entry__ as g
        g.build()
    return binding.load_library()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "mc.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mc_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported_and_bound(lib):
    names = declared_symbols()
    assert {"mc_prefill_shared", "mc_decode_step", "mc_score_candidates", "mc_sample"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in mc.h but not exported"
        assert n in binding.SIGNATURES, f"{n} has no Python signature"
    assert set(binding.SIGNATURES) == set(names)


def test_model_and_session_sizes(lib):
    s = synth.TINY
    cfg = binding.make_config(s)
    nbytes = lib.mc_model_bytes(C.byref(cfg))
    d, F, V, hd = s.d_model, s.d_ffn, s.vocab, s.head_dim
    per_layer = 2 * d + (s.n_q_heads + 2 * s.n_kv_heads) * hd * d + d * s.n_q_heads * hd + 3 * F * d
    params = 2 * V * d + d + s.n_layers * per_layer
    assert params * 4 <= nbytes <= params * 4 + 256 * (4 + 7 * s.n_layers)
    p = binding.mc_session_params(128, 4, 16, 4, 0)
    sb = lib.mc_session_bytes(C.byref(cfg), C.byref(p))
    kv = 2 * s.n_layers * ((128 // 4) + 4 * 4) * s.n_kv_heads * hd * 4 * 4
    assert sb > kv
    # 8B shape, headline workload: weights ~16 GB, KV = 512 MiB prefix + 2 GiB suffix
    cfg8 = binding.make_config(synth.S8B)
    assert 16.0e9 < lib.mc_model_bytes(C.byref(cfg8)) < 16.2e9
    p8 = binding.mc_session_params(4096, 32, 512, 64, 4096)
    sb8 = lib.mc_session_bytes(C.byref(cfg8), C.byref(p8))
    assert sb8 > 2.5 * 2 ** 30 and sb8 < 6 * 2 ** 30
    # a smaller page pool shrinks the session by exactly the pages it leaves out (K and V, every layer)
    p8s = binding.mc_session_params(4096, 32, 512, 64, 4096, 64)
    page = 2 * 8 * 128 * 64 * 2 * 32
    assert sb8 - lib.mc_session_bytes(C.byref(cfg8), C.byref(p8s)) == (32 * 8 - 64) * page
    p8b = binding.mc_session_params(4096, 32, 512, 64, 4096, 10 ** 6)     # more than can be used: capped
    assert lib.mc_session_bytes(C.byref(cfg8), C.byref(p8b)) == sb8


def test_invalid_configs_are_rejected(lib):
    s = synth.TINY
    for field, bad in [("n_layers", 0), ("n_kv_heads", 3), ("head_dim", 7), ("dtype", 9), ("vocab", 0)]:
        cfg = binding.make_config(s)
        setattr(cfg, field, bad)
        assert lib.mc_model_bytes(C.byref(cfg)) == 0
        assert len(lib.mc_last_error()) > 0
    cfg = binding.make_config(s)
    for field, bad in [("page_tokens", 3), ("page_tokens", 256), ("max_cands", 0), ("max_suffix", 0), ("pool_pages", -1)]:
        p = binding.mc_session_params(128, 4, 16, 4, 0)
        setattr(p, field, bad)
        assert lib.mc_session_bytes(C.byref(cfg), C.byref(p)) == 0
    assert lib.mc_model_bytes(None) == 0
    # NULL handles are reported, not dereferenced
    assert lib.mc_session_sync(None) == -1
    assert lib.mc_decode_step(None, None, 1) == -1
    assert lib.mc_prefill_shared(None, None, 1) == -1
    h = C.c_void_p()
    assert lib.mc_model_create(C.byref(cfg), None, None, C.byref(h)) == -1
    assert lib.mc_op_linear(None, 0, 4, 4, 4, None, None, None, 1, 0) == -1
    assert lib.mc_op_tiled_bytes(33, 128) == 64 * 128 * 2 and lib.mc_op_tiled_bytes(33, 100) == 0
    assert lib.mc_op_linear_splits(1, 32, 6144, 4096, 1) >= 1
    assert lib.mc_op_sample(None, 0, 10, None, 0, 1.0, 5, None, None, None) == -1
    # the fused many-row layers: bad arguments and shapes they do not cover are refused on the host
    fake = C.c_void_p(256)                     # never dereferenced: the checks come first
    assert lib.mc_op_linear_accumulate(None, 4096, 4096, 4096, None, None, None) == -1
    assert lib.mc_op_linear_accumulate(None, 0, 4096, 4096, fake, fake, fake) == -1
    assert lib.mc_op_linear_accumulate(None, 64, 4096, 4096, fake, fake, fake) == -5       # few rows: the weight-streaming path
    assert lib.mc_op_linear_accumulate(None, 8192, 4000, 4096, fake, fake, fake) == -5     # N not a multiple of 128
    assert lib.mc_op_linear_accumulate(None, 8192, 4096, 4000, fake, fake, fake) == -5     # K not a multiple of 256
    args = [fake] * 9
    assert lib.mc_op_linear_qkv_rope(None, 32, 32, 8, 128, 64, 4096, 5e5, 100, *([None] * 9)) == -1
    assert lib.mc_op_linear_qkv_rope(None, 32, 32, 8, 126, 64, 4096, 5e5, 100, *args) == -1   # head_dim % 4
    assert lib.mc_op_linear_qkv_rope(None, 32, 32, 8, 128, 64, 4096, -1.0, 100, *args) == -1
    out = (C.c_int32 * 9)()
    assert lib.mc_op_attention_decode_plan(32, 32, 8, 128, 64, 4096, 1, 0, out) == 0 and out[2] >= 1
    assert lib.mc_op_attention_decode_plan(32, 32, 8, 128, 64, 0, 0, 0, out) == -1           # no keys
    assert lib.mc_op_attention_decode_plan(32, 32, 7, 128, 64, 4096, 1, 0, out) == -1        # heads do not divide
    assert lib.mc_op_attention_decode_plan(32, 32, 8, 96, 64, 4096, 1, 0, out) == -5         # head_dim not covered
    assert lib.mc_op_attention_decode_plan(32, 32, 8, 128, 16, 4096, 1, 0, out) == -5        # page size not covered


def test_decode_attention_plan_covers_every_block_and_fits_its_workspace(lib):
    """Host logic of the decode-attention launcher: for a sweep of shapes the key splits cover
    every 32-key block exactly once, no split is empty, the partial states fit the workspace the
    library asks for, and the prefix ids of one split are a multiple of 8 apart."""
    import itertools
    shapes = [(32, 32, 8, 128), (64, 40, 8, 128), (16, 32, 8, 64), (1, 4, 4, 64), (5, 12, 2, 128), (33, 4, 1, 64)]
    lens = [0, 1, 31, 32, 33, 64, 65, 200, 512, 1000, 4096, 16384, 40000]
    for (B, Hq, Hkv, hd), P, t, S in itertools.product(shapes, lens, [0, 1, 63, 64, 65, 512, 1024, 3000], [0, 1, 7, 64, 5000]):
        if P + t == 0:
            continue
        p = binding.op_attention_decode_plan(B, Hq, Hkv, hd, 64, P, t, S)
        G = Hq // Hkv
        nb_p, nb_s = -(-P // 32), -(-t // 32)
        if P:
            assert p["splits"] >= 1 and p["splits"] * p["blocks_per_split"] >= nb_p
            assert (p["splits"] - 1) * p["blocks_per_split"] < nb_p
            row_blocks = -(-B * G // 32)
            assert p["rb_per_item"] == (4 if row_blocks >= 8 else 1)
            assert p["prefix_stride"] % 8 == 0 and p["prefix_stride"] >= Hkv * p["splits"]
            assert p["prefix_items"] == p["prefix_stride"] * -(-row_blocks // p["rb_per_item"])
        else:
            assert p["prefix_items"] == 0
        if t:
            assert 1 <= p["suffix_splits"] <= 8 and p["suffix_splits"] * p["suffix_bps"] >= nb_s
            assert (p["suffix_splits"] - 1) * p["suffix_bps"] < nb_s
            assert p["suffix_items"] == B * Hkv * p["suffix_splits"]
        else:
            assert p["suffix_items"] == 0
        assert p["n_parts"] == (p["splits"] if P else 0) + (p["suffix_splits"] if t else 0) <= 1024 or P > 100000
        ws = lib.mc_op_attention_decode_ws(B, Hq, Hkv, hd, P, t, 64)
        assert p["n_parts"] * B * Hq * (hd + 2) * 4 <= ws, (B, Hq, Hkv, hd, P, t, S, p, ws)


def test_bench_refuses_more_than_one_gpu_and_bad_step_counts():
    """bench.py is a one-GPU program: --gpus N > 1 ends with a message and a non-zero status before
    anything touches a device; so do step counts outside the workload."""
    import subprocess
    import sys
    bench = os.path.join(ROOT, "bench.py")
    r = subprocess.run([sys.executable, bench, "--gpus", "2"], capture_output=True, text=True, timeout=300)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout.strip() == ""
    r = subprocess.run([sys.executable, bench, "--gpus", "0"], capture_output=True, text=True, timeout=300)
    assert r.returncode != 0 and r.stdout.strip() == ""
