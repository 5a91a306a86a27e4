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


def test_invalid_configs_are_rejected(lib):
    s = synth.TINY
    for field, bad in [("n_layers", 0), ("n_kv_heads", 3), ("head_dim", 7), ("dtype", 9), ("vocab", 0)]:
        cfg = binding.make_config(s)
        setattr(cfg, field, bad)
        assert lib.mc_model_bytes(C.byref(cfg)) == 0
        assert len(lib.mc_last_error()) > 0
    cfg = binding.make_config(s)
    for field, bad in [("page_tokens", 3), ("page_tokens", 256), ("max_cands", 0), ("max_suffix", 0)]:
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
