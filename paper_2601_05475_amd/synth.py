"""Seeded synthetic inputs: model shapes, weights, token ids, uniforms.

This module holds no transformer arithmetic.  It fills arrays from a counter-based
generator (``csrc/synth_gen.c``) so that the HIP path and any checker can be handed
the very same bytes.  The shapes are the five workloads this library is built for
(a tiny fp32 decoder, 1B-, 8B- and 32B-shape bf16 decoders, and a reranking run on
the 8B shape); the fan-out sizes mirror the search budgets of the MaxCode paper
(Sec. 4, experimental setup: 8 candidates per step, 64 flat samples) and its
sampling temperatures (0.6 for generation, 0.7 for the reward model).

bf16 tensors are returned as ``uint16`` bit patterns; ``bf16_bits_to_f32`` widens
them without changing a value.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass, replace
from typing import Dict

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "csrc", "synth_gen.c")
_LIB = os.path.join(_HERE, "libmc_synth.so")


def build_synth(force: bool = False) -> str:
    """Compile the generator with gcc (host code only)."""
    if force or not os.path.exists(_LIB):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build_synth())
        u64, sz, dbl, vp = ctypes.c_uint64, ctypes.c_size_t, ctypes.c_double, ctypes.c_void_p
        lib.synth_normal_f32.argtypes = [u64, u64, u64, sz, dbl, dbl, vp]
        lib.synth_normal_bf16.argtypes = [u64, u64, u64, sz, dbl, dbl, vp]
        lib.synth_tokens.argtypes = [u64, u64, u64, sz, ctypes.c_int32, vp]
        lib.synth_uniform_f32.argtypes = [u64, u64, u64, sz, vp]
        for f in (lib.synth_normal_f32, lib.synth_normal_bf16, lib.synth_tokens,
                  lib.synth_uniform_f32):
            f.restype = None
        _lib = lib
    return _lib


@dataclass(frozen=True)
class Shape:
    """Decoder shape.  ``dtype`` is 'f32' or 'bf16' (weights, activations, KV)."""
    name: str
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    rope_base: float
    dtype: str
    rms_eps: float = 1e-6

    def with_layers(self, n_layers: int) -> "Shape":
        return replace(self, n_layers=n_layers, name=f"{self.name}-L{n_layers}")


@dataclass(frozen=True)
class Workload:
    shape: Shape
    prefix_len: int
    n_cands: int
    n_steps: int          # decode steps, or suffix length for reranking
    temperature: float
    top_k: int
    page_tokens: int
    seed_weights: int
    seed_tokens: int
    seed_uniforms: int


TINY = Shape("tiny", 2, 256, 4, 2, 64, 688, 4096, 1.0e4, "f32")
S1B = Shape("1b", 16, 2048, 32, 8, 64, 8192, 32000, 1.0e4, "bf16")
S8B = Shape("8b", 32, 4096, 32, 8, 128, 14336, 128256, 5.0e5, "bf16")
S32B = Shape("32b", 64, 5120, 40, 8, 128, 27648, 152064, 1.0e6, "bf16")

WORKLOADS: Dict[str, Workload] = {
    "tiny": Workload(TINY, 128, 4, 16, 0.8, 50, 4, 1001, 2001, 3001),
    "1b": Workload(S1B, 2048, 16, 256, 0.7, 50, 64, 1002, 2002, 3002),
    "8b": Workload(S8B, 4096, 32, 512, 0.7, 50, 64, 1003, 2003, 3003),
    "8b-rerank": Workload(S8B, 4096, 64, 1024, 0.7, 50, 64, 1003, 2004, 3004),
    "32b": Workload(S32B, 16384, 64, 1024, 0.7, 50, 64, 1005, 2005, 3005),
}

# stream ids of the generator, one per tensor
_ST_EMBED, _ST_FINAL_NORM, _ST_LM_HEAD = 1, 2, 3
_ST_LAYER0, _ST_LAYER_STRIDE = 100, 16
_LAYER_TENSORS = ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down")
_ST_TOKENS_PREFIX, _ST_TOKENS_SUFFIX, _ST_UNIFORMS, _ST_REWARD_IDS = 1, 2, 1, 3


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns to the fp32 values they denote (exact)."""
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def normal(seed: int, stream: int, shape, mean: float, std: float, dtype: str) -> np.ndarray:
    n = int(np.prod(shape))
    lib = _load()
    if dtype == "f32":
        out = np.empty(n, dtype=np.float32)
        lib.synth_normal_f32(seed, stream, 0, n, mean, std, out.ctypes.data)
    elif dtype == "bf16":
        out = np.empty(n, dtype=np.uint16)
        lib.synth_normal_bf16(seed, stream, 0, n, mean, std, out.ctypes.data)
    else:
        raise ValueError(dtype)
    return out.reshape(shape)


def tokens(seed: int, stream: int, shape, vocab: int) -> np.ndarray:
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.int32)
    _load().synth_tokens(seed, stream, 0, n, vocab, out.ctypes.data)
    return out.reshape(shape)


def uniforms(seed: int, stream: int, shape) -> np.ndarray:
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.float32)
    _load().synth_uniform_f32(seed, stream, 0, n, out.ctypes.data)
    return out.reshape(shape)


def layer_tensor_shapes(s: Shape) -> Dict[str, tuple]:
    d, hd = s.d_model, s.head_dim
    return {
        "attn_norm": (d,), "wq": (s.n_q_heads * hd, d), "wk": (s.n_kv_heads * hd, d),
        "wv": (s.n_kv_heads * hd, d), "wo": (d, s.n_q_heads * hd), "ffn_norm": (d,),
        "w_gate": (s.d_ffn, d), "w_up": (s.d_ffn, d), "w_down": (d, s.d_ffn),
    }


def make_layer(s: Shape, seed: int, layer: int) -> Dict[str, np.ndarray]:
    """One layer's tensors, row-major [out_features][in_features].

    Matrices are N(0, 0.02^2); norm gains are 1 + N(0, 0.02^2) so that a missing
    gain cannot go unnoticed."""
    out = {}
    shapes = layer_tensor_shapes(s)
    for j, name in enumerate(_LAYER_TENSORS):
        stream = _ST_LAYER0 + _ST_LAYER_STRIDE * layer + j
        mean = 1.0 if name.endswith("norm") else 0.0
        out[name] = normal(seed, stream, shapes[name], mean, 0.02, s.dtype)
    return out


def make_weights(s: Shape, seed: int) -> Dict[str, object]:
    """All tensors of a model: {'embed', 'final_norm', 'lm_head', 'layers': [ {...} ]}."""
    return {
        "embed": normal(seed, _ST_EMBED, (s.vocab, s.d_model), 0.0, 0.02, s.dtype),
        "final_norm": normal(seed, _ST_FINAL_NORM, (s.d_model,), 1.0, 0.02, s.dtype),
        "lm_head": normal(seed, _ST_LM_HEAD, (s.vocab, s.d_model), 0.0, 0.02, s.dtype),
        "layers": [make_layer(s, seed, l) for l in range(s.n_layers)],
    }


def weights_as_f32(w: Dict[str, object]) -> Dict[str, object]:
    """The same values as fp32 arrays (bf16 bit patterns widened; fp32 passed through)."""
    def conv(a):
        return bf16_bits_to_f32(a) if a.dtype == np.uint16 else a
    out = {k: conv(v) for k, v in w.items() if k != "layers"}
    out["layers"] = [{k: conv(v) for k, v in lw.items()} for lw in w["layers"]]
    return out


def prefix_tokens(wl: Workload, n: int | None = None) -> np.ndarray:
    return tokens(wl.seed_tokens, _ST_TOKENS_PREFIX, (n or wl.prefix_len,), wl.shape.vocab)


def suffix_tokens(wl: Workload, n_cands: int | None = None, n: int | None = None) -> np.ndarray:
    """Teacher-forcing / reranking suffixes, [B][n]."""
    return tokens(wl.seed_tokens, _ST_TOKENS_SUFFIX,
                  (n_cands or wl.n_cands, n or wl.n_steps), wl.shape.vocab)


def step_uniforms(wl: Workload, n_cands: int | None = None, n: int | None = None) -> np.ndarray:
    """Uniforms in [0,1) for sampling, [n_steps][B]."""
    return uniforms(wl.seed_uniforms, _ST_UNIFORMS, (n or wl.n_steps, n_cands or wl.n_cands))


def reward_token_ids(wl: Workload, n_reward: int) -> np.ndarray:
    """n_reward distinct token ids (first distinct draws of the stream)."""
    draw = tokens(wl.seed_tokens, _ST_REWARD_IDS, (64 * n_reward,), wl.shape.vocab)
    _, first = np.unique(draw, return_index=True)
    ids = draw[np.sort(first)][:n_reward]
    assert len(ids) == n_reward
    return ids.astype(np.int32)
