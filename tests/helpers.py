"""Adapters between the seeded input generator and the two sides under test."""
import numpy as np

from oracle import transformer as otf
from paper_2601_05475_amd import synth


def oracle_config(s: synth.Shape) -> otf.Config:
    return otf.Config(s.n_layers, s.d_model, s.n_q_heads, s.n_kv_heads, s.head_dim,
                      s.d_ffn, s.vocab, s.rope_base, s.rms_eps)


def small_shape(name="t", L=2, d=16, Hq=4, Hkv=2, hd=4, F=12, V=32, base=1.0e4, dtype="f32"):
    return synth.Shape(name, L, d, Hq, Hkv, hd, F, V, base, dtype)
