"""Adapters between the seeded input generator and the two sides under test."""
import numpy as np

from oracle import transformer as otf
from paper_2601_05475_amd import synth


def oracle_config(s: synth.Shape, exact: bool = False) -> otf.Config:
    """Oracle configuration of a shape.  bf16 shapes get bf16 activation tensors, as their
    specification says; exact=True switches every rounding off."""
    act = "bf16" if (s.dtype == "bf16" and not exact) else "f64"
    return otf.Config(s.n_layers, s.d_model, s.n_q_heads, s.n_kv_heads, s.head_dim,
                      s.d_ffn, s.vocab, s.rope_base, s.rms_eps, act)


def small_shape(name="t", L=2, d=16, Hq=4, Hkv=2, hd=4, F=12, V=32, base=1.0e4, dtype="f32"):
    return synth.Shape(name, L, d, Hq, Hkv, hd, F, V, base, dtype)
