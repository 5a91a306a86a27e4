"""CPU oracle: the plain definition of the decoder step, in float64.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this package;
it shares no code with the HIP kernels.  It is slow on purpose: every candidate is
an independent sequence [prefix ; suffix], attention is a full softmax over all
earlier positions, nothing is tiled, split, paged or fused.

What it computes is the computation the MaxCode search (Sec. 3, "The Markov
Decision Process": the policy is a frozen autoregressive LLM from which several
candidates are sampled for the same state) spends its time in: a pre-norm
decoder-only transformer with grouped-query attention, rotary position embedding
(rotate-half pairing), RMSNorm and a SwiGLU feed-forward block.  The paper leaves
the architecture open; the readings taken here are:
  * RMSNorm over the model width, y = x * g / sqrt(mean(x^2) + eps); no QK-norm;
  * RoPE angle pos * base^(-2i/hd) on coordinate pairs (i, i + hd/2) of q and k;
  * query head a uses KV head a // (Hq / Hkv); scores scaled by 1/sqrt(hd);
    key j visible from position p iff j <= p; no biases; untied LM head.

Weights arrive as fp32 arrays (for bf16 models: the bf16 values widened, i.e. the
same numbers the GPU holds); everything else is float64.

Precision of bf16 models.  The bf16 workloads are specified as "bf16 weights and
activations with fp32 accumulation".  Read literally, every activation tensor the
model defines is a bf16 tensor: the RMSNorm outputs, q/k/v after the projection and
rotation (which is also what the KV cache holds), the attention output and the SwiGLU
product.  With ``Config.act_dtype == "bf16"`` the oracle rounds exactly those tensors
to the nearest bf16 value (ties to even) and nothing else: the residual stream, all
sums, the softmax and its probabilities stay float64.  With "f64" (default) nothing
is rounded; that mode is the reference of fp32 models and shows how far bf16
arithmetic itself is from exact.

Parity pins live in tests/test_oracle_*.py: an element-by-element brute force on
tiny shapes, closed forms for RMSNorm / RoPE / softmax, shared == unshared,
decode == prefill.  Matrix products use numpy's matmul as a library step.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Optional

import numpy as np

F64 = np.float64


@dataclass(frozen=True)
class Config:
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    rope_base: float
    rms_eps: float = 1e-6
    act_dtype: str = "f64"        # "f64": nothing rounded; "bf16": activation tensors are bf16


def round_bf16(x: np.ndarray) -> np.ndarray:
    """Nearest bfloat16 value (8 significand bits, ties to even) of each element, as float64.

    Done on the fp32 bit pattern: add 0x7FFF plus the lowest kept bit, clear the low 16 bits."""
    f = np.ascontiguousarray(x, np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(f.shape).astype(F64)


def store(cfg: "Config", x: np.ndarray) -> np.ndarray:
    """An activation tensor as the model holds it."""
    return round_bf16(x) if cfg.act_dtype == "bf16" else np.asarray(x, F64)


def rmsnorm(x: np.ndarray, g: np.ndarray, eps: float) -> np.ndarray:
    """Row-wise y = x * g / sqrt(mean(x^2) + eps).  x: [..., d], g: [d]."""
    x = np.asarray(x, F64)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x * np.asarray(g, F64) / np.sqrt(ms + eps)


def rope(z: np.ndarray, pos: np.ndarray, base: float) -> np.ndarray:
    """Rotate head vectors.  z: [T, H, hd], pos: [T] integer positions.

    Coordinates i and i + hd/2 form a pair rotated by the angle pos * base^(-2i/hd).
    """
    z = np.asarray(z, F64)
    hd = z.shape[-1]
    half = hd // 2
    i = np.arange(half, dtype=F64)
    theta = np.power(F64(base), -2.0 * i / hd)                      # [half]
    ang = np.asarray(pos, F64)[:, None] * theta[None, :]           # [T, half]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]        # [T, 1, half]
    lo, hi = z[..., :half], z[..., half:]
    return np.concatenate([lo * c - hi * s, hi * c + lo * s], axis=-1)


def softmax_rows(s: np.ndarray) -> np.ndarray:
    m = np.max(s, axis=-1, keepdims=True)
    e = np.exp(s - m)
    return e / np.sum(e, axis=-1, keepdims=True)


def attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, q_pos: np.ndarray,
              k_pos: np.ndarray) -> np.ndarray:
    """Full-softmax grouped-query attention.

    q: [T, Hq, hd] (rotated), k, v: [S, Hkv, hd] (k rotated), q_pos: [T], k_pos: [S].
    Key j is visible to query i iff k_pos[j] <= q_pos[i].  Returns [T, Hq, hd]."""
    T, Hq, hd = q.shape
    Hkv = k.shape[1]
    G = Hq // Hkv
    visible = np.asarray(k_pos)[None, :] <= np.asarray(q_pos)[:, None]     # [T, S]
    out = np.empty((T, Hq, hd), F64)
    for a in range(Hq):
        kvh = a // G
        s = (q[:, a, :] @ k[:, kvh, :].T) / np.sqrt(F64(hd))               # [T, S]
        s = np.where(visible, s, -np.inf)
        out[:, a, :] = softmax_rows(s) @ v[:, kvh, :]
    return out


def silu(z: np.ndarray) -> np.ndarray:
    return z / (1.0 + np.exp(-z))


class KVCache:
    """Per-layer rotated keys and values of the positions seen so far."""

    def __init__(self, n_layers: int):
        self.k: List[Optional[np.ndarray]] = [None] * n_layers   # [S, Hkv, hd]
        self.v: List[Optional[np.ndarray]] = [None] * n_layers
        self.length = 0

    def copy(self) -> "KVCache":
        c = KVCache(len(self.k))
        c.k = [None if a is None else a.copy() for a in self.k]
        c.v = [None if a is None else a.copy() for a in self.v]
        c.length = self.length
        return c


def layer_forward(cfg: Config, lw: Dict[str, np.ndarray], x: np.ndarray, pos: np.ndarray,
                  k_past: Optional[np.ndarray], v_past: Optional[np.ndarray]):
    """One decoder layer on rows x [T, d] sitting at positions pos [T].

    k_past / v_past hold earlier positions 0..len-1 of the same sequence (or None).
    Returns (x_out, k_all, v_all)."""
    T = x.shape[0]
    Hq, Hkv, hd = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    h = store(cfg, rmsnorm(x, lw["attn_norm"], cfg.rms_eps))
    q = (h @ np.asarray(lw["wq"], F64).T).reshape(T, Hq, hd)
    k = (h @ np.asarray(lw["wk"], F64).T).reshape(T, Hkv, hd)
    v = store(cfg, (h @ np.asarray(lw["wv"], F64).T).reshape(T, Hkv, hd))
    q = store(cfg, rope(q, pos, cfg.rope_base))
    k = store(cfg, rope(k, pos, cfg.rope_base))
    if k_past is not None:
        k_all = np.concatenate([k_past, k], axis=0)
        v_all = np.concatenate([v_past, v], axis=0)
        k_pos = np.concatenate([np.arange(k_past.shape[0]), np.asarray(pos)])
    else:
        k_all, v_all, k_pos = k, v, np.asarray(pos)
    o = store(cfg, attention(q, k_all, v_all, pos, k_pos).reshape(T, Hq * hd))
    x = x + o @ np.asarray(lw["wo"], F64).T
    h2 = store(cfg, rmsnorm(x, lw["ffn_norm"], cfg.rms_eps))
    gate = h2 @ np.asarray(lw["w_gate"], F64).T
    up = h2 @ np.asarray(lw["w_up"], F64).T
    x = x + store(cfg, silu(gate) * up) @ np.asarray(lw["w_down"], F64).T
    return x, k_all, v_all


def lm_logits(cfg: Config, w: Dict[str, object], x: np.ndarray) -> np.ndarray:
    """Final RMSNorm and LM head on rows x [T, d] -> [T, V]."""
    return store(cfg, rmsnorm(x, w["final_norm"], cfg.rms_eps)) @ np.asarray(w["lm_head"], F64).T


def forward(cfg: Config, w: Dict[str, object], tokens: np.ndarray,
            cache: Optional[KVCache] = None, logits_rows: Optional[np.ndarray] = None):
    """Run tokens [T] through the model, continuing the sequence held in ``cache``.

    Returns (logits [len(logits_rows) or T, V] float64, cache).  ``cache`` is updated
    in place (a fresh one is made when None)."""
    tokens = np.asarray(tokens)
    if cache is None:
        cache = KVCache(cfg.n_layers)
    T = tokens.shape[0]
    pos = cache.length + np.arange(T)
    x = np.asarray(w["embed"], F64)[tokens]                     # [T, d]
    for l in range(cfg.n_layers):
        x, cache.k[l], cache.v[l] = layer_forward(cfg, w["layers"][l], x, pos,
                                                  cache.k[l], cache.v[l])
    cache.length += T
    rows = np.arange(T) if logits_rows is None else np.asarray(logits_rows)
    return lm_logits(cfg, w, x[rows]), cache


def forward_unshared(cfg: Config, w, prefix: np.ndarray, suffix: np.ndarray) -> np.ndarray:
    """The definition: one independent pass over [prefix ; suffix].  Logits of all rows."""
    return forward(cfg, w, np.concatenate([prefix, suffix]))[0]


def forward_shared(cfg: Config, w, prefix: np.ndarray, suffixes: np.ndarray):
    """Prefix computed once, every candidate continued from a copy of its cache.

    suffixes: [B, n].  Returns (prefix_last_logits [V], suffix_logits [B, n, V])."""
    plog, pcache = forward(cfg, w, prefix)
    outs = []
    for b in range(suffixes.shape[0]):
        lg, _ = forward(cfg, w, suffixes[b], cache=pcache.copy())
        outs.append(lg)
    return plog[-1], np.stack(outs)


# ---- single-operation helpers used by the kernel-level parity tests ---------------

def attention_one(q: np.ndarray, keys: np.ndarray, values: np.ndarray) -> np.ndarray:
    """One query vector [hd] against all given keys/values [S, hd]: softmax(q.k/sqrt(hd)) v."""
    q = np.asarray(q, F64)
    keys = np.asarray(keys, F64)
    s = keys @ q / np.sqrt(F64(q.shape[0]))
    p = softmax_rows(s[None, :])[0]
    return p @ np.asarray(values, F64)


def linear(x: np.ndarray, w: np.ndarray) -> np.ndarray:
    """y = x W^T with W row-major [out][in]."""
    return np.asarray(x, F64) @ np.asarray(w, F64).T
