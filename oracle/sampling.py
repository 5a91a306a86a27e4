"""CPU oracle: temperature / top-k sampling, reward-token log-probs, score, ranking.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

Sampling is the stochastic token sampling that makes one search state yield several
distinct candidates (MaxCode Sec. 3, policy paragraph); the temperatures used there
are 0.6 (generation) and 0.7 (reward model) (Sec. 4, experimental setup).  The
random number is an input (one uniform in [0,1) per draw), so the draw is a
deterministic function.  Because a floating-point comparison decides an integer
here, the arithmetic is carried out in fp32, the precision of the kernel it checks:
    z_v   = logit_v / T                                  (IEEE fp32 division)
    S     = the k largest entries under the total order (z descending, id ascending)
    e_i   = exp(z_(i) - z_(1)),  Z = e_1 + e_2 + ... (left to right),  c_i = (e_1+..+e_i)/Z
    token = id_(i*),  i* = first i with c_i > u,  or the k-th entry if there is none.
T <= 0 or k == 1 mean argmax (lowest id on exact ties); k <= 0 or k >= V mean all V.

Scoring follows the generative value function (Sec. 3.3, categorical reward and the
softmax over reward categories; value-guided search picks the highest expected
estimated value): the label tokens' log-probabilities are read at the candidate's
last position, renormalised inside the label set at temperature Ts, and the score is
the expectation of the label values.  This part is float64.
"""
from __future__ import annotations

import numpy as np

F32 = np.float32
F64 = np.float64


def topk_order(z: np.ndarray, k: int) -> np.ndarray:
    """Ids of the k largest entries of z under (value descending, id ascending), sorted."""
    ids = np.arange(z.shape[0])
    order = np.lexsort((ids, -z.astype(F64)))      # primary: -z ascending; ties: id ascending
    return order[:k]


def sample(logits: np.ndarray, temperature: float, top_k: int, u: float):
    """One draw.  Returns (token, topk_ids, margin); margin = min_i |u - c_i| (inf for argmax).

    ``logits`` is taken as fp32 values; ``u`` in [0, 1)."""
    lg = np.asarray(logits, F32)
    V = lg.shape[0]
    if temperature <= 0 or top_k == 1:
        tok = int(np.flatnonzero(lg == lg.max())[0])
        return tok, np.array([tok]), np.inf
    k = V if (top_k <= 0 or top_k >= V) else int(top_k)
    z = lg / F32(temperature)
    ids = topk_order(z, k)
    zs = z[ids]
    e = np.exp((zs - zs[0]).astype(F32)).astype(F32)
    csum = np.cumsum(e, dtype=F32)                 # left-to-right fp32 accumulation
    c = (csum / csum[-1]).astype(F32)
    hit = np.flatnonzero(c > F32(u))
    i = int(hit[0]) if hit.size else k - 1
    margin = float(np.min(np.abs(c.astype(F64) - F64(u))))
    return int(ids[i]), ids, margin


def reward_logprobs(logits: np.ndarray, reward_ids: np.ndarray) -> np.ndarray:
    """log-softmax over the whole vocabulary, read at the reward tokens.  [V] -> [R]."""
    lg = np.asarray(logits, F64)
    m = lg.max()
    lse = m + np.log(np.sum(np.exp(lg - m)))
    return lg[np.asarray(reward_ids)] - lse


def expected_value(logprobs: np.ndarray, reward_values: np.ndarray, score_temperature: float) -> float:
    """sum_r w_r * softmax_r(lp_r / Ts): expectation of the label value inside the label set."""
    t = np.asarray(logprobs, F64) / F64(score_temperature)
    p = np.exp(t - t.max())
    p = p / p.sum()
    return float(np.sum(np.asarray(reward_values, F64) * p))


def rank(scores: np.ndarray) -> np.ndarray:
    """Candidate indices, best first: score descending, index ascending on equal scores."""
    s = np.asarray(scores)
    return np.lexsort((np.arange(s.shape[0]), -s.astype(F64))).astype(np.int32)
