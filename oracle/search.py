"""Host-side bookkeeping of the max-reward search, written out from the paper's definitions.

TEST INFRASTRUCTURE ONLY: slow, plain, float64 Python.  Only tests/, the smoke check and the
benchmark's CPU baseline may import this package; the library never does.

Passages followed (Sec. 3 = "Method", Sec. 4 = "Experiments and Results"):
  reward_bin          Sec. 3.3, "Categorical Reward Formulation": the five-way binning f_r with
                      thresholds (s1, s2, s3); Sec. 4 "Experimental Setup" prints the three triples.
  best_so_far         Sec. 3.2: u_i = max_{j <= i} gamma^{d_j} f(e_j), d_j the depth of state j.
  value_targets       Sec. 3.3: along one trajectory e_1..e_T, u_t = max_{k <= t} gamma^{k-1} f_r(e_k)
                      and v*_t = max(u_t / gamma, max_{k >= t} gamma^{k-t} f_r(e_k)).
  max_reward_return   Sec. 3.1: G_t = max_{k >= 1} gamma^{k-1} r_{t+k}; the best trajectory of a set
                      is the one with the largest max_t gamma^{t-1} f_r(e_t).
  select_candidate    Sec. 3.2, CUDA-LLM step: if any candidate is correct and faster (f(e) > 1) go on
                      with the arg max, else none is selected.
  median_of_max_speedup, average_rank
                      Sec. 4, "Evaluation Metrics": per problem the maximum speedup over all
                      generations; over problems its median, and the average over problems of a
                      method's rank among the methods on that problem.
Readings: ties in an arg max go to the lowest index; methods with equal maximum speedup on a
problem share the best (lowest) rank of their group; the median of an even number of problems is
the mean of the two middle values.
"""
from __future__ import annotations

from typing import List, Optional, Sequence

THRESHOLDS = {                      # Sec. 4, experimental setup: (s1, s2, s3) in percent
    "kernelbench_l1": (140.0, 320.0, 475.0),
    "kernelbench_l2": (120.0, 170.0, 215.0),
    "pie": (125.0, 180.0, 260.0),
}


def reward_bin(speedup_percent: float, correct: bool, thresholds: Sequence[float]) -> int:
    s1, s2, s3 = thresholds
    if not correct or speedup_percent <= 100.0:
        return 0
    if speedup_percent <= s1:
        return 1
    if speedup_percent <= s2:
        return 2
    if speedup_percent <= s3:
        return 3
    return 4


def best_so_far(rewards: Sequence[float], depths: Sequence[int], gamma: float) -> List[float]:
    out, best = [], None
    for r, d in zip(rewards, depths):
        v = (gamma ** d) * r
        best = v if best is None or v > best else best
        out.append(best)
    return out


def value_targets(rewards: Sequence[float], gamma: float):
    """rewards[k-1] = f_r(e_k), k = 1..T.  Returns (u, v_star), entries t = 1..T."""
    T = len(rewards)
    u, v = [], []
    for t in range(1, T + 1):
        u_t = max((gamma ** (k - 1)) * rewards[k - 1] for k in range(1, t + 1))
        future = max((gamma ** (k - t)) * rewards[k - 1] for k in range(t, T + 1))
        u.append(u_t)
        v.append(max(u_t / gamma, future))
    return u, v


def max_reward_return(rewards_after_t: Sequence[float], gamma: float) -> float:
    """G_t for rewards r_{t+1}, r_{t+2}, ..."""
    return max((gamma ** k) * r for k, r in enumerate(rewards_after_t))


def best_trajectory(trajectories: Sequence[Sequence[float]], gamma: float) -> int:
    scores = [max_reward_return(tr, gamma) for tr in trajectories]
    return scores.index(max(scores))


def select_candidate(speedups: Sequence[float]) -> Optional[int]:
    """speedups[j] = f(e_ij) as a ratio (0 for an incorrect candidate)."""
    best = None
    for j, f in enumerate(speedups):
        if f > 1.0 and (best is None or f > speedups[best]):
            best = j
    return best


def median(values: Sequence[float]) -> float:
    v = sorted(values)
    n = len(v)
    return v[n // 2] if n % 2 else 0.5 * (v[n // 2 - 1] + v[n // 2])


def median_of_max_speedup(speedups_per_problem: Sequence[Sequence[float]]) -> float:
    return median([max(g) for g in speedups_per_problem])


def average_rank(max_speedup: Sequence[Sequence[float]]) -> List[float]:
    """max_speedup[m][p]: method m on problem p.  Rank 1 = largest; equal values share the
    lowest rank of their group."""
    n_m, n_p = len(max_speedup), len(max_speedup[0])
    total = [0.0] * n_m
    for p in range(n_p):
        col = [max_speedup[m][p] for m in range(n_m)]
        for m in range(n_m):
            total[m] += 1 + sum(1 for x in col if x > col[m])
    return [t / n_p for t in total]
