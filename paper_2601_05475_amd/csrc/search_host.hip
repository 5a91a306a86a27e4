// Host-side bookkeeping of the max-reward search loop (no device work): reward binning,
// best-reward-so-far, value targets, the beam selection rule and the two evaluation statistics.
// Plain C++ behind the C ABI; every function validates its arguments and reports through
// mc_last_error like the rest of the library.
#include "common.h"

#include <math.h>

#include <algorithm>
#include <vector>

using namespace mc;

extern "C" int32_t mc_reward_bin(double speedup_percent, int32_t correct, const double *thresholds) {
  if (!thresholds || !(thresholds[0] >= 100.0) || !(thresholds[1] >= thresholds[0]) || !(thresholds[2] >= thresholds[1]) ||
      isnan(speedup_percent))
    MC_FAIL(MC_ERR_INVALID, "thresholds must satisfy 100 <= s1 <= s2 <= s3 and the speedup must be a number");
  if (!correct || speedup_percent <= 100.0) return 0;
  int bin = 1;
  for (int i = 0; i < 3; ++i)
    if (speedup_percent > thresholds[i]) bin = i + 2;
  return bin;
}

static int check_gamma(double gamma) {
  if (!(gamma > 0.0 && gamma <= 1.0)) MC_FAIL(MC_ERR_INVALID, "gamma %g outside (0, 1]", gamma);
  return MC_OK;
}

extern "C" int mc_best_so_far(const double *rewards, const int32_t *depths, int32_t n, double gamma, double *u_out) {
  if (!rewards || !depths || !u_out || n < 1) MC_FAIL(MC_ERR_INVALID, "NULL argument or n < 1");
  MC_TRY(check_gamma(gamma));
  double best = 0.0;
  for (int i = 0; i < n; ++i) {
    if (depths[i] < 0 || isnan(rewards[i])) MC_FAIL(MC_ERR_INVALID, "depth %d negative or reward %d not a number", i, i);
    const double v = pow(gamma, (double)depths[i]) * rewards[i];
    best = (i == 0 || v > best) ? v : best;
    u_out[i] = best;
  }
  return MC_OK;
}

extern "C" int mc_value_targets(const double *rewards, int32_t n, double gamma, double *u_out, double *v_out) {
  if (!rewards || !u_out || !v_out || n < 1) MC_FAIL(MC_ERR_INVALID, "NULL argument or n < 1");
  MC_TRY(check_gamma(gamma));
  for (int i = 0; i < n; ++i)
    if (isnan(rewards[i])) MC_FAIL(MC_ERR_INVALID, "reward %d is not a number", i);
  // forward: u_t = max_{k <= t} gamma^{k-1} r_k; backward: w_t = max_{k >= t} gamma^{k-t} r_k
  //          = max(r_t, gamma * w_{t+1})
  double best = 0.0, g = 1.0;
  for (int t = 0; t < n; ++t) {
    const double v = g * rewards[t];
    best = (t == 0 || v > best) ? v : best;
    u_out[t] = best;
    g *= gamma;
  }
  double w = 0.0;
  for (int t = n - 1; t >= 0; --t) {
    w = (t == n - 1) ? rewards[t] : std::max(rewards[t], gamma * w);
    v_out[t] = std::max(u_out[t] / gamma, w);
  }
  return MC_OK;
}

extern "C" int32_t mc_select_candidate(const double *speedups, int32_t n) {
  if (!speedups || n < 1) MC_FAIL(MC_ERR_INVALID, "NULL argument or n < 1");
  int best = -1;
  for (int j = 0; j < n; ++j) {
    if (isnan(speedups[j])) MC_FAIL(MC_ERR_INVALID, "speedup %d is not a number", j);
    if (speedups[j] > 1.0 && (best < 0 || speedups[j] > speedups[best])) best = j;
  }
  return best < 0 ? MC_SELECT_NONE : best;
}

extern "C" int mc_median_of_max(const double *speedups, const int32_t *counts, int32_t n_problems, double *out) {
  if (!speedups || !counts || !out || n_problems < 1) MC_FAIL(MC_ERR_INVALID, "NULL argument or n_problems < 1");
  std::vector<double> mx((size_t)n_problems);
  size_t at = 0;
  for (int p = 0; p < n_problems; ++p) {
    if (counts[p] < 1) MC_FAIL(MC_ERR_INVALID, "problem %d has no generation", p);
    double m = speedups[at];
    for (int i = 0; i < counts[p]; ++i) {
      if (isnan(speedups[at + i])) MC_FAIL(MC_ERR_INVALID, "a speedup of problem %d is not a number", p);
      m = std::max(m, speedups[at + i]);
    }
    mx[p] = m;
    at += (size_t)counts[p];
  }
  std::sort(mx.begin(), mx.end());
  const int n = n_problems;
  *out = (n % 2) ? mx[n / 2] : 0.5 * (mx[n / 2 - 1] + mx[n / 2]);
  return MC_OK;
}

extern "C" int mc_average_rank(const double *max_speedup, int32_t n_methods, int32_t n_problems, double *avg_rank) {
  if (!max_speedup || !avg_rank || n_methods < 1 || n_problems < 1) MC_FAIL(MC_ERR_INVALID, "NULL argument or empty table");
  for (size_t i = 0; i < (size_t)n_methods * n_problems; ++i)
    if (isnan(max_speedup[i])) MC_FAIL(MC_ERR_INVALID, "entry %zu is not a number", i);
  for (int m = 0; m < n_methods; ++m) {
    double total = 0.0;
    for (int p = 0; p < n_problems; ++p) {
      const double mine = max_speedup[(size_t)m * n_problems + p];
      int above = 0;
      for (int o = 0; o < n_methods; ++o) above += max_speedup[(size_t)o * n_problems + p] > mine;
      total += 1 + above;
    }
    avg_rank[m] = total / n_problems;
  }
  return MC_OK;
}
