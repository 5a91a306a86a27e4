"""Host-side bookkeeping of the search loop: the oracle (oracle/search.py) against what the
paper prints and against closed forms, then the library's C functions against the oracle.
No GPU work."""
import itertools

import numpy as np
import pytest

from oracle import search as osearch
from paper_2601_05475_amd import binding

from golden_io import paper_values

PV = paper_values()


# ---------------------------------------------------------------- the oracle against its pins
def test_thresholds_are_the_printed_triples():
    assert osearch.THRESHOLDS["kernelbench_l1"] == tuple(PV["reward_thresholds_kernelbench_l1"])
    assert osearch.THRESHOLDS["kernelbench_l2"] == tuple(PV["reward_thresholds_kernelbench_l2"])
    assert osearch.THRESHOLDS["pie"] == tuple(PV["reward_thresholds_pie"])


def test_reward_bin_boundaries_as_printed():
    """Sec. 3.3: 0 for speedup <= 100 % or incorrect, then (100, s1], (s1, s2], (s2, s3], > s3."""
    th = PV["reward_thresholds_kernelbench_l1"]
    cases = [(50, 0), (100, 0), (100.001, 1), (140, 1), (140.001, 2), (320, 2), (320.5, 3), (475, 3), (475.001, 4), (1e6, 4)]
    for sp, want in cases:
        assert osearch.reward_bin(sp, True, th) == want, sp
        assert osearch.reward_bin(sp, False, th) == 0
    # the five labels are exactly the printed ones
    seen = {osearch.reward_bin(sp, True, th) for sp in np.linspace(0, 600, 601)}
    assert sorted(seen) == [int(v) for v in PV["reward_labels"]]


def test_value_targets_closed_forms():
    # gamma = 1 (the paper's setting): u is the running maximum and every target equals the
    # maximum reward of the whole trajectory
    assert PV["discount_gamma"] == 1
    r = [1, 0, 3, 2, 4, 0]
    u, v = osearch.value_targets(r, 1.0)
    assert u == [1, 1, 3, 3, 4, 4] and v == [4] * 6
    # worked by hand for gamma = 1/2, rewards (1, 0, 3): u = (1, 1, 1); the future maxima are
    # max(1, 0, 3/4), max(0, 3/2), 3; u / gamma = 2
    u, v = osearch.value_targets([1, 0, 3], 0.5)
    assert u == [1, 1, 1] and v == [2, 2, 3]
    # the return G_t of Sec. 3.1 and the best-trajectory rule
    assert osearch.max_reward_return([0, 2, 8], 0.5) == 2.0
    assert osearch.best_trajectory([[0, 1, 1], [0, 0, 4], [3, 0, 0]], 1.0) == 1
    assert osearch.best_trajectory([[0, 1, 1], [0, 0, 4], [3, 0, 0]], 0.5) == 2
    # u with depths: the same state visited at different depths
    assert osearch.best_so_far([2, 4, 1], [0, 2, 1], 0.5) == [2, 2, 2]


def test_select_candidate_rule():
    assert osearch.select_candidate([0.5, 1.0, 0.9]) is None          # 1.0 is not faster
    assert osearch.select_candidate([0.0, 2.49, 2.49, 1.2]) == 1      # lowest index on ties
    assert osearch.select_candidate([1.0000001]) == 0


def test_rank_reading_is_the_one_table1_allows():
    """Five methods: with no ties the ranks on a problem are a permutation of 1..5 and the
    averages add up to 15.  Table 1's columns add up to less, which only the reading 'equal
    values share the lowest rank' produces (mean ranks would give exactly 15)."""
    for key in ("table1_avg_rank_kernelbench_l1", "table1_avg_rank_kernelbench_l2", "table1_avg_rank_pie"):
        assert sum(PV[key]) < 15 - 1.5
    rng = np.random.default_rng(3)
    t = rng.random((5, 40)) + 1
    assert abs(sum(osearch.average_rank(t)) - 15) < 1e-12
    t[1:4, :20] = 1.0                                                 # three methods tie at the bottom
    assert sum(osearch.average_rank(t)) == pytest.approx(15 - 20 * 3 / 40)   # ranks 3, 3, 3 instead of 3, 4, 5
    # brute force on a tiny table
    tiny = [[3.0, 1.0], [3.0, 2.0], [1.0, 2.0]]
    assert osearch.average_rank(tiny) == [(1 + 3) / 2, (1 + 1) / 2, (3 + 1) / 2]


def test_median_of_max_speedup():
    assert osearch.median_of_max_speedup([[1, 3], [2], [0.5, 0.7, 0.6]]) == 2
    assert osearch.median_of_max_speedup([[1, 3], [2], [0.5], [10]]) == 2.5
    # invariant under permutations of problems and of generations
    g = [[1.0, 2.5], [0.9], [4.0, 1.0, 3.0], [1.2, 1.1]]
    for perm in itertools.permutations(range(4)):
        assert osearch.median_of_max_speedup([g[i][::-1] for i in perm]) == pytest.approx((1.2 + 2.5) / 2)


# ---------------------------------------------------------------- the library against the oracle
@pytest.fixture(scope="module")
def lib():
    return binding.load_library()


def test_library_matches_oracle(lib):
    rng = np.random.default_rng(11)
    for name, th in osearch.THRESHOLDS.items():
        for sp in list(rng.uniform(0, 600, 200)) + [100.0, th[0], th[1], th[2]]:
            for ok in (True, False):
                assert binding.reward_bin(sp, ok, th) == osearch.reward_bin(sp, ok, th)
    for gamma in (1.0, 0.9, 0.5):
        for n in (1, 2, 7, 30):
            r = rng.integers(0, 5, n).astype(np.float64)
            u, v = binding.value_targets(r, gamma)
            wu, wv = osearch.value_targets(list(r), gamma)
            np.testing.assert_allclose(u, wu, rtol=1e-12)
            np.testing.assert_allclose(v, wv, rtol=1e-12)
            d = rng.integers(0, 8, n)
            np.testing.assert_allclose(binding.best_so_far(r, d, gamma), osearch.best_so_far(list(r), list(d), gamma), rtol=1e-12)
    for n in (1, 3, 8):
        for _ in range(20):
            f = np.round(rng.uniform(0, 3, n), 1)
            assert binding.select_candidate(f) == osearch.select_candidate(list(f))
    groups = [list(rng.uniform(0.5, 4, rng.integers(1, 9))) for _ in range(11)]
    assert binding.median_of_max(groups) == osearch.median_of_max_speedup(groups)
    assert binding.median_of_max(groups[:10]) == osearch.median_of_max_speedup(groups[:10])
    t = np.round(rng.uniform(1, 2, (5, 30)), 1)                       # rounding makes ties
    np.testing.assert_allclose(binding.average_rank(t), osearch.average_rank(t.tolist()), rtol=1e-15)


def test_library_rejects_bad_arguments(lib):
    with pytest.raises(binding.McError):
        binding.reward_bin(150, True, [140, 120, 475])
    with pytest.raises(binding.McError):
        binding.value_targets([1, 2], 0.0)
    with pytest.raises(binding.McError):
        binding.value_targets([1, float("nan")], 1.0)
    with pytest.raises(binding.McError):
        binding.best_so_far([1.0], [-1], 1.0)
    with pytest.raises(binding.McError):
        binding.select_candidate([float("nan")])
