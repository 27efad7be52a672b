"""Pins for the oracle's selection / unstructured pruning (CPU only).

The oracle is checked against things it does not compute itself: a brute-force
O(N^2) rank written here from the definition, exhaustive optimality of the
compression mapping C(w) = argmin ||w - D(Theta)||^2 (Section 3.3), numpy's
partition, the closed-form Gaussian quantile, and the invariants that follow
from sparsity being the proportion of zero-valued parameters (Introduction) and
from pruning zeroing the weights of lowest magnitude (Section 3.3).
"""
import itertools
import math

import numpy as np
import pytest
from scipy.stats import norm

import oracle
import workloads


def brute_keep(keys, k):
    """rank_i = #{key_j > key_i} + #{j < i, key_j == key_i}; keep rank < k."""
    n = len(keys)
    keep = []
    for i in range(n):
        rank = sum(1 for j in range(n) if keys[j] > keys[i]) + sum(1 for j in range(i) if keys[j] == keys[i])
        keep.append(1 if rank < k else 0)
    return keep


def mag_key(x):
    return int(np.float32(x).view(np.uint32)) & 0x7FFFFFFF


CASES = {
    "random": lambda r: r.standard_normal(40).astype(np.float32),
    "all_equal": lambda r: np.full(17, 0.25, np.float32),
    "all_zero": lambda r: np.zeros(9, np.float32),
    "signed_zero_mix": lambda r: np.array([0.0, -0.0, 1.0, -0.0, 0.0, -1.0, 0.0], np.float32),
    "planted_ties": lambda r: np.array([3, -2, 2, 1, -2, 2, 5, -2, 0.5, 2], np.float32),
    "few_values": lambda r: r.integers(-3, 4, 64).astype(np.float32),
    "inf_nan": lambda r: np.array([1.0, np.inf, -np.inf, np.nan, 0.0, -3.0, 1e-40, -1e-40], np.float32),
    "single": lambda r: np.array([-7.0], np.float32),
}


@pytest.mark.parametrize("name", sorted(CASES))
def test_select_matches_brute_force_rank(name):
    rng = np.random.default_rng(7)
    x = CASES[name](rng)
    keys = [mag_key(v) for v in x]
    n = len(x)
    for k in sorted({0, 1, 2, n // 3, n // 2, n - 1, n} & set(range(n + 1))):
        sel, keep = oracle.select_keep(oracle.magnitude_keys(x), k)
        want = brute_keep(keys, k)
        assert keep.tolist() == want, (name, k)
        assert sel["k"] == k and sel["n"] == n
        assert int(keep.sum()) == k
        if k == 0:
            assert sel["threshold_key"] == 2**64 - 1 and sel["tie_end"] == 0
            assert sel["n_gt"] == sel["n_tie"] == sel["n_tie_kept"] == 0
            continue
        T = sorted(keys, reverse=True)[k - 1]
        assert sel["threshold_key"] == T
        assert sel["n_gt"] == sum(1 for q in keys if q > T)
        assert sel["n_tie"] == sum(1 for q in keys if q == T)
        assert sel["n_tie_kept"] == k - sel["n_gt"]
        assert 1 <= sel["n_tie_kept"] <= sel["n_tie"]
        # ties kept are exactly the ties below tie_end
        ties = [i for i in range(n) if keys[i] == T]
        kept_ties = [i for i in ties if keep[i]]
        assert kept_ties == [i for i in ties if i < sel["tie_end"]]
        if sel["n_tie_kept"] == sel["n_tie"]:
            assert sel["tie_end"] == n
        else:
            assert sel["tie_end"] == kept_ties[-1] + 1


def test_magnitude_key_is_abs_bit_pattern():
    x = np.array([1.5, -1.5, 0.0, -0.0, np.inf, -np.inf, 1e-45, -3.25], np.float32)
    keys = oracle.magnitude_keys(x)
    want = np.abs(x).view(np.uint32).astype(np.uint64)
    assert keys.tolist() == want.tolist()
    assert keys[2] == keys[3] == 0


def test_prune_is_the_optimal_k_sparse_projection():
    """C(w): no other choice of k kept positions is closer to w (Section 3.3)."""
    rng = np.random.default_rng(11)
    for n in (5, 8, 11):
        x = rng.standard_normal(n).astype(np.float32)
        for k in range(n + 1):
            res = oracle.prune([x], [k / n])[0]
            assert res["select"]["k"] == k
            theta = res["theta"][0].astype(np.float64)
            best = float(np.sum((x.astype(np.float64) - theta) ** 2))
            for kept in itertools.combinations(range(n), k):
                cand = np.zeros(n)
                cand[list(kept)] = x[list(kept)]
                assert best <= float(np.sum((x - cand) ** 2)) + 1e-18


def test_threshold_matches_numpy_partition_and_invariants():
    rng = np.random.default_rng(3)
    for n, d in [(1000, 0.1), (4097, 0.5), (10000, 0.003), (777, 0.999)]:
        x = (rng.standard_normal(n) * 0.02).astype(np.float32)
        res = oracle.prune([x], [d])[0]
        k = res["select"]["k"]
        assert k == int(math.floor(d * n + 0.5))
        mask = res["mask"][0].astype(bool)
        assert int(mask.sum()) == k
        a = np.abs(x)
        kth = np.partition(a, n - k)[n - k]
        assert res["select"]["threshold_key"] == int(kth.view(np.uint32))
        assert a[mask].min() >= a[~mask].max()
        theta = res["theta"][0]
        assert np.array_equal(theta[mask].view(np.uint32), x[mask].view(np.uint32))
        assert np.all(theta[~mask].view(np.uint32) == 0)


def test_pruned_positions_are_positive_zero_and_kept_values_bit_exact():
    x = np.array([-0.0, -5.0, 1e-30, -1e-30, 2.0, -0.0], np.float32)
    res = oracle.prune([x], [0.5])[0]
    assert res["mask"][0].tolist() == [0, 1, 1, 0, 1, 0]
    assert res["theta"][0].view(np.uint32).tolist() == [0, x[1:2].view(np.uint32)[0], x[2:3].view(np.uint32)[0], 0,
                                                        x[4:5].view(np.uint32)[0], 0]
    # keeping everything copies -0 bit for bit
    res = oracle.prune([x], [1.0])[0]
    assert np.array_equal(res["theta"][0].view(np.uint32), x.view(np.uint32))


def test_kept_count_rounds_half_away_from_zero():
    assert oracle.kept_count(0.02, 1024 * 1024) == 20972        # 20971.52
    assert oracle.kept_count(0.5, 5) == 3                       # 2.5 -> 3 (not banker's 2)
    assert oracle.kept_count(0.5, 7) == 4
    assert oracle.kept_count(0.25, 2) == 1                      # 0.5 -> 1
    assert oracle.kept_count(0.0, 10) == 0
    assert oracle.kept_count(1.0, 10) == 10
    assert oracle.kept_count(0.1, 1207959552) == 120795955
    assert oracle.kept_count(0.3, 2032) == 610


def test_single_matrix_workload_count_and_gaussian_quantile():
    """1024x1024 N(0, 0.02^2) at density 0.02: exactly 20 972 kept and the
    threshold sits at sigma * Phi^-1(1 - d/2) within sampling error."""
    (w,) = workloads.single_matrix()
    res = oracle.prune([w], [0.02])[0]
    sel = res["select"]
    assert sel["k"] == 20972 and int(res["mask"][0].sum()) == 20972
    t = float(np.array([sel["threshold_key"]], np.uint32).view(np.float32)[0])
    d = 0.02
    q = 0.02 * norm.ppf(1 - d / 2)
    # s.e. of the quantile: sqrt(p(1-p)/n) / pdf
    se = math.sqrt(d * (1 - d) / w.size) / (2 * norm.pdf(q / 0.02) / 0.02)
    assert abs(t - q) < 5 * se


def test_global_scope_spans_tensors_in_list_order():
    a = np.array([[1.0, -4.0], [2.0, 2.0]], np.float32)
    b = np.array([2.0, -3.0, 2.0], np.float32)
    res = oracle.prune([a, b], [4 / 7])[0]         # k = 4: 4, 3, then two of the four 2s (lowest flat index)
    assert res["select"]["k"] == 4
    assert res["mask"][0].tolist() == [[0, 1], [1, 1]]
    assert res["mask"][1].tolist() == [0, 1, 0]
    assert res["select"]["n_tie"] == 4 and res["select"]["n_tie_kept"] == 2 and res["select"]["tie_end"] == 4
    per = oracle.prune([a, b], [0.5], scope=oracle.SCOPE_PER_TENSOR)[0]
    assert per["mask"][0].tolist() == [[0, 1], [1, 0]]
    assert per["mask"][1].tolist() == [1, 1, 0]       # k = llround(1.5) = 2: 3 and the first 2
    assert [s["k"] for s in per["select"]] == [2, 2]


def test_multi_density_results_are_nested_and_monotone():
    rng = np.random.default_rng(5)
    ts = [rng.standard_normal((8, 3, 3, 3)).astype(np.float32), rng.standard_normal((10, 16)).astype(np.float32)]
    ds = workloads.search_densities()
    multi = oracle.prune(ts, ds)
    prev_mask, prev_t = None, None
    for d, res in zip(ds, multi):
        single = oracle.prune(ts, [d])[0]
        assert single["select"] == res["select"]
        for m1, m2 in zip(single["mask"], res["mask"]):
            assert np.array_equal(m1, m2)
        flat = np.concatenate([m.reshape(-1) for m in res["mask"]])
        if prev_mask is not None:
            assert np.all(flat >= prev_mask)                  # nested masks
            assert res["select"]["threshold_key"] <= prev_t   # thresholds fall as density grows
        prev_mask, prev_t = flat, res["select"]["threshold_key"]


def test_planted_mistakes_are_caught_by_the_brute_force():
    """The brute-force rank distinguishes the usual slips (>= for >, highest index wins)."""
    keys = [2, 5, 2, 2, 1]
    assert brute_keep(keys, 3) == [1, 1, 1, 0, 0]
    wrong_highest_index = [0, 1, 1, 1, 0]
    assert brute_keep(keys, 3) != wrong_highest_index
