"""Pins of the grouping oracle (oracle/grouping.py): recover planted partitions.

The paper (Sec. 2.2, Fig. 3) reports 14 groups of 6 or 8 SMs, found from the
pair heatmap; the planted matrices below have that shape and the shape expected
of the target GPU (8 equal groups), with noise, and with unit ids shuffled so
that contiguity of ids cannot be what is detected.
"""
import numpy as np
import pytest

from oracle.grouping import groups_from_heatmap


def planted(sizes, seed, slow=0.6, noise=0.02, shuffle=True, per_unit=100.0):
    rng = np.random.default_rng(seed)
    n = sum(sizes)
    truth = np.repeat(np.arange(len(sizes)), sizes)
    if shuffle:
        truth = truth[rng.permutation(n)]
    T = np.zeros((n, n))
    for a in range(n):
        for b in range(a + 1, n):
            base = 2 * per_unit * (slow if truth[a] == truth[b] else 1.0)
            T[a, b] = T[b, a] = base * (1 + noise * rng.standard_normal())
    return T, truth


def same_partition(g1, g2):
    pairs1 = {(a, b) for a in range(len(g1)) for b in range(len(g1)) if g1[a] == g1[b]}
    pairs2 = {(a, b) for a in range(len(g2)) for b in range(len(g2)) if g2[a] == g2[b]}
    return pairs1 == pairs2


@pytest.mark.parametrize("sizes", [[8] * 8, [8, 6, 8, 8, 6, 8, 8, 8, 8, 8, 8, 8, 8, 8], [2] * 16, [1, 1, 30]])
@pytest.mark.parametrize("use_singles", [False, True])
def test_recovers_planted_partition(sizes, use_singles):
    T, truth = planted(sizes, seed=len(sizes))
    singles = np.full(len(truth), 100.0) if use_singles else None
    group, order, thr = groups_from_heatmap(T, singles)
    assert same_partition(group, truth)
    assert sorted(order) == list(range(len(truth)))
    # re-ordered matrix is block diagonal: group ids non-decreasing along the order
    assert all(group[order[i]] <= group[order[i + 1]] for i in range(len(order) - 1))
    assert 0.6 < thr < 1.0 if not use_singles else 0.6 < thr < 1.0


def test_groups_numbered_by_smallest_member():
    T, truth = planted([3, 3, 3], seed=3)
    group, _, _ = groups_from_heatmap(T)
    firsts = [int(np.flatnonzero(group == g)[0]) for g in range(3)]
    assert firsts == sorted(firsts) and group[0] == 0


def test_flat_matrix_has_no_structure():
    T, _ = planted([12], seed=1, slow=1.0, noise=0.01)
    group, order, thr = groups_from_heatmap(T)
    assert list(group) == list(range(12)) and np.isnan(thr)
    assert list(order) == list(range(12))


def test_two_by_two_boxes():
    """Adjacent ids sharing a resource (the paper's 2-by-2 dark boxes, Sec. 2.2)."""
    T, truth = planted([2] * 8, seed=5, shuffle=False)
    group, _, _ = groups_from_heatmap(T)
    assert list(group) == [i // 2 for i in range(16)]


def sym(n, entries):
    T = np.zeros((n, n))
    for (a, b), v in entries.items():
        T[a, b] = T[b, a] = v
    return T


def test_first_of_two_equal_largest_gaps_splits():
    """Worked by hand from the rule's statement (step 2: the first of equal gaps).  Ratios T/max are
    0.25, 0.25, 0.625, 0.625, 1, 1 (all exact in binary): the gaps 0.25 -> 0.625 and 0.625 -> 1 are both 0.375.
    The first one splits: threshold 0.4375, only the 0.25 pairs are linked -> {0,1}, {2,3}.  Taking the last of
    the equal gaps instead would give 0.8125 and one group of four."""
    T = sym(4, {(0, 1): 0.25, (2, 3): 0.25, (0, 2): 0.625, (1, 3): 0.625, (0, 3): 1.0, (1, 2): 1.0})
    group, order, thr = groups_from_heatmap(T, None, 0.05)
    assert group.tolist() == [0, 0, 1, 1] and order.tolist() == [0, 1, 2, 3] and thr == 0.4375


def test_gap_exactly_at_min_gap_times_median_counts_as_structure():
    """Step 3 says "smaller than": ratios 0.5, 1, 1 -> largest gap 0.5, median 1.  With min_gap = 0.5 the gap is
    not smaller than min_gap x median, so the matrix has structure (threshold 0.75, units 0 and 1 linked); with
    min_gap just above, it has none."""
    T = sym(3, {(0, 1): 50.0, (0, 2): 100.0, (1, 2): 100.0})
    group, order, thr = groups_from_heatmap(T, None, 0.5)
    assert group.tolist() == [0, 0, 1] and thr == 0.75
    group, order, thr = groups_from_heatmap(T, None, 0.5 + 2.0 ** -40)
    assert group.tolist() == [0, 1, 2] and np.isnan(thr)
    # the same with single-unit rates: ratio = T / (S_a + S_b) = 0.25, 0.5, 0.5 -> gap 0.25 = 0.5 x median 0.5
    group, order, thr = groups_from_heatmap(T, np.array([100.0, 100.0, 100.0]), 0.5)
    assert group.tolist() == [0, 0, 1] and thr == 0.375


@pytest.mark.parametrize("bad", ["nan", "negative", "zero", "single_zero", "single_nan"])
def test_matrices_the_rule_is_not_defined_for_are_refused(bad):
    T = sym(3, {(0, 1): 50.0, (0, 2): 100.0, (1, 2): 100.0})
    singles = None
    if bad == "nan":
        T[0, 2] = T[2, 0] = float("nan")
    elif bad == "negative":
        T[0, 1] = T[1, 0] = -1.0
    elif bad == "zero":
        T[:] = 0.0
    elif bad == "single_zero":
        singles = np.array([100.0, 0.0, 100.0])
    else:
        singles = np.array([100.0, float("nan"), 100.0])
    with pytest.raises(ValueError):
        groups_from_heatmap(T, singles)
