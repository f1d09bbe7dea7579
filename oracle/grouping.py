"""CPU oracle for the "heatmap -> compute-unit groups" step.

TEST INFRASTRUCTURE ONLY; never imported by the product package.

Paper, Sec. 2.2: the access kernel is run on exactly two SMs for all pairs;
pairs that share a memory-side resource run slower than pairs that do not, and
re-arranging the indices makes the groups visible (Fig. 2, Fig. 3).  The paper
gives no algorithm for the re-arrangement.  The reading taken here:

  1. every unordered pair (a,b), a<b, gets a ratio
         r_ab = T[a][b] / (S[a] + S[b])      if single-unit throughputs S are given,
         r_ab = T[a][b] / max_{c<d} T[c][d]  otherwise;
     a pair that does not interfere has r close to 1, one that does has r lower;
  2. sort the ratios ascending; the split point is the largest gap between
     neighbours (first one on ties);
  3. if that gap is smaller than `min_gap` times the median ratio the matrix has
     no structure: every unit is its own group;
  4. otherwise the threshold is the midpoint of the gap, pairs below it are
     "linked", and the groups are the connected components of the link graph;
  5. groups are numbered by their smallest member; the re-ordered index lists
     units by (group, unit id).

The partition is the result; the order within it is one valid choice.
Everything is done in float64 with plain loops so that it can be read against
the five steps above.
"""
from typing import Optional, Tuple

import numpy as np


def groups_from_heatmap(T: np.ndarray, singles: Optional[np.ndarray] = None,
                        min_gap: float = 0.05) -> Tuple[np.ndarray, np.ndarray, float]:
    """Return (group_of_unit[n], order[n], threshold).  threshold is NaN if no structure."""
    T = np.asarray(T, dtype=np.float64)
    n = T.shape[0]
    assert T.shape == (n, n)
    pairs = [(a, b) for a in range(n) for b in range(a + 1, n)]
    if not pairs:
        return np.zeros(n, dtype=np.int64), np.arange(n, dtype=np.int64), float("nan")
    # the rule is defined for ordinary throughputs only: finite, not negative, not all zero, singles positive
    if any(not np.isfinite(T[a, b]) or T[a, b] < 0 for a, b in pairs):
        raise ValueError("pair throughputs must be finite and non-negative")
    if singles is not None and any(not np.isfinite(x) or not x > 0 for x in np.asarray(singles, dtype=np.float64)):
        raise ValueError("single-unit throughputs must be finite and positive")
    if singles is None and not max(T[a, b] for a, b in pairs) > 0:
        raise ValueError("every pair throughput is zero")
    if singles is not None:
        S = np.asarray(singles, dtype=np.float64)
        r = np.array([T[a, b] / (S[a] + S[b]) for a, b in pairs], dtype=np.float64)
    else:
        top = max(T[a, b] for a, b in pairs)
        r = np.array([T[a, b] / top for a, b in pairs], dtype=np.float64)
    rs = np.sort(r)
    m = rs.size
    best_gap, best_i = -1.0, -1
    for i in range(m - 1):
        gap = rs[i + 1] - rs[i]
        if gap > best_gap:
            best_gap, best_i = gap, i
    # median of the sorted ratios (mean of the two middle ones when m is even)
    median = rs[m // 2] if m % 2 == 1 else 0.5 * (rs[m // 2 - 1] + rs[m // 2])
    group = -np.ones(n, dtype=np.int64)
    if best_i < 0 or best_gap < min_gap * median:
        group = np.arange(n, dtype=np.int64)
        threshold = float("nan")
    else:
        threshold = 0.5 * (rs[best_i] + rs[best_i + 1])
        linked = np.zeros((n, n), dtype=bool)
        for (a, b), rab in zip(pairs, r):
            if rab < threshold:
                linked[a, b] = linked[b, a] = True
        next_group = 0
        for start in range(n):
            if group[start] >= 0:
                continue
            group[start] = next_group
            frontier = [start]
            while frontier:
                u = frontier.pop()
                for v in range(n):
                    if linked[u, v] and group[v] < 0:
                        group[v] = next_group
                        frontier.append(v)
            next_group += 1
    order = np.array(sorted(range(n), key=lambda u: (group[u], u)), dtype=np.int64)
    return group, order, threshold
