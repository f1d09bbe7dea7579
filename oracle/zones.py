"""CPU oracle for the "pair rates -> memory zones" step.

TEST INFRASTRUCTURE ONLY; never imported by the product package.

Not in the paper as such: it is the paper's pair probe (Sec. 2.2: run the access
kernel on two units at a time and see which pairs slow each other down) applied
to pieces of memory instead of compute units.  The region is cut into n equal
windows; rate(a, b) is the read rate when half of the device reads window a
while the other half reads window b.  On the MI355X a pair of windows inside
one memory zone runs a few per cent faster than a pair across two zones.  The
rule that turns such rates into a zone per window, step by step:

  1. anchor: a window paired with itself certainly shares a zone with itself.
     same = the largest of rate(p, p) over p in {0, n/3, 2n/3, n-1}, taken once
     before and once after step 2 (a process' first launches can run slow, and
     what disturbs a launch only ever makes it slower: hence "largest").
  2. first row: row[b] = rate(0, b) for b = 1 .. n-1.
  3. cut: low = the row entries below same * (1 - min_gap).  If there are at
     least two of them and their median lies below same * (1 - 1.4 * min_gap),
     the row has two clusters and cut = (same + median(low)) / 2; otherwise
     cut = same * (1 - min_gap).  band = (same - cut) / 4.
  4. "a and b run together" means rate(a, b) >= cut; a rate closer to the cut
     than band is taken again (rate(a, b, again=True)) and the larger of the two
     counts.
  5. window 0 opens zone 0 and takes every b that runs together with it (row[b]
     is the first measurement of that pair).  Then, as long as a window is
     without a zone: the first such window opens the next zone and takes every
     later window without a zone that runs together with it.
  6. more than max_zones zones: no usable structure, every window gets zone 0.
  7. merge: rates taken while the process was still starting up can be a few
     per cent low (seen on the GPU: the first 50 launches of one process in
     five), which makes windows of zone 0 look foreign in step 2; they then
     open a zone of their own in step 5.  So the zones' first windows are
     compared once more, each pair with the longer measurement of step 4
     (again=True): going through the zones in order, a zone whose first window
     runs together (rate >= cut) with the first window of an earlier zone that
     is still on its own joins that zone (the earliest such one).  Ids are then
     renumbered in order of first appearance.

Zone ids are thereby numbered in order of first appearance.  With k zones
before merging the rule consults at most 8 + (n - 1) + (k - 1)(n - 2) rates in
steps 1-5 (for zones that are found large first, far fewer) and at most
k (k - 1) / 2 in step 7.
"""
from statistics import median
from typing import Callable, Dict, List, Optional


def zones_from_pair_rates(rate: Callable[..., float], n: int, min_gap: float = 0.02, max_zones: int = 16,
                          details: Optional[Dict] = None) -> List[int]:
    """zone_of_window[n].  rate(a, b) or rate(a, b, again=True) returns the pair's read rate."""
    assert n >= 1 and min_gap > 0
    picks = sorted({0, n // 3, 2 * n // 3, n - 1})
    same = max(rate(p, p) for p in picks)                       # step 1, first half
    row = {b: rate(0, b) for b in range(1, n)}                  # step 2
    same = max(same, max(rate(p, p) for p in picks))            # step 1, second half
    low = [r for r in row.values() if r < same * (1.0 - min_gap)]                 # step 3
    if len(low) >= 2 and median(low) < same * (1.0 - 1.4 * min_gap):
        cut = 0.5 * (same + median(low))
    else:
        cut = same * (1.0 - min_gap)
    band = 0.25 * (same - cut)
    consulted = [2 * len(picks) + len(row)]

    def together(a: int, b: int, first: Optional[float] = None) -> bool:        # step 4
        r = first
        if r is None:
            r = rate(a, b)
            consulted[0] += 1
        if abs(r - cut) < band:
            r = max(r, rate(a, b, again=True))
        return r >= cut

    zone = [-1] * n                                                              # step 5
    n_zones = 0
    gave_up = False
    while -1 in zone:
        if n_zones == max_zones:                                                 # step 6
            gave_up = True
            zone = [0] * n
            n_zones = 1
            break
        ref = zone.index(-1)
        zone[ref] = n_zones
        for b in range(ref + 1, n):
            if zone[b] == -1 and together(ref, b, row[b] if ref == 0 else None):
                zone[b] = n_zones
        n_zones += 1
    before = list(zone)
    merge_rates = 0
    if not gave_up:                                                              # step 7
        firsts = [zone.index(z) for z in range(n_zones)]
        joined = list(range(n_zones))
        for zb in range(1, n_zones):
            for za in range(zb):
                if joined[za] != za:
                    continue
                merge_rates += 1
                if rate(firsts[za], firsts[zb], again=True) >= cut:
                    joined[zb] = za
                    break
        ids: Dict[int, int] = {}
        zone = [ids.setdefault(joined[z], len(ids)) for z in zone]
        n_zones = len(ids)
    if details is not None:
        details.update(same=same, cut=cut, band=band, n_zones=n_zones, pair_rates=consulted[0], gave_up=gave_up,
                       row=[row[b] for b in range(1, n)], merge_rates=merge_rates, zones_before_merging=before)
    return zone
