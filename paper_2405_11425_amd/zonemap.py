"""Which parts of an allocation lie in the same memory zone: a quick probe for the zone-phased read.

The full pair matrix is the "zones" experiment of the sweep driver; this is the short form for
callers that only want the map.  Two windows are read at the same time (even CUs one, odd CUs the
other); a pair inside one zone runs several per cent faster than a pair across zones (measured:
4 % apart, single launches scatter by 0.5 % inside a zone and 0.8 % across, and on a busy box a good
part of the launches is slower by up to 10 %: a pair's rate is therefore the upper quartile of its
launches, the second fastest of six, not the median).

The decision is made against a fixed cut, not against the best rate seen.  A window paired with
itself gives the rate of a pair that certainly shares a zone; the first row (window 0 with every
other one) shows whether there is a slower cluster, and the cut goes halfway between the two (or,
with no slower cluster, `min_gap` below the same-zone rate).  A rate close to the cut is measured
again with three times the launches.  Windows are then assigned greedily (the first unassigned
window opens a zone and takes every window that runs with it), zones whose first windows run
together are merged, and every window gets a second opinion against the first window of its zone:
one that fails it, or sits alone, moves to a zone whose first window it does run with.
"""
import statistics
from typing import List, Optional

import numpy as np

from . import binding as rl
from . import workloads as wl


def detect_zone_map(region, region_bytes: int, n_cus: int, n_windows: int = 32, reps: int = 6,
                    min_gap: float = 0.02, max_zones: int = 16, unroll: int = 8, warmup: int = 64,
                    details: Optional[dict] = None) -> List[int]:
    """zone_of_window[n_windows] for the first region_bytes of `region` (ids in order of first appearance).
    The probe launches use the ring-of-8 build of the read kernel by default, so that in a kernel trace they
    stay apart from a caller's own launches of the default (ring of 16) kernel.  `details`, if given, receives
    what the decision rests on: the same-zone rate, the cut, the first row of pair rates, the zones before merging."""
    if region_bytes % (n_windows * 128) != 0:
        raise ValueError("region_bytes must be a multiple of n_windows lines")
    waves = wl.resident_logical_waves(n_cus)
    iters = 4096
    parity = (np.arange(n_cus) % 2).astype(np.uint16)

    def pair_rate(a: int, b: int, n: int = reps) -> float:
        wm = rl.WindowMap(n_windows, parity, np.array([a, b], np.uint16))
        call = lambda seed: rl.rand_read(region, 128, waves * iters, iters, seed, wm, region_bytes=region_bytes,
                                         unroll=unroll)
        call(1000)                                     # the first launch with a new map is several per cent slower
        ms = sorted(call(wl.READ_SEED + i).kernel_ms_event for i in range(n))
        # What disturbs a launch makes it slower (on a busy box by up to 10 %, and often); launches faster than
        # the rest by more than 1 % have not been seen.  The upper quartile stands for the pair: the second
        # fastest of six launches, the fifth fastest of eighteen.
        return waves * iters * 128 / ms[n // 4] / 1e6

    # The first launches of a process can run 2-3 % slow for some tens of milliseconds (seen: the first 50): a
    # warm-up, and the anchor below is measured before and after the first row, the faster of the two counts.
    for i in range(warmup):
        rl.rand_read(region, 128, waves * iters, iters, 2000 + i, rl.WindowMap(n_windows, parity, np.array([0, 0], np.uint16)),
                     region_bytes=region_bytes, unroll=unroll)
    # the rate of a pair that certainly shares a zone: a window with itself
    picks = sorted({0, n_windows // 3, 2 * n_windows // 3, n_windows - 1})
    before = statistics.median(pair_rate(w, w) for w in picks)
    # first row: window 0 with every other one; the rates fall into one or two clusters
    row = {b: pair_rate(0, b) for b in range(1, n_windows)}
    same = max(before, statistics.median(pair_rate(w, w) for w in picks))
    low = [r for r in row.values() if r < same * (1.0 - min_gap)]
    if len(low) >= 2 and statistics.median(low) < same * (1.0 - 1.4 * min_gap):
        cut = 0.5 * (same + statistics.median(low))    # two clusters: halfway between them
        band = 0.25 * (same - cut)
    else:                                              # nothing clearly slower so far
        cut = same * (1.0 - min_gap)
        band = 0.5 * min_gap * same

    if details is not None:
        details.update(gbps_same_zone=round(same, 1), gbps_cut=round(cut, 1), gbps_retest_band=round(band, 1),
                       gbps_window0_with=[round(row[b], 1) for b in range(1, n_windows)])

    def together(a: int, b: int, first=None) -> bool:
        r = pair_rate(a, b) if first is None else first
        if abs(r - cut) < band:                        # too close to call: measure again, longer
            r = pair_rate(a, b, 3 * reps)
        return r >= cut

    zone = [-1] * n_windows
    n_zones = 0
    while -1 in zone:
        if n_zones == max_zones:
            if details is not None:
                details.update(gave_up_with=list(zone))
            return [0] * n_windows
        ref = zone.index(-1)
        zone[ref] = n_zones
        for b in range(n_windows):
            if zone[b] == -1 and together(ref, b, row.get(b) if ref == 0 else None):
                zone[b] = n_zones
        n_zones += 1
    if details is not None:
        details.update(zones_before_merging=list(zone))
    # zones whose first windows run together are one zone
    firsts = [zone.index(z) for z in range(n_zones)]
    merged = list(range(n_zones))
    for a in range(n_zones):
        for b in range(a + 1, n_zones):
            if merged[b] == b and merged[a] == a and pair_rate(firsts[a], firsts[b], 3 * reps) >= cut:
                merged[b] = a
    zone = [merged[z] for z in zone]
    # second opinion on every window: it must run together with the first window of its zone; one that does not, or
    # that is alone, moves to a zone whose first window it does run with (if there is one)
    for w in range(n_windows):
        first = zone.index(zone[w])
        alone = zone.count(zone[w]) == 1
        if (first == w and not alone) or (first != w and together(first, w)):
            continue
        for z in sorted(set(zone) - {zone[w]}):
            if zone.index(z) != w and pair_rate(zone.index(z), w, 3 * reps) >= cut:
                zone[w] = z
                break
    order = {z: i for i, z in enumerate(dict.fromkeys(zone))}
    return [order[z] for z in zone]
