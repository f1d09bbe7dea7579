"""Which parts of an allocation lie in the same memory zone: a quick probe for the zone-phased read.

The full pair matrix is the "zones" experiment of the sweep driver; this is the short form for
callers that only want the map.  Two windows are read at the same time (even CUs one, odd CUs the
other); a pair inside one zone runs several per cent faster than a pair across zones.  Windows are
assigned greedily: the first unassigned window opens a zone and takes with it every window whose
pair rate with it is within `tolerance` of the best one seen for that reference.  A second pass then
pairs every window with one representative per zone and moves it to the zone it runs fastest with,
which absorbs windows that a noisy measurement had left on their own.
"""
import statistics
from typing import List

import numpy as np

from . import binding as rl
from . import workloads as wl


def detect_zone_map(region, region_bytes: int, n_cus: int, n_windows: int = 32, reps: int = 3,
                    tolerance: float = 0.02, max_zones: int = 16, unroll: int = 8) -> List[int]:
    """zone_of_window[n_windows] for the first region_bytes of `region` (ids in order of first appearance).
    The probe launches use the ring-of-8 build of the read kernel by default, so that in a kernel trace they
    stay apart from a caller's own launches of the default (ring of 16) kernel."""
    if region_bytes % (n_windows * 128) != 0:
        raise ValueError("region_bytes must be a multiple of n_windows lines")
    waves = wl.resident_logical_waves(n_cus)
    iters = 4096
    parity = (np.arange(n_cus) % 2).astype(np.uint16)

    def pair_rate(a: int, b: int, n: int = reps) -> float:
        wm = rl.WindowMap(n_windows, parity, np.array([a, b], np.uint16))
        call = lambda seed: rl.rand_read(region, 128, waves * iters, iters, seed, wm, region_bytes=region_bytes,
                                         unroll=unroll)
        call(1000)
        ms = statistics.median(call(wl.READ_SEED + i).kernel_ms_event for i in range(n))
        return waves * iters * 128 / ms / 1e6

    zone = [-1] * n_windows
    n_zones = 0
    while -1 in zone:
        if n_zones == max_zones:                      # no clear structure: give up, everything in one zone
            return [0] * n_windows
        ref = zone.index(-1)
        zone[ref] = n_zones
        rates = {b: pair_rate(ref, b) for b in range(n_windows) if zone[b] == -1}
        if rates:
            best = max(max(rates.values()), pair_rate(ref, ref))
            for b, r in rates.items():
                if abs(r / best - (1.0 - tolerance)) < 0.5 * tolerance:     # too close to call: measure again, longer
                    r = pair_rate(ref, b, 3 * reps)
                if r >= (1.0 - tolerance) * best:
                    zone[b] = n_zones
        n_zones += 1
    if n_zones > 1:
        sizes = [zone.count(z) for z in range(n_zones)]
        keep = [z for z in range(n_zones) if sizes[z] > 1] or list(range(n_zones))
        reps_of = {z: zone.index(z) for z in keep}
        for w in range(n_windows):
            rates = {z: pair_rate(reps_of[z], w) for z in keep}
            zone[w] = max(rates, key=rates.get)
        order = {z: i for i, z in enumerate(dict.fromkeys(zone))}      # renumber by first appearance
        zone = [order[z] for z in zone]
    return zone
