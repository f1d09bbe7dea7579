"""Seeded, synthetic workload definitions shared by the tests, the sweep driver
and bench.py: sizes, seeds, window maps, CU samples.

This module holds none of the benchmark's arithmetic (no fill function, no
index hash, no checksum): it only names inputs.  Random choices use numpy's
seeded generator.

The paper's workload (Sec. 2.1) is fully synthetic -- uniformly random lines in
a region of varying size -- so these inputs do not stand in for a dataset; they
are the workload itself, at MI355X sizes (regions of 1..256 GiB instead of up
to 80 GB).
"""
from dataclasses import dataclass
from typing import List, Optional, Sequence, Tuple

import numpy as np

GiB = 1 << 30
MiB = 1 << 20

FILL_SEED = 1
READ_SEED = 7
ITERS_PER_WAVE = 4096

# hardware shape of one MI355X in SPX mode: 8 XCDs x 32 CUs, 4 SIMDs per CU, 8 waves per SIMD
N_XCD = 8
CUS_PER_XCD = 32
WAVES_PER_CU = 32


@dataclass(frozen=True)
class ReadConfig:
    """One rand_read invocation: region, line shape, logical waves x iterations."""
    name: str
    region_bytes: int
    line_bytes: int
    lanes_per_line: int
    logical_waves: int
    iters_per_wave: int
    fill_seed: int = FILL_SEED
    read_seed: int = READ_SEED

    @property
    def n_reads(self) -> int:
        return self.logical_waves * self.iters_per_wave

    @property
    def bytes_read(self) -> int:
        return self.n_reads * self.line_bytes


def resident_logical_waves(n_cus: int = N_XCD * CUS_PER_XCD, lanes_per_line: int = 32) -> int:
    """Logical waves that fill every wave slot of the device exactly once."""
    return n_cus * WAVES_PER_CU * (64 // lanes_per_line)


def pr1_reference() -> ReadConfig:
    """256 MiB region, 2^20 random 128-byte lines (32 lanes x 4 B), 256 logical waves x 4096."""
    return ReadConfig("pr1-256MiB", 256 * MiB, 128, 32, 256, ITERS_PER_WAVE)


SWEEP_REGIONS_GIB = [1, 2, 4, 8, 16, 32, 64, 128, 192, 256]


def region_sweep(max_region_bytes: int = 256 * GiB, n_cus: int = N_XCD * CUS_PER_XCD) -> List[ReadConfig]:
    """Region-size sweep: all wave slots occupied, each logical wave reads 4096 random 128-byte lines."""
    W = resident_logical_waves(n_cus, 32)
    return [ReadConfig(f"sweep-{s}GiB", s * GiB, 128, 32, W, ITERS_PER_WAVE)
            for s in SWEEP_REGIONS_GIB if s * GiB <= max_region_bytes]


LINE_SHAPES = [(128, 32), (256, 32), (512, 32), (256, 64)]  # (line_bytes, lanes_per_line)


def line_width_sweep(region_bytes: int, total_reads: int = 1 << 30) -> List[ReadConfig]:
    """32 lanes x {4,8,16} B and 64 lanes x 4 B, 2^30 reads in total, at one region size."""
    out = []
    for line_bytes, lanes in LINE_SHAPES:
        W = total_reads // ITERS_PER_WAVE
        out.append(ReadConfig(f"line-{lanes}x{line_bytes // lanes}B-{region_bytes // GiB}GiB", region_bytes,
                              line_bytes, lanes, W, ITERS_PER_WAVE))
    return out


def probe_config(region_bytes: int = 16 * GiB) -> ReadConfig:
    """Pair probe: 2^22 random 128-byte reads per pair (1024 logical waves x 4096)."""
    return ReadConfig("probe-16GiB", region_bytes, 128, 32, (1 << 22) // ITERS_PER_WAVE, ITERS_PER_WAVE)


# ----------------------------------------------------------------------------- window maps

def window_map_random_per_cu(n_cus: int, n_windows: int, seed: int) -> Tuple[np.ndarray, np.ndarray]:
    """The paper's baseline placement (Sec. 2.1): every CU is its own group and
    draws its window independently and uniformly (not balanced)."""
    rng = np.random.default_rng(seed)
    group_of_cu = np.arange(n_cus, dtype=np.uint16)
    window_of_group = rng.integers(0, n_windows, size=n_cus).astype(np.uint16)
    return group_of_cu, window_of_group


def window_map_own_per_cu(n_cus: int) -> Tuple[np.ndarray, np.ndarray]:
    """Every CU is its own group with a window of its own (n_windows = n_cus): the finest placement."""
    ids = np.arange(n_cus, dtype=np.uint16)
    return ids, ids.copy()


def window_map_for_selected_cus(n_cus: int, selected: Sequence[int], windows: Sequence[int]) -> Tuple[np.ndarray, np.ndarray]:
    """Only the selected CUs take part, the i-th of them as group i reading windows[i]; all others are excluded."""
    group_of_cu = np.full(n_cus, 0xFFFF, dtype=np.uint16)
    group_of_cu[np.asarray(selected, dtype=np.int64)] = np.arange(len(selected), dtype=np.uint16)
    return group_of_cu, np.asarray(windows, dtype=np.uint16)


def window_map_by_xcd(cu_table: np.ndarray, n_windows: int) -> Tuple[np.ndarray, np.ndarray]:
    """Group = XCD (the first hardware coordinate); XCD x reads window x mod n_windows
    (the paper's group-to-chunk placement, Sec. 2.4, with the XCD as the group)."""
    xcc = np.asarray(cu_table)[:, 0].astype(np.int64)
    ids = np.unique(xcc)
    group_of_cu = np.searchsorted(ids, xcc).astype(np.uint16)
    window_of_group = (np.arange(ids.size) % n_windows).astype(np.uint16)
    return group_of_cu, window_of_group


def window_map_by_se(cu_table: np.ndarray, n_windows: int) -> Tuple[np.ndarray, np.ndarray]:
    """Group = shader engine, i.e. the pair (xcc, se) -- the 8-CU groups that the block pair probe
    finds on the MI355X; group g reads window g mod n_windows."""
    t = np.asarray(cu_table).astype(np.int64)
    key = t[:, 0] * 64 + t[:, 1]
    ids = np.unique(key)
    group_of_cu = np.searchsorted(ids, key).astype(np.uint16)
    window_of_group = (np.arange(ids.size) % n_windows).astype(np.uint16)
    return group_of_cu, window_of_group


def window_map_from_groups(group_of_cu: Sequence[int], n_windows: int) -> Tuple[np.ndarray, np.ndarray]:
    """Placement for an arbitrary CU grouping (e.g. the one inferred from the pair probe)."""
    g = np.asarray(group_of_cu, dtype=np.uint16)
    n_groups = int(g[g != 0xFFFF].max()) + 1
    return g, (np.arange(n_groups) % n_windows).astype(np.uint16)


def synthetic_cu_table(n_xcd: int = N_XCD, n_se: int = 4, cus_per_se: int = 8) -> np.ndarray:
    """A CU table shaped like the device's, for host-side tests: rows (xcc, se, sh, cu)."""
    rows = [(x, s, 0, c) for x in range(n_xcd) for s in range(n_se) for c in range(cus_per_se)]
    return np.array(rows, dtype=np.uint32)


def probe_cu_sample(cu_table: np.ndarray, n: int = 64) -> np.ndarray:
    """CUs for the pair probe: n / n_xcd per XCD, taken as adjacent-id pairs spread over the
    XCD's shader engines, so that both "neighbouring CUs share something" and per-SE / per-XCD
    structure can show up in the heatmap."""
    table = np.asarray(cu_table)
    xcds = np.unique(table[:, 0])
    per_xcd = n // xcds.size
    picked: List[int] = []
    for x in xcds:
        ids = np.flatnonzero(table[:, 0] == x)
        n_pairs = per_xcd // 2
        starts = np.linspace(0, ids.size - 2, n_pairs).round().astype(int)
        starts -= starts % 2
        for s in starts:
            picked.extend([int(ids[s]), int(ids[s + 1])])
    return np.array(sorted(set(picked)), dtype=np.uint32)
