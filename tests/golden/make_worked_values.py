#!/usr/bin/env python3
"""Recompute every entry of worked_values.txt from the definitions, with numpy only.

    python tests/golden/make_worked_values.py            # print the entries
    python tests/golden/make_worked_values.py --check    # compare with worked_values.txt

This script is a third implementation of the checksum contract: it uses neither the C oracle nor
the HIP library (and nothing from the product package); arithmetic is numpy uint64 with wrap-around.
The region is never materialised: words are regenerated from their 64-bit index.
"""
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
GAMMA = np.uint64(0x9E3779B97F4A7C15)
np.seterr(over="ignore")


def mix64(z):
    z = np.asarray(z, dtype=np.uint64)
    z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
    z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
    return z ^ (z >> np.uint64(31))


def sm(seed, k):
    """k-th output (array allowed) of SplitMix64 seeded with `seed` (array allowed)."""
    return mix64(np.asarray(seed, dtype=np.uint64) + (np.asarray(k, dtype=np.uint64) + np.uint64(1)) * GAMMA)


def fill_words(seed, idx):
    idx = np.asarray(idx, dtype=np.uint64)
    q = sm(seed, idx >> np.uint64(1))
    return np.where(idx & np.uint64(1), q >> np.uint64(32), q & np.uint64(0xFFFFFFFF))


def line_indices(R, B, W, I, read_seed, n_windows=1, window_of_group=None):
    L = R // B
    L_win = L // n_windows
    w = np.arange(W, dtype=np.uint64)
    wave_seed = sm(read_seed, w)                                   # [W]
    h = sm(wave_seed[:, None], np.arange(I, dtype=np.uint64)[None, :])  # [W, I]
    idx = h % np.uint64(L_win)
    if window_of_group is not None:
        G = len(window_of_group)
        base = np.asarray(window_of_group, dtype=np.uint64)[(w % np.uint64(G)).astype(np.int64)] * np.uint64(L_win)
        idx = idx + base[:, None]
    return idx


def checksum(R, B, W, I, fill_seed, read_seed, n_windows=1, window_of_group=None, block=1 << 14):
    idx = line_indices(R, B, W, I, read_seed, n_windows, window_of_group).reshape(-1)
    wpl = B // 4
    total = np.uint64(0)
    offs = np.arange(wpl, dtype=np.uint64)
    for s in range(0, idx.size, block):
        words = idx[s:s + block, None] * np.uint64(wpl) + offs[None, :]
        total = total + fill_words(fill_seed, words).sum(dtype=np.uint64)
    return int(total)


def entries():
    out = {}
    out["sm_seed0"] = [int(x) for x in sm(0, np.arange(3))]
    out["fill_seed1_words0to7"] = [int(x) for x in fill_words(1, np.arange(8))]
    out["hash_seed7_wave0"] = [int(x) for x in sm(sm(7, 0), np.arange(3))]
    out["hash_seed7_wave1"] = [int(x) for x in sm(sm(7, 1), np.arange(3))]
    out["tiny_R4096_B128"] = [checksum(4096, 128, 4, 8, 1, 7)]
    out["tiny_R4096_B256"] = [checksum(4096, 256, 4, 8, 1, 7)]
    out["tiny_R4096_B512"] = [checksum(4096, 512, 4, 8, 1, 7)]
    out["tiny_R12288_B128"] = [checksum(12288, 128, 4, 8, 1, 7)]
    out["tiny_windowed_R4096_B128"] = [checksum(4096, 128, 4, 8, 1, 7, 2, [1, 0])]
    out["one_line_R128"] = [checksum(128, 128, 2, 3, 1, 7)]
    R = 1 << 28
    c = checksum(R, 128, 256, 4096, 1, 7)
    out["pr1_W256_I4096"] = [c]
    out["pr1_W1024_I1024"] = [checksum(R, 128, 1024, 1024, 1, 7)]
    idx = line_indices(R, 128, 256, 4096, 7)
    out["pr1_wave0_first_indices"] = [int(x) for x in idx[0, :4]]
    out["pr1_distinct_lines"] = [int(np.unique(idx).size)]
    out["pr1_mean_word"] = [c // (256 * 4096 * 32)]
    return out


def stored():
    vals = {}
    with open(os.path.join(HERE, "worked_values.txt")) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if "=" in line:
                k, v = line.split("=", 1)
                vals[k.strip()] = [int(t, 0) for t in v.split()]
    return vals


def main():
    got = entries()
    if "--check" in sys.argv:
        want = stored()
        bad = [k for k in want if got.get(k) != want[k]]
        print("worked_values.txt:", "all %d entries reproduced" % len(want) if not bad else "MISMATCH " + ", ".join(bad))
        return 1 if bad else 0
    for k, v in got.items():
        print(k, "=", " ".join(str(x) for x in v))
    return 0


if __name__ == "__main__":
    sys.exit(main())
