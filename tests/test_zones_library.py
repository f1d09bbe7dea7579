"""The library's "pair rates -> memory zones" rule (rr_zones_from_pair_rates, the rule rr_detect_zones applies to the
rates it measures) against the oracle's (oracle/zones.py), fed with the same rate functions: same zones, same
anchor, cut and band, same number of rates consulted, same order of questions.  CPU only."""
import itertools

import numpy as np
import pytest

import paper_2405_11425_amd as rl
from oracle.zones import zones_from_pair_rates as oracle_zones
from test_zones_oracle import canonical, launch_noise_rate, planted_rate, table_rate


def both(make_rate, n, min_gap=0.02, max_zones=16):
    """Run the oracle and the library on two fresh copies of one rate function; assert that they agree in everything
    they report and asked the same questions in the same order.  Returns (zones, details)."""
    logs, outs, dets = [], [], []
    for fn in (oracle_zones, rl.zones_from_pair_rates):
        rate = make_rate()
        log = []

        def logged(a, b, again=False, rate=rate, log=log):
            log.append((a, b, bool(again)))
            return rate(a, b, again) if again else rate(a, b)
        d = {}
        outs.append(fn(logged, n, min_gap, max_zones, details=d))
        logs.append(log)
        dets.append(d)
    assert outs[0] == outs[1]
    assert logs[0] == logs[1]
    for key in ("same", "cut", "band", "n_zones", "pair_rates", "gave_up", "row", "merge_rates", "zones_before_merging"):
        assert dets[0][key] == dets[1][key], key
    return outs[1], dets[1]


def test_worked_examples():
    t = {(p, p): 100.0 for p in range(4)}
    t.update({(0, 1): 100.0, (0, 2): 95.0, (0, 3): 95.2, (2, 3): 99.5})
    zones, d = both(lambda: table_rate(t), 4)
    assert zones == [0, 0, 1, 1] and d["pair_rates"] == 12 and d["retakes"] == 0
    assert d["cut"] == pytest.approx(97.55, abs=1e-12) and d["band"] == pytest.approx(0.6125, abs=1e-12)
    t2 = {(p, p): 100.0 for p in range(4)}
    t2.update({(0, 1): 99.9, (0, 2): 97.0, (0, 3): 99.2, (2, 3): 90.0})
    zones, d = both(lambda: table_rate(t2), 4)
    assert zones == [0, 0, 1, 0] and d["cut"] == 98.0 and d["band"] == 0.5
    t3 = {(p, p): 100.0 for p in range(4)}
    t3.update({(0, 1): (97.3, 99.8), (0, 2): 95.0, (0, 3): 95.2, (2, 3): (97.8, 94.0)})
    zones, d = both(lambda: table_rate(t3), 4)
    assert zones == [0, 0, 1, 1] and d["retakes"] == 2


def test_every_partition_of_six_windows():
    seen = set()
    for labels in itertools.product(range(3), repeat=6):
        truth = tuple(canonical(labels))
        if truth in seen:
            continue
        seen.add(truth)
        zones, _ = both(lambda: planted_rate(truth), 6)
        assert zones == list(truth)


@pytest.mark.parametrize("truth", [
    [0] * 12 + [1] * 12 + [2] * 8,
    [0] * 8 + [1] * 8 + [2] * 4 + [0] * 4 + [2] * 6 + [1] * 2,
    [0] * 32,
    [0, 1] * 16,
    [0] + [1] * 31,
    list(range(16)) * 2,
    list(range(17)),                  # gives up
    [0] * 22 + [1] * 21 + [2] * 21,   # 64 windows
])
def test_planted_maps_under_noise(truth):
    for seed in range(10):
        zones, d = both(lambda: planted_rate(truth, noise=0.003, seed=seed), len(truth))
        if max(truth) < 16:
            assert zones == truth
        else:
            assert d["gave_up"] and zones == [0] * len(truth)


@pytest.mark.parametrize("truth", [
    [0] * 12 + [1] * 12 + [2] * 8,
    [0] * 8 + [1] * 8 + [2] * 4 + [0] * 4 + [2] * 6 + [1] * 2,
    [0] * 32,
    [0, 1] * 16,
])
def test_fastest_of_three_launches_recovers_planted_maps(truth):
    for stream in range(24):
        zones, d = both(lambda: launch_noise_rate(truth, stream), len(truth))
        assert zones == truth, (stream, zones, d)


def test_arguments_and_failures():
    ok = planted_rate([0, 0, 1, 1])
    for kw, needle in (({"n_windows": 0}, "n_windows"), ({"n_windows": 65}, "n_windows"),
                       ({"min_gap": 0.0}, "min_gap"), ({"min_gap": 0.5}, "min_gap"), ({"min_gap": float("nan")}, "min_gap"),
                       ({"max_zones": 0}, "max_zones"), ({"max_zones": 17}, "max_zones")):
        args = {"n_windows": 4, "min_gap": 0.02, "max_zones": 16}
        args.update(kw)
        with pytest.raises(rl.RandlineError) as e:
            rl.zones_from_pair_rates(ok, **args)
        assert e.value.code == rl.RR_EINVAL and needle in str(e.value)
    for bad in (float("nan"), float("inf"), -1.0):
        with pytest.raises(rl.RandlineError) as e:
            rl.zones_from_pair_rates(lambda a, b, again=False: bad if (a, b) == (0, 2) else 100.0, 4)
        assert e.value.code == rl.RR_EINVAL and "rate(0, 2)" in str(e.value)

    def raising(a, b, again=False):
        if (a, b) == (0, 3):
            raise KeyError("no such pair")
        return 100.0
    with pytest.raises(KeyError):
        rl.zones_from_pair_rates(raising, 4)


def test_detect_zones_validates_before_touching_a_device():
    cases = [
        (dict(region=(0, 1 << 30)), "region is NULL"),
        (dict(region=(4096 + 64, 1 << 30)), "aligned"),
        (dict(region=(4096, (1 << 30) + 128)), "multiple of n_windows"),
        (dict(region=(4096, 0)), "multiple of n_windows"),
        (dict(n_windows=0), "n_windows"),
        (dict(n_windows=65), "n_windows"),
        (dict(min_gap=0.7), "min_gap"),
        (dict(max_zones=17), "max_zones"),
        (dict(launches=65), "launches"),
        (dict(warmup=5000), "warm-up"),
        (dict(unroll=3), "unroll"),
        (dict(region=(4096, 1 << 40), n_windows=32), "2^32 lines"),
    ]
    for kw, needle in cases:
        args = dict(region=(4096, 1 << 30), n_windows=32)
        args.update(kw)
        with pytest.raises(rl.RandlineError) as e:
            rl.detect_zones(**args)
        assert e.value.code == rl.RR_EINVAL and needle in str(e.value), (kw, str(e.value))
