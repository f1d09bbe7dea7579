"""Do the pins of the zone oracle have teeth?  Each case plants one plausible mistake into a copy of the source of
oracle/zones.py, and the pins of tests/test_zones_oracle.py (worked examples, exhaustive partitions, planted maps
under noise, counts of rates consulted) are run against the mutated rule: every planted mistake must make at least one
of them fail, and the unmodified source must pass them all.  CPU only."""
import inspect
import os

import pytest

import test_zones_oracle as pins
from oracle import zones as zones_module

SRC = inspect.getsource(zones_module)

MISTAKES = [
    ("anchor is the smallest rate, not the largest", "same = max(rate(p, p) for p in picks)                       # step 1, first half",
     "same = min(rate(p, p) for p in picks)                       # step 1, first half"),
    ("anchor not taken again after the row", "same = max(same, max(rate(p, p) for p in picks))            # step 1, second half",
     "same = max(same, 0.0)"),
    ("cut at the slow cluster instead of halfway", "cut = 0.5 * (same + median(low))", "cut = median(low)"),
    ("row always split in two clusters", "if len(low) >= 2 and median(low) < same * (1.0 - 1.4 * min_gap):", "if len(low) >= 1:"),
    ("no retake band", "band = 0.25 * (same - cut)", "band = 0.0"),
    ("the smaller of two measurements counts", "r = max(r, rate(a, b, again=True))", "r = min(r, rate(a, b, again=True))"),
    ("a zone also takes windows that already have one", "if zone[b] == -1 and together(ref, b, row[b] if ref == 0 else None):",
     "if together(ref, b, row[b] if ref == 0 else None):"),
    ("the first row is not reused for window 0", "together(ref, b, row[b] if ref == 0 else None)", "together(ref, b, None)"),
    ("one zone too many before giving up", "if n_zones == max_zones:", "if n_zones > max_zones:"),
    ("no merge step", "if not gave_up:                                                              # step 7", "if False:"),
    ("merged zones keep their old numbers", "zone = [ids.setdefault(joined[z], len(ids)) for z in zone]", "zone = [joined[z] for z in zone]"),
    ("merge compares with the first measurement, not the longer one", "if rate(firsts[za], firsts[zb], again=True) >= cut:",
     "if rate(firsts[za], firsts[zb]) >= cut:"),
    ("a joined zone can still be joined to", "if joined[za] != za:\n                    continue", "if False:\n                    continue"),
]


def rule_from(source):
    namespace = {}
    exec(compile(source, "zones_variant.py", "exec"), namespace)
    return namespace["zones_from_pair_rates"]


def run_pins(rule, monkeypatch):
    """Names of the pins that fail for this rule."""
    monkeypatch.setattr(pins, "zones_from_pair_rates", rule)
    failed = []
    for name, fn in sorted(vars(pins).items()):
        if not name.startswith("test_") or not callable(fn):
            continue
        cases = [()]
        for mark in getattr(fn, "pytestmark", []):
            if mark.name == "parametrize":
                cases = [(v,) if not isinstance(v, tuple) else v for v in mark.args[1]]
        for args in cases:
            try:
                fn(*args)
            except Exception:          # an assertion, or the rule asking for a pair the worked example does not hold
                failed.append(name)
                break
    return failed


def test_unmodified_rule_passes_every_pin(monkeypatch):
    assert run_pins(rule_from(SRC), monkeypatch) == []


@pytest.mark.parametrize("name,old,new", MISTAKES, ids=[m[0] for m in MISTAKES])
def test_planted_mistake_is_caught(monkeypatch, name, old, new):
    assert SRC.count(old) == 1, f"mistake '{name}': snippet to replace occurs {SRC.count(old)} times in the oracle"
    failed = run_pins(rule_from(SRC.replace(old, new)), monkeypatch)
    assert failed, f"no pin noticed: {name}"
