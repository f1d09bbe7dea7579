"""CPU-only checks of the product's host side: the C ABI library loads and exports what the
header declares, rejects bad arguments before touching a device, clusters heatmaps exactly like
the grouping oracle, and the workload/window-map generators produce valid inputs."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2405_11425_amd as rl
from paper_2405_11425_amd import workloads as wl
from oracle.grouping import groups_from_heatmap as oracle_groups
from test_grouping_oracle import planted, same_partition


def _has_gpu():
    try:
        import torch
        return torch.cuda.is_available()
    except ImportError:
        return False

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "randline.h")).read()
    declared = set(re.findall(r"\b(rr_[a-z_]+)\s*\(", header))
    assert declared >= {"rr_fill", "rr_rand_read", "rr_probe_pair", "rr_enumerate_cus"}
    lib = C.CDLL(rl.library_path())
    for name in sorted(declared):
        assert hasattr(lib, name), f"{name} is declared in randline.h but not exported"
    assert declared == set(rl.binding.EXPORTS)


def test_header_is_plain_c(tmp_path):
    """The boundary is a C ABI: the header must compile as C99 (and as C++) on its own, with no HIP or torch types, and
    the structs the binding mirrors must have the sizes and field offsets the C compiler gives them."""
    import subprocess
    inc = os.path.join(os.path.dirname(os.path.abspath(__file__)), "..", "include")
    b = rl.binding
    mirrors = {"rr_launch_opts_t": b._Opts, "rr_result_t": b._Result, "rr_window_map_t": b._WindowMap,
               "rr_chase_result_t": b._ChaseResult, "rr_read_item_t": b._ReadItem,
               "rr_zone_probe_opts_t": b._ZoneProbeOpts, "rr_zone_probe_t": b._ZoneProbe, "rr_read_plan_t": b._ReadPlan}
    prints = []
    for cname, mirror in mirrors.items():
        prints.append(f'printf("%zu\\n", sizeof({cname}));')
        prints += [f'printf("%zu\\n", offsetof({cname}, {field}));' for field, _ in mirror._fields_]
    src = tmp_path / "abi.c"
    src.write_text('#include "randline.h"\n#include <stddef.h>\n#include <stdio.h>\nint main(void) {\n'
                   + "\n".join(prints) + "\nreturn RR_OK; }\n")
    exe = tmp_path / "abi"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", inc, "-o", str(exe), str(src)],
                   check=True)
    subprocess.run(["g++", "-std=c++11", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", inc, "-fsyntax-only", "-x", "c++",
                    str(src)], check=True)
    got = [int(x) for x in subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()]
    want = []
    for mirror in mirrors.values():
        want.append(C.sizeof(mirror))
        want += [getattr(mirror, field).offset for field, _ in mirror._fields_]
    assert got == want


def test_plans_of_reads_beyond_the_translation_reach():
    """rr_describe_read: what a call would do, from the host alone.  Over more than 256 GiB a plain read becomes one zone
    of at most 64 power-of-two windows, divided between the two halves of the XCDs so that of every pair of windows
    256 GiB apart each half may read at most one; every window stays readable by somebody; windows without a partner
    256 GiB away by both."""
    GiB = 1 << 30
    plan = lambda gib, B=128, **kw: rl.describe_read((1 << 21, gib * GiB), B, 16384 * 4096, 4096, **kw)
    for gib in (1, 64, 255, 256, 257, 260, 263):       # by default only from one whole window beyond 256 GiB on
        d = plan(gib)
        assert (d["mode"], d["zone_kernel"], d["xcd_split"]) == (rl.MODE_STREAM, 0, 0), gib
    for gib in list(range(257, 300)) + [320, 384, 448, 511, 512]:
        for B in (128, 512):
            d = plan(gib, B, xcd_split=rl.SPLIT_ON if gib < 264 else rl.SPLIT_DEFAULT)
            n, w = d["n_zone_windows"], d["zone_window_bytes"]
            assert (d["mode"], d["zone_kernel"], d["n_zones"], d["xcd_split"]) == (rl.MODE_STREAM, 1, 1, 1), gib
            assert w & (w - 1) == 0 and n <= 64 and (n - 1) * w < gib * GiB <= n * w
            assert 64 * (w // 2) < gib * GiB                                                    # the smallest such window
            all_windows = (1 << n) - 1
            assert d["zone_windows"] == [all_windows]
            lo, hi = d["split_windows"]
            reach = (256 * GiB) // w
            assert lo | hi == all_windows
            for k in range(n):
                partner = k + reach
                if partner < n:
                    for half in (lo, hi):
                        assert not ((half >> k) & 1 and (half >> partner) & 1), (gib, k)     # never both
                    assert ((lo >> k) & 1) != ((hi >> k) & 1) and ((lo >> partner) & 1) != ((hi >> partner) & 1)
                elif k - reach < 0:
                    assert (lo >> k) & 1 and (hi >> k) & 1, (gib, k)                          # nobody displaces it
            left_out = [bin(all_windows & ~half).count("1") for half in (lo, hi)]
            assert abs(left_out[0] - left_out[1]) <= 1 and sum(left_out) == 2 * max(0, n - reach)
    # switched off; asked for in vain; asked for on a small region (7/8 of it in place of 256 GiB); with a zone map
    assert plan(280, xcd_split=rl.SPLIT_OFF)["zone_kernel"] == 0
    assert plan(280, mode=rl.MODE_FLAT)["zone_kernel"] == 0 and plan(280, mode=rl.MODE_TICKET)["xcd_split"] == 0
    d = rl.describe_read((1 << 21, 280 * GiB), 128, 16384 * 100, 100)              # 100 reads per wave: no chunks of 64
    assert (d["zone_kernel"], d["xcd_split"], d["mode"]) == (0, 0, rl.MODE_FLAT)
    d = plan(1, xcd_split=rl.SPLIT_ON)
    assert d["xcd_split"] == 1 and d["n_zone_windows"] == 64 and bin(d["split_windows"][0]).count("1") == 56
    zm = [0] * 12 + [1] * 12 + [2] * 11
    d = plan(280, zone_of_window=zm)
    assert (d["n_zones"], d["xcd_split"], d["n_zone_windows"]) == (3, 0, 35)
    assert d["zone_windows"] == [0xFFF, 0xFFF000, 0x7FF000000]
    assert plan(280, zone_of_window=zm, zone_descending=True)["zone_windows"] == [0x7FF000000, 0xFFF000, 0xFFF]
    d = plan(280, zone_of_window=zm, xcd_split=rl.SPLIT_ON)      # several zones: one half gives up the upper windows, the other the lower
    assert d["xcd_split"] == 1 and d["split_windows"] == [(1 << 32) - 1, ((1 << 35) - 1) & ~0b111]
    with pytest.raises(rl.RandlineError) as e:       # the same checks as the call itself
        rl.describe_read((0, GiB), 128, 64, 64)
    assert e.value.code == rl.RR_EINVAL and "NULL" in str(e.value)


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU; asked for more it says so and exits before touching a device."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=60)
    assert r.returncode == 2 and "single-GPU" in r.stderr and r.stdout == ""


def test_strerror_and_codes():
    L = rl.lib()
    assert L.rr_strerror(0) == b"success"
    for code in (rl.RR_EINVAL, rl.RR_EHIP, rl.RR_EPLACE, -99):
        assert L.rr_strerror(code)


FAKE = (1 << 21, 1 << 20)  # an aligned, non-null "device pointer" that is never dereferenced on these paths


@pytest.mark.parametrize("args,kw,needle", [
    (((0, 4096), 128, 8, 8, 7), {}, "NULL"),
    ((FAKE, 100, 8, 8, 7), {}, "line_bytes"),
    ((FAKE, 128, 8, 8, 7), {"lanes_per_line": 64}, "4, 8 or 16"),
    ((FAKE, 128, 8, 8, 7), {"lanes_per_line": 16}, "lanes_per_line"),
    (((1 << 21, 1000), 128, 8, 8, 7), {}, "multiple of line_bytes"),
    (((1 << 21, 0), 128, 8, 8, 7), {}, "multiple of line_bytes"),
    ((((1 << 21) + 64, 4096), 128, 8, 8, 7), {}, "aligned"),
    (((1 << 21, (1 << 39) + (1 << 38)), 128, 8, 8, 7), {}, "2^32"),
    ((FAKE, 128, 9, 8, 7), {}, "multiple of iters_per_wave"),
    ((FAKE, 128, 8, 0, 7), {}, "at least 1"),
    ((FAKE, 128, 8, 8, 7), {"block_threads": 96}, "block_threads"),
    ((FAKE, 128, 8, 8, 7), {"unroll": 3}, "unroll"),
    ((FAKE, 512, 8, 8, 7), {"unroll": 16}, "unroll"),
    ((FAKE, 128, 8, 8, 7), {"bcast": 9}, "bcast"),
    ((FAKE, 128, 8, 8, 7), {"mode": 5}, "mode"),
    ((FAKE, 128, 8, 8, 7), {"nontemporal": 3}, "nontemporal"),
    ((FAKE, 128, 8, 8, 7), {"zone_bytes": 100}, "zone_bytes"),
    ((FAKE, 128, 8, 8, 7), {"zone_bytes": 128}, "at most 16"),
    ((FAKE, 128, 8, 8, 7), {"zone_bytes": 1 << 18, "chunk_iters": 64}, "chunk_iters"),
    ((FAKE, 128, 8, 8, 7), {"zone_bytes": 1 << 18, "zone_of_window": [0, 1]}, "not both"),
    ((FAKE, 128, 8, 8, 7), {"zone_of_window": [0, 1, 2]}, "divide"),
    ((FAKE, 128, 8, 8, 7), {"zone_of_window": [0, 16]}, "below 16"),
    ((FAKE, 128, 8, 8, 7), {"zone_of_window": [0] * 65}, "n_zone_windows"),
    ((FAKE, 128, 8, 8, 7), {"zone_of_window": [0, 1], "zone_descending": 2}, "zone_descending"),
    ((FAKE, 128, 8, 8, 7), {"xcd_split": 3}, "xcd_split"),
    ((FAKE, 128, 8, 8, 7), {"xcd_split": 1}, "xcd_split"),                       # 8 reads per wave: no chunks of 64
    ((FAKE, 128, 128, 64, 7), {"xcd_split": 1, "mode": 2}, "xcd_split"),
    (((1 << 21, 128), 128, 128, 64, 7), {"xcd_split": 1}, "2 to 64 zone windows"),  # a single line
    ((FAKE, 128, 8, 8, 7), {"zone_descending": True}, "zone_descending needs"),
    (((1 << 21, 3 << 20), 128, 8, 8, 7), {"zone_of_window": [0, 1]}, "power-of-two"),
])
def test_rand_read_rejects_bad_arguments_without_a_device(args, kw, needle):
    with pytest.raises(rl.RandlineError) as e:
        rl.rand_read(*args, **kw)
    assert e.value.code == rl.RR_EINVAL and needle in str(e.value)


def _expected_to_pass(ptr, nbytes, B, lanes, iters, wm, kw):
    """The header's argument rules, restated (for calls with n_reads = 0, which return before any device work)."""
    if ptr == 0 or B not in (128, 256, 512) or lanes not in (32, 64) or B // lanes not in (4, 8, 16):
        return False
    if nbytes == 0 or nbytes % B or ptr % B or nbytes // B > 1 << 32 or iters == 0:
        return False
    n_lines, G = nbytes // B, 1
    if wm is not None:
        G = wm.n_groups
        if not 1 <= G <= 1024 or wm.n_windows == 0 or n_lines % wm.n_windows or not 1 <= wm.group_of_cu.size <= 1024:
            return False
        if any(g != 0xFFFF and g >= G for g in wm.group_of_cu) or any(w >= wm.n_windows for w in wm.window_of_group):
            return False
    if kw.get("block_threads", 0) not in (0, 64, 128, 256) or kw.get("bcast", 0) > 3 or kw.get("nontemporal", 0) > 2:
        return False
    mode = kw.get("mode", 0)
    if mode > 3 or kw.get("chunk_iters", 0) % 64 or kw.get("first_wave", 0) % G:
        return False
    wdw = B // lanes // 4
    # the stream kernel: no map, DPP broadcast, 256 threads, ring of 8 or 16, chunks of a multiple of 16 that divide iters
    chunk = kw.get("chunk_iters", 0) or next((c for c in (256, 128, 64, 32, 16) if iters % c == 0), 16)
    streams = (wm is None and kw.get("bcast", 0) in (0, 2) and kw.get("block_threads", 0) in (0, 256)
               and (kw.get("unroll", 0) or (8 if wdw == 4 else 16)) in (8, 16) and iters % chunk == 0 and chunk % 16 == 0)
    if mode == rl.MODE_STREAM:
        return streams
    if not (mode == rl.MODE_AUTO and streams) and kw.get("unroll", 0) not in ((0, 2, 4, 8) if wdw == 4 else (0, 4, 8, 16)):
        return False
    if wm is not None and kw.get("mode", 0) == rl.MODE_FLAT and (G > 1 or (wm.group_of_cu == 0xFFFF).any()):
        return False
    return True


def test_argument_rules_hold_for_generated_calls():
    """Property test of rr_rand_read's validation: generated argument combinations are accepted or rejected as the
    header says.  Every call has n_reads = 0, so an accepted call returns before any device work (also on a GPU machine)."""
    from hypothesis import given, settings, strategies as st

    maps = st.none() | st.builds(
        lambda G, nw, cus, goc_bad, wog_bad: rl.WindowMap(
            nw, np.array([(c % max(G, 1)) if not (goc_bad and c == 1) else G + 3 for c in range(cus)], np.uint16)
            if cus else np.zeros(0, np.uint16),
            np.array([(g % max(nw, 1)) if not (wog_bad and g == 0) else nw + 1 for g in range(G)], np.uint16)),
        st.sampled_from([0, 1, 2, 8, 256, 1024, 1025]), st.sampled_from([0, 1, 2, 3, 8, 64]),
        st.sampled_from([0, 1, 4, 256, 1024]), st.booleans(), st.booleans())
    launch = st.fixed_dictionaries({}, optional={
        "block_threads": st.sampled_from([0, 64, 96, 128, 256, 512]), "unroll": st.sampled_from([0, 2, 4, 8, 16, 32]),
        "mode": st.sampled_from([0, 1, 2, 3]), "bcast": st.sampled_from([0, 1, 2, 3, 4]),
        "nontemporal": st.sampled_from([0, 1, 2, 3]), "chunk_iters": st.sampled_from([0, 64, 100, 512]),
        "first_wave": st.sampled_from([0, 1, 2, 8, 1024])})

    @settings(max_examples=600, deadline=None)
    # the value lists lean towards valid entries, so that a good third of the calls pass every rule
    @given(ptr=st.sampled_from([1 << 21] * 5 + [0, (1 << 21) + 64, (1 << 21) + 256]),
           nbytes=st.sampled_from([4096, 12288, 1 << 20, 3 << 20, 1 << 30, 1 << 39, 0, 1000, (1 << 39) + (1 << 38)]),
           B=st.sampled_from([128, 128, 256, 512, 64, 100, 1024]), lanes=st.sampled_from([32, 32, 32, 64, 16, 48]),
           iters=st.sampled_from([1, 7, 4096, 4096, 0]), wm=maps, kw=launch)
    def check(ptr, nbytes, B, lanes, iters, wm, kw):
        want = _expected_to_pass(ptr, nbytes, B, lanes, iters, wm, kw)
        try:
            got = rl.rand_read((ptr, nbytes), B, 0, iters, 7, wm, lanes_per_line=lanes, **kw)
            assert want, ("accepted", ptr, nbytes, B, lanes, iters, wm, kw)
            assert (got.checksum, got.waves_run, got.launches) == (0, 0, 0)
        except rl.RandlineError as e:
            assert e.code == rl.RR_EINVAL and not want, (str(e), ptr, nbytes, B, lanes, iters, wm, kw)

    check()


@pytest.mark.parametrize("wm,n_reads,kw,needle", [
    (rl.WindowMap(3, np.zeros(4, np.uint16), np.zeros(1, np.uint16)), 8, {}, "divide"),
    (rl.WindowMap(2, np.array([0, 2], np.uint16), np.array([0, 1], np.uint16)), 16, {}, "group_of_cu"),
    (rl.WindowMap(2, np.array([0, 1], np.uint16), np.array([0, 2], np.uint16)), 16, {}, "window_of_group"),
    (rl.WindowMap(2, np.array([0, 1], np.uint16), np.array([0, 1], np.uint16)), 24, {}, "multiple of n_groups"),
    (rl.WindowMap(2, np.array([0, 1], np.uint16), np.array([0, 1], np.uint16)), 16, {"first_wave": 1}, "first_wave"),
    (rl.WindowMap(2, np.array([0, 1], np.uint16), np.array([0, 1], np.uint16)), 16, {"mode": rl.MODE_FLAT}, "flat"),
    (rl.WindowMap(1, np.array([0, 0xFFFF], np.uint16), np.array([0], np.uint16)), 16, {"mode": rl.MODE_FLAT}, "flat"),
])
def test_window_map_validation(wm, n_reads, kw, needle):
    with pytest.raises(rl.RandlineError) as e:
        rl.rand_read(FAKE, 128, n_reads, 8, 7, wm, **kw)
    assert e.value.code == rl.RR_EINVAL and needle in str(e.value)


def test_fill_and_probe_validation():
    with pytest.raises(rl.RandlineError):
        rl.fill((0, 4096), 1)
    with pytest.raises(rl.RandlineError):
        rl.fill(((1 << 21) + 8, 4096), 1)
    with pytest.raises(rl.RandlineError):
        rl.fill((1 << 21, 4100), 1)
    with pytest.raises(rl.RandlineError) as e:
        rl.probe_pair(FAKE, 3, 3, 8, 8, 7)
    assert "differ" in str(e.value)
    with pytest.raises(rl.RandlineError) as e:
        rl.probe_cus(FAKE, [1, 2, 1], 8, 8, 7)
    assert "twice" in str(e.value)
    with pytest.raises(rl.RandlineError):
        rl.probe_cus(FAKE, [], 8, 8, 7)
    # a pinned run cannot be zone-phased (that kernel knows no excluded compute units) nor flat
    for kw in ({"zone_bytes": 1 << 19}, {"zone_of_window": [0, 1]}, {"mode": rl.MODE_FLAT}):
        with pytest.raises(rl.RandlineError) as e:
            rl.probe_cus(FAKE, [0, 1], 8, 8, 7, **kw)
        assert e.value.code == rl.RR_EINVAL and "pinned" in str(e.value)
        with pytest.raises(rl.RandlineError) as e:
            rl.probe_pair(FAKE, 0, 1, 8, 8, 7, **kw)
        assert e.value.code == rl.RR_EINVAL and "pinned" in str(e.value)


def test_noalloc_entry_point_validates_like_rand_read_and_knows_its_limit():
    """Same argument rules as rr_rand_read, checked before any device work; on top of them the fixed capacity
    of its placement log."""
    for args, kw, needle in ((((0, 4096), 128, 8, 8, 7), {}, "NULL"), ((FAKE, 100, 8, 8, 7), {}, "line_bytes"),
                             ((FAKE, 128, 9, 8, 7), {}, "multiple of iters_per_wave"),
                             ((FAKE, 128, 8, 8, 7), {"unroll": 3}, "unroll")):
        with pytest.raises(rl.RandlineError) as e:
            rl.rand_read_noalloc(*args, **kw)
        assert e.value.code == rl.RR_EINVAL and needle in str(e.value)
    W = 65536 + 1
    with pytest.raises(rl.RandlineError) as e:
        rl.rand_read_noalloc(FAKE, 128, W * 2, 2, 7, want_placement=True)
    assert e.value.code == rl.RR_EINVAL and "beyond" in str(e.value)
    assert rl.rand_read_noalloc(FAKE, 128, 0, 8, 7).checksum == 0         # nothing to read: no device work at all
    header = open(os.path.join(ROOT, "include", "randline.h")).read()
    assert "#define RR_NOALLOC_MAX_PLACEMENT 65536u" in header


def test_rand_update_validation():
    with pytest.raises(rl.RandlineError) as e:
        rl.rand_update(FAKE, 128, 8, 8, 7, 3, 1)
    assert "op must be" in str(e.value)
    with pytest.raises(rl.RandlineError):
        rl.rand_update(FAKE, 100, 8, 8, 7, rl.OP_WRITE, 1)
    with pytest.raises(rl.RandlineError):
        rl.rand_update((0, 4096), 128, 8, 8, 7, rl.OP_ADD, 1)


def test_chase_validation():
    for args, needle in ((((0, 4096), 128, 0, 0, 0, 1), "NULL"), ((FAKE, 100, 0, 0, 0, 1), "line_bytes"),
                         ((FAKE, 128, 1 << 13, 0, 0, 1), "start"), ((FAKE, 128, 0, 0, 0, 0), "hops"),
                         (((1 << 21, 1000), 128, 0, 0, 0, 1), "multiple")):
        with pytest.raises(rl.RandlineError) as e:
            rl.chase(*args)
        assert e.value.code == rl.RR_EINVAL and needle in str(e.value)
    for args, kw, needle in (((FAKE, 128, 0, 0, 0, 1), {"cu": 1024}, "out of range"), ((FAKE, 128, 0, 0, 0, 0), {"cu": 3}, "hops"),
                             (((0, 4096), 128, 0, 0, 0, 1), {"cu": 0}, "NULL")):
        with pytest.raises(rl.RandlineError) as e:                      # the pinned walk checks the same, and its CU
            rl.chase(*args, **kw)
        assert e.value.code == rl.RR_EINVAL and needle in str(e.value)


def test_verify_sweep_tool(tmp_path, worked):
    """The result checker recomputes a row's checksum from what the row says: a row holding the worked PR1 value
    matches, the same row with one bit flipped does not, rows without a checksum are skipped."""
    import io
    import json
    import verify_sweep
    pr1 = int(worked["pr1_W256_I4096"][0])
    base = {"experiment": "region", "region_gib": 0.25, "line_bytes": 128, "lanes_per_line": 32, "n_reads": 1 << 20,
            "iters_per_wave": 4096}
    rows = [{"key": "good", **base, "checksum_first_seed": pr1},
            {"key": "bad", **base, "checksum_first_seed": pr1 ^ 2},
            {"key": "big", **base, "n_reads": 1 << 40, "checksum_first_seed": 0},
            {"key": "other", "experiment": "groups"}]
    path = tmp_path / "r.jsonl"
    path.write_text("\n".join(json.dumps(r) for r in rows) + "\n")
    out = io.StringIO()
    assert verify_sweep.verify(str(path), 2, 3e8, out) == (1, 1, 2)
    text = out.getvalue()
    assert "good: match" in text and "bad: MISMATCH" in text and "big: skipped" in text and "other: skipped" in text
    assert verify_sweep.main([str(path), "--threads", "2"]) == 1
    path.write_text(json.dumps(rows[0]) + "\n")
    assert verify_sweep.main([str(path), "--threads", "2"]) == 0


def test_report_renders_every_kind_of_row():
    """The Markdown report of a result file: a table or sentence for each experiment, and no crash on a file that
    holds only some of them."""
    from paper_2405_11425_amd import report
    env = {"device": "d", "arch": "gfx950", "compute_units": 256, "memory_gib": 288.0, "rocm": "7.2.0",
           "compute_partition": "SPX", "memory_partition": "NPS1", "mclk": "2000Mhz"}
    rows = [
        {"experiment": "region", "scheme": "uniform", "region_gib": 1.0, "gbps": 6900.0, "environment": env},
        {"experiment": "region", "scheme": "uniform, zone by zone", "region_gib": 256.0, "gbps": 6700.0},
        {"experiment": "region", "scheme": "uniform", "launch_size": "16x", "region_gib": 256.0, "gbps": 6400.0},
        {"experiment": "lines", "region_gib": 128.0, "line_bytes": 256, "lanes_per_line": 64, "order": "plain", "gbps": 6650.0},
        {"experiment": "windows", "region_gib": 256.0, "scheme": "xcd", "n_windows": 8, "gbps": 6200.0},
        {"experiment": "stream", "kind": "sequential read", "region_gib": 16, "gbps": 7000.0},
        {"experiment": "updates", "op": "write", "region_gib": 16, "gbps_lines": 5000.0},
        {"experiment": "zones", "n_zones": 2, "zone_ranges_gib": [[[0.0, 96.0]], [[96.0, 128.0]]], "region_gib": 128,
         "gbps_same_zone_median": 6800.0, "gbps_cross_zone_median": 6500.0, "gbps_uniform_plain": 6550.0,
         "gbps_uniform_zone_by_zone": 6700.0},
        {"experiment": "probe", "n_units": 64, "unit_cus": 4, "n_pairs": 2016, "ratio_min": 0.72, "ratio_max": 1.0,
         "ratio_median": 0.99, "threshold": 0.87, "n_groups": 32, "group_sizes_in_cus": [8], "distinct_checksums": 1},
        {"experiment": "groups", "gbps_by_xcd": {"0": 1200.0, "1": 1190.0}, "cus_per_xcd": 32},
        {"experiment": "latency", "footprint_mib": 1, "ns_per_hop": 155.0},
        {"experiment": "pages", "distance_bytes": 1 << 30, "n_lines": 33, "ns_per_hop": 200.0},
        {"experiment": "pieces-size", "region_mib": 512.0, "pieces_in_region": 4096, "n_pieces": 24576, "piece_kib": 128,
         "gbps_uniform": 280.0, "gbps_own_per_cu": 6600.0},
        {"experiment": "pieces-reach", "window_pieces": [16, 96], "gbps": [56.0, 10.0]},
        {"experiment": "pieces-share", "window_pieces": 48, "cus_of_one_xcd": [4, 6], "gbps_per_cu_one_xcd": [50.0, 11.0],
         "cus_per_xcd_all_xcds": [4], "gbps_per_cu_all_xcds": [49.0]},
        {"experiment": "pieces-probe", "unit_cus": 4, "window_pieces": 48, "ratio_min": 0.18, "ratio_max": 1.01, "n_groups": 8,
         "group_sizes_in_cus": [32], "groups_are_xcds": True},
        {"experiment": "latency-per-xcd", "footprint_mib": 64, "cus": [0, 32], "ns_per_hop": [401.0, 405.0], "all_cus_agree": True},
        {"experiment": "pieces-latency", "footprint_pieces": [16, 64], "ns_per_hop_by_cu": {"0": [410.0, 733.0]}},
        {"experiment": "pieces-flat-curve", "by_grouping": {"cu": {"groups": 256, "reach_pieces": 24, "own_window_pieces": [16, 32],
         "own_window_gbps": [6900.0, 2800.0], "curve": [{"windows": 2, "region_mib": 6.0, "gbps_windowed": 6100.0, "gbps_uniform": 900.0}]}}},
        {"experiment": "beyond", "scheme": "uniform", "launch_size": "1x", "region_gib": 280.0, "gbps": 4006.0, "allocation_gib": 280},
        {"experiment": "beyond", "scheme": "windows 1/8, xcd", "launch_size": "1x", "region_gib": 280.0, "gbps": 6200.0, "allocation_gib": 280},
        {"experiment": "beyond", "scheme": "uniform, zone by zone", "launch_size": "16x", "region_gib": 264.0, "gbps": 6864.0, "allocation_gib": 280},
        {"experiment": "beyond-latency", "footprint_mib": 286720, "ns_per_hop": 545.0},
        {"experiment": "beyond-pages", "distance_bytes": 130 << 20, "n_lines": 2200, "translations": 2200, "ns_per_hop": 238.0},
        {"experiment": "beyond-pages", "distance_bytes": 128 << 20, "n_lines": 2239, "translations": 2239, "ns_per_hop": 304.0},
        {"experiment": "beyond-switch", "top_gib": 280, "iters_per_wave": 1024, "us_each_region_repeated": 317.9,
         "us_regions_in_a_cycle": 381.4, "us_in_a_cycle_after_a_touch_of_32768_lines": 379.0},
    ]
    text = report.report(rows)
    for needle in ("an allocation of 280 GiB", "| uniform |  | 4006 |", "| windows 1/8, xcd |  | 6200 |",
                   "| uniform, zone by zone, 16x longer launches | 6864 |  |", "280 GiB: 545", "one line per 130 MiB: 2200 [2200]: 238",
                   "one line per 128 MiB: 2239 [2239]: 304", "| 280 GiB | 1024 | 317.9 | 381.4 | +63.5 | 379.0 |"):
        assert needle in text, needle
    for needle in ("Throughput vs region size", "| 256 GiB |  | 6700 (83.8 %) |  | 6400 (80.0 %) |", "64 x 4 B = 256 B", "xcd | 8",
                   "sequential read", "write | 16 GiB |", "2 zones", "32 groups of [8] CUs", "1190-1200 GB/s", "| 1 MiB | 155.0 |",
                   "| 33 | 200.0 |", "| 512 MiB | 4096 | 280 |", "96: 10", "6: 11.0", "the groups are the XCDs: True",
                   "401, 405 ns per hop", "64: 733", "reach 24 pieces", "| 2 | 6 MiB | 6100 | 900 |"):
        assert needle in text, needle
    assert "Line width" not in report.report(rows[:1])


def test_knee_finder_on_synthetic_curves():
    """The knee of a throughput-vs-size curve (paper Sec. 2.1, Fig. 1: flat up to the translation reach, then a cliff)."""
    from paper_2405_11425_amd.report import find_knee, knee_sentence
    sizes = [1, 2, 4, 8, 16, 32, 64, 128, 192, 256]
    flat = [6950, 6960, 6940, 6930, 6945, 6935, 6925, 6600, 6610, 6250]            # two steps of 4-5 %: no cliff at 10 %
    assert find_knee(sizes, flat, 0.10) == (None, 6932.5)
    assert find_knee(sizes, flat, 0.03)[0] == 128                                   # ... but a knee at 3 %
    a100 = [1400, 1405, 1398, 1402, 1400, 1399, 1401, 600, 420, 380]               # the paper's picture: collapse above 64
    assert find_knee(sizes, a100, 0.10) == (128, 1400)
    assert find_knee(sizes[::-1], a100[::-1], 0.10) == (128, 1400)                  # order of the points does not matter
    dip = [1400, 1400, 1400, 1100, 1400, 1400, 1400, 1400, 1400, 1400]             # one bad point that recovers: no knee
    assert find_knee(sizes, dip, 0.10)[0] is None
    late = [100.0] * 9 + [94.9]
    assert find_knee(sizes, late, 0.05) == (256, 100.0) and find_knee(sizes, late, 0.06)[0] is None
    rng = np.random.default_rng(5)
    for knee_at in range(2, 10):                                                    # noisy plateau (1 %), then a drop of 30 %
        curve = [1000 * (1 + 0.01 * rng.standard_normal()) * (0.7 if i >= knee_at else 1.0) for i in range(10)]
        assert find_knee(sizes, curve, 0.10)[0] == sizes[knee_at]
    assert find_knee([1, 2], [5.0, 1.0], 0.1) == (2, 5.0) and find_knee([1], [5.0], 0.1) == (None, 5.0)
    assert "no knee up to 256 GiB" in knee_sentence("x", sizes, flat, 0.1) and "knee at 128 GiB" in knee_sentence("x", sizes, a100, 0.1)


def test_region_create_validation():
    """Argument checks of the piecewise region come before any HIP call."""
    for args, needle in (((0, 4096), "multiple of piece_bytes"), ((8192, 0), "multiple of piece_bytes"),
                         ((8192, 12288), "multiple of piece_bytes"), ((3000, 1000), "4096"),
                         ((1 << 40, 4096), "30000 pieces")):
        with pytest.raises(rl.RandlineError) as e:
            rl.region_create(*args)
        assert e.value.code == rl.RR_EINVAL and needle in str(e.value)
    out = C.c_void_p(77)
    assert rl.lib().rr_region_create(0, 4096, C.byref(out)) == rl.RR_EINVAL and out.value == 77
    assert rl.lib().rr_region_create(4096, 4096, None) == rl.RR_EINVAL
    assert rl.lib().rr_region_destroy(12345) == rl.RR_EINVAL
    assert rl.lib().rr_region_granularity(None, None) == rl.RR_EINVAL


def test_out_left_untouched_on_failure():
    res = rl.binding._Result(123, 1.0, 2.0, 4, 5)
    rc = rl.lib().rr_rand_read(1 << 21, 1000, 128, 32, 8, 8, None, 7, None, None, C.byref(res))
    assert rc == rl.RR_EINVAL and (res.checksum, res.waves_run, res.launches) == (123, 4, 5)
    assert rl.lib().rr_rand_read(1 << 21, 4096, 128, 32, 8, 8, None, 7, None, None, None) == rl.RR_EINVAL


def test_batch_validation_comes_before_any_launch():
    """Every item is checked, and out stays as it was, before the device is touched."""
    fake = 1 << 21                                    # never dereferenced: all of these fail or do nothing on the host
    with pytest.raises(rl.RandlineError, match="at most 64"):
        rl.rand_read_batch(fake, [(4096, 1)] * 65, 128, 8, 8)
    with pytest.raises(rl.RandlineError, match="line_bytes"):
        rl.rand_read_batch(fake, [(4096, 1)], 100, 8, 8)
    with pytest.raises(rl.RandlineError, match="multiple"):
        rl.rand_read_batch(fake, [(4096, 1), (4096, 2), (1000, 3)], 128, 8, 8)
    with pytest.raises(rl.RandlineError, match="not available in a batch"):
        o = rl.binding._Opts()
        o.cu_waves_out = (C.c_uint32 * 4)()
        item = (rl.binding._ReadItem * 1)()
        item[0].region_bytes, item[0].read_seed, item[0].opts = 4096, 1, C.pointer(o)
        res = (rl.binding._Result * 1)()
        rl.binding._check(rl.lib().rr_rand_read_batch(fake, item, 1, 128, 32, 8, 8, None, res))
    res = (rl.binding._Result * 2)()
    res[1].checksum = 99
    items = (rl.binding._ReadItem * 2)()
    items[0].region_bytes, items[1].region_bytes = 4096, 1000
    assert rl.lib().rr_rand_read_batch(fake, items, 2, 128, 32, 8, 8, None, res) == rl.RR_EINVAL and res[1].checksum == 99
    assert rl.lib().rr_rand_read_batch(fake, None, 2, 128, 32, 8, 8, None, res) == rl.RR_EINVAL
    assert rl.lib().rr_rand_read_batch(fake, items, 1, 128, 32, 8, 8, None, None) == rl.RR_EINVAL
    assert rl.lib().rr_rand_read_batch(fake, None, 0, 128, 32, 8, 8, None, None) == rl.RR_OK     # an empty batch
    # nothing to read: every result is written (zeros) without a launch
    res[0].checksum = res[1].checksum = 5
    items[1].region_bytes = 4096
    assert rl.lib().rr_rand_read_batch(fake, items, 2, 128, 32, 0, 8, None, res) == rl.RR_OK
    assert (res[0].checksum, res[1].checksum, res[1].launches) == (0, 0, 0)


# ------------------------------------------------------------------ heatmap clustering: library vs oracle
@pytest.mark.parametrize("sizes,seed", [([8] * 8, 1), ([8, 6, 8, 8, 6, 8, 8, 8, 8, 8, 8, 8, 8, 8], 2),
                                        ([2] * 32, 3), ([1, 1, 30], 4), ([64], 5), ([3, 5, 7, 11], 6)])
@pytest.mark.parametrize("use_singles", [False, True])
def test_groups_from_heatmap_matches_oracle(sizes, seed, use_singles):
    slow = 1.0 if len(sizes) == 1 else 0.6
    T, truth = planted(sizes, seed, slow=slow)
    rng = np.random.default_rng(seed)
    singles = 100.0 * (1 + 0.01 * rng.standard_normal(len(truth))) if use_singles else None
    g_lib, order_lib, thr_lib = rl.groups_from_heatmap(T, singles)
    g_orc, order_orc, thr_orc = oracle_groups(T, singles)
    assert g_lib.tolist() == g_orc.tolist()
    assert order_lib.tolist() == order_orc.tolist()
    assert (np.isnan(thr_lib) and np.isnan(thr_orc)) or thr_lib == thr_orc
    if len(sizes) > 1:
        assert same_partition(g_lib, truth)


def test_groups_from_heatmap_noisy_random_matrices_match_oracle():
    rng = np.random.default_rng(0)
    for n in (2, 3, 5, 17, 40):
        A = rng.uniform(50, 200, size=(n, n))
        T = (A + A.T) / 2
        for gap in (0.0, 0.05, 0.5):
            g_lib, o_lib, t_lib = rl.groups_from_heatmap(T, None, gap)
            g_orc, o_orc, t_orc = oracle_groups(T, None, gap)
            assert g_lib.tolist() == g_orc.tolist() and o_lib.tolist() == o_orc.tolist()
            assert (np.isnan(t_lib) and np.isnan(t_orc)) or t_lib == t_orc


def test_groups_from_heatmap_tie_break_and_boundary_match_oracle():
    """The two corners of the rule that planted matrices do not reach: the first of two equal largest gaps
    splits, and a gap exactly at min_gap x median still counts as structure (values worked by hand in
    tests/test_grouping_oracle.py)."""
    T = np.zeros((4, 4))
    for (a, b), v in {(0, 1): 0.25, (2, 3): 0.25, (0, 2): 0.625, (1, 3): 0.625, (0, 3): 1.0, (1, 2): 1.0}.items():
        T[a, b] = T[b, a] = v
    g, o, t = rl.groups_from_heatmap(T, None, 0.05)
    assert g.tolist() == [0, 0, 1, 1] and t == 0.4375
    assert oracle_groups(T, None, 0.05)[0].tolist() == g.tolist()
    T = np.array([[0, 50.0, 100.0], [50.0, 0, 100.0], [100.0, 100.0, 0]])
    for gap, groups in ((0.5, [0, 0, 1]), (0.5 + 2.0 ** -40, [0, 1, 2])):
        g, o, t = rl.groups_from_heatmap(T, None, gap)
        g_orc, _, t_orc = oracle_groups(T, None, gap)
        assert g.tolist() == groups == g_orc.tolist()
        assert (np.isnan(t) and np.isnan(t_orc)) or t == t_orc == 0.75


def test_groups_from_heatmap_refuses_what_the_rule_is_not_defined_for():
    """NaN, negative or all-zero matrices and non-positive single rates: RR_EINVAL with a message of its own
    (never a stale one), outputs untouched; the oracle refuses the same inputs."""
    good = np.array([[0, 50.0, 100.0], [50.0, 0, 100.0], [100.0, 100.0, 0]])
    cases = []
    T = good.copy(); T[0, 2] = T[2, 0] = np.nan; cases.append((T, None, "T[0][2]"))
    T = good.copy(); T[0, 1] = T[1, 0] = -1.0; cases.append((T, None, "T[0][1]"))
    T = good.copy(); T[1, 2] = T[2, 1] = np.inf; cases.append((T, None, "T[1][2]"))
    cases.append((np.zeros((3, 3)), None, "zero"))
    cases.append((good, np.array([100.0, 0.0, 100.0]), "singles[1]"))
    cases.append((good, np.array([100.0, 100.0, np.nan]), "singles[2]"))
    for T, singles, word in cases:
        with pytest.raises(ValueError):
            oracle_groups(T, singles)
        rl.lib().rr_rand_read(None, 0, 0, 0, 0, 0, None, 0, None, None, None)      # leaves some other message behind
        with pytest.raises(rl.RandlineError) as e:
            rl.groups_from_heatmap(T, singles)
        assert e.value.code == rl.RR_EINVAL and word in str(e.value), str(e.value)
    # raw call: NULL matrix, n out of range, bad min_gap -- each with its own message, outputs untouched
    group = (C.c_uint16 * 3)(7, 7, 7)
    order = (C.c_uint32 * 3)(9, 9, 9)
    ng, thr = C.c_uint32(5), C.c_double(-2.0)
    Tp = good.ctypes.data_as(C.POINTER(C.c_double))
    L = rl.lib()
    for args, word in (((None, 3, None, 0.05), "NULL"), ((Tp, 0, None, 0.05), "n must"), ((Tp, 2000, None, 0.05), "n must"),
                       ((Tp, 3, None, float("nan")), "min_gap"), ((Tp, 3, None, -0.1), "min_gap")):
        assert L.rr_groups_from_heatmap(args[0], args[1], args[2], args[3], group, order, C.byref(ng), C.byref(thr)) == rl.RR_EINVAL
        assert word in L.rr_last_error().decode()
    assert L.rr_groups_from_heatmap(Tp, 3, None, 0.05, None, order, C.byref(ng), C.byref(thr)) == rl.RR_EINVAL
    assert "output" in L.rr_last_error().decode()
    assert list(group) == [7, 7, 7] and list(order) == [9, 9, 9] and ng.value == 5 and thr.value == -2.0


def test_copy_reports_time_on_success_only():
    """rr_copy writes *kernel_ms when it succeeds (an empty copy: 0) and leaves it alone on every failure."""
    L = rl.lib()
    ms = C.c_double(-1.0)
    assert L.rr_copy(0x1000, 0x2000, 0, None, C.byref(ms)) == rl.RR_OK and ms.value == 0.0
    ms = C.c_double(-1.0)
    assert L.rr_copy(0x1000, 0x1008, 64, None, C.byref(ms)) == rl.RR_EINVAL and ms.value == -1.0     # misaligned
    assert L.rr_copy(0x1000, 0x1010, 64, None, C.byref(ms)) == rl.RR_EINVAL and ms.value == -1.0     # overlap
    if not _has_gpu():
        # without a device the call fails in the HIP runtime, after validation: still untouched
        assert L.rr_copy(0x10000, 0x20000, 64, None, C.byref(ms)) == rl.RR_EHIP and ms.value == -1.0


def test_groups_from_heatmap_single_unit():
    g, o, t = rl.groups_from_heatmap(np.zeros((1, 1)))
    assert g.tolist() == [0] and o.tolist() == [0] and np.isnan(t)


# ------------------------------------------------------------------ workload generators
def test_window_maps_are_valid():
    table = wl.synthetic_cu_table()
    for nw in (1, 2, 4, 8):
        g, w = wl.window_map_by_xcd(table, nw)
        assert g.shape == (256,) and w.shape == (8,) and g.max() == 7 and w.max() == min(nw, 8) - 1
        assert all((g[table[:, 0] == x] == x).all() for x in range(8))
        g, w = wl.window_map_random_per_cu(256, nw, seed=4)
        assert g.tolist() == list(range(256)) and w.max() < nw
        assert np.array_equal(w, wl.window_map_random_per_cu(256, nw, seed=4)[1])   # seeded
    g, w = wl.window_map_by_se(table, 4)
    assert w.shape == (32,) and g.max() == 31 and all(np.sum(g == k) == 8 for k in range(32))
    assert all(len({(int(x), int(s)) for x, s in table[g == k][:, :2]}) == 1 for k in range(32))
    g, w = wl.window_map_from_groups([0, 0, 1, 1, 2, 0xFFFF], 2)
    assert w.tolist() == [0, 1, 0]
    g, w = wl.window_map_own_per_cu(256)
    assert g.tolist() == list(range(256)) == w.tolist()
    g, w = wl.window_map_for_selected_cus(16, [9, 3], [5, 0])
    assert w.tolist() == [5, 0] and g[9] == 0 and g[3] == 1 and (np.delete(g, [3, 9]) == 0xFFFF).all()


def test_probe_sample_and_configs():
    table = wl.synthetic_cu_table()
    s = wl.probe_cu_sample(table)
    assert len(s) == 64 and len(set(s.tolist())) == 64
    assert all(np.sum(table[s, 0] == x) == 8 for x in range(8))
    assert all(s[i + 1] == s[i] + 1 for i in range(0, 64, 2))       # adjacent-id pairs
    sweep = wl.region_sweep()
    assert [c.region_bytes >> 30 for c in sweep] == [1, 2, 4, 8, 16, 32, 64, 128, 192, 256]
    assert all(c.n_reads == 1 << 26 and c.line_bytes == 128 for c in sweep)
    assert wl.pr1_reference().n_reads == 1 << 20
    assert all(c.n_reads == 1 << 30 for c in wl.line_width_sweep(128 << 30))
    assert wl.probe_config().n_reads == 1 << 22


# ------------------------------------------------------------------ the exact-remainder recipe of the kernel
def test_reciprocal_remainder_recipe_is_exact():
    """The read kernel reduces a 64-bit draw h modulo a non-power-of-two L <= 2^32 as
    q = mulhi64(h, M), M = floor((2^64-1)/L), r = h - q*L, one conditional subtraction.
    Shown here with Python integers: q is floor(h/L) or one less, so one step suffices."""
    rng = np.random.default_rng(1)
    Ls = [3, 5, 96, 3 << 30, (1 << 32) - 1, (1 << 31) + 1, 3 << 29, 1000003, 7 << 28]
    Ls += [int(x) for x in rng.integers(3, 1 << 32, size=200) if int(x) & (int(x) - 1)]
    hs = [0, 1, (1 << 64) - 1, (1 << 63), (1 << 63) - 1] + [int(x) for x in rng.integers(0, 1 << 64, size=300, dtype=np.uint64)]
    for L in Ls:
        M = ((1 << 64) - 1) // L
        for h in hs + [L - 1, L, L + 1, ((1 << 64) - 1) // L * L, ((1 << 64) - 1) // L * L - 1]:
            q = (h * M) >> 64
            r = h - q * L
            assert 0 <= r < 2 * L
            if r >= L:
                r -= L
            assert r == h % L
