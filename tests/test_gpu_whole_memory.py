"""GPU parity beyond 256 GiB: one allocation of nearly the whole memory of the card (280 GiB on an idle MI355X).

What is new out here: line indices above 2^31 and word indices above 2^36, a region of 35 (not 32) zone windows, and a
footprint larger than what the second-level translation cache of an XCD covers, where the paper's windows per group
(Sec. 2.4) matter on this GPU.  Everything is integer work and is compared bit-exactly with the CPU oracle.  This module
runs after test_gpu_parity.py and takes its memory over; it gives the memory back when it is done.
"""
import gc
import os

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import paper_2405_11425_amd as rl                      # noqa: E402
from paper_2405_11425_amd import workloads as wl       # noqa: E402
from oracle import randline as orc                     # noqa: E402

GiB = 1 << 30
ORACLE_THREADS = 16


@pytest.fixture(scope="module")
def whole():
    assert torch.cuda.is_available(), "these tests need the GPU"
    assert os.path.exists(rl.library_path()), "librandline.so is not built"
    gc.collect()
    torch.cuda.empty_cache()
    free, _ = torch.cuda.mem_get_info()
    gib = min(280, int((free - 6 * GiB) // (8 * GiB)) * 8)
    if gib < 264:
        pytest.skip(f"needs one allocation well beyond 256 GiB; {free / GiB:.1f} GiB are free")
    buf = torch.empty(gib * GiB, dtype=torch.uint8, device="cuda")
    rl.fill(buf, wl.FILL_SEED)
    print(f"\n[whole-memory fixture] {free / GiB:.1f} GiB free, allocated {gib} GiB", flush=True)
    yield buf
    buf.untyped_storage().resize_(0)     # pytest still holds the tensor: let go of its memory, not of the object
    del buf
    gc.collect()
    torch.cuda.empty_cache()


def oracle(R, B, W, I, **kw):
    return orc.checksum(R, B, W, I, wl.FILL_SEED, wl.READ_SEED, n_threads=ORACLE_THREADS, **kw)


def test_fill_and_streaming_sum_at_the_top(whole):
    n_words = whole.numel() // 4
    assert n_words > 1 << 36
    for off in ((1 << 36) - 2048, (1 << 36) + 4096 * 3, n_words - 4096):
        got = whole[off * 4:(off + 4096) * 4].cpu().numpy().view(np.uint32)
        assert np.array_equal(got, orc.fill_words(wl.FILL_SEED, off, 4096)), f"word offset {off}"
    top = whole.numel() - GiB
    assert rl.seq_read(whole[top:]).checksum == orc.sum_words(wl.FILL_SEED, top // 4, GiB // 4, n_threads=ORACLE_THREADS)


def test_walk_over_the_whole_allocation(whole):
    R = whole.numel()
    assert R // 128 > 1 << 31
    want = orc.chase(R, 128, wl.FILL_SEED, 0, 0, 0xFFFFFFFF, 20000)
    for cu in (None, 0):
        got = rl.chase(whole, 128, 0, 0, 0xFFFFFFFF, 20000, cu=cu)
        assert (got.final_line, got.word_sum) == want, cu
    # a closed walk over one line per 128 MiB: 2239 lines, more translations than the second level holds
    stride = (128 << 20) + 128
    n = min(2239, R // stride)
    got = rl.chase(whole, 128, 0, stride // 128, 0, 3 * n + 5, region_bytes=n * stride, cu=0)
    assert (got.final_line, got.word_sum) == orc.chase(n * stride, 128, wl.FILL_SEED, 0, stride // 128, 0, 3 * n + 5)
    assert got.final_line == 5 * (stride // 128)     # three laps and five hops


def test_every_scheme_over_the_whole_allocation(whole):
    """Full occupancy, 4096 reads per logical wave, over all of the allocation: uniform reads by every kernel (by default
    the zone stream kernel with the region divided between the halves of the XCDs), in zone order in both directions with
    and without that division, one window per XCD and windows drawn per CU."""
    R = whole.numel()
    cus = rl.enumerate_cus()
    n = len(cus)
    W, I = wl.resident_logical_waves(n), wl.ITERS_PER_WAVE
    want = oracle(R, 128, W, I)
    read = lambda wm=None, **kw: rl.rand_read(whole, 128, W * I, I, wl.READ_SEED, wm, **kw)
    rates = {}
    for name, kw, kernel in (("default (XCD halves split)", {}, "rand_read_zone_stream_kernel<"),
                             ("stream", dict(xcd_split=rl.SPLIT_OFF), "rand_read_stream_kernel<"),
                             ("flat", dict(mode=rl.MODE_FLAT), "rand_read_flat_kernel<"),
                             ("ticketed", dict(mode=rl.MODE_TICKET), "rand_read_kernel<")):
        got = read(**kw)
        assert got.checksum == want, name
        assert rl.last_kernel().startswith(kernel), (name, rl.last_kernel())
        rates[name] = W * I * 128 / got.kernel_ms_event / 1e6
    n_win = R // (8 * GiB)
    zm = rl.detect_zones(whole, n_win)
    assert len(zm) == n_win and max(zm) < 16
    for name, kw in (("zone order", {}), ("zone order, descending", dict(zone_descending=True)),
                     ("zone order, XCD halves split", dict(xcd_split=rl.SPLIT_ON)),
                     ("zone order, XCD halves split, descending", dict(xcd_split=rl.SPLIT_ON, zone_descending=True)),
                     ("zone order, ticketed, descending", dict(zone_descending=True, mode=rl.MODE_TICKET))):
        got = read(zone_of_window=zm, **kw)
        assert got.checksum == want, name
        rates[name] = W * I * 128 / got.kernel_ms_event / 1e6
    for k, scheme in ((8, "xcd"), (2, "random")):
        g_of_cu, w_of_g = (wl.window_map_by_xcd(cus, k) if scheme == "xcd" else wl.window_map_random_per_cu(n, k, seed=k))
        got = read(rl.WindowMap(k, g_of_cu, w_of_g))
        assert got.checksum == oracle(R, 128, W, I, n_windows=k, window_of_group=w_of_g), (k, scheme)
        rates[f"windows 1/{k}, {scheme}"] = W * I * 128 / got.kernel_ms_event / 1e6
    print(f"\n[{R // GiB} GiB, zones {zm}; one launch each, nothing warmed up] " + ", ".join(f"{k}: {v:.0f} GB/s" for k, v in rates.items()), flush=True)


def test_shapes_of_the_papers_figures_beyond_the_reach(whole):
    """The qualitative shapes of the paper's Fig. 1 and Fig. 5 where this GPU shows them, with wide margins (measured:
    factors of 1.3-1.55): over more than the second-level translation reach, windows per resource group keep the rate
    that windows drawn per CU lose (Sec. 2.4 against Sec. 2.1), and so does the library's division of a plain read."""
    R = whole.numel()
    if R < 272 * GiB:
        pytest.skip("the effect is measured on an allocation of 272 GiB or more")
    import statistics
    cus = rl.enumerate_cus()
    n = len(cus)
    W, I = wl.resident_logical_waves(n), wl.ITERS_PER_WAVE

    def rate(wm=None, **kw):
        for i in range(3):
            rl.rand_read(whole, 128, W * I, I, 100 + i, wm, **kw)
        ms = statistics.median(rl.rand_read(whole, 128, W * I, I, wl.READ_SEED + i, wm, **kw).kernel_ms_event for i in range(5))
        return W * I * 128 / ms / 1e6
    rate()                                                       # clocks up
    xcd = rate(rl.WindowMap(8, *wl.window_map_by_xcd(cus, 8)))
    per_cu = rate(rl.WindowMap(8, *wl.window_map_random_per_cu(n, 8, seed=8)))
    divided, undivided = rate(), rate(xcd_split=rl.SPLIT_OFF)
    print(f"\n[{R // GiB} GiB] one window of 8 per XCD {xcd:.0f}, drawn per CU {per_cu:.0f}; plain read divided {divided:.0f}, "
          f"undivided {undivided:.0f} GB/s", flush=True)
    assert xcd > 1.15 * per_cu
    assert divided > 1.15 * undivided
    assert abs(xcd - divided) < 0.1 * xcd                        # the division reaches the rate of the windows


def test_other_entry_points_over_the_whole_allocation(whole):
    """The entry point that allocates nothing and the batched one take the same path over more than 256 GiB (the region
    divided between the XCD halves) and return the same checksums."""
    R = whole.numel()
    n = len(rl.enumerate_cus())
    W, I = wl.resident_logical_waves(n) // 4, 1024
    want = oracle(R, 128, W, I)
    assert rl.rand_read(whole, 128, W * I, I, wl.READ_SEED).checksum == want
    got = rl.rand_read_noalloc(whole, 128, W * I, I, wl.READ_SEED)
    assert got.checksum == want and rl.last_kernel().startswith("rand_read_zone_stream_kernel<")
    half = (R // (2 * GiB)) * GiB
    items = [(R, wl.READ_SEED), (half, wl.READ_SEED), (R, wl.READ_SEED, dict(xcd_split=rl.SPLIT_OFF))]
    res = rl.rand_read_batch(whole, items, 128, W * I, I)
    assert [r.checksum for r in res] == [want, oracle(half, 128, W, I), want]


@pytest.mark.parametrize("R,B,lanes,W,I,zone", [
    (3 << 24, 128, 32, 301, 1100, 1 << 24),         # odd wave count: the ticketed zone kernel
    (3 << 24, 256, 32, 64, 1024, 5 << 22),          # the zone stream kernel, uneven zones
    (5 << 22, 512, 32, 32, 512, 1 << 22),           # 16-byte lanes, 5 zones
    (1 << 26, 256, 64, 32, 704, 1 << 25),           # 64-lane lines
    (1 << 26, 128, 32, 10, 2100, 1 << 26),          # a single zone: both directions are the same launch
])
def test_zone_direction_does_not_change_the_checksum(whole, R, B, lanes, W, I, zone):
    want = orc.checksum(R, B, W, I, wl.FILL_SEED, wl.READ_SEED, n_threads=ORACLE_THREADS)
    if W * lanes % 64 == 0 and I % 64 == 0 and R > zone:   # what the zone stream kernel takes: also split between the XCD halves
        for down in (False, True):
            got = rl.rand_read(whole, B, W * I, I, wl.READ_SEED, lanes_per_line=lanes, region_bytes=R, zone_bytes=zone,
                               zone_descending=down, xcd_split=rl.SPLIT_ON)
            assert got.checksum == want, ("split", down)
    for mode in (rl.MODE_AUTO, rl.MODE_TICKET, rl.MODE_FLAT):
        for down in (False, True):
            got = rl.rand_read(whole, B, W * I, I, wl.READ_SEED, lanes_per_line=lanes, region_bytes=R, zone_bytes=zone,
                               mode=mode, zone_descending=down)
            assert got.checksum == want, (mode, down)
    # a scattered map, descending, equals the plain read too
    if (R // B) % 8 == 0 and ((R // B // 8) & (R // B // 8 - 1)) == 0:
        got = rl.rand_read(whole, B, W * I, I, wl.READ_SEED, lanes_per_line=lanes, region_bytes=R,
                           zone_of_window=[2, 0, 1, 0, 2, 2, 1, 0], zone_descending=True)
        assert got.checksum == want


@pytest.mark.parametrize("B,lanes", [(128, 32), (256, 64), (512, 32)])
def test_zz_updates_over_the_whole_allocation(whole, B, lanes):
    """Random line writes and atomic adds over all of the allocation (line indices above 2^31 for 128-byte lines; the launch
    divided between the XCD halves): checksum, and the lines a few logical waves drew read back and compared with the
    oracle's values.  Runs last in this module and restores the fill."""
    R, W, I = whole.numel(), 1024, 4096
    idx = orc.indices(R, B, W, I, 11)
    assert B != 128 or int(idx.max()) > 1 << 31
    lines, hits = np.unique(idx, return_counts=True)
    count = dict(zip(lines.tolist(), hits.tolist()))
    words = B // 4
    # lines in the first and the last window of 8 GiB (what changes hands between the halves), and the busiest line
    first = [int(x) for x in lines[lines < (8 * GiB) // B][:4]]
    last = [int(x) for x in lines[lines >= (R - 8 * GiB) // B][-4:]]
    try:
        for op in (rl.OP_WRITE, rl.OP_ADD):
            got = rl.rand_update(whole, B, W * I, I, 11, op, 99, lanes_per_line=lanes)
            assert got.checksum == orc.update_checksum(R, B, W, I, 11, 99)
            for line in list(idx[0, :4]) + list(idx[W - 1, -4:]) + first + last + [int(lines[np.argmax(hits)])]:
                line = int(line)
                now = whole[line * B:(line + 1) * B].cpu().numpy().view(np.uint32).astype(np.uint64)
                old = orc.fill_words(wl.FILL_SEED, line * words, words).astype(np.uint64)
                v = np.array([orc.update_value(99, line * words + j) for j in range(words)], dtype=np.uint64)
                want = v if op == rl.OP_WRITE else (old + count[line] * v) % (1 << 32)
                assert np.array_equal(now, want), (op, line)
            untouched = int(np.setdiff1d(np.arange(lines[-1] - 1000, lines[-1]), lines)[0])   # nobody drew it: still the fill
            now = whole[untouched * B:(untouched + 1) * B].cpu().numpy().view(np.uint32)
            assert np.array_equal(now, orc.fill_words(wl.FILL_SEED, untouched * words, words))
            rl.fill(whole, wl.FILL_SEED)
    finally:
        rl.fill(whole, wl.FILL_SEED)
