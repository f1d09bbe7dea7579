"""The entry point that allocates nothing (rr_rand_read_noalloc) against rr_rand_read, through the C ABI.

Integer work: every checksum and placement is compared bit-exactly.  The first test makes two calls in a
row, the second with a smaller input, which is what shows stale contents of the device array if a call
forgets to clear something.
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import paper_2405_11425_amd as rl                      # noqa: E402
from paper_2405_11425_amd import workloads as wl       # noqa: E402
from oracle import randline as orc                     # noqa: E402

GiB = 1 << 30
MiB = 1 << 20


@pytest.fixture(scope="module")
def region():
    assert torch.cuda.is_available(), "these tests need the GPU"
    buf = torch.empty(1 * GiB, dtype=torch.uint8, device="cuda")
    rl.fill(buf, wl.FILL_SEED)
    return buf


def same(a, b):
    assert a.checksum == b.checksum
    assert a.launches == b.launches == 1


def test_two_calls_in_a_row_second_smaller(region):
    """Launches without a map: 8192 logical waves x 512 over 1 GiB (stream kernel by default, flat on request), then
    96 x 100 over 12 KiB (96 lines: exact remainder; 100 iterations: the flat kernel)."""
    big = dict(line_bytes=128, n_reads=8192 * 512, iters_per_wave=512, read_seed=7)
    small = dict(line_bytes=128, n_reads=96 * 100, iters_per_wave=100, read_seed=11, region_bytes=12288)
    got_big = rl.rand_read_noalloc(region, **big)
    got_small = rl.rand_read_noalloc(region, **small)
    want_big = rl.rand_read(region, **big)
    want_small = rl.rand_read(region, **small)
    same(got_big, want_big)
    same(got_small, want_small)
    assert got_big.waves_run == want_big.waves_run == 8 * len(rl.enumerate_cus())     # the stream kernel: 8 waves per CU
    flat_big = rl.rand_read_noalloc(region, mode=rl.MODE_FLAT, **big)                   # one wavefront per pair
    same(flat_big, want_big)
    assert flat_big.waves_run == rl.rand_read(region, mode=rl.MODE_FLAT, **big).waves_run == 4096
    assert got_small.waves_run == want_small.waves_run == 48
    assert got_big.kernel_ms_device > 0 and got_big.kernel_ms_event == 0.0
    # and both equal the oracle
    assert got_big.checksum == orc.checksum(1 * GiB, 128, 8192, 512, wl.FILL_SEED, 7, n_threads=16)
    assert got_small.checksum == orc.checksum(12288, 128, 96, 100, wl.FILL_SEED, 11, n_threads=16)
    # the smaller call again, and the bigger one again: nothing is left over either way
    same(rl.rand_read_noalloc(region, **small), want_small)
    same(rl.rand_read_noalloc(region, **big), want_big)


def test_windows_tickets_and_placement(region):
    """Ticketed launches with a window map (groups = XCDs), then a smaller one with per-CU windows;
    placement log and per-CU counts as from rr_rand_read."""
    cus = rl.enumerate_cus()
    n_cus = len(cus)
    g_of_cu, w_of_g = wl.window_map_by_xcd(cus, 4)
    G = len(w_of_g)
    W = G * 64
    first = dict(line_bytes=128, n_reads=W * 2048, iters_per_wave=2048, read_seed=7,
                 window_map=rl.WindowMap(4, g_of_cu, w_of_g))
    got = rl.rand_read_noalloc(region, want_placement=True, want_cu_waves=True, **first)
    want = rl.rand_read(region, **first)
    same(got, want)
    assert got.checksum == orc.checksum(1 * GiB, 128, W, 2048, wl.FILL_SEED, 7, n_threads=16, n_windows=4,
                                        window_of_group=w_of_g)
    assert got.placement.shape == (W,) and (got.placement < n_cus).all()
    assert np.array_equal(g_of_cu[got.placement], np.arange(W) % G)    # every logical wave ran on a CU of its group
    assert int(got.cu_waves.sum()) == got.waves_run
    # smaller, other shape: 256-byte lines, every CU its own group, 2 windows, odd quota per group
    g2, w2 = wl.window_map_random_per_cu(n_cus, 2, seed=5)
    W2 = n_cus * 3
    second = dict(line_bytes=256, n_reads=W2 * 200, iters_per_wave=200, read_seed=9,
                  window_map=rl.WindowMap(2, g2, w2), region_bytes=256 * MiB)
    got2 = rl.rand_read_noalloc(region, want_placement=True, **second)
    want2 = rl.rand_read(region, **second)
    same(got2, want2)
    assert np.array_equal(g2[got2.placement], np.arange(W2) % n_cus)
    assert got2.checksum == orc.checksum(256 * MiB, 256, W2, 200, wl.FILL_SEED, 9, n_threads=16, n_windows=2,
                                         window_of_group=w2)


def test_zone_phased_and_line_shapes(region):
    for B, lanes in wl.LINE_SHAPES:
        kw = dict(line_bytes=B, lanes_per_line=lanes, n_reads=512 * 1024, iters_per_wave=1024, read_seed=13)
        same(rl.rand_read_noalloc(region, **kw), rl.rand_read(region, **kw))
    kw = dict(line_bytes=128, n_reads=2048 * 2048, iters_per_wave=2048, read_seed=17, zone_bytes=384 * MiB)
    same(rl.rand_read_noalloc(region, **kw), rl.rand_read(region, **kw))
    assert rl.rand_read_noalloc(region, 128, 0, 64, 7).checksum == 0     # empty read


def test_limit_and_no_allocation(region):
    # the placement log has a fixed capacity
    W = 65536 + 2
    with pytest.raises(rl.RandlineError) as e:
        rl.rand_read_noalloc(region, 128, W * 64, 64, 7, want_placement=True)
    assert e.value.code == rl.RR_EINVAL and "beyond" in str(e.value)
    ok = rl.rand_read_noalloc(region, 128, 65536 * 64, 64, 7, want_placement=True)     # the maximum itself
    assert ok.checksum == rl.rand_read(region, 128, 65536 * 64, 64, 7).checksum
    # device memory in use does not change over calls of this entry point
    torch.cuda.synchronize()
    free0, _ = torch.cuda.mem_get_info()
    for seed in range(3):
        rl.rand_read_noalloc(region, 128, 4096 * 256, 256, seed)
    torch.cuda.synchronize()
    free1, _ = torch.cuda.mem_get_info()
    assert free1 == free0
