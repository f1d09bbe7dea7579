"""GPU parity: the HIP library (through its C ABI binding) against the CPU oracle.

Checksums, indices and placements are integer work: everything is compared bit-exactly.
Run on the GPU machine with `pytest -m gpu`.
"""
import os

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import paper_2405_11425_amd as rl                      # noqa: E402
from paper_2405_11425_amd import workloads as wl       # noqa: E402
from oracle import randline as orc                     # noqa: E402

GiB = 1 << 30
M64 = (1 << 64) - 1
ORACLE_THREADS = 16


@pytest.fixture(scope="module")
def region():
    """One device allocation, as large as fits (256 GiB on an idle MI355X), filled with seed 1."""
    assert torch.cuda.is_available(), "these tests need the GPU"
    assert os.path.exists(rl.library_path()), "librandline.so is not built"
    torch.cuda.empty_cache()              # what an earlier test module may have left in torch's allocator
    free, _ = torch.cuda.mem_get_info()
    gib = min(256, int((free - 6 * GiB) // GiB))
    assert gib >= 2, "not enough free device memory"
    buf = torch.empty(gib * GiB, dtype=torch.uint8, device="cuda")
    rl.fill(buf, wl.FILL_SEED)
    print(f"\n[region fixture] {free / GiB:.1f} GiB free, allocated {gib} GiB", flush=True)
    return buf


def need(region, gib):
    """Skip (with the reason) a case that needs a larger allocation than this card gave."""
    if region.numel() < gib * GiB:
        pytest.skip(f"needs a {gib} GiB region, the allocation is {region.numel() // GiB} GiB")


@pytest.fixture(scope="module")
def cu_table():
    return rl.enumerate_cus()


def oracle(cfg_bytes, B, W, I, read_seed=wl.READ_SEED, **kw):
    return orc.checksum(cfg_bytes, B, W, I, wl.FILL_SEED, read_seed, n_threads=ORACLE_THREADS, **kw)


# ------------------------------------------------------------------ CU enumeration
def test_enumerate_cus(cu_table):
    n = torch.cuda.get_device_properties(0).multi_processor_count
    assert cu_table.shape == (n, 4)
    keys = [tuple(r) for r in cu_table.tolist()]
    assert keys == sorted(set(keys))                      # distinct and in dense-id order
    xcc, counts = np.unique(cu_table[:, 0], return_counts=True)
    assert len(set(counts.tolist())) == 1                 # same CU count on every XCD
    assert np.array_equal(rl.enumerate_cus(), cu_table)   # stable across calls


# ------------------------------------------------------------------ fill
def test_fill_matches_oracle_words(region):
    n_words = region.numel() // 4
    offsets = [0, 1, 1023, (1 << 20) - 512, n_words // 2 - 7, n_words - 4096]
    if n_words > (1 << 32):
        offsets += [(1 << 32) - 100, (1 << 32) + 12345, n_words - (1 << 31) - 3]  # beyond 32-bit word indices
    rng = np.random.default_rng(3)
    offsets += [int(x) for x in rng.integers(0, n_words - 4096, size=24)]
    for off in offsets:
        off -= off % 4                                     # keep the byte offset 16-aligned for the view
        got = region[off * 4:(off + 4096) * 4].cpu().numpy().view(np.uint32)
        assert np.array_equal(got, orc.fill_words(wl.FILL_SEED, off, 4096)), f"word offset {off}"


def test_fill_ragged_sizes_and_other_seed():
    """Sizes that are not a multiple of the grid's stride, incl. the 16-byte minimum; empty fill."""
    for nbytes in (16, 48, 4096 + 16, (1 << 20) + 16 * 37, 3 * (1 << 22) + 16):
        buf = torch.zeros(nbytes + 64, dtype=torch.uint8, device="cuda")
        rl.fill(buf, 0xDEADBEEF12345, region_bytes=nbytes)
        host = buf.cpu().numpy()
        assert np.array_equal(host[:nbytes].view(np.uint32), orc.fill_words(0xDEADBEEF12345, 0, nbytes // 4))
        assert not host[nbytes:].any()                     # nothing written past the end
    buf = torch.zeros(64, dtype=torch.uint8, device="cuda")
    rl.fill(buf, 5, region_bytes=0)
    assert not buf.cpu().numpy().any()


# ------------------------------------------------------------------ streaming read and copy
@pytest.mark.parametrize("nbytes", [16, 4096, (1 << 20) + 48, 3 * (1 << 26) + 16 * 5, 1 << 32])
def test_seq_read_matches_oracle_sum(region, nbytes):
    got = rl.seq_read(region, nbytes)
    assert got.checksum == orc.sum_words(wl.FILL_SEED, 0, nbytes // 4, n_threads=ORACLE_THREADS)
    assert rl.seq_read(region, 0).checksum == 0


def test_seq_read_full_region_by_parts(region):
    """Whole allocation: the sum over the region equals the sum of its 1 GiB slices (GPU), and
    sampled slices equal the oracle."""
    n_gib = region.numel() // GiB
    whole = rl.seq_read(region).checksum
    total = 0
    for g in range(n_gib):
        part = rl.seq_read(region[g * GiB:(g + 1) * GiB]).checksum
        total += part
        if g in (0, n_gib // 2, n_gib - 1):
            assert part == orc.sum_words(wl.FILL_SEED, g * GiB // 4, GiB // 4, n_threads=ORACLE_THREADS), g
    assert total & M64 == whole


def test_copy_kernel():
    n = (1 << 24) + 16 * 3
    src = torch.empty(n, dtype=torch.uint8, device="cuda")
    dst = torch.zeros(n + 32, dtype=torch.uint8, device="cuda")
    rl.fill(src, 21)
    ms = rl.copy(dst[:n], src)
    assert ms > 0
    host = dst.cpu().numpy()
    assert np.array_equal(host[:n].view(np.uint32), orc.fill_words(21, 0, n // 4)) and not host[n:].any()
    with pytest.raises(rl.RandlineError):
        rl.copy(src[16:n], src[:n - 16])       # overlap


# ------------------------------------------------------------------ dependent-load walk
@pytest.mark.parametrize("R,B,start,stride,mask,hops", [
    (1 << 16, 128, 0, 0, 0xFFFFFFFF, 1000),          # data-driven walk inside the L2
    (12288, 128, 95, 7, 0xFF, 500),                  # 96 lines, exact remainder
    (3 << 20, 256, 5, 12345, 0, 2000),               # strided
    (5 << 19, 512, 1, 0, 0xFFFFFFFF, 1),             # a single hop
    (1 << 34, 128, 12345, 1 << 14, 0xFFFFFFFF, 5000),  # 16 GiB, one new 2 MiB page per hop on top of the data term
])
def test_chase_matches_oracle(region, R, B, start, stride, mask, hops):
    got = rl.chase(region, B, start, stride, mask, hops, region_bytes=R)
    assert (got.final_line, got.word_sum) == orc.chase(R, B, wl.FILL_SEED, start, stride, mask, hops)
    assert got.ns_per_hop > 0


def test_chase_on_a_chosen_cu(region, cu_table):
    """The walk pinned to a compute unit (Sec. 2.2's pinning applied to the latency probe): same result as the
    oracle's walk whatever the CU, and it ran where it was told to (the library checks the CU's key and would
    report RR_EPLACE); one CU of every XCD, the first and the last CU."""
    n = len(cu_table)
    one_per_xcd = [int(np.flatnonzero(cu_table[:, 0] == x)[0]) for x in sorted(set(cu_table[:, 0].tolist()))]
    R, hops = 1 << 30, 3000
    want = orc.chase(R, 128, wl.FILL_SEED, 5, 0, 0xFFFFFFFF, hops)
    for cu in sorted(set(one_per_xcd + [0, n - 1])):
        got = rl.chase(region, 128, 5, 0, 0xFFFFFFFF, hops, region_bytes=R, cu=cu)
        assert (got.final_line, got.word_sum) == want, cu
        assert 50 < got.ns_per_hop < 5000
    with pytest.raises(rl.RandlineError) as e:
        rl.chase(region, 128, 5, 0, 0xFFFFFFFF, hops, region_bytes=R, cu=n)
    assert e.value.code == rl.RR_EINVAL


def test_chase_full_region(region):
    R = region.numel()
    got = rl.chase(region, 128, 0, 0, 0xFFFFFFFF, 20000)
    assert (got.final_line, got.word_sum) == orc.chase(R, 128, wl.FILL_SEED, 0, 0, 0xFFFFFFFF, 20000)


@pytest.mark.parametrize("dist,n", [(4 << 10, 16), (2 << 20, 33), (32 << 20, 128), (1 << 30, 64)])
def test_chase_closed_cycle_over_pages(region, dist, n):
    """The walk of the page-reach experiment: n lines, one per (dist + 128) bytes, region of exactly n strides,
    data term masked off.  It returns to its start after every n hops, and visits what the oracle visits."""
    stride = dist + 128
    R = n * stride
    if R > region.numel():
        pytest.skip("region too small")
    for hops in (n, 3 * n + 5):
        got = rl.chase(region, 128, 0, stride // 128, 0, hops, region_bytes=R)
        assert (got.final_line, got.word_sum) == orc.chase(R, 128, wl.FILL_SEED, 0, stride // 128, 0, hops)
        assert got.final_line == (hops % n) * (stride // 128)


def test_detected_zone_map_drives_the_phased_read(region):
    """The quick zone probe returns a usable map (one id per window, ids numbered by first appearance), and a read
    ordered by that map returns the checksum of the plain read."""
    R = (region.numel() // (32 * GiB)) * 32 * GiB
    if R == 0:
        pytest.skip("region too small for 32 windows of whole GiB")
    d = {}
    zm = rl.detect_zones(region, 32, region_bytes=R, details=d)
    print(f"\n[zones] {zm}\n[zones] " + str({k: v for k, v in d.items() if k != "row"}), flush=True)
    assert len(zm) == 32 and zm[0] == 0 and max(zm) < 16 and d["n_zones"] == max(zm) + 1
    assert d["launches"] >= 3 * d["pair_rates"] and d["cut"] < d["same"] and len(d["row"]) == 31
    assert all(z <= max(zm[:i]) + 1 for i, z in enumerate(zm) if i)          # numbered by first appearance
    W, I = 4096, 512
    plain = rl.rand_read(region, 128, W * I, I, 21, region_bytes=R)
    phased = rl.rand_read(region, 128, W * I, I, 21, region_bytes=R, zone_of_window=zm)
    assert plain.checksum == phased.checksum == orc.checksum(R, 128, W, I, wl.FILL_SEED, 21, n_threads=ORACLE_THREADS)


def test_measured_pair_rates_give_the_same_zones_through_library_and_oracle(region):
    """Pair rates of eight 32 GiB windows, measured here the way rr_detect_zones measures them (even CUs on one window,
    odd CUs on the other, the fastest of three launches; of six when taken again), recorded, and fed to the library's
    rule and to the oracle's: same zones, same cut, same questions.  And rr_detect_zones itself finds the same
    partition of the same windows."""
    from oracle.zones import zones_from_pair_rates as oracle_zones
    need(region, 256)
    n, R, iters = 8, 256 * GiB, 2048
    n_cus = len(rl.enumerate_cus())
    W = n_cus * 64
    parity = (np.arange(n_cus) % 2).astype(np.uint16)

    def measure(a, b, launches):
        wm = rl.WindowMap(n, parity, np.array([a, b], np.uint16))
        ms = [rl.rand_read(region, 128, W * iters, iters, 100 + i, wm, region_bytes=R, unroll=16).kernel_ms_event
              for i in range(launches)]
        return W * iters * 128 / min(ms) / 1e6
    for i in range(24):
        measure(0, 0, 1)                                   # the process' first launches can run slow
    table = {(a, b): (measure(a, b, 3), measure(a, b, 6)) for a in range(n) for b in range(a, n)}

    def rate(a, b, again=False):
        return table[(min(a, b), max(a, b))][1 if again else 0]
    d_lib, d_orc = {}, {}
    got = rl.zones_from_pair_rates(rate, n, details=d_lib)
    want = oracle_zones(rate, n, details=d_orc)
    print(f"\n[measured zones] {got}  same {d_lib['same']:.0f} cut {d_lib['cut']:.0f} GB/s, row {[round(x) for x in d_lib['row']]}",
          flush=True)
    assert got == want
    for key in ("same", "cut", "band", "n_zones", "pair_rates", "merge_rates", "gave_up", "row", "zones_before_merging"):
        assert d_lib[key] == d_orc[key], key
    assert 2 <= d_lib["n_zones"] <= 4                      # a 256 GiB allocation spans the card's three zones
    assert rl.detect_zones(region, n, region_bytes=R) == got


def test_calls_on_a_side_stream():
    """Every entry point works on the stream it is given (explicitly, or torch's current one) and is ordered
    after what that stream already holds."""
    side = torch.cuda.Stream()
    R = 1 << 24
    with torch.cuda.stream(side):
        buf = torch.empty(R + 256, dtype=torch.uint8, device="cuda")
        buf.fill_(0xAB)                                   # queued on the side stream; rr_fill must come after it
        rl.fill(buf, 5, region_bytes=R, stream=side)
        got = rl.rand_read(buf, 128, 64 * 100, 100, 3, region_bytes=R, stream=side)
        tick = rl.rand_read(buf, 128, 64 * 100, 100, 3, region_bytes=R, stream=side, mode=rl.MODE_TICKET)
        wide = rl.rand_read(buf, 256, 33 * 7, 7, 9, region_bytes=R)        # stream=None -> torch's current stream
        seq = rl.seq_read(buf, R, stream=side)
        walk = rl.chase(buf, 128, 1, 3, 0xFFF, 500, region_bytes=R, stream=side)
        both = rl.rand_read_batch(buf, [(R, 3), (R, 3, dict(mode=rl.MODE_TICKET))], 128, 64 * 100, 100, stream=side)
    side.synchronize()
    assert got.checksum == tick.checksum == orc.checksum(R, 128, 64, 100, 5, 3)
    assert [r.checksum for r in both] == [got.checksum] * 2
    assert wide.checksum == orc.checksum(R, 256, 33, 7, 5, 9)
    assert seq.checksum == orc.sum_words(5, 0, R // 4)
    assert (walk.final_line, walk.word_sum) == orc.chase(R, 128, 5, 1, 3, 0xFFF, 500)
    assert (buf[R:].cpu() == 0xAB).all()


def test_concurrent_callers_are_serialised(region):
    """Two host threads calling at once (ctypes drops the GIL): the library's lock keeps the shared scratch of the
    device to one call at a time, so every call still returns its own exact checksum."""
    import threading
    R = 1 << 26
    jobs = {0: (128, 96, 50, 11, rl.MODE_AUTO), 1: (256, 40, 77, 12, rl.MODE_TICKET), 2: (128, 64, 31, 13, "batch")}
    want = {k: orc.checksum(R, B, W, I, wl.FILL_SEED, seed) for k, (B, W, I, seed, _) in jobs.items()}
    bad = []

    def worker(k):
        B, W, I, seed, mode = jobs[k]
        stream = torch.cuda.Stream()
        for _ in range(40):
            if mode == "batch":     # three launches per call, one of them ticketed, on scratch slots of their own
                got = rl.rand_read_batch(region, [(R, seed), (R, seed, dict(mode=rl.MODE_TICKET)), (R, seed)], B, W * I, I,
                                         stream=stream)
                if [g.checksum for g in got] != [want[k]] * 3:
                    bad.append((k, [g.checksum for g in got]))
                continue
            got = rl.rand_read(region, B, W * I, I, seed, region_bytes=R, stream=stream, mode=mode)
            if got.checksum != want[k]:
                bad.append((k, got.checksum))

    threads = [threading.Thread(target=worker, args=(k,)) for k in jobs]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not bad


# ------------------------------------------------------------------ regions mapped in pieces
def test_piecewise_region_behaves_like_any_region():
    """A region backed by separate 128 KiB allocations: same bytes after the fill, same checksums (with and
    without windows, pinned CUs included), and the library gives the memory back."""
    lo, rec = rl.region_granularity()
    assert lo > 0 and rec >= lo
    piece = 128 << 10
    assert piece % lo == 0
    reg = rl.region_create(96 * piece, piece)
    assert reg.ptr % piece == 0
    R = reg.numel()
    rl.fill(reg, wl.FILL_SEED)
    back = torch.empty(R, dtype=torch.uint8, device="cuda")
    rl.copy(back, reg)
    assert np.array_equal(back.cpu().numpy(), orc.fill_buffer(R, wl.FILL_SEED))
    got = rl.rand_read(reg, 128, 300 * 200, 200, 7)
    assert got.checksum == orc.checksum(R, 128, 300, 200, wl.FILL_SEED, 7)
    n = len(rl.enumerate_cus())
    g, w = wl.window_map_for_selected_cus(n, [5, n - 1, 17], [1, 3, 0])
    got = rl.rand_read(reg, 128, 30 * 64, 64, 9, rl.WindowMap(4, g, w))
    assert got.checksum == orc.checksum(R, 128, 30, 64, wl.FILL_SEED, 9, 4, w)
    reg.destroy()
    reg.destroy()                                              # a second call is a no-op of the wrapper
    with pytest.raises(rl.RandlineError):
        rl.binding._check(rl.lib().rr_region_destroy(back.data_ptr()))   # not ours
    free_before, _ = torch.cuda.mem_get_info()
    with rl.region_create(128 << 21, 2 << 20) as again:        # the library can map again: 256 MiB in 2 MiB pieces
        free_during, _ = torch.cuda.mem_get_info()
        rl.fill(again, 3)
        assert rl.seq_read(again, again.numel()).checksum == orc.sum_words(3, 0, again.numel() // 4)
    free_after, _ = torch.cuda.mem_get_info()
    assert free_before - free_during >= 200 << 20 and free_after - free_during >= 200 << 20   # taken, and given back


# ------------------------------------------------------------------ random line write / add
@pytest.mark.parametrize("R,B,lanes,W,I", [
    (4096, 128, 32, 4, 8), (12288, 128, 32, 5, 37), (1 << 20, 128, 32, 7, 100), (3 << 20, 256, 32, 77, 95),
    (5 << 19, 512, 32, 31, 129), (1 << 20, 256, 64, 9, 70), (3 << 20, 512, 64, 33, 257), (128, 128, 32, 3, 50),
    (1 << 24, 128, 32, 1024, 256),     # heavy reuse: every line hit about twice
])
@pytest.mark.parametrize("op", [rl.OP_WRITE, rl.OP_ADD])
def test_rand_update_region_content(R, B, lanes, W, I, op):
    """Whole region compared byte for byte with the oracle's sequential application of the updates."""
    dev = torch.zeros(R + 512, dtype=torch.uint8, device="cuda")
    rl.fill(dev, wl.FILL_SEED, region_bytes=R)
    got = rl.rand_update(dev, B, W * I, I, 7, op, 0x1234567890ABC, lanes_per_line=lanes, region_bytes=R)
    host = orc.fill_buffer(R, wl.FILL_SEED)
    orc.apply_updates(host, B, W, I, 7, op, 0x1234567890ABC)
    out = dev.cpu().numpy()
    assert np.array_equal(out[:R], host)
    assert not out[R:].any()                                   # nothing written past the region
    assert got.checksum == orc.update_checksum(R, B, W, I, 7, 0x1234567890ABC)
    assert got.waves_run == (W * lanes + 63) // 64


def test_rand_update_large_region_sampled():
    """4 GiB region, 2^22 updates: checksum, and the lines drawn by a few logical waves read back
    and compared with old + hits * value (add) resp. value (write)."""
    R, B, W, I = 4 * GiB, 128, 1024, 4096
    dev = torch.empty(R, dtype=torch.uint8, device="cuda")
    idx = orc.indices(R, B, W, I, 11)
    lines, hits = np.unique(idx, return_counts=True)
    count = dict(zip(lines.tolist(), hits.tolist()))
    for op in (rl.OP_WRITE, rl.OP_ADD):
        rl.fill(dev, wl.FILL_SEED)
        got = rl.rand_update(dev, B, W * I, I, 11, op, 99)
        assert got.checksum == orc.update_checksum(R, B, W, I, 11, 99)
        for line in list(idx[0, :8]) + list(idx[W - 1, -8:]) + [int(lines[np.argmax(hits)])]:
            line = int(line)
            now = dev[line * B:(line + 1) * B].cpu().numpy().view(np.uint32).astype(np.uint64)
            old = orc.fill_words(wl.FILL_SEED, line * 32, 32).astype(np.uint64)
            v = np.array([orc.update_value(99, line * 32 + j) for j in range(32)], dtype=np.uint64)
            want = v if op == rl.OP_WRITE else (old + count[line] * v) % (1 << 32)
            assert np.array_equal(now, want), (op, line)
        probe = int(np.setdiff1d(np.arange(1000), lines)[0])         # a line nobody hit keeps the fill
        now = dev[probe * B:(probe + 1) * B].cpu().numpy().view(np.uint32)
        assert np.array_equal(now, orc.fill_words(wl.FILL_SEED, probe * 32, 32))


# ------------------------------------------------------------------ rand_read, small cases
SMALL = [
    # region bytes, line, lanes, W, I
    (4096, 128, 32, 4, 8),
    (4096, 256, 32, 4, 8),
    (4096, 512, 32, 4, 8),
    (12288, 128, 32, 4, 8),            # 96 lines: exact remainder path
    (128, 128, 32, 2, 3),              # one-line region
    (512, 512, 32, 1, 1),              # one line, one wave, one read
    (1 << 20, 128, 32, 1, 1),          # single logical wave: upper half of the wavefront shadows
    (1 << 20, 128, 32, 7, 100),        # odd W, I not a multiple of the batch
    (1 << 20, 128, 32, 513, 33),       # several workgroups + ragged tail
    (3 << 20, 256, 32, 77, 95),        # non-power-of-two lines, 8-byte lanes
    (5 << 19, 512, 32, 31, 129),       # 16-byte lanes
    (1 << 20, 256, 64, 9, 70),         # 64-lane lines
    (3 << 20, 512, 64, 33, 257),
    (1 << 28, 128, 32, 256, 4096),     # the small reference configuration
    (1 << 28, 128, 32, 1024, 1024),
]


@pytest.mark.parametrize("R,B,lanes,W,I", SMALL)
def test_rand_read_small(region, R, B, lanes, W, I):
    want = oracle(R, B, W, I)
    got = rl.rand_read(region, B, W * I, I, wl.READ_SEED, lanes_per_line=lanes, region_bytes=R, mode=rl.MODE_FLAT)
    assert got.checksum == want
    assert got.launches == 1 and got.waves_run == (W * lanes + 63) // 64
    # the default: the stream kernel where it applies (whole wavefronts, iterations a multiple of 16), else the flat one
    auto = rl.rand_read(region, B, W * I, I, wl.READ_SEED, lanes_per_line=lanes, region_bytes=R)
    assert auto.checksum == want and auto.launches == 1
    streams = (W * lanes) % 64 == 0 and I % 16 == 0
    if streams:
        tickets = (W * lanes // 64) * (I // next(c for c in (256, 128, 64, 32, 16) if I % c == 0))
        assert 1 <= auto.waves_run <= min(tickets, 8 * len(rl.enumerate_cus()))
        explicit = rl.rand_read(region, B, W * I, I, wl.READ_SEED, lanes_per_line=lanes, region_bytes=R, mode=rl.MODE_STREAM)
        assert explicit.checksum == want
    else:
        assert auto.waves_run == got.waves_run
        with pytest.raises(rl.RandlineError, match="stream mode does not work with"):
            rl.rand_read(region, B, W * I, I, wl.READ_SEED, lanes_per_line=lanes, region_bytes=R, mode=rl.MODE_STREAM)


def test_reference_configuration_value(region, worked):
    """The first configuration against the stored worked value (not only the live oracle)."""
    got = rl.rand_read(region, 128, 1 << 20, 4096, 7, region_bytes=1 << 28)
    assert got.checksum == worked["pr1_W256_I4096"][0]


def test_empty_read(region):
    got = rl.rand_read(region, 128, 0, 4096, 7, region_bytes=1 << 20)
    assert got.checksum == 0 and got.waves_run == 0


@pytest.mark.parametrize("B,lanes,unrolls", [(128, 32, (4, 8, 16)), (256, 32, (4, 8, 16)), (512, 32, (2, 4, 8)),
                                             (256, 64, (4, 8, 16)), (512, 64, (4, 8, 16))])
def test_launch_geometry_does_not_change_checksum(region, B, lanes, unrolls):
    """Broadcast path, ring depth, cache hint, block size, flat vs ticketed, grid size."""
    R, W, I = 3 << 24, 301, 197
    want = oracle(R, B, W, I)
    for bcast in (rl.BCAST_LDS, rl.BCAST_DPP, rl.BCAST_READLANE):
        for unroll in unrolls:
            for nt in (rl.NT_ON, rl.NT_OFF):
                got = rl.rand_read(region, B, W * I, I, wl.READ_SEED, lanes_per_line=lanes, region_bytes=R,
                                   bcast=bcast, unroll=unroll, nontemporal=nt)
                assert got.checksum == want, (bcast, unroll, nt)
    for block in (64, 128, 256):
        for mode, grid in ((rl.MODE_FLAT, 0), (rl.MODE_TICKET, 0), (rl.MODE_TICKET, 3), (rl.MODE_TICKET, 1000)):
            got = rl.rand_read(region, B, W * I, I, wl.READ_SEED, lanes_per_line=lanes, region_bytes=R,
                               block_threads=block, mode=mode, grid_blocks=grid)
            assert got.checksum == want, (block, mode, grid)


@pytest.mark.parametrize("B,lanes", wl.LINE_SHAPES)
def test_stream_geometry_does_not_change_checksum(region, B, lanes):
    """The stream kernel (ranges of tickets per workgroup, chunks handed out from LDS, loads kept in flight across
    chunks): ring depth, cache hint, chunk size, grid size from one workgroup to more workgroups than tickets, a
    first wave other than 0, a region that is not a power of two."""
    R, W, I = 3 << 24, 300, 192
    want = oracle(R, B, W, I)
    for unroll in (8, 16):
        for nt in (rl.NT_ON, rl.NT_OFF):
            for chunk, grid in ((0, 0), (64, 1), (64, 7), (192, 3), (64, 1000), (64, 5000)):
                got = rl.rand_read(region, B, W * I, I, wl.READ_SEED, lanes_per_line=lanes, region_bytes=R,
                                   mode=rl.MODE_STREAM, unroll=unroll, nontemporal=nt, chunk_iters=chunk, grid_blocks=grid)
                assert got.checksum == want, (unroll, nt, chunk, grid)
    first = 64
    got = rl.rand_read(region, B, W * I, I, 5, lanes_per_line=lanes, region_bytes=R, mode=rl.MODE_STREAM, first_wave=first)
    assert got.checksum == oracle(R, B, W, I, read_seed=5, first_wave=first)
    # iterations that only 16 divides; one ticket per unit
    got = rl.rand_read(region, B, 64 * 48, 48, 5, lanes_per_line=lanes, region_bytes=1 << 20, mode=rl.MODE_STREAM)
    assert got.checksum == oracle(1 << 20, B, 64, 48, read_seed=5)
    got = rl.rand_read(region, B, W * I, I, 5, lanes_per_line=lanes, region_bytes=R, mode=rl.MODE_STREAM, want_cu_waves=True)
    assert got.checksum == oracle(R, B, W, I, read_seed=5) and int(got.cu_waves.sum()) == got.waves_run > 0
    for kw in (dict(bcast=rl.BCAST_LDS), dict(block_threads=128), dict(chunk_iters=128), dict(want_placement=True)):
        with pytest.raises(rl.RandlineError, match="stream mode does not work with"):
            rl.rand_read(region, B, W * I, I, 5, lanes_per_line=lanes, region_bytes=R, mode=rl.MODE_STREAM, **kw)


def test_last_kernel_names_what_was_launched(region):
    """rr_last_kernel: the name a kernel trace shows for the kernel the last read call chose."""
    R, W, I = 1 << 26, 64, 256
    kw = dict(region_bytes=R)
    rl.rand_read(region, 128, W * I, I, 7, **kw)
    assert rl.last_kernel() == "rand_read_stream_kernel<32, 1, 16, 1>"
    rl.rand_read(region, 128, W * I, I, 7, mode=rl.MODE_FLAT, nontemporal=rl.NT_OFF, **kw)
    assert rl.last_kernel() == "rand_read_flat_kernel<32, 1, 16, 2, 0>"
    rl.rand_read(region, 512, W * I, I, 7, mode=rl.MODE_TICKET, unroll=4, bcast=rl.BCAST_LDS, **kw)
    assert rl.last_kernel() == "rand_read_kernel<32, 4, 4, 1, 1>"
    rl.rand_read(region, 256, W * I, I, 7, lanes_per_line=64, zone_bytes=1 << 24, **kw)
    assert rl.last_kernel() == "rand_read_zone_stream_kernel<64, 1, 16, 1>"
    rl.rand_read(region, 512, W * I, I, 7, zone_bytes=1 << 24, **kw)
    assert rl.last_kernel() == "rand_read_zone_stream_kernel<32, 4, 8, 1>"
    rl.rand_read(region, 128, W * I, I, 7, zone_bytes=1 << 24, mode=rl.MODE_TICKET, **kw)
    assert rl.last_kernel() == "rand_read_phased_kernel<32, 1, 32, 1>"
    rl.probe_pair(region, 0, 1, W * I, I, 7, **kw)
    assert rl.last_kernel() == "rand_read_kernel<32, 1, 16, 2, 1>"


def test_additivity_over_wave_ranges(region):
    R, B, I = 1 << 26, 128, 64
    whole = rl.rand_read(region, B, 1000 * I, I, 9, region_bytes=R).checksum
    assert whole == oracle(R, B, 1000, I, read_seed=9)
    parts = 0
    for first, n in ((0, 1), (1, 333), (334, 666)):
        got = rl.rand_read(region, B, n * I, I, 9, region_bytes=R, first_wave=first).checksum
        assert got == oracle(R, B, n, I, read_seed=9, first_wave=first)
        parts += got
    assert parts & M64 == whole


def test_line_shapes_with_equal_bytes_agree(region):
    """256-byte lines as 32 x 8 B and as 64 x 4 B read the same words (same W)."""
    R, W, I = 1 << 27, 128, 500
    a = rl.rand_read(region, 256, W * I, I, 7, lanes_per_line=32, region_bytes=R).checksum
    b = rl.rand_read(region, 256, W * I, I, 7, lanes_per_line=64, region_bytes=R).checksum
    assert a == b == oracle(R, 256, W, I)


def test_per_cu_counts_in_flat_mode(region, cu_table):
    R, W, I = 1 << 28, 1000, 64
    res = rl.rand_read(region, 128, W * I, I, 7, region_bytes=R, want_cu_waves=True)
    assert res.checksum == oracle(R, 128, W, I)
    assert int(res.cu_waves[:len(cu_table)].sum()) == res.waves_run == 500
    res = rl.rand_read(region, 128, W * I, I, 7, region_bytes=R, want_cu_waves=True, want_placement=True)
    counts = np.bincount(res.placement, minlength=len(cu_table))
    assert np.array_equal(counts, 2 * res.cu_waves[:len(cu_table)])       # two logical waves per wavefront


def test_repeatable(region):
    R, W, I = 1 << 30, 2048, 512
    seen = {rl.rand_read(region, 128, W * I, I, 5, region_bytes=R).checksum for _ in range(5)}
    assert seen == {oracle(R, 128, W, I, read_seed=5)}


# ------------------------------------------------------------------ zone-phased order
@pytest.mark.parametrize("R,B,lanes,W,I,zone", [
    (1 << 20, 128, 32, 4, 8, 1 << 18),              # tiny, 4 zones
    (1 << 20, 128, 32, 7, 100, 3 << 17),            # odd W, ragged chunk, last zone shorter
    (12288, 128, 32, 5, 37, 4096),                  # 96 lines in 3 zones, exact remainder path
    (3 << 24, 128, 32, 301, 1100, 1 << 24),         # several chunks per wave, 3 zones
    (3 << 24, 256, 32, 77, 600, 5 << 22),           # 8-byte lanes, uneven zones
    (5 << 22, 512, 32, 31, 513, 1 << 22),           # 16-byte lanes, 5 zones
    (1 << 26, 256, 64, 33, 700, 1 << 25),           # 64-lane lines
    (1 << 26, 512, 64, 9, 70, 1 << 26),             # a single zone
    (1 << 26, 128, 32, 10, 2100, 1 << 26),          # a single zone and full chunks: every list filled to capacity
    (1 << 26, 256, 64, 5, 2048, 1 << 26),           # the same with 64-lane lines
    (1 << 28, 128, 32, 256, 4096, 96 << 20),        # the small reference configuration in 3 zones
])
def test_zone_phased_reads_same_checksum(region, R, B, lanes, W, I, zone):
    want = oracle(R, B, W, I)
    for nt in (rl.NT_ON, rl.NT_OFF):
        got = rl.rand_read(region, B, W * I, I, wl.READ_SEED, lanes_per_line=lanes, region_bytes=R,
                           zone_bytes=zone, nontemporal=nt, mode=rl.MODE_FLAT)
        assert got.checksum == want
        assert got.waves_run == (W * lanes + 63) // 64
        for grid in (0, 5):                      # zone-major tickets; a tiny grid finishes by stealing
            got = rl.rand_read(region, B, W * I, I, wl.READ_SEED, lanes_per_line=lanes, region_bytes=R,
                               zone_bytes=zone, nontemporal=nt, mode=rl.MODE_TICKET, grid_blocks=grid)
            assert got.checksum == want, grid


@pytest.mark.parametrize("B,lanes", wl.LINE_SHAPES)
def test_zone_stream_geometry_does_not_change_checksum(region, B, lanes):
    """Zone by zone with the stream kernel (the default for zoned reads where it applies): per-wave queues in LDS
    filled zone by zone, loads kept in flight across tickets and zones, the last batch filled up with line 0 and
    corrected.  Contiguous and scattered zones, one zone, sixteen zones, chunk sizes, grids from one workgroup to more
    workgroups than units, cache hints, a first wave other than 0, a region that is not a power of two."""
    R, W, I = 3 << 24, 300, 192
    want = oracle(R, B, W, I)
    scattered = [0, 1, 2, 0, 2, 1]                       # six windows of 2^23 bytes
    for kw in (dict(zone_bytes=1 << 24), dict(zone_of_window=scattered), dict(zone_of_window=[0] * 6),
               dict(zone_bytes=3 << 20), dict(zone_of_window=[5, 0, 5, 0, 1, 1])):
        for nt in (rl.NT_ON, rl.NT_OFF):
            for chunk, grid in ((0, 0), (64, 1), (64, 7), (192, 3), (64, 1000)):
                got = rl.rand_read(region, B, W * I, I, wl.READ_SEED, lanes_per_line=lanes, region_bytes=R,
                                   mode=rl.MODE_STREAM, nontemporal=nt, chunk_iters=chunk, grid_blocks=grid, **kw)
                assert got.checksum == want, (kw, nt, chunk, grid)
        assert rl.rand_read(region, B, W * I, I, wl.READ_SEED, lanes_per_line=lanes, region_bytes=R,
                            **kw).checksum == want, kw       # the default mode
    got = rl.rand_read(region, B, W * I, I, 5, lanes_per_line=lanes, region_bytes=R, zone_bytes=1 << 24, first_wave=64)
    assert got.checksum == oracle(R, B, W, I, read_seed=5, first_wave=64)
    got = rl.rand_read(region, B, W * I, I, 5, lanes_per_line=lanes, region_bytes=R, zone_bytes=1 << 24, want_cu_waves=True)
    assert got.checksum == oracle(R, B, W, I, read_seed=5) and int(got.cu_waves.sum()) == got.waves_run > 0
    # a region whose last zone is short, and few enough reads that most waves end on a filled-up batch
    got = rl.rand_read(region, B, 8 * 64, 64, 5, lanes_per_line=lanes, region_bytes=5 << 22, zone_bytes=1 << 23,
                       mode=rl.MODE_STREAM)
    assert got.checksum == oracle(5 << 22, B, 8, 64, read_seed=5)
    # what the stream kernel does not take goes to the ticketed zone-phased kernel by default, and is refused on request
    odd = rl.rand_read(region, B, W * 100, 100, 5, lanes_per_line=lanes, region_bytes=R, zone_bytes=1 << 24)
    assert odd.checksum == oracle(R, B, W, 100, read_seed=5)
    with pytest.raises(rl.RandlineError, match="stream mode does not work with"):
        rl.rand_read(region, B, W * 100, 100, 5, lanes_per_line=lanes, region_bytes=R, zone_bytes=1 << 24, mode=rl.MODE_STREAM)


@pytest.mark.parametrize("R,B,lanes,W,I", [
    (1 << 28, 128, 32, 256, 4096),        # the small reference configuration: 64 windows, 8 pairs divided
    (12288, 128, 32, 64, 128),            # 96 lines: 48 windows of 2 lines
    (3 << 24, 256, 32, 130, 576),         # 8-byte lanes, a line count that is no power of two, 48 windows
    ((1 << 26) + (1 << 20), 512, 32, 32, 192),   # 16-byte lanes; the last window is shorter than the others
    (5 << 22, 256, 64, 33, 320),          # 64-lane lines, odd wave count
])
def test_plain_read_divided_between_the_xcd_halves(region, R, B, lanes, W, I):
    """xcd_split on a read without a zone map: the zone stream kernel with the region as one zone of up to 64 windows, every
    unit gone through by a workgroup of each half of the XCDs.  Same checksum as the plain kernels', whatever the grid."""
    want = oracle(R, B, W, I)
    plain = rl.rand_read(region, B, W * I, I, wl.READ_SEED, lanes_per_line=lanes, region_bytes=R)
    assert plain.checksum == want and rl.last_kernel().startswith("rand_read_stream_kernel<")
    for grid in (0, 8, 64, 1024):
        got = rl.rand_read(region, B, W * I, I, wl.READ_SEED, lanes_per_line=lanes, region_bytes=R, xcd_split=rl.SPLIT_ON,
                           grid_blocks=grid)
        assert got.checksum == want, grid
        assert rl.last_kernel().startswith("rand_read_zone_stream_kernel<")
    for bad in (dict(grid_blocks=12), dict(mode=rl.MODE_FLAT), dict(mode=rl.MODE_TICKET), dict(chunk_iters=0, placement=True)):
        want_placement = bad.pop("placement", False)
        with pytest.raises(rl.RandlineError) as e:
            rl.rand_read(region, B, W * I, I, wl.READ_SEED, lanes_per_line=lanes, region_bytes=R, xcd_split=rl.SPLIT_ON,
                         want_placement=want_placement, **bad)
        assert e.value.code == rl.RR_EINVAL and "xcd_split" in str(e.value), bad


def test_stream_kernels_on_seeded_random_shapes(region):
    """Sixty seeded random launches of the two stream kernels -- line shape, region size (powers of two and not),
    logical waves, iterations, chunk, grid, first wave, and for the zoned ones a random assignment of 2-64 windows to
    1-16 zones -- each against the oracle."""
    rng = np.random.default_rng(20240511)
    for case in range(60):
        B, lanes = wl.LINE_SHAPES[int(rng.integers(len(wl.LINE_SHAPES)))]
        lpw = 64 // lanes
        W = lpw * int(rng.integers(1, 120))
        zoned = case % 2 == 1
        unit = 64 if zoned else 16
        I = unit * int(rng.integers(1, 12))
        chunks = [c for c in range(unit, I + 1, unit) if I % c == 0 and c % 64 == 0]      # chunk_iters must be a multiple of 64
        chunk = int(rng.choice(chunks)) if chunks and rng.integers(2) else 0
        grid = int(rng.choice([0, 1, 2, 5, 64, 511, 513, 2000]))
        first = lpw * int(rng.integers(0, 50))
        kw = {}
        if zoned:
            n_win = int(rng.choice([2, 3, 4, 6, 8, 16, 32, 64]))
            win_lines = 1 << int(rng.integers(6, 14))
            R = n_win * win_lines * B
            n_zones = int(rng.integers(1, min(16, n_win) + 1))
            zmap = rng.integers(0, n_zones, n_win).tolist()
            zmap[:n_zones] = list(range(n_zones))                 # every zone id up to the largest is used
            kw = dict(zone_of_window=zmap)
        else:
            R = B * int(rng.integers(1, 1 << 16)) if rng.integers(2) else B << int(rng.integers(0, 18))
        seed = int(rng.integers(1, 1 << 40))
        got = rl.rand_read(region, B, W * I, I, seed, lanes_per_line=lanes, region_bytes=R, mode=rl.MODE_STREAM,
                           chunk_iters=chunk, grid_blocks=grid, first_wave=first, **kw)
        want = oracle(R, B, W, I, read_seed=seed, first_wave=first)
        assert got.checksum == want, (case, B, lanes, R, W, I, chunk, grid, first, kw)
        if zoned:   # the same in descending zone order, and divided between the XCD halves where the grid allows it
            kw["zone_descending"] = True
            if grid % 8 == 0:
                kw["xcd_split"] = rl.SPLIT_ON
            got = rl.rand_read(region, B, W * I, I, seed, lanes_per_line=lanes, region_bytes=R, mode=rl.MODE_STREAM,
                               chunk_iters=chunk, grid_blocks=grid, first_wave=first, **kw)
            assert got.checksum == want, (case, B, lanes, R, W, I, chunk, grid, first, kw)


def test_zone_map_with_scattered_zones(region):
    """Zones given window by window, not contiguous (the way physical zones show up in an allocation)."""
    R, W, I = 1 << 30, 200, 777
    want = oracle(R, 128, W, I)
    zmap = [0] * 8 + [1] * 8 + [2] * 4 + [0] * 4 + [2] * 6 + [1] * 2
    for mode in (rl.MODE_FLAT, rl.MODE_TICKET, rl.MODE_AUTO):
        got = rl.rand_read(region, 128, W * I, I, wl.READ_SEED, region_bytes=R, zone_of_window=zmap, mode=mode)
        assert got.checksum == want, mode
    got = rl.rand_read(region, 256, W * I, I, wl.READ_SEED, lanes_per_line=64, region_bytes=R, zone_of_window=[3, 0])
    assert got.checksum == oracle(R, 256, W, I)


def test_zone_phase_ticks(region):
    """Per-wave phase end times: one non-decreasing row of clock values per hardware wave."""
    W, I, Z = 64, 600, 3
    ticks = torch.zeros(32 * Z, dtype=torch.int64, device="cuda")
    got = rl.rand_read(region, 128, W * I, I, 7, region_bytes=3 << 24, zone_bytes=1 << 24, phase_ticks=ticks,
                       mode=rl.MODE_FLAT)
    assert got.checksum == oracle(3 << 24, 128, W, I)
    t = ticks.cpu().numpy().reshape(32, Z)
    assert (t > 0).all() and (np.diff(t, axis=1) >= 0).all()


def test_zone_phased_full_size(region, cu_table):
    """The sweep's largest points in 96 GiB zones, as the bench's phased leg launches them."""
    for cfg in wl.region_sweep(region.numel(), len(cu_table))[-3:]:
        got = rl.rand_read(region, 128, cfg.n_reads, cfg.iters_per_wave, cfg.read_seed,
                           region_bytes=cfg.region_bytes, zone_bytes=96 * GiB)
        assert got.checksum == oracle(cfg.region_bytes, 128, cfg.logical_waves, cfg.iters_per_wave), cfg.name


# ------------------------------------------------------------------ windows
def check_placement(res, W, G, group_of_cu):
    assert res.placement is not None and res.placement.shape == (W,)
    assert (res.placement != 0xFFFF).all()                         # every logical wave was executed
    for w in range(W):
        assert group_of_cu[res.placement[w]] == w % G, f"logical wave {w} ran on CU {res.placement[w]}"


@pytest.mark.parametrize("n_windows", [1, 2, 4, 8])
def test_windows_by_xcd(region, cu_table, n_windows):
    R, B, I = 1 << 30, 128, 256
    g_of_cu, w_of_g = wl.window_map_by_xcd(cu_table, n_windows)
    G = len(w_of_g)
    W = G * 12
    want = oracle(R, B, W, I, n_windows=n_windows, window_of_group=w_of_g)
    res = rl.rand_read(region, B, W * I, I, wl.READ_SEED, rl.WindowMap(n_windows, g_of_cu, w_of_g),
                       region_bytes=R, want_placement=True, want_cu_waves=True)
    assert res.checksum == want
    check_placement(res, W, G, g_of_cu)
    assert int(res.cu_waves.sum()) == res.waves_run


@pytest.mark.parametrize("n_windows", [2, 8])
def test_windows_random_per_cu(region, cu_table, n_windows):
    """Every CU its own group: each CU must turn up for its own logical waves."""
    R, B, I = 3 << 28, 128, 64
    n = len(cu_table)
    g_of_cu, w_of_g = wl.window_map_random_per_cu(n, n_windows, seed=11)
    W = n * 4
    want = oracle(R, B, W, I, n_windows=n_windows, window_of_group=w_of_g)
    res = rl.rand_read(region, B, W * I, I, wl.READ_SEED, rl.WindowMap(n_windows, g_of_cu, w_of_g),
                       region_bytes=R, want_placement=True)
    assert res.checksum == want
    check_placement(res, W, n, g_of_cu)


def test_windows_by_shader_engine(region, cu_table):
    R, B, I = 1 << 31, 128, 128
    g_of_cu, w_of_g = wl.window_map_by_se(cu_table, 4)
    G = len(w_of_g)
    W = G * 6
    want = oracle(R, B, W, I, n_windows=4, window_of_group=w_of_g)
    res = rl.rand_read(region, B, W * I, I, wl.READ_SEED, rl.WindowMap(4, g_of_cu, w_of_g), region_bytes=R,
                       want_placement=True)
    assert res.checksum == want
    check_placement(res, W, G, g_of_cu)


def test_small_grids_still_finish_by_stealing(region, cu_table):
    """Fewer workgroups than CUs: the waves that do run must drain the shares of the CUs that got none."""
    R, B, I = 1 << 28, 128, 200
    g_of_cu, w_of_g = wl.window_map_by_xcd(cu_table, 2)
    G = len(w_of_g)
    W = G * 40
    want = oracle(R, B, W, I, n_windows=2, window_of_group=w_of_g)
    for grid in (64, 500):
        res = rl.rand_read(region, B, W * I, I, wl.READ_SEED, rl.WindowMap(2, g_of_cu, w_of_g), region_bytes=R,
                           grid_blocks=grid, chunk_iters=64, want_placement=True)
        assert res.checksum == want, grid
        check_placement(res, W, G, g_of_cu)


def test_windows_other_shapes_and_odd_quota(region, cu_table):
    """512-byte and 64-lane lines under a map; odd number of logical waves per group."""
    R, I = 3 << 27, 77
    g_of_cu, w_of_g = wl.window_map_by_xcd(cu_table, 4)
    G = len(w_of_g)
    for B, lanes in ((512, 32), (256, 64), (256, 32)):
        W = G * 5
        want = oracle(R, B, W, I, n_windows=4, window_of_group=w_of_g)
        res = rl.rand_read(region, B, W * I, I, wl.READ_SEED, rl.WindowMap(4, g_of_cu, w_of_g),
                           lanes_per_line=lanes, region_bytes=R, want_placement=True)
        assert res.checksum == want
        check_placement(res, W, G, g_of_cu)


def test_degenerate_maps_equal_no_map(region, cu_table):
    R, B, W, I = 1 << 28, 128, 256, 128
    plain = rl.rand_read(region, B, W * I, I, wl.READ_SEED, region_bytes=R).checksum
    n = len(cu_table)
    one = rl.WindowMap(1, np.zeros(n, np.uint16), np.zeros(1, np.uint16))
    assert rl.rand_read(region, B, W * I, I, wl.READ_SEED, one, region_bytes=R).checksum == plain
    g_of_cu, _ = wl.window_map_by_xcd(cu_table, 1)
    many = rl.WindowMap(1, g_of_cu, np.zeros(int(g_of_cu.max()) + 1, np.uint16))
    assert rl.rand_read(region, B, W * I, I, wl.READ_SEED, many, region_bytes=R).checksum == plain


def test_group_without_cu_is_reported(region, cu_table):
    n = len(cu_table)
    wm = rl.WindowMap(2, np.zeros(n, np.uint16), np.array([0, 1], np.uint16))   # group 1 owns no CU
    with pytest.raises(rl.RandlineError) as e:
        rl.rand_read(region, 128, 2 * 8, 8, 7, wm, region_bytes=1 << 20)
    assert e.value.code == rl.RR_EPLACE


# ------------------------------------------------------------------ pinned probe
def test_probe_pairs(region, cu_table):
    R, I, W = 1 << 30, 256, 64
    want = oracle(R, 128, W, I)
    n = len(cu_table)
    for a, b in ((0, 1), (0, n - 1), (n // 2, 5), (n - 2, n - 1)):
        res = rl.probe_cus(region, [a, b], W * I, I, wl.READ_SEED, region_bytes=R,
                           want_placement=True, want_cu_waves=True)
        assert res.checksum == want                               # the same for every pair
        assert set(np.unique(res.placement).tolist()) <= {a, b}
        others = np.delete(res.cu_waves[:n], [a, b])
        assert not others.any() and res.cu_waves[[a, b]].sum() == res.waves_run > 0
        assert rl.probe_pair(region, a, b, W * I, I, wl.READ_SEED, region_bytes=R).checksum == want


def test_probe_single_cu_and_group(region, cu_table):
    R, I, W = 1 << 30, 128, 32
    want = oracle(R, 128, W, I)
    res = rl.probe_cus(region, [17], W * I, I, wl.READ_SEED, region_bytes=R, want_placement=True)
    assert res.checksum == want and set(res.placement.tolist()) == {17}
    xcd0 = np.flatnonzero(cu_table[:, 0] == cu_table[0, 0]).tolist()
    res = rl.probe_cus(region, xcd0, W * I, I, wl.READ_SEED, region_bytes=R, want_placement=True)
    assert res.checksum == want and set(res.placement.tolist()) <= set(xcd0)


def test_groups_scale_and_are_independent(region, cu_table):
    """The shapes of the paper's Sec. 2.3 with this GPU's groups, with wide margins: compute units inside one XCD add up
    (1, 2, 4 CUs of different shader engines: 54, 108, 215 GB/s measured), and two XCDs reading disjoint halves of a
    region together reach the sum of what each reaches alone (measured 0.98-1.01).  Checksums against the oracle."""
    import statistics
    need(region, 80)
    n = len(cu_table)
    xcc = cu_table[:, 0]
    I = 1024

    def pinned(group_of_cu, window_of_group, n_windows, R, W):
        wm = rl.WindowMap(n_windows, group_of_cu, window_of_group)
        want = oracle(R, 128, W, I, n_windows=n_windows, window_of_group=window_of_group)
        rl.rand_read(region, 128, W * I, I, 99, wm, region_bytes=R)
        res = [rl.rand_read(region, 128, W * I, I, wl.READ_SEED, wm, region_bytes=R) for _ in range(3)]
        assert all(r.checksum == want for r in res)
        return W * I * 128 / statistics.median(r.kernel_ms_device for r in res) / 1e6

    # k CUs of XCD 0, one per shader engine (CUs of one shader engine share a path: four of them reach 215 GB/s, eight 320)
    ids0 = np.flatnonzero(xcc == xcc[0])
    by_se = [int(ids0[np.flatnonzero(cu_table[ids0, 1] == se)[0]]) for se in sorted(set(cu_table[ids0, 1].tolist()))]
    rates = {}
    for k in (1, 2, 4):
        if k > len(by_se):
            continue
        g = np.full(n, rl.RR_CU_EXCLUDED, np.uint16)
        g[by_se[:k]] = 0
        rates[k] = pinned(g, np.zeros(1, np.uint16), 1, 16 * GiB, 2048 * k)
    for k in rates:
        assert 0.8 * k * rates[1] < rates[k] < 1.2 * k * rates[1], rates
    # two XCDs, each on its own 40 GiB half
    xs = sorted(set(xcc.tolist()))[:2]
    R, W = 80 * GiB, 16384
    alone = []
    for i, x in enumerate(xs):
        g = np.full(n, rl.RR_CU_EXCLUDED, np.uint16)
        g[xcc == x] = 0
        alone.append(pinned(g, np.array([i], np.uint16), 2, R, W))
    g = np.full(n, rl.RR_CU_EXCLUDED, np.uint16)
    g[xcc == xs[0]] = 0
    g[xcc == xs[1]] = 1
    both = pinned(g, np.array([0, 1], np.uint16), 2, R, 2 * W)
    print(f"\n[groups] CUs of one XCD {rates}; XCDs alone {alone[0]:.0f}, {alone[1]:.0f}, together {both:.0f} GB/s", flush=True)
    assert 0.85 * sum(alone) < both < 1.15 * sum(alone)


def test_probe_rejects_bad_targets(region, cu_table):
    n = len(cu_table)
    for cus in ([3, 3], [0, n], []):
        with pytest.raises(rl.RandlineError) as e:
            rl.probe_cus(region, cus, 64, 8, 7, region_bytes=1 << 20)
        assert e.value.code == rl.RR_EINVAL


# ------------------------------------------------------------------ full sizes, as bench.py launches them
def test_allocation_is_256_gib(region):
    """The tests below are 'full size' only if the allocation is: on an idle MI355X (288 GB) the fixture gets its
    256 GiB.  A smaller one fails here, loudly, instead of letting the full-size tests pass at a smaller size."""
    assert region.numel() == 256 * GiB, f"the allocation is only {region.numel() // GiB} GiB: the card is not idle"


def test_region_sweep_full_size(region, cu_table):
    """Every point of the region-size sweep (all wave slots occupied, 4096 reads per logical
    wave, default launch options -- what bench.py times) against the oracle."""
    for cfg in wl.region_sweep(region.numel(), len(cu_table)):
        want = oracle(cfg.region_bytes, cfg.line_bytes, cfg.logical_waves, cfg.iters_per_wave)
        # the default launch: the stream kernel, two workgroups of four wavefronts per compute unit
        got = rl.rand_read(region, cfg.line_bytes, cfg.n_reads, cfg.iters_per_wave, cfg.read_seed,
                           lanes_per_line=cfg.lanes_per_line, region_bytes=cfg.region_bytes)
        assert got.checksum == want, cfg.name
        assert got.waves_run == 8 * len(cu_table)
        # one wavefront per pair of logical waves, every wave slot of the device occupied
        flat = rl.rand_read(region, cfg.line_bytes, cfg.n_reads, cfg.iters_per_wave, cfg.read_seed,
                            lanes_per_line=cfg.lanes_per_line, region_bytes=cfg.region_bytes, mode=rl.MODE_FLAT)
        assert flat.checksum == want, cfg.name
        assert flat.waves_run == cfg.logical_waves // 2


def test_batch_equals_single_calls(region):
    """A batch of small calls -- flat, zone by zone with tickets, zone by zone flat, odd sizes, other
    launch options -- returns what the same calls return one by one, and what the oracle says."""
    W, I, B = 300, 517, 128
    zmap = [0] * 4 + [1] * 4 + [2] * 8
    items = [(1 << 30, 11), (3 << 26, 12), (1 << 30, 13, dict(zone_of_window=zmap)),
             (1 << 30, 14, dict(zone_bytes=1 << 28, mode=rl.MODE_FLAT)), (5 * 128 * 1000, 15),
             (1 << 27, 16, dict(mode=rl.MODE_TICKET, chunk_iters=128)), (1 << 30, 11, dict(unroll=4, block_threads=64)),
             (1 << 31, 17, dict(first_wave=64))]
    got = rl.rand_read_batch(region, items, B, W * I, I)
    assert len(got) == len(items)
    for it, g in zip(items, got):
        kw = dict(it[2]) if len(it) > 2 else {}
        one = rl.rand_read(region, B, W * I, I, it[1], region_bytes=it[0], **kw)
        assert g.checksum == one.checksum, it
        assert g.waves_run == one.waves_run and g.launches == 1
        assert g.kernel_ms_event > 0
        if "first_wave" not in kw:
            assert g.checksum == oracle(it[0], B, W, I, read_seed=it[1]), it
    # again, in another order and with other line shapes: nothing is left over from the first batch
    for B2, lanes in ((256, 64), (512, 32)):
        items2 = [(1 << 30, 21, dict(zone_bytes=1 << 29)), (1 << 29, 22), (1 << 30, 23)]
        got2 = rl.rand_read_batch(region, items2, B2, W * I, I, lanes_per_line=lanes)
        for it, g in zip(items2, got2):
            assert g.checksum == oracle(it[0], B2, W, I, read_seed=it[1]), (B2, it)
    # a prepared batch, run again with other seeds
    prepared = rl.ReadBatch(region, [(1 << 30, 0), (1 << 29, 0, dict(zone_bytes=1 << 27))], 128, W * I, I)
    for seed in (5, 6, 5):
        for it_bytes, g in zip((1 << 30, 1 << 29), prepared.run(read_seed=seed)):
            assert g.checksum == oracle(it_bytes, 128, W, I, read_seed=seed), seed
    assert rl.rand_read_batch(region, [], 128, W * I, I) == []
    assert [r.checksum for r in rl.rand_read_batch(region, [(1 << 20, 1)] * 3, 128, 0, 7)] == [0, 0, 0]


def test_batch_full_size(region, cu_table):
    """The bench's step: the whole region-size sweep as one batch, the largest points zone by zone."""
    cfgs = wl.region_sweep(region.numel(), len(cu_table))
    c0 = cfgs[0]
    items = [(c.region_bytes, c.read_seed) if c.region_bytes <= 96 * GiB else
             (c.region_bytes, c.read_seed, dict(zone_bytes=96 * GiB)) for c in cfgs]
    for rep in range(2):
        got = rl.rand_read_batch(region, items, c0.line_bytes, c0.n_reads, c0.iters_per_wave)
        for c, g in zip(cfgs, got):
            assert g.checksum == oracle(c.region_bytes, c.line_bytes, c.logical_waves, c.iters_per_wave), (rep, c.name)
            assert 0.5 < g.kernel_ms_event < 5.0


def test_batch_rejects_what_it_cannot_do(region):
    with pytest.raises(rl.RandlineError, match="at most 64"):
        rl.rand_read_batch(region, [(1 << 20, 1)] * 65, 128, 64, 1)
    with pytest.raises(rl.RandlineError):
        rl.rand_read_batch(region, [(1 << 20, 1), (1 << 20 | 64, 2)], 128, 64, 1)   # second item's size is no multiple of a line
    ticks = torch.zeros(64, dtype=torch.int64, device="cuda")
    with pytest.raises(rl.RandlineError, match="not available in a batch"):
        rl.rand_read_batch(region, [(3 << 24, 1, dict(zone_bytes=1 << 24, phase_ticks=ticks, mode=rl.MODE_FLAT))], 128, 64, 1)
    assert rl.rand_read(region, 128, 640, 10, 5, region_bytes=1 << 20).checksum == oracle(1 << 20, 128, 64, 10, read_seed=5)


@pytest.fixture(scope="module")
def zone_map(region):
    """zone_of_window for the whole allocation in 32 windows, from the quick probe (what bench.py orders its
    largest regions by)."""
    need(region, 256)
    zm = rl.detect_zones(region, 32, region_bytes=256 * GiB)
    print(f"\n[zone map] {zm}", flush=True)
    return zm


@pytest.mark.parametrize("gib", [128, 256])
@pytest.mark.parametrize("line_bytes,lanes", wl.LINE_SHAPES)
def test_line_width_sweep_full_size(region, zone_map, gib, line_bytes, lanes):
    """2^30 reads of every line shape over 128 and 256 GiB (paper Sec. 2.1: the wider accesses), in plain order
    and zone by zone: the checksum of the whole launch against the oracle's for all 2^30 reads."""
    need(region, gib)
    cfg = [c for c in wl.line_width_sweep(gib * GiB) if (c.line_bytes, c.lanes_per_line) == (line_bytes, lanes)][0]
    assert cfg.n_reads == 1 << 30
    want = oracle(cfg.region_bytes, cfg.line_bytes, cfg.logical_waves, cfg.iters_per_wave)
    kw = dict(lanes_per_line=cfg.lanes_per_line, region_bytes=cfg.region_bytes)
    plain = rl.rand_read(region, cfg.line_bytes, cfg.n_reads, cfg.iters_per_wave, cfg.read_seed, **kw)
    assert plain.checksum == want, "plain order"
    windows = zone_map[:32 * gib // 256]                   # windows of 8 GiB
    ids = {z: i for i, z in enumerate(dict.fromkeys(windows))}
    zoned = rl.rand_read(region, cfg.line_bytes, cfg.n_reads, cfg.iters_per_wave, cfg.read_seed,
                         zone_of_window=[ids[z] for z in windows], **kw)
    assert zoned.checksum == want, "zone order"
    gbps = lambda r: cfg.bytes_read / r.kernel_ms_event / 1e6
    print(f"\n[{cfg.name}] plain {gbps(plain):.0f} GB/s, zone order ({len(ids)} zones) {gbps(zoned):.0f} GB/s", flush=True)


def test_windowed_full_size(region, cu_table):
    """Largest region, windows of 1/2, 1/4, 1/8, XCD-aware and random-per-CU, full occupancy."""
    R = region.numel()
    if R >= 256 * GiB:
        R = 256 * GiB
    n = len(cu_table)
    W, I = wl.resident_logical_waves(n), wl.ITERS_PER_WAVE
    for n_windows in (2, 4, 8):
        for scheme in ("xcd", "random"):
            g_of_cu, w_of_g = (wl.window_map_by_xcd(cu_table, n_windows) if scheme == "xcd"
                               else wl.window_map_random_per_cu(n, n_windows, seed=n_windows))
            want = oracle(R, 128, W, I, n_windows=n_windows, window_of_group=w_of_g)
            got = rl.rand_read(region, 128, W * I, I, wl.READ_SEED, rl.WindowMap(n_windows, g_of_cu, w_of_g),
                               region_bytes=R)
            assert got.checksum == want, (n_windows, scheme)


def oracle_groups_equal_library(T, singles, min_gap=0.05):
    """The measured matrix through the library's clustering and through the oracle's: identical groups, order, threshold."""
    from oracle.grouping import groups_from_heatmap as oracle_groups
    g_lib, o_lib, t_lib = rl.groups_from_heatmap(T, singles, min_gap)
    g_orc, o_orc, t_orc = oracle_groups(T, singles, min_gap)
    assert g_lib.tolist() == g_orc.tolist() and o_lib.tolist() == o_orc.tolist()
    assert (np.isnan(t_lib) and np.isnan(t_orc)) or t_lib == t_orc
    return g_lib, t_lib


def probe_matrix(region, units, cfg, want):
    """Singles and all pairs of the probe units (lists of CUs): every run must return the one checksum `want`
    and must have had working waves on every one of its CUs."""
    n_reads = cfg.n_reads * len(units[0])
    gbps = lambda r: n_reads * cfg.line_bytes / r.kernel_ms_device / 1e6
    run = lambda cus: rl.probe_cus(region, cus, n_reads, cfg.iters_per_wave, cfg.read_seed, region_bytes=cfg.region_bytes,
                                   want_cu_waves=True)
    m = len(units)
    singles, T = np.zeros(m), np.zeros((m, m))
    run(units[0] + units[1])
    for i in range(m):
        r = run(units[i])
        assert r.checksum == want, f"unit {i} alone"
        singles[i] = gbps(r)
    for i in range(m):
        for j in range(i + 1, m):
            cus = units[i] + units[j]
            r = run(cus)
            assert r.checksum == want, f"pair {i},{j}"
            assert (r.cu_waves[cus] > 0).all() and r.cu_waves.sum() == r.cu_waves[cus].sum() == r.waves_run
            T[i, j] = T[j, i] = gbps(r)
    return singles, T


def test_probe_all_pairs_full_size(region, cu_table):
    """Paper Sec. 2.2 at full extent: the access kernel on every pair of the 64 sampled compute units (2016 pairs,
    16 GiB, 2^22 reads each) and on each alone.  Every run returns the checksum of one oracle evaluation; the
    measured heatmap gives the same groups through the library's clustering and through the oracle's."""
    need(region, 16)
    cfg = wl.probe_config(16 * GiB)
    want = oracle(cfg.region_bytes, 128, cfg.logical_waves, cfg.iters_per_wave)
    sample = wl.probe_cu_sample(cu_table)
    assert len(sample) == 64
    singles, T = probe_matrix(region, [[int(c)] for c in sample], cfg, want)
    group, thr = oracle_groups_equal_library(T, singles)
    iu = np.triu_indices(64, 1)
    ratio = (T / (singles[:, None] + singles[None, :]))[iu]
    print(f"\n[probe 64x1] single {np.median(singles):.1f} GB/s, pair ratio {ratio.min():.3f}..{ratio.max():.3f}, "
          f"threshold {thr}, {group.max() + 1} groups", flush=True)


def test_probe_blocks_of_four_full_size(region, cu_table):
    """The same with blocks of four adjacent compute units as probe units (all 256 CUs in 64 blocks): two CUs
    cannot load a shared resource on this GPU, two blocks can.  Library and oracle must agree on the measured
    matrix whatever it shows; what it showed so far (32 groups of two blocks, the shader engines) is printed."""
    need(region, 16)
    n = len(cu_table)
    if n % 4 != 0 or n // 4 < 2:
        pytest.skip(f"{n} compute units do not split into blocks of four")
    cfg = wl.probe_config(16 * GiB)
    want = oracle(cfg.region_bytes, 128, cfg.logical_waves * 4, cfg.iters_per_wave)
    m = min(64, n // 4)
    step = (n // 4) / m
    units = [list(range(int(i * step) * 4, int(i * step) * 4 + 4)) for i in range(m)]
    singles, T = probe_matrix(region, units, cfg, want)
    group, thr = oracle_groups_equal_library(T, singles)
    sizes = np.bincount(group)
    print(f"\n[probe {m}x4] single {np.median(singles):.1f} GB/s, threshold {thr}, {group.max() + 1} groups of "
          f"{sorted(set((sizes * 4).tolist()))} CUs", flush=True)
    if not np.isnan(thr):
        # whatever was linked shares a shader engine: blocks of different XCDs are never in one group
        for g in range(group.max() + 1):
            members = np.flatnonzero(group == g)
            assert len({int(cu_table[units[u][0], 0]) for u in members}) == 1


def test_planted_heatmaps_library_equals_oracle():
    """The clustering is host code; run here as well so that the suite on the GPU machine exercises it."""
    from test_grouping_oracle import planted, same_partition
    for sizes, seed in (([8] * 8, 1), ([8, 6, 8, 8, 6, 8, 8, 8, 8, 8, 8, 8, 8, 8], 2), ([2] * 32, 3)):
        T, truth = planted(sizes, seed)
        group, _ = oracle_groups_equal_library(T, None)
        assert same_partition(group, truth)
