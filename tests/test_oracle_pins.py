"""Pins of the CPU oracle (oracle/randline_oracle.c) to things other than itself.

 * the published SplitMix64 test vector (constants, shifts, increment);
 * worked values fixed by the benchmark's checksum contract (tests/golden/);
 * brute force through real byte addresses on tiny regions (tests/pybrute.py);
 * closed forms (one-line region; all-ones buffer; power-of-two mask == remainder);
 * invariants (additivity over wave ranges, thread-count independence, window range,
   degenerate window maps, recompute mode == materialised mode);
 * statistics the uniform distribution fixes (distinct-line count, chi-square, mean word).

Each pin names the mistake it is there to catch.
"""
import math
import os

import numpy as np
import pytest

from conftest import read_golden_values
from oracle import randline as orc
import pybrute

M64 = (1 << 64) - 1


# ---------------------------------------------------------------- generator pins
def test_splitmix64_published_vector():
    """Wrong constant, wrong shift, or gamma added after instead of before mixing."""
    want = read_golden_values("splitmix64_seed1234567.txt")["_list"]
    assert [orc.sm(1234567, k) for k in range(5)] == want
    g = pybrute.SplitMix64(1234567)
    assert [g.next() for _ in range(5)] == want  # the brute-force helper is pinned by the same vector


def test_worked_generator_values(worked):
    assert [orc.sm(0, k) for k in range(3)] == worked["sm_seed0"]
    # low half first: a swapped half order flips every even/odd pair
    assert [orc.fill_word(1, i) for i in range(8)] == worked["fill_seed1_words0to7"]
    # split generator per wave: a flat counter sm(seed, w*I+it) fails here
    assert [orc.index_hash(7, 0, i) for i in range(3)] == worked["hash_seed7_wave0"]
    assert [orc.index_hash(7, 1, i) for i in range(3)] == worked["hash_seed7_wave1"]


def test_fill_is_the_little_endian_generator_stream():
    """fill_buffer bytes == the published generator's outputs packed little-endian."""
    buf = orc.fill_buffer(4096, 99).tobytes()
    assert buf == pybrute.region_bytes(4096, 99)
    words = np.frombuffer(buf, dtype="<u4")
    assert np.array_equal(words, orc.fill_words(99, 0, 1024))
    # word index beyond 32 bits (a 256 GiB region has 2^36 words): 32-bit truncation would alias
    hi = (1 << 35) + 6
    g = pybrute.SplitMix64((99 + (hi // 2) * 0x9E3779B97F4A7C15) & M64)
    assert orc.fill_word(99, hi) == g.next() & 0xFFFFFFFF
    assert orc.fill_word(99, hi) != orc.fill_word(99, hi & 0xFFFFFFFF)


# ---------------------------------------------------------------- worked checksums
@pytest.mark.parametrize("key,R,B", [("tiny_R4096_B128", 4096, 128), ("tiny_R4096_B256", 4096, 256),
                                     ("tiny_R4096_B512", 4096, 512), ("tiny_R12288_B128", 12288, 128)])
def test_worked_tiny_checksums(worked, key, R, B):
    assert orc.checksum(R, B, 4, 8, 1, 7) == worked[key][0]


def test_worked_windowed_checksum(worked):
    got = orc.checksum(4096, 128, 4, 8, 1, 7, n_windows=2, window_of_group=[1, 0])
    assert got == worked["tiny_windowed_R4096_B128"][0]
    # swapping the map must change it (window base really applied)
    assert orc.checksum(4096, 128, 4, 8, 1, 7, n_windows=2, window_of_group=[0, 1]) != got


def test_worked_first_configuration(worked):
    """R=2^28, B=128, fill seed 1, read seed 7 (the small reference configuration)."""
    R = 1 << 28
    assert orc.checksum(R, 128, 256, 4096, 1, 7, n_threads=4) == worked["pr1_W256_I4096"][0]
    assert orc.checksum(R, 128, 1024, 1024, 1, 7, n_threads=4) == worked["pr1_W1024_I1024"][0]
    idx = orc.indices(R, 128, 256, 4096, 7)
    assert list(idx[0, :4]) == worked["pr1_wave0_first_indices"]
    assert np.unique(idx).size == worked["pr1_distinct_lines"][0]


def test_stored_values_are_reproduced_by_the_numpy_script():
    """tests/golden/make_worked_values.py (numpy only, no oracle, no GPU) regenerates the fixture."""
    import subprocess
    import sys
    script = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "make_worked_values.py")
    out = subprocess.run([sys.executable, script, "--check"], capture_output=True, text=True)
    assert out.returncode == 0 and "all 15 entries reproduced" in out.stdout, out.stdout + out.stderr


# ---------------------------------------------------------------- brute force via byte addresses
@pytest.mark.parametrize("R,B,W,I,nw,wog", [
    (4096, 128, 4, 8, 1, None),
    (4096, 256, 4, 8, 1, None),
    (4096, 512, 3, 5, 1, None),
    (12288, 128, 4, 8, 1, None),          # 96 lines: non power of two
    (15 * 512, 512, 5, 7, 1, None),       # 15 lines of 512 B
    (4096, 128, 4, 8, 2, [1, 0]),
    (8192, 128, 12, 5, 4, [3, 3, 0]),     # G=3 does not divide n_windows; a window reused, some unused
    (24576, 256, 8, 9, 3, [2, 0, 1, 1]),  # 96 lines, 3 windows of 32
])
def test_bruteforce_byte_addresses(R, B, W, I, nw, wog):
    region = pybrute.region_bytes(R, 1)
    want, touched = pybrute.checksum(region, B, W, I, 7, nw, wog)
    assert orc.checksum(R, B, W, I, 1, 7, nw, wog) == want
    got_idx = orc.indices(R, B, W, I, 7, nw, wog).reshape(-1)
    assert list(got_idx) == touched


def test_bruteforce_first_wave_offset():
    region = pybrute.region_bytes(8192, 5)
    want, _ = pybrute.checksum(region, 128, 3, 6, 11, first_wave=5)
    assert orc.checksum(8192, 128, 3, 6, 5, 11, first_wave=5) == want


# ---------------------------------------------------------------- closed forms
def test_one_line_region_closed_form(worked):
    """R == B: every read is line 0, checksum = n_reads * sum of the line's words."""
    for B in (128, 256, 512):
        line_sum = int(orc.fill_words(1, 0, B // 4).astype(np.uint64).sum())
        for W, I in ((2, 3), (5, 1), (1, 17)):
            assert orc.checksum(B, B, W, I, 1, 7) == (W * I * line_sum) & M64
    assert orc.checksum(128, 128, 2, 3, 1, 7) == worked["one_line_R128"][0]


def test_all_ones_buffer_counts_words():
    """On a buffer of 0x00000001 words the materialised checksum is the number of words read:
    a dropped or doubled word, or a 64-bit instead of 32-bit load, changes the count."""
    for B in (128, 256, 512):
        buf = np.ones(4096 // 4, dtype="<u4").view(np.uint8)
        assert orc.checksum_materialised(buf, B, 6, 11, 3) == 6 * 11 * (B // 4)
    # 0xFFFFFFFF words: zero-extension, not sign-extension, and no 32-bit wrap of the sum
    buf = np.full(4096 // 4, 0xFFFFFFFF, dtype="<u4").view(np.uint8)
    assert orc.checksum_materialised(buf, 128, 4, 5, 3) == 4 * 5 * 32 * 0xFFFFFFFF


def test_line_identifying_buffer_recovers_indices():
    """Buffer where every word of line l holds l: checksum = words_per_line * sum of indices."""
    B, L = 128, 96
    buf = np.repeat(np.arange(L, dtype="<u4"), B // 4).view(np.uint8)
    idx = orc.indices(L * B, B, 5, 9, 21)
    assert orc.checksum_materialised(buf, B, 5, 9, 21) == (B // 4) * int(idx.sum())


def test_power_of_two_remainder_is_a_mask():
    idx = orc.indices(1 << 20, 128, 3, 50, 7)
    for w in range(3):
        for it in range(50):
            assert idx[w, it] == orc.index_hash(7, w, it) & ((1 << 13) - 1)


def test_non_power_of_two_remainder_is_exact():
    """3*2^30 lines (a 192 GiB region of 128-B lines): python big-int remainder."""
    R = 192 << 30
    L = R // 128
    idx = orc.indices(R, 128, 2, 40, 7)
    for w in range(2):
        for it in range(40):
            assert idx[w, it] == orc.index_hash(7, w, it) % L


# ---------------------------------------------------------------- invariants
def test_additivity_and_thread_independence():
    R, B, W, I = 1 << 16, 128, 37, 13
    whole = orc.checksum(R, B, W, I, 1, 7)
    parts = sum(orc.checksum(R, B, n, I, 1, 7, first_wave=f) for f, n in ((0, 10), (10, 1), (11, 26)))
    assert parts & M64 == whole
    for t in (2, 3, 8):
        assert orc.checksum(R, B, W, I, 1, 7, n_threads=t) == whole


def test_recompute_equals_materialised():
    for R, B in ((1 << 20, 128), (3 << 18, 256), (1 << 20, 512)):
        buf = orc.fill_buffer(R, 1)
        for nw, wog in ((1, None), (2, [1, 0]), (4, [2, 0, 3, 1, 1, 2, 0, 3])):
            W = 16
            assert orc.checksum_materialised(buf, B, W, 64, 7, nw, wog, n_threads=2) == \
                orc.checksum(R, B, W, 64, 1, 7, nw, wog)


def test_recompute_equals_materialised_256MiB():
    """The first configuration end to end through host memory."""
    R = 1 << 28
    buf = orc.fill_buffer(R, 1)
    assert orc.checksum_materialised(buf, 128, 256, 4096, 7, n_threads=8) == \
        orc.checksum(R, 128, 256, 4096, 1, 7, n_threads=8)


def test_window_indices_in_range():
    R, B, nw = 1 << 22, 128, 8
    L = R // B
    wog = [5, 0, 7, 7, 2, 1]
    idx = orc.indices(R, B, 24, 200, 7, nw, wog)
    for w in range(24):
        v = wog[w % 6]
        assert idx[w].min() >= v * (L // nw) and idx[w].max() < (v + 1) * (L // nw)
    # within its window the offset is the unwindowed draw reduced modulo the window length
    for it in range(5):
        assert idx[3, it] - wog[3] * (L // nw) == orc.index_hash(7, 3, it) % (L // nw)


def test_degenerate_window_maps_equal_no_map():
    R, B, W, I = 1 << 18, 128, 24, 31
    plain = orc.checksum(R, B, W, I, 1, 7)
    assert orc.checksum(R, B, W, I, 1, 7, 1, [0]) == plain
    assert orc.checksum(R, B, W, I, 1, 7, 1, [0] * 8) == plain       # one window, any grouping
    assert orc.checksum(R, B, W, I, 1, 7, 2, [0, 0]) != plain        # a real restriction differs


def test_line_width_only_regroups_words():
    """256-B lines read as 2 x 128-B halves: same draw stream -> sum over line 2k and 2k+1."""
    R, W, I = 1 << 16, 4, 16
    idx256 = orc.indices(R, 256, W, I, 7).reshape(-1)
    want = 0
    for l in idx256:
        want += int(orc.fill_words(1, int(l) * 64, 64).astype(np.uint64).sum())
    assert orc.checksum(R, 256, W, I, 1, 7) == want & M64


def test_invalid_arguments_rejected():
    with pytest.raises(ValueError):
        orc.checksum(4096, 64, 1, 1, 1, 7)
    with pytest.raises(ValueError):
        orc.checksum(4096 + 4, 128, 1, 1, 1, 7)
    with pytest.raises(ValueError):
        orc.checksum(4096, 128, 1, 1, 1, 7, n_windows=3, window_of_group=[0])
    with pytest.raises(ValueError):
        orc.checksum(4096, 128, 1, 1, 1, 7, n_windows=2, window_of_group=[2])


# ---------------------------------------------------------------- statistics of the uniform draw
def test_uniformity_statistics(worked):
    R, B = 1 << 28, 128
    L = R // B
    idx = orc.indices(R, B, 256, 4096, 7).reshape(-1)
    n = idx.size
    # distinct lines among n uniform draws from L: L(1-exp(-n/L)) +- a few sigma
    expect = L * (1 - math.exp(-n / L))
    assert abs(np.unique(idx).size - expect) < 5 * math.sqrt(expect)
    # chi-square over 1024 equal bins
    counts = np.bincount((idx >> np.uint64(11)).astype(np.int64), minlength=1024)
    chi2 = float(((counts - n / 1024) ** 2 / (n / 1024)).sum())
    assert 1023 - 6 * math.sqrt(2 * 1023) < chi2 < 1023 + 6 * math.sqrt(2 * 1023)
    # mean of the words read is close to 2^31 (uniform 32-bit words)
    mean = orc.checksum(R, B, 256, 4096, 1, 7, n_threads=4) / (n * 32)
    assert int(mean) == worked["pr1_mean_word"][0]
    assert abs(mean - 2 ** 31) < 5 * (2 ** 32 / math.sqrt(12)) / math.sqrt(n * 32) * 40  # lines repeat


# ---------------------------------------------------------------- dependent-load walk
def test_chase_bruteforce_byte_addresses():
    """The walk through real byte addresses of a materialised region (wrong word, wrong modulus,
    stride or mask dropped)."""
    import struct
    for R, B in ((1 << 16, 128), (96 * 256, 256), (15 * 512, 512)):
        region = pybrute.region_bytes(R, 1)
        L = R // B
        for start, stride, mask, hops in ((0, 0, 0xFFFFFFFF, 100), (5, 7, 0, 1000), (3, 123456789, 0xFFFF, 257),
                                          (L - 1, 1, 0, 3), (2, 0, 0, 9)):
            line, total = start, 0
            for k in range(hops):
                word = struct.unpack_from("<I", region, line * B)[0]
                total += word
                line = (line + stride + ((word ^ (k * 0x9E3779B9 & 0xFFFFFFFF)) & mask)) % L
            assert orc.chase(R, B, 1, start, stride, mask, hops) == (line, total & M64)


def test_chase_closed_forms():
    R, B = 192 << 30, 128                     # 3 * 2^30 lines: 64-bit line arithmetic
    L = R // B
    final, total = orc.chase(R, B, 1, 17, 1 << 14, 0, 1000)
    assert final == (17 + 1000 * (1 << 14)) % L      # mask 0: a pure strided walk
    lines = [(17 + k * (1 << 14)) % L for k in range(1000)]
    assert total == sum(orc.fill_word(1, l * 32) for l in lines) & M64
    assert orc.chase(R, B, 1, 5, 0, 0, 10) == (5, 10 * orc.fill_word(1, 5 * 32))   # standing still
    with pytest.raises(ValueError):
        orc.chase(R, B, 1, L, 0, 0, 1)


# ---------------------------------------------------------------- random line write / add
def test_update_bruteforce_on_bytes():
    """Writes and adds applied with struct on a bytearray (wrong word index, value not truncated to
    32 bits, add without wrap, write that depends on the old content)."""
    import struct
    for R, B, W, I in ((4096, 128, 4, 8), (96 * 256, 256, 5, 13), (15 * 512, 512, 3, 40)):
        L = R // B
        for op in (orc.OP_WRITE, orc.OP_ADD):
            ref = bytearray(pybrute.region_bytes(R, 1))
            total = 0
            for w in range(W):
                for h in pybrute.wave_draws(7, w, I):
                    line = h % L
                    for j in range(B // 4):
                        i = line * (B // 4) + j
                        v = (0xABCDEF0123 + i * 0x9E3779B1) & 0xFFFFFFFF
                        total += v
                        old = struct.unpack_from("<I", ref, 4 * i)[0]
                        struct.pack_into("<I", ref, 4 * i, v if op == orc.OP_WRITE else (old + v) & 0xFFFFFFFF)
            buf = orc.fill_buffer(R, 1)
            orc.apply_updates(buf, B, W, I, 7, op, 0xABCDEF0123)
            assert buf.tobytes() == bytes(ref)
            assert orc.update_checksum(R, B, W, I, 7, 0xABCDEF0123) == total & M64


def test_update_closed_forms():
    B = 128
    old = orc.fill_words(1, 0, 32).astype(np.uint64)
    v = np.array([orc.update_value(5, j) for j in range(32)], dtype=np.uint64)
    buf = orc.fill_buffer(B, 1)                      # one-line region: every update hits line 0
    orc.apply_updates(buf, B, 3, 7, 9, orc.OP_ADD, 5)
    assert np.array_equal(buf.view("<u4").astype(np.uint64), (old + 21 * v) % (1 << 32))
    buf = orc.fill_buffer(B, 1)
    orc.apply_updates(buf, B, 3, 7, 9, orc.OP_WRITE, 5)
    assert np.array_equal(buf.view("<u4").astype(np.uint64), v)
    assert orc.update_checksum(B, B, 3, 7, 9, 5) == 21 * int(v.sum())
    # a write is idempotent, and lines that were not hit keep the fill
    R = 1 << 16
    a, b = orc.fill_buffer(R, 1), orc.fill_buffer(R, 1)
    orc.apply_updates(a, B, 4, 9, 7, orc.OP_WRITE, 3)
    orc.apply_updates(b, B, 4, 9, 7, orc.OP_WRITE, 3)
    orc.apply_updates(b, B, 4, 9, 7, orc.OP_WRITE, 3)
    assert np.array_equal(a, b)
    hit = set(orc.indices(R, B, 4, 9, 7).reshape(-1).tolist())
    words = a.view("<u4").reshape(-1, 32)
    fill = orc.fill_words(1, 0, R // 4).reshape(-1, 32)
    for line in range(R // B):
        assert np.array_equal(words[line], fill[line]) == (line not in hit)
    assert orc.update_value(0xFFFFFFFFFFFFFFFF, 1 << 36) == (0xFFFFFFFFFFFFFFFF + (1 << 36) * 0x9E3779B1) & 0xFFFFFFFF
