"""Do the oracle's pins have teeth?  Each case plants one plausible mistake into a copy of the
oracle's C source (a dropped term, a wrong shift, a swapped half, a transposed index ...), builds
it, and runs a battery of checks that never consult the real oracle: the published SplitMix64
vector, brute force through byte addresses (tests/pybrute.py), closed forms and invariants.
Every planted mistake must make at least one check fail; the unmodified source must pass them all.
Everything here runs on the CPU.
"""
import os
import struct
import subprocess

import numpy as np
import pytest

from conftest import read_golden_values
from oracle import randline as orc
import pybrute

M64 = (1 << 64) - 1
SRC = os.path.join(os.path.dirname(os.path.abspath(orc.__file__)), "randline_oracle.c")

MISTAKES = [
    ("mix64 first shift 31 instead of 30", "z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;", "z = (z ^ (z >> 31)) * 0xBF58476D1CE4E5B9ULL;"),
    ("mix64 second constant off by one digit", "0x94D049BB133111EBULL", "0x94D049BB133111EAULL"),
    ("generator output k uses k*gamma, not (k+1)*gamma", "return rlo_mix64(s + (k + 1) * GAMMA);", "return rlo_mix64(s + k * GAMMA);"),
    ("fill halves swapped", "return (i % 2 == 0) ? (uint32_t)(q & 0xFFFFFFFFULL) : (uint32_t)(q >> 32);",
     "return (i % 2 == 1) ? (uint32_t)(q & 0xFFFFFFFFULL) : (uint32_t)(q >> 32);"),
    ("fill word index not halved", "uint64_t q = rlo_sm(fill_seed, i / 2);", "uint64_t q = rlo_sm(fill_seed, i);"),
    ("draws from one flat stream instead of one generator per wave", "return rlo_sm(wave_seed, it);", "return rlo_sm(read_seed, w * 64 + it);"),
    ("wave seed taken from output w+1", "uint64_t wave_seed = rlo_sm(read_seed, w);", "uint64_t wave_seed = rlo_sm(read_seed, w + 1);"),
    ("multiply-shift instead of remainder", "return window * L_win + rlo_index_hash(read_seed, w, it) % L_win;",
     "return window * L_win + (uint64_t)(((unsigned __int128)rlo_index_hash(read_seed, w, it) * L_win) >> 64);"),
    ("window base dropped", "return window * L_win + rlo_index_hash(read_seed, w, it) % L_win;", "return rlo_index_hash(read_seed, w, it) % L_win;"),
    ("remainder by the whole region instead of the window", "return window * L_win + rlo_index_hash(read_seed, w, it) % L_win;",
     "return (window * L_win + rlo_index_hash(read_seed, w, it) % L) % L;"),
    ("group of a wave is w / G", "window_of_group[w % G] : 0;", "window_of_group[(w / G) % G] : 0;"),
    ("last word of every line skipped", "for (uint64_t j = 0; j < words_per_line; ++j)\n                wave_sum +=", "for (uint64_t j = 0; j + 1 < words_per_line; ++j)\n                wave_sum +="),
    ("words sign-extended", "wave_sum += (uint64_t)rlo_fill_word(fill_seed, first_word + j);", "wave_sum += (uint64_t)(int64_t)(int32_t)rlo_fill_word(fill_seed, first_word + j);"),
    ("line start assumes 32 words per line", "uint64_t first_word = line * words_per_line;", "uint64_t first_word = line * 32;"),
    ("materialised mode reads every other word", "for (uint32_t off = 0; off < line_bytes; off += 4) {", "for (uint32_t off = 0; off < line_bytes; off += 8) {"),
    ("materialised mode addresses lines as 128 bytes", "const unsigned char *p = base + line * (uint64_t)line_bytes;", "const unsigned char *p = base + line * 128;"),
    ("first_wave ignored in the recompute mode", "uint64_t w = first_wave + (uint64_t)a;\n        uint64_t wave_sum = 0;\n        for (uint64_t it = 0; it < I; ++it) {\n            uint64_t line = line_of(read_seed, w, it, L, G, n_windows, window_of_group);\n            uint64_t first_word",
     "uint64_t w = (uint64_t)a;\n        uint64_t wave_sum = 0;\n        for (uint64_t it = 0; it < I; ++it) {\n            uint64_t line = line_of(read_seed, w, it, L, G, n_windows, window_of_group);\n            uint64_t first_word"),
    ("fill buffer big endian", "p[8 * j + b] = (unsigned char)(q >> (8 * b));", "p[8 * j + b] = (unsigned char)(q >> (8 * (7 - b)));"),
    ("streaming sum starts one word late", "total += (uint64_t)rlo_fill_word(fill_seed, first_word + (uint64_t)k);", "total += (uint64_t)rlo_fill_word(fill_seed, first_word + (uint64_t)k + 1);"),
    ("walk without the hop salt", "uint32_t salt = (uint32_t)(k * 0x9E3779B9ULL);", "uint32_t salt = 0;"),
    ("walk ignores the mask", "(uint64_t)((word ^ salt) & mask)) % L;", "(uint64_t)(word ^ salt)) % L;"),
    ("walk loads word 1 of the line", "uint32_t word = rlo_fill_word(fill_seed, line * words_per_line);", "uint32_t word = rlo_fill_word(fill_seed, line * words_per_line + 1);"),
    ("update value not truncated consistently (index + 1)", "return (uint32_t)((value_seed + i * 0x9E3779B1ULL) & 0xFFFFFFFFULL);", "return (uint32_t)((value_seed + (i + 1) * 0x9E3779B1ULL) & 0xFFFFFFFFULL);"),
    ("write and add exchanged", "uint32_t now = (op == 1) ? v : (uint32_t)(old + v);", "uint32_t now = (op == 2) ? v : (uint32_t)(old + v);"),
    ("update checksum counts lines, not words", "total += (uint64_t)rlo_update_value(value_seed, line * words_per_line + j);", "total += (uint64_t)rlo_update_value(value_seed, line * words_per_line);"),
]


def build_variant(tmp_path, name, old, new):
    text = open(SRC).read()
    if old is not None:
        assert text.count(old) == 1, f"mistake '{name}': snippet to replace occurs {text.count(old)} times in the oracle"
        text = text.replace(old, new)
    c_file = tmp_path / "variant.c"
    so_file = tmp_path / "variant.so"
    c_file.write_text(text)
    subprocess.run(["gcc", "-O1", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-w", "-o", str(so_file), str(c_file)], check=True)
    return str(so_file)


def battery():
    """Independent checks of whatever library orc currently points at; returns the names of those that fail."""
    failed = []

    def check(name, fn):
        try:
            ok = fn()
        except Exception:                                   # a planted mistake may also make a call fail outright
            ok = False
        if not ok:
            failed.append(name)

    vector = read_golden_values("splitmix64_seed1234567.txt")["_list"]
    check("published vector", lambda: [orc.sm(1234567, k) for k in range(5)] == vector)
    check("fill bytes", lambda: orc.fill_buffer(4096, 99).tobytes() == pybrute.region_bytes(4096, 99))
    check("fill words", lambda: orc.fill_words(99, 6, 100).tobytes() == pybrute.region_bytes(4096, 99)[24:424])

    def brute_case(R, B, W, I, nw, wog, first=0):
        region = pybrute.region_bytes(R, 1)
        want, touched = pybrute.checksum(region, B, W, I, 7, nw, wog, first_wave=first)
        got = orc.checksum(R, B, W, I, 1, 7, nw, wog, first_wave=first)
        idx = orc.indices(R, B, W, I, 7, nw, wog, first_wave=first).reshape(-1).tolist()
        buf = np.frombuffer(region, dtype=np.uint8).copy()
        mat = orc.checksum_materialised(buf, B, W, I, 7, nw, wog, first_wave=first)
        return got == want and idx == touched and mat == want

    for case in ((4096, 128, 4, 8, 1, None), (12288, 128, 4, 8, 1, None), (15 * 512, 512, 5, 7, 1, None),
                 (24576, 256, 8, 9, 3, [2, 0, 1, 1]), (8192, 128, 12, 5, 4, [3, 3, 0]), (8192, 128, 3, 6, 1, None, 5)):
        check(f"brute force {case}", lambda c=case: brute_case(*c))

    def one_line():
        line_sum = sum(struct.unpack("<32I", pybrute.region_bytes(128, 1)))
        return orc.checksum(128, 128, 2, 3, 1, 7) == (6 * line_sum) & M64
    check("one-line closed form", one_line)
    check("all-ones buffer", lambda: orc.checksum_materialised(np.ones(1024, "<u4").view(np.uint8), 256, 6, 11, 3) == 6 * 11 * 64)
    check("all-0xFFFFFFFF buffer", lambda: orc.checksum_materialised(np.full(1024, 0xFFFFFFFF, "<u4").view(np.uint8), 128, 4, 5, 3)
          == 4 * 5 * 32 * 0xFFFFFFFF)
    check("high words zero-extended", lambda: orc.checksum(4096, 128, 4, 8, 1, 7) < (4 * 8 * 32) << 32)
    check("exact remainder", lambda: all(int(orc.indices(192 << 30, 128, 1, 8, 7)[0, it]) == orc.index_hash(7, 0, it) % ((192 << 30) // 128)
                                         for it in range(8)))
    check("streaming sum", lambda: orc.sum_words(3, 100, 50) == sum(struct.unpack("<1024I", pybrute.region_bytes(4096, 3))[100:150]))

    def walk(R, B, start, stride, mask, hops):
        region = pybrute.region_bytes(R, 1)
        L, line, total = R // B, start, 0
        for k in range(hops):
            word = struct.unpack_from("<I", region, line * B)[0]
            total += word
            line = (line + stride + ((word ^ (k * 0x9E3779B9 & 0xFFFFFFFF)) & mask)) % L
        return orc.chase(R, B, 1, start, stride, mask, hops) == (line, total & M64)
    check("walk data-driven", lambda: walk(1 << 16, 128, 0, 0, 0xFFFFFFFF, 100))
    check("walk masked", lambda: walk(96 * 256, 256, 3, 12345, 0xFFFF, 257))

    def updates(op):
        R, B, W, I = 96 * 256, 256, 5, 13
        ref = bytearray(pybrute.region_bytes(R, 1))
        total = 0
        for w in range(W):
            for h in pybrute.wave_draws(7, w, I):
                line = h % (R // B)
                for j in range(B // 4):
                    i = line * (B // 4) + j
                    v = (0xABCDEF0123 + i * 0x9E3779B1) & 0xFFFFFFFF
                    total += v
                    old = struct.unpack_from("<I", ref, 4 * i)[0]
                    struct.pack_into("<I", ref, 4 * i, v if op == 1 else (old + v) & 0xFFFFFFFF)
        buf = np.frombuffer(pybrute.region_bytes(R, 1), dtype=np.uint8).copy()
        orc.apply_updates(buf, B, W, I, 7, op, 0xABCDEF0123)
        return buf.tobytes() == bytes(ref) and orc.update_checksum(R, B, W, I, 7, 0xABCDEF0123) == total & M64
    check("random writes", lambda: updates(1))
    check("random adds", lambda: updates(2))
    return failed


@pytest.fixture
def swapped_library():
    saved = orc._lib
    yield
    orc._lib = saved


def test_unmodified_oracle_passes_the_battery(tmp_path, swapped_library):
    orc._lib = orc.bind(build_variant(tmp_path, "none", None, None))
    assert battery() == []


@pytest.mark.parametrize("name,old,new", MISTAKES, ids=[m[0] for m in MISTAKES])
def test_planted_mistake_is_caught(tmp_path, swapped_library, name, old, new):
    orc._lib = orc.bind(build_variant(tmp_path, name, old, new))
    failed = battery()
    assert failed, f"no independent check notices: {name}"
