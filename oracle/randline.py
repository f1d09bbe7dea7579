"""ctypes front end of the C oracle (oracle/randline_oracle.c).

TEST INFRASTRUCTURE ONLY.  Imported by tests/, by the smoke check and by the
CPU-baseline leg of bench.py; never by the product package.  Argument
marshalling only -- all arithmetic is in the C file.
"""
import ctypes as C
from typing import Optional, Sequence, Tuple

import numpy as np

from . import build as _build

_lib = None


def bind(path: str):
    """Load an oracle shared object and declare the signatures of its functions."""
    L = C.CDLL(path)
    u64, u32, i32 = C.c_uint64, C.c_uint32, C.c_int
    p16 = C.POINTER(C.c_uint16)
    L.rlo_mix64.restype = u64
    L.rlo_mix64.argtypes = [u64]
    L.rlo_sm.restype = u64
    L.rlo_sm.argtypes = [u64, u64]
    L.rlo_fill_word.restype = u32
    L.rlo_fill_word.argtypes = [u64, u64]
    L.rlo_index_hash.restype = u64
    L.rlo_index_hash.argtypes = [u64, u64, u64]
    L.rlo_indices.restype = i32
    L.rlo_indices.argtypes = [u64, u32, u64, u64, u32, u32, u32, p16, u64, C.POINTER(u64)]
    L.rlo_checksum.restype = i32
    L.rlo_checksum.argtypes = [u64, u32, u64, u64, u32, u32, u32, p16, u64, u64, i32,
                               C.POINTER(u64), C.POINTER(i32)]
    L.rlo_fill_buffer.restype = i32
    L.rlo_fill_buffer.argtypes = [C.c_void_p, u64, u64]
    L.rlo_checksum_materialised.restype = i32
    L.rlo_checksum_materialised.argtypes = [C.c_void_p, u64, u32, u64, u64, u32, u32, u32, p16,
                                            u64, i32, C.POINTER(u64), C.POINTER(i32)]
    L.rlo_fill_words.restype = i32
    L.rlo_fill_words.argtypes = [u64, u64, u64, C.POINTER(u32)]
    L.rlo_sum_words.restype = i32
    L.rlo_sum_words.argtypes = [u64, u64, u64, i32, C.POINTER(u64)]
    L.rlo_chase.restype = i32
    L.rlo_chase.argtypes = [u64, u32, u64, u64, u64, u32, u64, C.POINTER(u64), C.POINTER(u64)]
    L.rlo_update_value.restype = u32
    L.rlo_update_value.argtypes = [u64, u64]
    L.rlo_update_checksum.restype = i32
    L.rlo_update_checksum.argtypes = [u64, u32, u64, u32, u64, u64, C.POINTER(u64)]
    L.rlo_apply_updates.restype = i32
    L.rlo_apply_updates.argtypes = [C.c_void_p, u64, u32, u64, u32, u64, u32, u64]
    return L


def lib():
    global _lib
    if _lib is None:
        _lib = bind(_build.build())
    return _lib


def _wog(window_of_group: Optional[Sequence[int]]):
    if window_of_group is None:
        return None, 1, None
    arr = np.ascontiguousarray(np.asarray(window_of_group, dtype=np.uint16))
    return arr, int(arr.size), arr.ctypes.data_as(C.POINTER(C.c_uint16))


def mix64(z: int) -> int:
    return int(lib().rlo_mix64(z & (2**64 - 1)))


def sm(s: int, k: int) -> int:
    return int(lib().rlo_sm(s & (2**64 - 1), k))


def fill_word(fill_seed: int, i: int) -> int:
    return int(lib().rlo_fill_word(fill_seed, i))


def index_hash(read_seed: int, w: int, it: int) -> int:
    return int(lib().rlo_index_hash(read_seed, w, it))


def fill_words(fill_seed: int, first_word: int, n: int) -> np.ndarray:
    out = np.empty(n, dtype=np.uint32)
    rc = lib().rlo_fill_words(fill_seed, first_word, n, out.ctypes.data_as(C.POINTER(C.c_uint32)))
    if rc != 0:
        raise ValueError("rlo_fill_words: invalid argument")
    return out


def fill_buffer(n_bytes: int, fill_seed: int) -> np.ndarray:
    buf = np.empty(n_bytes, dtype=np.uint8)
    rc = lib().rlo_fill_buffer(buf.ctypes.data_as(C.c_void_p), n_bytes, fill_seed)
    if rc != 0:
        raise ValueError("rlo_fill_buffer: invalid argument")
    return buf


def indices(region_bytes: int, line_bytes: int, W: int, I: int, read_seed: int,
            n_windows: int = 1, window_of_group: Optional[Sequence[int]] = None,
            first_wave: int = 0) -> np.ndarray:
    arr, G, ptr = _wog(window_of_group)
    out = np.empty(W * I, dtype=np.uint64)
    rc = lib().rlo_indices(region_bytes, line_bytes, first_wave, W, I, G, n_windows, ptr, read_seed,
                           out.ctypes.data_as(C.POINTER(C.c_uint64)))
    if rc != 0:
        raise ValueError("rlo_indices: invalid argument")
    return out.reshape(W, I)


def checksum(region_bytes: int, line_bytes: int, W: int, I: int, fill_seed: int, read_seed: int,
             n_windows: int = 1, window_of_group: Optional[Sequence[int]] = None,
             first_wave: int = 0, n_threads: int = 1) -> int:
    return checksum_ex(region_bytes, line_bytes, W, I, fill_seed, read_seed, n_windows,
                       window_of_group, first_wave, n_threads)[0]


def checksum_ex(region_bytes: int, line_bytes: int, W: int, I: int, fill_seed: int, read_seed: int,
                n_windows: int = 1, window_of_group: Optional[Sequence[int]] = None,
                first_wave: int = 0, n_threads: int = 1) -> Tuple[int, int]:
    """Recompute-mode checksum; returns (checksum, threads actually used)."""
    arr, G, ptr = _wog(window_of_group)
    out = C.c_uint64(0)
    used = C.c_int(0)
    rc = lib().rlo_checksum(region_bytes, line_bytes, first_wave, W, I, G, n_windows, ptr,
                            fill_seed, read_seed, n_threads, C.byref(out), C.byref(used))
    if rc != 0:
        raise ValueError("rlo_checksum: invalid argument")
    return int(out.value), int(used.value)


def checksum_materialised(buf: np.ndarray, line_bytes: int, W: int, I: int, read_seed: int,
                          n_windows: int = 1, window_of_group: Optional[Sequence[int]] = None,
                          first_wave: int = 0, n_threads: int = 1) -> int:
    """Materialised-mode checksum over an existing host buffer (uint8 array)."""
    assert buf.dtype == np.uint8 and buf.flags["C_CONTIGUOUS"]
    arr, G, ptr = _wog(window_of_group)
    out = C.c_uint64(0)
    used = C.c_int(0)
    rc = lib().rlo_checksum_materialised(buf.ctypes.data_as(C.c_void_p), buf.size, line_bytes,
                                         first_wave, W, I, G, n_windows, ptr, read_seed, n_threads,
                                         C.byref(out), C.byref(used))
    if rc != 0:
        raise ValueError("rlo_checksum_materialised: invalid argument")
    return int(out.value)


def sum_words(fill_seed: int, first_word: int, n_words: int, n_threads: int = 1) -> int:
    """Wrapping 64-bit sum of a range of fill words (the sequential-read checksum)."""
    out = C.c_uint64(0)
    rc = lib().rlo_sum_words(fill_seed, first_word, n_words, n_threads, C.byref(out))
    if rc != 0:
        raise ValueError("rlo_sum_words: invalid argument")
    return int(out.value)


def chase(region_bytes: int, line_bytes: int, fill_seed: int, start: int, stride: int, mask: int,
          hops: int) -> Tuple[int, int]:
    """Dependent-load walk: (line reached, wrapping sum of the words loaded)."""
    final, total = C.c_uint64(0), C.c_uint64(0)
    rc = lib().rlo_chase(region_bytes, line_bytes, fill_seed, start, stride, mask, hops,
                         C.byref(final), C.byref(total))
    if rc != 0:
        raise ValueError("rlo_chase: invalid argument")
    return int(final.value), int(total.value)


OP_WRITE, OP_ADD = 1, 2


def update_value(value_seed: int, i: int) -> int:
    return int(lib().rlo_update_value(value_seed, i))


def update_checksum(region_bytes: int, line_bytes: int, W: int, I: int, draw_seed: int, value_seed: int) -> int:
    out = C.c_uint64(0)
    rc = lib().rlo_update_checksum(region_bytes, line_bytes, W, I, draw_seed, value_seed, C.byref(out))
    if rc != 0:
        raise ValueError("rlo_update_checksum: invalid argument")
    return int(out.value)


def apply_updates(buf: np.ndarray, line_bytes: int, W: int, I: int, draw_seed: int, op: int, value_seed: int) -> None:
    """Perform the random line writes / adds on a host buffer (uint8 array), in place."""
    assert buf.dtype == np.uint8 and buf.flags["C_CONTIGUOUS"]
    rc = lib().rlo_apply_updates(buf.ctypes.data_as(C.c_void_p), buf.size, line_bytes, W, I, draw_seed, op, value_seed)
    if rc != 0:
        raise ValueError("rlo_apply_updates: invalid argument")
