"""ctypes binding of librandline.so -- same names as the C ABI (include/randline.h).

Argument marshalling only: every step of the benchmark runs in the HIP library.
PyTorch is used by callers for device memory and streams; this module accepts a
torch tensor (its data_ptr/nbytes are taken) or a raw (pointer, bytes) pair.
There is no CPU fallback: if the library is missing, importing fails loudly.
"""
import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional, Sequence, Tuple

import numpy as np

from . import build as _build

RR_OK, RR_EINVAL, RR_EHIP, RR_EPLACE = 0, -1, -2, -3
RR_CU_EXCLUDED = 0xFFFF
BCAST_DEFAULT, BCAST_LDS, BCAST_DPP, BCAST_READLANE = 0, 1, 2, 3
MODE_AUTO, MODE_FLAT, MODE_TICKET, MODE_STREAM = 0, 1, 2, 3
SPLIT_DEFAULT, SPLIT_ON, SPLIT_OFF = 0, 1, 2
NT_DEFAULT, NT_ON, NT_OFF = 0, 1, 2
OP_WRITE, OP_ADD = 1, 2


class RandlineError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"randline error {code}: {message}")
        self.code = code


class _CU(C.Structure):
    _fields_ = [("xcc", C.c_uint32), ("se", C.c_uint32), ("sh", C.c_uint32), ("cu", C.c_uint32)]


class _WindowMap(C.Structure):
    _fields_ = [("n_groups", C.c_uint32), ("n_windows", C.c_uint32), ("n_cus", C.c_uint32),
                ("group_of_cu", C.POINTER(C.c_uint16)), ("window_of_group", C.POINTER(C.c_uint16))]


class _Result(C.Structure):
    _fields_ = [("checksum", C.c_uint64), ("kernel_ms_event", C.c_double),
                ("kernel_ms_device", C.c_double), ("waves_run", C.c_uint32), ("launches", C.c_uint32)]


class _ChaseResult(C.Structure):
    _fields_ = [("final_line", C.c_uint64), ("word_sum", C.c_uint64), ("kernel_ms_event", C.c_double),
                ("ns_per_hop", C.c_double)]


class _Opts(C.Structure):
    _fields_ = [("block_threads", C.c_uint32), ("grid_blocks", C.c_uint32), ("unroll", C.c_uint32),
                ("mode", C.c_uint32), ("bcast", C.c_uint32), ("nontemporal", C.c_uint32),
                ("chunk_iters", C.c_uint32), ("xcd_split", C.c_uint32), ("first_wave", C.c_uint64),
                ("zone_bytes", C.c_uint64), ("zone_of_window", C.POINTER(C.c_uint8)), ("n_zone_windows", C.c_uint32),
                ("zone_descending", C.c_uint32), ("phase_ticks", C.c_void_p), ("placement_out", C.POINTER(C.c_uint16)),
                ("cu_waves_out", C.POINTER(C.c_uint32))]


class _ReadPlan(C.Structure):
    _fields_ = [("mode", C.c_uint32), ("zone_kernel", C.c_uint32), ("n_zones", C.c_uint32), ("n_zone_windows", C.c_uint32),
                ("zone_window_bytes", C.c_uint64), ("zone_windows", C.c_uint64 * 16), ("xcd_split", C.c_uint32),
                ("chunk_iters", C.c_uint32), ("split_windows", C.c_uint64 * 2), ("block_threads", C.c_uint32),
                ("unroll", C.c_uint32), ("bcast", C.c_uint32), ("nontemporal", C.c_uint32)]


class _ZoneProbeOpts(C.Structure):
    _fields_ = [("min_gap", C.c_double), ("max_zones", C.c_uint32), ("launches", C.c_uint32),
                ("iters_per_wave", C.c_uint32), ("warmup", C.c_uint32), ("unroll", C.c_uint32),
                ("reserved", C.c_uint32)]


class _ZoneProbe(C.Structure):
    _fields_ = [("same", C.c_double), ("cut", C.c_double), ("band", C.c_double), ("row", C.c_double * 64),
                ("n_zones", C.c_uint32), ("pair_rates", C.c_uint32), ("retakes", C.c_uint32),
                ("gave_up", C.c_uint32), ("launches", C.c_uint32), ("merge_rates", C.c_uint32),
                ("seconds", C.c_double), ("before_merging", C.c_uint8 * 64)]


PAIR_RATE_FN = C.CFUNCTYPE(C.c_int, C.c_uint32, C.c_uint32, C.c_int, C.c_void_p, C.POINTER(C.c_double))
ZONE_NO_WARMUP = 0xFFFFFFFF


class _ReadItem(C.Structure):
    _fields_ = [("region_bytes", C.c_uint64), ("read_seed", C.c_uint64), ("opts", C.POINTER(_Opts))]


EXPORTS = ["rr_enumerate_cus", "rr_fill", "rr_rand_read", "rr_rand_read_noalloc", "rr_rand_read_batch", "rr_probe_pair", "rr_probe_cus", "rr_seq_read", "rr_copy", "rr_chase", "rr_chase_on_cu", "rr_rand_update",
           "rr_region_granularity", "rr_region_create", "rr_region_destroy",
           "rr_groups_from_heatmap", "rr_zones_from_pair_rates", "rr_detect_zones", "rr_shutdown", "rr_strerror", "rr_last_error", "rr_last_kernel", "rr_describe_read"]

_lib = None


def library_path() -> str:
    return _build.LIB


def lib():
    """Load the built library (build it only if nothing is built yet)."""
    global _lib
    if _lib is None:
        path = library_path()
        if not os.path.exists(path):
            _build.build()
        # PyTorch ships its own HIP runtime under the same soname.  Import it first so that this
        # library binds to that copy: two HIP runtimes in one process cannot both own the device.
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        L = C.CDLL(path)
        u64, u32, vp = C.c_uint64, C.c_uint32, C.c_void_p
        L.rr_enumerate_cus.restype = C.c_int
        L.rr_enumerate_cus.argtypes = [C.POINTER(_CU), u32, C.POINTER(u32), vp]
        L.rr_fill.restype = C.c_int
        L.rr_fill.argtypes = [vp, u64, u64, vp]
        L.rr_rand_read.restype = C.c_int
        L.rr_rand_read.argtypes = [vp, u64, u32, u32, u64, u32, C.POINTER(_WindowMap), u64, vp,
                                   C.POINTER(_Opts), C.POINTER(_Result)]
        L.rr_rand_read_noalloc.restype = C.c_int
        L.rr_rand_read_noalloc.argtypes = L.rr_rand_read.argtypes
        L.rr_rand_read_batch.restype = C.c_int
        L.rr_rand_read_batch.argtypes = [vp, C.POINTER(_ReadItem), u32, u32, u32, u64, u32, vp, C.POINTER(_Result)]
        L.rr_probe_pair.restype = C.c_int
        L.rr_probe_pair.argtypes = [vp, u64, u32, u32, u64, u32, u64, vp, C.POINTER(_Opts), C.POINTER(_Result)]
        L.rr_probe_cus.restype = C.c_int
        L.rr_probe_cus.argtypes = [vp, u64, C.POINTER(u32), u32, u64, u32, u64, vp, C.POINTER(_Opts),
                                   C.POINTER(_Result)]
        L.rr_seq_read.restype = C.c_int
        L.rr_seq_read.argtypes = [vp, u64, vp, C.POINTER(_Result)]
        L.rr_copy.restype = C.c_int
        L.rr_copy.argtypes = [vp, vp, u64, vp, C.POINTER(C.c_double)]
        L.rr_rand_update.restype = C.c_int
        L.rr_rand_update.argtypes = [vp, u64, u32, u32, u64, u32, u64, u32, u64, vp, C.POINTER(_Result)]
        L.rr_chase.restype = C.c_int
        L.rr_chase.argtypes = [vp, u64, u32, u64, u64, u32, u64, vp, C.POINTER(_ChaseResult)]
        L.rr_chase_on_cu.restype = C.c_int
        L.rr_chase_on_cu.argtypes = [vp, u64, u32, u64, u64, u32, u64, u32, vp, C.POINTER(_ChaseResult)]
        L.rr_region_granularity.restype = C.c_int
        L.rr_region_granularity.argtypes = [C.POINTER(u64), C.POINTER(u64)]
        L.rr_region_create.restype = C.c_int
        L.rr_region_create.argtypes = [u64, u64, C.POINTER(vp)]
        L.rr_region_destroy.restype = C.c_int
        L.rr_region_destroy.argtypes = [vp]
        L.rr_groups_from_heatmap.restype = C.c_int
        L.rr_groups_from_heatmap.argtypes = [C.POINTER(C.c_double), u32, C.POINTER(C.c_double), C.c_double,
                                             C.POINTER(C.c_uint16), C.POINTER(u32), C.POINTER(u32),
                                             C.POINTER(C.c_double)]
        L.rr_zones_from_pair_rates.restype = C.c_int
        L.rr_zones_from_pair_rates.argtypes = [PAIR_RATE_FN, vp, u32, C.c_double, u32, C.POINTER(C.c_uint8),
                                               C.POINTER(_ZoneProbe)]
        L.rr_detect_zones.restype = C.c_int
        L.rr_detect_zones.argtypes = [vp, u64, u32, C.POINTER(_ZoneProbeOpts), vp, C.POINTER(C.c_uint8),
                                      C.POINTER(_ZoneProbe)]
        L.rr_shutdown.restype = C.c_int
        L.rr_shutdown.argtypes = []
        L.rr_strerror.restype = C.c_char_p
        L.rr_strerror.argtypes = [C.c_int]
        L.rr_last_error.restype = C.c_char_p
        L.rr_last_error.argtypes = []
        L.rr_last_kernel.restype = C.c_char_p
        L.rr_last_kernel.argtypes = []
        L.rr_describe_read.restype = C.c_int
        L.rr_describe_read.argtypes = [vp, u64, u32, u32, u64, u32, C.POINTER(_WindowMap), C.POINTER(_Opts),
                                       C.POINTER(_ReadPlan)]
        _lib = L
    return _lib


def _check(rc: int):
    if rc != RR_OK:
        msg = lib().rr_last_error().decode() or lib().rr_strerror(rc).decode()
        raise RandlineError(rc, msg)


def _region(region, region_bytes: Optional[int]) -> Tuple[int, int]:
    """(device pointer, bytes) of a torch tensor, or of an explicit (ptr, bytes) pair."""
    if hasattr(region, "data_ptr"):
        nbytes = region.numel() * region.element_size()
        return int(region.data_ptr()), int(nbytes if region_bytes is None else region_bytes)
    if isinstance(region, tuple):
        return int(region[0]), int(region[1])
    if region_bytes is None:
        raise ValueError("region_bytes is required with a raw pointer")
    return int(region), int(region_bytes)


def _stream(stream) -> Optional[int]:
    if stream is None:
        try:
            import torch
            if torch.cuda.is_available():
                return int(torch.cuda.current_stream().cuda_stream) or None
        except ImportError:
            pass
        return None
    if hasattr(stream, "cuda_stream"):
        return int(stream.cuda_stream) or None
    return int(stream) or None


@dataclass
class WindowMap:
    """Host-side window map: CU -> group -> window (see rr_window_map_t)."""
    n_windows: int
    group_of_cu: np.ndarray       # uint16 [n_cus]; RR_CU_EXCLUDED keeps a CU out
    window_of_group: np.ndarray   # uint16 [G]

    def __post_init__(self):
        self.group_of_cu = np.ascontiguousarray(self.group_of_cu, dtype=np.uint16)
        self.window_of_group = np.ascontiguousarray(self.window_of_group, dtype=np.uint16)

    @property
    def n_groups(self) -> int:
        return int(self.window_of_group.size)

    def _c(self) -> _WindowMap:
        return _WindowMap(self.n_groups, self.n_windows, int(self.group_of_cu.size),
                          self.group_of_cu.ctypes.data_as(C.POINTER(C.c_uint16)),
                          self.window_of_group.ctypes.data_as(C.POINTER(C.c_uint16)))


@dataclass
class ReadResult:
    checksum: int
    kernel_ms_event: float
    kernel_ms_device: float
    waves_run: int
    launches: int
    placement: Optional[np.ndarray] = None   # dense CU id per logical wave, if requested
    cu_waves: Optional[np.ndarray] = None    # working hardware waves per CU, if requested


def _opts(W: int, n_cus_hint: int, block_threads=0, grid_blocks=0, unroll=0, mode=0, bcast=0,
          nontemporal=0, chunk_iters=0, first_wave=0, zone_bytes=0, zone_of_window=None, phase_ticks=None,
          zone_descending=False, xcd_split=0, want_placement=False, want_cu_waves=False):
    ticks_ptr = None
    if phase_ticks is not None:   # a torch int64 device tensor of hardware waves x zones elements
        ticks_ptr = int(phase_ticks.data_ptr())
    zmap_ptr, zmap_len = None, 0
    if zone_of_window is not None:
        zmap = np.ascontiguousarray(zone_of_window, dtype=np.uint8)
        zmap_ptr, zmap_len = zmap.ctypes.data_as(C.POINTER(C.c_uint8)), int(zmap.size)
    o = _Opts(block_threads, grid_blocks, unroll, mode, bcast, nontemporal, chunk_iters, xcd_split, first_wave, zone_bytes,
              zmap_ptr, zmap_len, int(zone_descending), ticks_ptr, None, None)
    o._keepalive = zone_of_window if zone_of_window is None else zmap
    placement = cu_waves = None
    if want_placement:
        placement = np.full(max(W, 1), 0xFFFF, dtype=np.uint16)
        o.placement_out = placement.ctypes.data_as(C.POINTER(C.c_uint16))
    if want_cu_waves:
        cu_waves = np.zeros(n_cus_hint, dtype=np.uint32)
        o.cu_waves_out = cu_waves.ctypes.data_as(C.POINTER(C.c_uint32))
    return o, placement, cu_waves


def enumerate_cus(stream=None) -> np.ndarray:
    """Array [n_cus, 4] of (xcc, se, sh, cu); row index = dense CU id."""
    n = C.c_uint32(0)
    buf = (_CU * 1024)()
    _check(lib().rr_enumerate_cus(buf, 1024, C.byref(n), _stream(stream)))
    return np.array([[buf[i].xcc, buf[i].se, buf[i].sh, buf[i].cu] for i in range(n.value)], dtype=np.uint32)


def fill(region, fill_seed: int, region_bytes: Optional[int] = None, stream=None) -> None:
    ptr, nbytes = _region(region, region_bytes)
    _check(lib().rr_fill(ptr, nbytes, fill_seed, _stream(stream)))


def _rand_read(entry, region, line_bytes, n_reads, iters_per_wave, read_seed, window_map, lanes_per_line,
               region_bytes, stream, want_placement, want_cu_waves, launch) -> ReadResult:
    ptr, nbytes = _region(region, region_bytes)
    W = n_reads // iters_per_wave if iters_per_wave else 0
    o, placement, cu_waves = _opts(W, 1024, want_placement=want_placement, want_cu_waves=want_cu_waves, **launch)
    res = _Result()
    wm = window_map._c() if window_map is not None else None
    _check(entry(ptr, nbytes, line_bytes, lanes_per_line, n_reads, iters_per_wave,
                 C.byref(wm) if wm is not None else None, read_seed, _stream(stream), C.byref(o), C.byref(res)))
    return ReadResult(int(res.checksum), res.kernel_ms_event, res.kernel_ms_device, int(res.waves_run),
                      int(res.launches), placement[:W] if placement is not None else None, cu_waves)


def rand_read(region, line_bytes: int, n_reads: int, iters_per_wave: int, read_seed: int,
              window_map: Optional[WindowMap] = None, lanes_per_line: int = 32,
              region_bytes: Optional[int] = None, stream=None, want_placement: bool = False,
              want_cu_waves: bool = False, **launch) -> ReadResult:
    return _rand_read(lib().rr_rand_read, region, line_bytes, n_reads, iters_per_wave, read_seed, window_map,
                      lanes_per_line, region_bytes, stream, want_placement, want_cu_waves, launch)


def rand_read_noalloc(region, line_bytes: int, n_reads: int, iters_per_wave: int, read_seed: int,
                      window_map: Optional[WindowMap] = None, lanes_per_line: int = 32,
                      region_bytes: Optional[int] = None, stream=None, want_placement: bool = False,
                      want_cu_waves: bool = False, **launch) -> ReadResult:
    """rand_read through the entry point that allocates nothing (see rr_rand_read_noalloc)."""
    return _rand_read(lib().rr_rand_read_noalloc, region, line_bytes, n_reads, iters_per_wave, read_seed, window_map,
                      lanes_per_line, region_bytes, stream, want_placement, want_cu_waves, launch)


class ReadBatch:
    """The arguments of one rr_rand_read_batch call, marshalled once and reusable: a caller that repeats a series
    of reads with new seeds (a benchmark step) pays for building the C structures only the first time.

    items: one (region_bytes, read_seed) or (region_bytes, read_seed, launch options as a dict) per call."""

    def __init__(self, region, items: Sequence, line_bytes: int, n_reads: int, iters_per_wave: int,
                 lanes_per_line: int = 32):
        self._ptr, _ = _region(region, 0)
        self._n = len(items)
        self._arr = (_ReadItem * max(self._n, 1))()
        self._keep = []
        for i, it in enumerate(items):
            self._arr[i].region_bytes, self._arr[i].read_seed = int(it[0]), int(it[1])
            launch = dict(it[2]) if len(it) > 2 and it[2] else None
            if launch is not None:
                o, _, _ = _opts(0, 1024, **launch)
                self._keep.append(o)
                self._arr[i].opts = C.pointer(o)
        self._res = (_Result * max(self._n, 1))()
        self._shape = (line_bytes, lanes_per_line, n_reads, iters_per_wave)
        self._call = lib().rr_rand_read_batch

    def run(self, read_seed: Optional[int] = None, stream=None):
        """Queue the calls and wait once; with read_seed, every item uses that seed.  A list of ReadResult."""
        if read_seed is not None:
            for i in range(self._n):
                self._arr[i].read_seed = read_seed
        line_bytes, lanes, n_reads, iters = self._shape
        _check(self._call(self._ptr, self._arr, self._n, line_bytes, lanes, n_reads, iters, _stream(stream), self._res))
        return [ReadResult(int(r.checksum), r.kernel_ms_event, r.kernel_ms_device, int(r.waves_run), int(r.launches))
                for r in self._res[:self._n]]


def rand_read_batch(region, items: Sequence, line_bytes: int, n_reads: int, iters_per_wave: int,
                    lanes_per_line: int = 32, stream=None):
    """Several rand_read calls queued back to back with one wait at the end (see rr_rand_read_batch).
    Returns a list of ReadResult, one per item of ReadBatch's `items`."""
    return ReadBatch(region, items, line_bytes, n_reads, iters_per_wave, lanes_per_line).run(stream=stream)


def probe_cus(region, cus: Sequence[int], n_reads: int, iters_per_wave: int, read_seed: int,
              region_bytes: Optional[int] = None, stream=None, want_placement: bool = False,
              want_cu_waves: bool = False, **launch) -> ReadResult:
    ptr, nbytes = _region(region, region_bytes)
    W = n_reads // iters_per_wave if iters_per_wave else 0
    o, placement, cu_waves = _opts(W, 1024, want_placement=want_placement, want_cu_waves=want_cu_waves, **launch)
    res = _Result()
    arr = (C.c_uint32 * max(len(cus), 1))(*[int(c) for c in cus])
    _check(lib().rr_probe_cus(ptr, nbytes, arr, len(cus), n_reads, iters_per_wave, read_seed, _stream(stream),
                              C.byref(o), C.byref(res)))
    return ReadResult(int(res.checksum), res.kernel_ms_event, res.kernel_ms_device, int(res.waves_run),
                      int(res.launches), placement[:W] if placement is not None else None, cu_waves)


def probe_pair(region, cu_a: int, cu_b: int, n_reads: int, iters_per_wave: int, read_seed: int,
               region_bytes: Optional[int] = None, stream=None, **launch) -> ReadResult:
    ptr, nbytes = _region(region, region_bytes)
    o, _, _ = _opts(0, 1024, **launch)
    res = _Result()
    _check(lib().rr_probe_pair(ptr, nbytes, cu_a, cu_b, n_reads, iters_per_wave, read_seed, _stream(stream),
                               C.byref(o), C.byref(res)))
    return ReadResult(int(res.checksum), res.kernel_ms_event, res.kernel_ms_device, int(res.waves_run),
                      int(res.launches))


def seq_read(region, region_bytes: Optional[int] = None, stream=None) -> ReadResult:
    ptr, nbytes = _region(region, region_bytes)
    res = _Result()
    _check(lib().rr_seq_read(ptr, nbytes, _stream(stream), C.byref(res)))
    return ReadResult(int(res.checksum), res.kernel_ms_event, res.kernel_ms_device, int(res.waves_run),
                      int(res.launches))


def copy(dst, src, nbytes: Optional[int] = None, stream=None) -> float:
    """Device-to-device copy with the library's plain copy kernel; returns the kernel time in ms."""
    dptr, dbytes = _region(dst, nbytes)
    sptr, sbytes = _region(src, nbytes)
    ms = C.c_double(0.0)
    _check(lib().rr_copy(dptr, sptr, min(dbytes, sbytes), _stream(stream), C.byref(ms)))
    return float(ms.value)


class Region:
    """A device region made by rr_region_create; accepted wherever a region tensor is (it has data_ptr/numel)."""

    def __init__(self, ptr: int, nbytes: int, piece_bytes: int):
        self.ptr, self.nbytes, self.piece_bytes = ptr, nbytes, piece_bytes

    def data_ptr(self) -> int:
        return self.ptr

    def numel(self) -> int:
        return self.nbytes

    def element_size(self) -> int:
        return 1

    def destroy(self) -> None:
        if self.ptr:
            _check(lib().rr_region_destroy(self.ptr))
            self.ptr = 0

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.destroy()


def region_granularity() -> Tuple[int, int]:
    """(minimum, recommended) physical allocation granularity of the current device, in bytes."""
    lo, rec = C.c_uint64(0), C.c_uint64(0)
    _check(lib().rr_region_granularity(C.byref(lo), C.byref(rec)))
    return int(lo.value), int(rec.value)


def region_create(nbytes: int, piece_bytes: int) -> Region:
    """Device region of nbytes backed by separate physical pieces of piece_bytes; see rr_region_create."""
    out = C.c_void_p(None)
    _check(lib().rr_region_create(nbytes, piece_bytes, C.byref(out)))
    return Region(int(out.value), nbytes, piece_bytes)


def rand_update(region, line_bytes: int, n_updates: int, iters_per_wave: int, draw_seed: int, op: int,
                value_seed: int, lanes_per_line: int = 32, region_bytes: Optional[int] = None,
                stream=None) -> ReadResult:
    """Random line write (OP_WRITE) or atomic add (OP_ADD); see rr_rand_update."""
    ptr, nbytes = _region(region, region_bytes)
    res = _Result()
    _check(lib().rr_rand_update(ptr, nbytes, line_bytes, lanes_per_line, n_updates, iters_per_wave, draw_seed, op,
                                value_seed, _stream(stream), C.byref(res)))
    return ReadResult(int(res.checksum), res.kernel_ms_event, res.kernel_ms_device, int(res.waves_run),
                      int(res.launches))


@dataclass
class ChaseResult:
    final_line: int
    word_sum: int
    kernel_ms_event: float
    ns_per_hop: float


def chase(region, line_bytes: int, start: int, stride: int, mask: int, hops: int,
          region_bytes: Optional[int] = None, stream=None, cu: Optional[int] = None) -> ChaseResult:
    """Dependent-load walk by one wavefront (latency probe); see rr_chase.  With cu: on that compute unit
    (rr_chase_on_cu)."""
    ptr, nbytes = _region(region, region_bytes)
    res = _ChaseResult()
    if cu is None:
        _check(lib().rr_chase(ptr, nbytes, line_bytes, start, stride, mask, hops, _stream(stream), C.byref(res)))
    else:
        _check(lib().rr_chase_on_cu(ptr, nbytes, line_bytes, start, stride, mask, hops, cu, _stream(stream), C.byref(res)))
    return ChaseResult(int(res.final_line), int(res.word_sum), res.kernel_ms_event, res.ns_per_hop)


def groups_from_heatmap(T: np.ndarray, singles: Optional[np.ndarray] = None, min_gap: float = 0.05):
    """(group_of_cu[n], order[n], threshold) from an n x n pair-throughput matrix."""
    T = np.ascontiguousarray(T, dtype=np.float64)
    n = T.shape[0]
    if T.shape != (n, n):
        raise ValueError("T must be square")
    s_ptr = None
    if singles is not None:
        singles = np.ascontiguousarray(singles, dtype=np.float64)
        s_ptr = singles.ctypes.data_as(C.POINTER(C.c_double))
    group = np.zeros(n, dtype=np.uint16)
    order = np.zeros(n, dtype=np.uint32)
    ng = C.c_uint32(0)
    thr = C.c_double(0.0)
    rc = lib().rr_groups_from_heatmap(T.ctypes.data_as(C.POINTER(C.c_double)), n, s_ptr, min_gap,
                                      group.ctypes.data_as(C.POINTER(C.c_uint16)),
                                      order.ctypes.data_as(C.POINTER(C.c_uint32)), C.byref(ng), C.byref(thr))
    _check(rc)
    return group, order, float(thr.value)


def _zone_details(d: _ZoneProbe, n: int) -> dict:
    return {"same": d.same, "cut": d.cut, "band": d.band, "row": [d.row[b] for b in range(1, n)],
            "n_zones": int(d.n_zones), "pair_rates": int(d.pair_rates), "retakes": int(d.retakes),
            "gave_up": bool(d.gave_up), "launches": int(d.launches), "seconds": d.seconds,
            "merge_rates": int(d.merge_rates), "zones_before_merging": [int(d.before_merging[b]) for b in range(n)]}


def zones_from_pair_rates(rate, n_windows: int, min_gap: float = 0.02, max_zones: int = 16,
                          details: Optional[dict] = None):
    """zone_of_window[n_windows] by the library's rule from rates the caller supplies: rate(a, b, again) -> float
    (see rr_zones_from_pair_rates).  An exception raised by `rate` ends the call and is raised again."""
    raised = []

    def trampoline(a, b, again, _user, out):
        try:
            out[0] = float(rate(a, b, bool(again)))
            return RR_OK
        except BaseException as e:   # must not propagate through the C frames
            raised.append(e)
            return RR_EINVAL
    zone = (C.c_uint8 * max(n_windows, 1))()
    d = _ZoneProbe()
    rc = lib().rr_zones_from_pair_rates(PAIR_RATE_FN(trampoline), None, n_windows, min_gap, max_zones, zone, C.byref(d))
    if raised:
        raise raised[0]
    _check(rc)
    if details is not None:
        details.update(_zone_details(d, n_windows))
    return [int(z) for z in zone[:n_windows]]


def detect_zones(region, n_windows: int = 32, region_bytes: Optional[int] = None, stream=None,
                 details: Optional[dict] = None, min_gap: float = 0.0, max_zones: int = 0, launches: int = 0,
                 iters_per_wave: int = 0, warmup: int = 0, unroll: int = 0):
    """zone_of_window[n_windows] of the region, measured by the library (see rr_detect_zones); rates in GB/s."""
    ptr, nbytes = _region(region, region_bytes)
    o = _ZoneProbeOpts(min_gap, max_zones, launches, iters_per_wave, warmup, unroll, 0)
    zone = (C.c_uint8 * max(n_windows, 1))()
    d = _ZoneProbe()
    _check(lib().rr_detect_zones(ptr, nbytes, n_windows, C.byref(o), _stream(stream), zone, C.byref(d)))
    if details is not None:
        details.update(_zone_details(d, n_windows))
    return [int(z) for z in zone[:n_windows]]


def describe_read(region, line_bytes: int, n_reads: int, iters_per_wave: int, window_map: Optional[WindowMap] = None,
                  lanes_per_line: int = 32, region_bytes: Optional[int] = None, **launch) -> dict:
    """What rand_read would do with these arguments (see rr_describe_read); needs no device."""
    ptr, nbytes = _region(region, region_bytes)
    o, _, _ = _opts(0, 1024, **launch)
    wm = window_map._c() if window_map is not None else None
    d = _ReadPlan()
    _check(lib().rr_describe_read(ptr, nbytes, line_bytes, lanes_per_line, n_reads, iters_per_wave,
                                  C.byref(wm) if wm is not None else None, C.byref(o), C.byref(d)))
    out = {name: getattr(d, name) for name, _ in _ReadPlan._fields_}
    out["zone_windows"] = [int(x) for x in d.zone_windows][:max(d.n_zones, 0)]
    out["split_windows"] = [int(x) for x in d.split_windows]
    return out


def last_kernel() -> str:
    """Name of the read kernel this thread's last read call launched (see rr_last_kernel)."""
    return lib().rr_last_kernel().decode()


def shutdown() -> None:
    _check(lib().rr_shutdown())
