// The streaming and latency companions of the random read: fill, sequential read, plain copy and
// the dependent-load walk, with their entry points.
#include <algorithm>
#include <cstring>

#include "rr_host.hpp"
#include "rr_read_kernel.hpp"

namespace rr {

// Region as uint64[]: element j = mix64(seed + (j+1)*gamma).  Each thread writes
// 16 bytes per step (two consecutive elements), grid-stride.
typedef u64 u64x2 __attribute__((ext_vector_type(2)));
__global__ void __launch_bounds__(256) fill_kernel(u64x2 *out, u64 n_pairs, u64 seed) {
    const u64 stride = (u64)gridDim.x * blockDim.x;
    u64 i = (u64)blockIdx.x * blockDim.x + threadIdx.x;
    u64 ctr = seed + (2 * i + 1) * kGamma;  // state of element 2i
    const u64 ctr_step = 2 * stride * kGamma;
    for (; i < n_pairs; i += stride) {
        u64x2 v;
        v.x = mix64(ctr);
        v.y = mix64(ctr + kGamma);
        __builtin_nontemporal_store(v, &out[i]);  // one 16-byte store per lane
        ctr += ctr_step;
    }
}

// Streaming counterpart of the random read: every 32-bit word of the region is
// read once (the sequential reads the paper expects to be faster than random
// lines, Sec. 2.1).  Each wave owns contiguous 8 KiB chunks (eight 16-byte loads
// per lane in flight, consecutive lanes on consecutive addresses) -- measured
// 3 % faster than a plain grid-stride loop; what does not fill a chunk is read
// grid-stride.  Same checksum convention:
// wrapping 64-bit sum of zero-extended words, one atomic per wave.
__global__ void __launch_bounds__(256) seq_read_kernel(const u32x4 *src, u64 n_vec, Scratch *s, u32 block_chunks) {
    typedef const u32x4 __attribute__((address_space(1))) *gptr;
    constexpr u32 kLoads = 8;
    gptr g = (gptr)(u64)src;
    const u32 lane = threadIdx.x & 63;
    const u64 wave = ((u64)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const u64 n_chunks = n_vec / (64 * kLoads);
    const u64 t0 = clock_ticks();
    Acc acc{0u, 0u};
    if (block_chunks == 0) {
        // small regions: chunks dealt round-robin to the waves, no counters
        const u64 n_waves = ((u64)gridDim.x * blockDim.x) >> 6;
        for (u64 c = wave; c < n_chunks; c += n_waves) {
            const u64 base = c * (64 * kLoads) + lane;
            u32x4 v[kLoads];
#pragma unroll
            for (u32 k = 0; k < kLoads; ++k) v[k] = __builtin_nontemporal_load(g + base + k * 64);
#pragma unroll
            for (u32 k = 0; k < kLoads; ++k) acc.add(v[k]);
        }
    } else {
        // Large regions: blocks of block_chunks consecutive chunks are handed out in address order from one
        // counter.  However unevenly the waves advance, the device as a whole then sweeps through the region front
        // to back and reads one memory zone after the other; with the fixed round-robin assignment the slow waves
        // fall so far behind that all zones are read at once.  The blocks are large
        // because an atomic on one address takes about 12 ns.
        const u64 n_blocks = (n_chunks + block_chunks - 1) / block_chunks;
        for (;;) {
            u32 t = 0;
            if (lane == 0) t = atomicAdd(&s->tickets[0], 1u);
            const u64 b = __builtin_amdgcn_readfirstlane(t);
            if (b >= n_blocks) break;
            const u64 c_end = min((b + 1) * block_chunks, n_chunks);
            for (u64 c = b * block_chunks; c < c_end; ++c) {
                const u64 base = c * (64 * kLoads) + lane;
                u32x4 v[kLoads];
#pragma unroll
                for (u32 k = 0; k < kLoads; ++k) v[k] = __builtin_nontemporal_load(g + base + k * 64);
#pragma unroll
                for (u32 k = 0; k < kLoads; ++k) acc.add(v[k]);
            }
        }
    }
    const u64 stride = (u64)gridDim.x * blockDim.x;
    for (u64 i = n_chunks * (64 * kLoads) + (u64)blockIdx.x * blockDim.x + threadIdx.x; i < n_vec; i += stride)
        acc.add(__builtin_nontemporal_load(g + i));
    const u64 total = wave_sum(acc.value());
    const u64 t1 = clock_ticks();
    if (lane == 0) {
        Cell *c = &s->cells[wave & (kNumCells - 1)];
        atomicAdd(&c->sum, total);
        atomicMin(&c->t_min, t0);
        atomicMax(&c->t_max, t1);
        atomicAdd(&c->waves, 1u);
    }
}

// Dependent-load walk by a single wavefront; every lane follows the same chain
// (uniform address, broadcast load), lane 0 reports.
struct ChaseOut {
    u64 final_line, word_sum, ticks;
    u32 claimed;  // pinned walk: set by the wavefront that does the walk
    u32 ran_key;  // ... and the key of the compute unit it ran on
};
__device__ __forceinline__ void walk(const char *region, const Reducer &red, u32 log2_line, u64 start, u64 stride,
                                     u32 mask, u64 hops, ChaseOut *out) {
    typedef const u32 __attribute__((address_space(1))) *gptr;
    u64 line = start, sum = 0;
    const u64 t0 = clock_ticks();
    for (u64 k = 0; k < hops; ++k) {
        const u32 word = *(gptr)((u64)region + (line << log2_line));
        sum += word;
        const u32 salt = (u32)k * 0x9E3779B9u;  // hop-dependent, so the walk cannot close into a short cycle
        line = reduce_to_line(line + stride + (u64)((word ^ salt) & mask), red);
    }
    const u64 t1 = clock_ticks();
    if (threadIdx.x == 0) {
        out->final_line = line;
        out->word_sum = sum;
        out->ticks = t1 - t0;
    }
}
__global__ void __launch_bounds__(64) chase_kernel(const char *region, Reducer red, u32 log2_line, u64 start,
                                                   u64 stride, u32 mask, u64 hops, ChaseOut *out) {
    walk(region, red, log2_line, start, stride, mask, hops, out);
}
// The same walk on a chosen compute unit (the pinning of the paper's two-SM probe, Sec. 2.2): many one-wave
// workgroups are launched, those that land elsewhere leave at once, and of those on the target the first to
// claim the walk does it.
__global__ void __launch_bounds__(64) chase_pinned_kernel(const char *region, Reducer red, u32 log2_line, u64 start,
                                                          u64 stride, u32 mask, u64 hops, ChaseOut *out, u32 target_key) {
    const u32 key = cu_key();
    if (key != target_key) return;
    u32 won = 0;
    if (threadIdx.x == 0) won = atomicCAS(&out->claimed, 0u, 1u) == 0u ? 1u : 0u;
    if (!__builtin_amdgcn_readfirstlane(won)) return;
    if (threadIdx.x == 0) out->ran_key = key;
    walk(region, red, log2_line, start, stride, mask, hops, out);
}

// Plain copy, 16 bytes per lane and step, grid-stride: a kernel of exactly known
// HBM traffic (bytes read = bytes written = n_vec * 16).
__global__ void __launch_bounds__(256) copy_kernel(u32x4 *dst, const u32x4 *src, u64 n_vec) {
    const u64 stride = (u64)gridDim.x * blockDim.x;
    for (u64 i = (u64)blockIdx.x * blockDim.x + threadIdx.x; i < n_vec; i += stride)
        __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

}  // namespace rr

using namespace rr;

extern "C" int rr_fill(void *region, uint64_t region_bytes, uint64_t fill_seed, void *hip_stream) {
    if (!region) return fail(RR_EINVAL, "region is NULL");
    if ((uintptr_t)region % 16 != 0) return fail(RR_EINVAL, "region is not 16-byte aligned");
    if (region_bytes % 16 != 0) return fail(RR_EINVAL, "region_bytes must be a multiple of 16");
    if (region_bytes == 0) return RR_OK;
    hipStream_t stream = (hipStream_t)hip_stream;
    int dev = 0, n_cu = 0;
    HIP_TRY(hipGetDevice(&dev));
    HIP_TRY(hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev));
    const u64 n_pairs = region_bytes / 16;
    u64 blocks = (n_pairs + 255) / 256;
    const u64 cap = (u64)n_cu * 32;  // grid-stride beyond this; stores want many waves (256 GiB: 7.1 TB/s, with 8 per CU 6.8)
    if (blocks > cap) blocks = cap;
    hipLaunchKernelGGL(fill_kernel, dim3((u32)blocks), dim3(256), 0, stream, (u64x2 *)region, n_pairs,
                       (u64)fill_seed);
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipStreamSynchronize(stream));
    return RR_OK;
}

extern "C" int rr_seq_read(const void *region, uint64_t region_bytes, void *hip_stream, rr_result_t *out) {
    if (!out) return fail(RR_EINVAL, "out is NULL");
    if (!region) return fail(RR_EINVAL, "region is NULL");
    if ((uintptr_t)region % 16 != 0) return fail(RR_EINVAL, "region is not 16-byte aligned");
    if (region_bytes % 16 != 0) return fail(RR_EINVAL, "region_bytes must be a multiple of 16");
    rr_result_t res;
    memset(&res, 0, sizeof res);
    if (region_bytes == 0) {
        *out = res;
        return RR_OK;
    }
    hipStream_t stream = (hipStream_t)hip_stream;
    std::lock_guard<std::mutex> lock(g_mutex);
    DeviceState *st = nullptr;
    int rc = get_state(stream, &st);
    if (rc != RR_OK) return rc;
    const u64 n_vec = region_bytes / 16;
    u64 blocks = (n_vec + 255) / 256;
    // One workgroup per compute unit, each wave looping over its chunks with 8 KiB in flight: 32 KB per CU, as for
    // the random reads, is what reads fastest (64 GiB: 7.26 TB/s; with 4 workgroups per CU 7.03, with 16 7.05).
    const u64 cap = st->n_cus;
    if (blocks > cap) blocks = cap;
    // Regions that may span several memory zones (more than 96 GiB) are swept front to back in blocks of 2 MiB
    // from one counter, so that the device reads one zone after the other: 7.19 / 7.16 TB/s over 128 / 256 GiB.  Inside
    // one zone the static assignment is used (7.40 / 7.37 TB/s at 16 / 64 GiB: no claims, no imbalance from the
    // coarse blocks).
    const u32 block_chunks = region_bytes > (96ull << 30) ? 256u : 0u;
    rc = begin_cells(*st, stream);
    if (rc != RR_OK) return rc;
    if (block_chunks) {
        rc = launch_reset(*st, 2u, stream);
        if (rc != RR_OK) return rc;
    }
    HIP_TRY(hipEventRecord(st->ev0, stream));
    hipLaunchKernelGGL(seq_read_kernel, dim3((u32)blocks), dim3(256), 0, stream, (const u32x4 *)region, n_vec,
                       st->scratch, block_chunks);
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipEventRecord(st->ev1, stream));
    rc = finish_and_wait(*st, 0u, 1u, 0u, stream);
    if (rc != RR_OK) return rc;
    float ms = 0.f;
    HIP_TRY(hipEventElapsedTime(&ms, st->ev0, st->ev1));
    res.checksum = st->head->checksum;
    res.kernel_ms_event = ms;
    res.kernel_ms_device = (double)(st->head->t_max - st->head->t_min) / (double)st->wall_khz;
    res.waves_run = st->head->waves_run;
    res.launches = 1;
    *out = res;
    return RR_OK;
}

namespace {
// cu: dense id of the compute unit that is to do the walk, or kAnyCu
constexpr u32 kAnyCu = 0xFFFFFFFFu;
int chase_impl(const void *region, uint64_t region_bytes, uint32_t line_bytes, uint64_t start, uint64_t stride,
               uint32_t mask, uint64_t hops, u32 cu, void *hip_stream, rr_chase_result_t *out) {
    if (!out) return fail(RR_EINVAL, "out is NULL");
    if (!region) return fail(RR_EINVAL, "region is NULL");
    if (line_bytes != 128 && line_bytes != 256 && line_bytes != 512)
        return fail(RR_EINVAL, "line_bytes must be 128, 256 or 512 (got %u)", line_bytes);
    if (region_bytes == 0 || region_bytes % line_bytes != 0)
        return fail(RR_EINVAL, "region_bytes must be a positive multiple of line_bytes");
    if ((uintptr_t)region % line_bytes != 0) return fail(RR_EINVAL, "region is not aligned to line_bytes");
    const u64 n_lines = region_bytes / line_bytes;
    if (n_lines > (1ull << 32)) return fail(RR_EINVAL, "region has more than 2^32 lines");
    if (start >= n_lines) return fail(RR_EINVAL, "start must be below the number of lines");
    if (hops == 0) return fail(RR_EINVAL, "hops must be at least 1");
    hipStream_t stream = (hipStream_t)hip_stream;
    std::lock_guard<std::mutex> lock(g_mutex);
    DeviceState *st = nullptr;
    int rc = get_state(stream, &st);
    if (rc != RR_OK) return rc;
    if (cu != kAnyCu && cu >= st->n_cus) return fail(RR_EINVAL, "compute unit id %u is not below %u", cu, st->n_cus);
    // the walk's result words go through the (otherwise idle) key-mark area of the scratch
    ChaseOut *dev_out = (ChaseOut *)st->scratch->key_seen;
    const u32 log2_line = line_bytes == 128 ? 7 : line_bytes == 256 ? 8 : 9;
    ChaseOut host;
    float ms = 0.f;
    if (cu == kAnyCu) {
        HIP_TRY(hipEventRecord(st->ev0, stream));
        hipLaunchKernelGGL(chase_kernel, dim3(1), dim3(64), 0, stream, (const char *)region, make_reducer(n_lines),
                           log2_line, (u64)start, (u64)(stride % n_lines), mask, (u64)hops, dev_out);
        HIP_TRY(hipGetLastError());
        HIP_TRY(hipEventRecord(st->ev1, stream));
        HIP_TRY(hipMemcpyAsync(&host, dev_out, sizeof host, hipMemcpyDeviceToHost, stream));
        HIP_TRY(hipStreamSynchronize(stream));
    } else {
        // 64 one-wave workgroups per wave slot of the device, as the pinned read launches: most leave at once
        const u32 target_key = key_of(st->cus[cu]);
        const u32 grid = st->n_cus * 32u * 64u;
        for (int launch = 0;; ++launch) {
            rc = launch_reset(*st, 8u, stream);  // clears the key-mark area, the claim flag with it
            if (rc != RR_OK) return rc;
            HIP_TRY(hipEventRecord(st->ev0, stream));
            hipLaunchKernelGGL(chase_pinned_kernel, dim3(grid), dim3(64), 0, stream, (const char *)region,
                               make_reducer(n_lines), log2_line, (u64)start, (u64)(stride % n_lines), mask, (u64)hops,
                               dev_out, target_key);
            HIP_TRY(hipGetLastError());
            HIP_TRY(hipEventRecord(st->ev1, stream));
            HIP_TRY(hipMemcpyAsync(&host, dev_out, sizeof host, hipMemcpyDeviceToHost, stream));
            HIP_TRY(hipStreamSynchronize(stream));
            if (host.claimed) break;
            if (launch + 1 >= 8)
                return fail(RR_EPLACE, "in 8 launches no workgroup landed on compute unit %u", cu);
        }
        if (host.ran_key != target_key)
            return fail(RR_EPLACE, "the walk ran on the compute unit with key %#x, not on %#x", host.ran_key, target_key);
    }
    HIP_TRY(hipEventElapsedTime(&ms, st->ev0, st->ev1));
    out->final_line = host.final_line;
    out->word_sum = host.word_sum;
    out->kernel_ms_event = ms;
    out->ns_per_hop = (double)host.ticks * 1e6 / (double)st->wall_khz / (double)hops;
    return RR_OK;
}
}  // namespace

extern "C" int rr_chase(const void *region, uint64_t region_bytes, uint32_t line_bytes, uint64_t start,
                        uint64_t stride, uint32_t mask, uint64_t hops, void *hip_stream, rr_chase_result_t *out) {
    return chase_impl(region, region_bytes, line_bytes, start, stride, mask, hops, kAnyCu, hip_stream, out);
}

extern "C" int rr_chase_on_cu(const void *region, uint64_t region_bytes, uint32_t line_bytes, uint64_t start,
                              uint64_t stride, uint32_t mask, uint64_t hops, uint32_t cu, void *hip_stream,
                              rr_chase_result_t *out) {
    if (cu >= RR_MAX_CUS) return fail(RR_EINVAL, "compute unit id %u is out of range", cu);
    return chase_impl(region, region_bytes, line_bytes, start, stride, mask, hops, cu, hip_stream, out);
}

extern "C" int rr_copy(void *dst, const void *src, uint64_t bytes, void *hip_stream, double *kernel_ms) {
    if (!dst || !src) return fail(RR_EINVAL, "dst or src is NULL");
    if ((uintptr_t)dst % 16 != 0 || (uintptr_t)src % 16 != 0 || bytes % 16 != 0)
        return fail(RR_EINVAL, "dst, src and bytes must be multiples of 16");
    const uintptr_t d = (uintptr_t)dst, c = (uintptr_t)src;
    if (d < c + bytes && c < d + bytes && bytes > 0) return fail(RR_EINVAL, "dst and src overlap");
    if (bytes == 0) {
        if (kernel_ms) *kernel_ms = 0.0;
        return RR_OK;
    }
    hipStream_t stream = (hipStream_t)hip_stream;
    std::lock_guard<std::mutex> lock(g_mutex);
    DeviceState *st = nullptr;
    int rc = get_state(stream, &st);
    if (rc != RR_OK) return rc;
    const u64 n_vec = bytes / 16;
    u64 blocks = (n_vec + 255) / 256;
    const u64 cap = (u64)st->n_cus * 3;  // measured best (2-4 per CU within 5 %; 8 and more 10-15 % slower)
    if (blocks > cap) blocks = cap;
    HIP_TRY(hipEventRecord(st->ev0, stream));
    hipLaunchKernelGGL(copy_kernel, dim3((u32)blocks), dim3(256), 0, stream, (u32x4 *)dst, (const u32x4 *)src, n_vec);
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipEventRecord(st->ev1, stream));
    HIP_TRY(hipStreamSynchronize(stream));
    float ms = 0.f;
    HIP_TRY(hipEventElapsedTime(&ms, st->ev0, st->ev1));
    if (kernel_ms) *kernel_ms = ms;
    return RR_OK;
}
