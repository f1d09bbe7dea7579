// Host side of the C ABI declared in include/randline.h, plus the small
// kernels (fill, CU enumeration, scratch reset).  The read kernel itself is in
// rr_read_kernel.hpp and is instantiated in the rr_inst_*.hip files.
#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <map>
#include <mutex>
#include <string>
#include <vector>

#include "../../include/randline.h"
#include "rr_phased_kernel.hpp"
#include "rr_update_kernel.hpp"

namespace rr {

// ------------------------------------------------------------------ small kernels

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

// Marks the key of the CU each workgroup runs on; a short sleep keeps the
// workgroup resident so that the dispatcher has to use the other CUs too.
__global__ void __launch_bounds__(64) enumerate_kernel(Scratch *s, u32 naps) {
    if (threadIdx.x == 0) s->key_seen[cu_key()] = 1u;
    for (u32 i = 0; i < naps; ++i) __builtin_amdgcn_s_sleep(100);
}

// Streaming counterpart of the random read: every 32-bit word of the region is
// read once (the sequential reads the paper expects to be faster than random
// lines, Sec. 2.1).  Each wave owns contiguous 8 KiB chunks (eight 16-byte loads
// per lane in flight, consecutive lanes on consecutive addresses), chunks dealt
// round-robin to the waves -- measured 3 % faster than a plain grid-stride loop;
// what does not fill a chunk is read grid-stride.  Same checksum convention:
// wrapping 64-bit sum of zero-extended words, one atomic per wave.
__global__ void __launch_bounds__(256) seq_read_kernel(const u32x4 *src, u64 n_vec, Scratch *s) {
    typedef const u32x4 __attribute__((address_space(1))) *gptr;
    constexpr u32 kLoads = 8;
    gptr g = (gptr)(u64)src;
    const u32 lane = threadIdx.x & 63;
    const u64 wave = ((u64)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const u64 n_waves = ((u64)gridDim.x * blockDim.x) >> 6;
    const u64 n_chunks = n_vec / (64 * kLoads);
    const u64 t0 = clock_ticks();
    Acc acc{0u, 0u};
    for (u64 c = wave; c < n_chunks; c += n_waves) {
        const u64 base = c * (64 * kLoads) + lane;
        u32x4 v[kLoads];
#pragma unroll
        for (u32 k = 0; k < kLoads; ++k) v[k] = __builtin_nontemporal_load(g + base + k * 64);
#pragma unroll
        for (u32 k = 0; k < kLoads; ++k) acc.add(v[k]);
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
};
__global__ void __launch_bounds__(64) chase_kernel(const char *region, Reducer red, u32 log2_line, u64 start,
                                                   u64 stride, u32 mask, u64 hops, ChaseOut *out) {
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

// Plain copy, 16 bytes per lane and step, grid-stride: a kernel of exactly known
// HBM traffic (bytes read = bytes written = n_vec * 16).
__global__ void __launch_bounds__(256) copy_kernel(u32x4 *dst, const u32x4 *src, u64 n_vec) {
    const u64 stride = (u64)gridDim.x * blockDim.x;
    for (u64 i = (u64)blockIdx.x * blockDim.x + threadIdx.x; i < n_vec; i += stride)
        __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

// what: bit 0 result cells; bit 1 ticket counters; bit 2 per-CU wave counts; bit 3 key marks
__global__ void __launch_bounds__(256) reset_kernel(Scratch *s, u32 what) {
    const u32 t = threadIdx.x;
    if (what & 1u) {
        for (u32 i = t; i < kNumCells; i += blockDim.x) {
            s->cells[i].sum = 0;
            s->cells[i].t_min = ~0ull;
            s->cells[i].t_max = 0;
            s->cells[i].waves = 0;
        }
    }
    if (what & 2u)
        for (u32 i = t; i < kMaxCus; i += blockDim.x) s->tickets[i * kTicketStride] = 0;
    if (what & 4u)
        for (u32 i = t; i < kMaxCus; i += blockDim.x) s->cu_waves[i] = 0;
    if (what & 8u)
        for (u32 i = t; i < kNumKeys; i += blockDim.x) s->key_seen[i] = 0;
}

// After a read launch (one block of kNumCells threads, one result cell each):
// fold the cells into the result head (pinned host memory mapped into the
// device, so no copy follows), leave them cleared for the next launch, and count
// the compute units whose share of tickets has not been fully claimed.
__global__ void __launch_bounds__(kNumCells) finish_kernel(Scratch *s, ResultHead *head, const Tables *tb,
                                                           u32 n_cus, u32 cpw, u32 ticket_mode) {
    __shared__ u64 sh_sum[kNumCells], sh_min[kNumCells], sh_max[kNumCells];
    __shared__ u32 sh_waves[kNumCells], sh_open[kNumCells];
    const u32 t = threadIdx.x;
    Cell *c = &s->cells[t];
    sh_sum[t] = c->sum;
    sh_min[t] = c->t_min;
    sh_max[t] = c->t_max;
    sh_waves[t] = c->waves;
    c->sum = 0;
    c->t_min = ~0ull;
    c->t_max = 0;
    c->waves = 0;
    u32 open = 0;
    if (ticket_mode && t < n_cus && s->tickets[t * kTicketStride] < tb->cu_unit_count[t] * cpw) open = 1;
    sh_open[t] = open;
    __syncthreads();
    for (u32 step = kNumCells / 2; step > 0; step >>= 1) {
        if (t < step) {
            sh_sum[t] += sh_sum[t + step];
            sh_min[t] = sh_min[t + step] < sh_min[t] ? sh_min[t + step] : sh_min[t];
            sh_max[t] = sh_max[t + step] > sh_max[t] ? sh_max[t + step] : sh_max[t];
            sh_waves[t] += sh_waves[t + step];
            sh_open[t] += sh_open[t + step];
        }
        __syncthreads();
    }
    if (t == 0) {
        head->checksum = sh_sum[0];
        head->t_min = sh_min[0];
        head->t_max = sh_max[0];
        head->waves_run = sh_waves[0];
        head->unfinished = sh_open[0];
    }
}
static_assert(kMaxCus <= kNumCells, "finish_kernel checks one compute unit per thread");

}  // namespace rr

using namespace rr;

// ------------------------------------------------------------------ errors

static thread_local std::string g_last_error;

static int fail(int code, const char *fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_last_error = buf;
    return code;
}

#define HIP_TRY(expr)                                                                          \
    do {                                                                                       \
        hipError_t e_ = (expr);                                                                \
        if (e_ != hipSuccess)                                                                  \
            return fail(RR_EHIP, "%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_), __FILE__, \
                        __LINE__);                                                             \
    } while (0)

extern "C" const char *rr_strerror(int code) {
    switch (code) {
        case RR_OK: return "success";
        case RR_EINVAL: return "invalid argument";
        case RR_EHIP: return "HIP runtime error";
        case RR_EPLACE: return "a group or target compute unit received no resident wave";
        default: return "unknown error code";
    }
}

extern "C" const char *rr_last_error(void) { return g_last_error.c_str(); }

// ------------------------------------------------------------------ per-device state

namespace {


struct DeviceState {
    bool ready = false;
    Scratch *scratch = nullptr;
    Tables *tables = nullptr;       // device
    Tables *tables_host = nullptr;  // pinned staging copy
    Tables *tables_last = nullptr;  // what the device copy holds (plain host memory), to skip equal uploads
    bool tables_valid = false;
    bool cells_clean = false;       // result cells are in their cleared state
    u16 *placement = nullptr;
    size_t placement_cap = 0;
    ResultHead *head = nullptr;      // pinned host memory, mapped ...
    ResultHead *head_dev = nullptr;  // ... and its address as the device sees it
    u32 *cu_waves_host = nullptr;    // pinned staging for the per-CU wave counts
    bool flat_tables_ready = false;  // the device tables are those of a call without a window map
    hipEvent_t ev0 = nullptr, ev1 = nullptr;
    int wall_khz = 0;
    std::vector<rr_cu_t> cus;             // dense id -> coordinates
    std::vector<u16> dense_of_key_host;   // [kNumKeys], kExcluded if no such CU
};

constexpr int kMaxDevices = 16;
DeviceState g_state[kMaxDevices];
std::mutex g_mutex;

u32 key_of(const rr_cu_t &c) { return (c.xcc << 8) | (c.se << 5) | (c.sh << 4) | c.cu; }

int enumerate(DeviceState &st, hipStream_t stream) {
    int dev = 0, n_expected = 0;
    HIP_TRY(hipGetDevice(&dev));
    HIP_TRY(hipDeviceGetAttribute(&n_expected, hipDeviceAttributeMultiprocessorCount, dev));
    std::vector<u32> seen(kNumKeys);
    u32 found = 0;
    for (int attempt = 0; attempt < 4 && (int)found < n_expected; ++attempt) {
        hipLaunchKernelGGL(reset_kernel, dim3(1), dim3(256), 0, stream, st.scratch, 8u);
        HIP_TRY(hipGetLastError());
        const u32 blocks = (u32)n_expected * 64u << attempt;
        hipLaunchKernelGGL(enumerate_kernel, dim3(blocks), dim3(64), 0, stream, st.scratch, 4u << attempt);
        HIP_TRY(hipGetLastError());
        HIP_TRY(hipMemcpyAsync(seen.data(), st.scratch->key_seen, kNumKeys * sizeof(u32),
                               hipMemcpyDeviceToHost, stream));
        HIP_TRY(hipStreamSynchronize(stream));
        found = 0;
        for (u32 k = 0; k < kNumKeys; ++k) found += seen[k] ? 1u : 0u;
    }
    if (found == 0 || found > kMaxCus)
        return fail(RR_EPLACE, "CU enumeration found %u compute units (device reports %d)", found, n_expected);
    if ((int)found != n_expected)
        return fail(RR_EPLACE, "CU enumeration found %u of %d compute units", found, n_expected);
    st.cus.clear();
    st.dense_of_key_host.assign(kNumKeys, kExcluded);
    for (u32 k = 0; k < kNumKeys; ++k) {  // ascending key == sorted (xcc, se, sh, cu)
        if (!seen[k]) continue;
        rr_cu_t c;
        c.xcc = k >> 8;
        c.se = (k >> 5) & 7u;
        c.sh = (k >> 4) & 1u;
        c.cu = k & 15u;
        st.dense_of_key_host[k] = (u16)st.cus.size();
        st.cus.push_back(c);
    }
    return RR_OK;
}

// Create (once per device) the scratch, tables, events and the CU list.
int get_state(hipStream_t stream, DeviceState **out) {
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(RR_EHIP, "device index %d not supported", dev);
    DeviceState &st = g_state[dev];
    if (!st.ready) {
        if (!st.scratch) HIP_TRY(hipMalloc((void **)&st.scratch, sizeof(Scratch)));
        if (!st.tables) HIP_TRY(hipMalloc((void **)&st.tables, sizeof(Tables)));
        if (!st.tables_host) HIP_TRY(hipHostMalloc((void **)&st.tables_host, sizeof(Tables), hipHostMallocDefault));
        if (!st.tables_last) st.tables_last = new Tables;
        if (!st.head) {
            HIP_TRY(hipHostMalloc((void **)&st.head, sizeof(ResultHead), hipHostMallocMapped));
            HIP_TRY(hipHostGetDevicePointer((void **)&st.head_dev, st.head, 0));
        }
        if (!st.cu_waves_host) HIP_TRY(hipHostMalloc((void **)&st.cu_waves_host, kMaxCus * sizeof(u32), hipHostMallocDefault));
        if (!st.ev0) HIP_TRY(hipEventCreate(&st.ev0));
        if (!st.ev1) HIP_TRY(hipEventCreate(&st.ev1));
        HIP_TRY(hipDeviceGetAttribute(&st.wall_khz, hipDeviceAttributeWallClockRate, dev));
        if (st.wall_khz <= 0) st.wall_khz = 100000;  // s_memrealtime: 100 MHz
        int rc = enumerate(st, stream);
        if (rc != RR_OK) return rc;
        st.ready = true;
    }
    *out = &st;
    return RR_OK;
}

struct Family {
    u32 lanes, wdw;
    kernel_handle (*find)(u32, u32, u32);
    u32 default_unroll;
};
const Family kFamilies[] = {
    // default ring depth: the deepest one built (measured best for every shape, by 1-3 %)
    {32, 1, find_read_kernel_32_1, 16}, {32, 2, find_read_kernel_32_2, 16}, {32, 4, find_read_kernel_32_4, 8},
    {64, 1, find_read_kernel_64_1, 16}, {64, 2, find_read_kernel_64_2, 16},
};

const Family *find_family(u32 lanes, u32 wdw) {
    for (const Family &f : kFamilies)
        if (f.lanes == lanes && f.wdw == wdw) return &f;
    return nullptr;
}

// Validated description of one read call.
struct Plan {
    u64 n_lines = 0, W = 0, first_wave = 0;
    u32 log2_line = 0, lanes = 0, wdw = 0, G = 1, n_windows = 1;
    u32 block = 256, unroll = 0, bcast = RR_BCAST_DPP, nt = 1, mode = RR_MODE_AUTO, grid_blocks = 0;
    u32 chunk_iters = 0;
    u32 n_zones = 0;     // > 0: zone-phased kernel
    u32 zone_shift = 0;
    u64 zone_mask[16] = {};
    bool pinned = false;
    const Family *family = nullptr;
    kernel_handle kernel = nullptr;
};

// Device-independent checks (everything that can be rejected without HIP).
int make_plan(const void *region, uint64_t region_bytes, uint32_t line_bytes, uint32_t lanes,
              uint64_t n_reads, uint32_t iters, const rr_window_map_t *wm,
              const rr_launch_opts_t *opts, const void *out, Plan &pl) {
    if (!out) return fail(RR_EINVAL, "out is NULL");
    if (!region) return fail(RR_EINVAL, "region is NULL");
    if (line_bytes != 128 && line_bytes != 256 && line_bytes != 512)
        return fail(RR_EINVAL, "line_bytes must be 128, 256 or 512 (got %u)", line_bytes);
    if (lanes != 32 && lanes != 64) return fail(RR_EINVAL, "lanes_per_line must be 32 or 64 (got %u)", lanes);
    const u32 width = line_bytes / lanes;
    if (width * lanes != line_bytes || (width != 4 && width != 8 && width != 16))
        return fail(RR_EINVAL, "line_bytes/lanes_per_line must be 4, 8 or 16 bytes (got %u/%u)", line_bytes, lanes);
    pl.lanes = lanes;
    pl.wdw = width / 4;
    pl.family = find_family(pl.lanes, pl.wdw);
    if (!pl.family) return fail(RR_EINVAL, "%u lanes x %u bytes is not a supported line shape", lanes, width);
    if (region_bytes == 0 || region_bytes % line_bytes != 0)
        return fail(RR_EINVAL, "region_bytes must be a positive multiple of line_bytes");
    if ((uintptr_t)region % line_bytes != 0) return fail(RR_EINVAL, "region is not aligned to line_bytes");
    pl.n_lines = region_bytes / line_bytes;
    if (pl.n_lines > (1ull << 32)) return fail(RR_EINVAL, "region has more than 2^32 lines");
    pl.log2_line = line_bytes == 128 ? 7 : line_bytes == 256 ? 8 : 9;
    if (iters == 0) return fail(RR_EINVAL, "iters_per_wave must be at least 1");
    if (n_reads % iters != 0) return fail(RR_EINVAL, "n_reads must be a multiple of iters_per_wave");
    pl.W = n_reads / iters;
    if (wm) {
        if (wm->n_groups == 0 || wm->n_groups > RR_MAX_GROUPS)
            return fail(RR_EINVAL, "n_groups must be in [1, %u]", RR_MAX_GROUPS);
        if (wm->n_windows == 0 || pl.n_lines % wm->n_windows != 0)
            return fail(RR_EINVAL, "n_windows must be positive and divide the number of lines");
        if (!wm->group_of_cu || !wm->window_of_group) return fail(RR_EINVAL, "window map arrays are NULL");
        if (wm->n_cus == 0 || wm->n_cus > RR_MAX_CUS) return fail(RR_EINVAL, "window map n_cus out of range");
        for (u32 c = 0; c < wm->n_cus; ++c)
            if (wm->group_of_cu[c] != RR_CU_EXCLUDED && wm->group_of_cu[c] >= wm->n_groups)
                return fail(RR_EINVAL, "group_of_cu[%u] = %u is not below n_groups", c, wm->group_of_cu[c]);
        for (u32 g = 0; g < wm->n_groups; ++g)
            if (wm->window_of_group[g] >= wm->n_windows)
                return fail(RR_EINVAL, "window_of_group[%u] = %u is not below n_windows", g, wm->window_of_group[g]);
        if (pl.W % wm->n_groups != 0) return fail(RR_EINVAL, "the number of logical waves must be a multiple of n_groups");
        pl.G = wm->n_groups;
        pl.n_windows = wm->n_windows;
    }
    if (pl.W / pl.G >= (1ull << 31)) return fail(RR_EINVAL, "too many logical waves per group");
    pl.unroll = pl.family->default_unroll;
    if (opts) {
        if (opts->block_threads) {
            if (opts->block_threads != 64 && opts->block_threads != 128 && opts->block_threads != 256)
                return fail(RR_EINVAL, "block_threads must be 64, 128 or 256");
            pl.block = opts->block_threads;
        }
        if (opts->unroll) pl.unroll = opts->unroll;
        if (opts->bcast > RR_BCAST_READLANE) return fail(RR_EINVAL, "unknown bcast value");
        if (opts->bcast) pl.bcast = opts->bcast;
        if (opts->nontemporal > RR_NT_OFF) return fail(RR_EINVAL, "nontemporal must be 0, 1 or 2");
        if (opts->nontemporal) pl.nt = opts->nontemporal == RR_NT_ON ? 1u : 0u;
        if (opts->mode > RR_MODE_TICKET) return fail(RR_EINVAL, "unknown mode value");
        pl.mode = opts->mode;
        pl.grid_blocks = opts->grid_blocks;
        if (opts->chunk_iters % 64 != 0) return fail(RR_EINVAL, "chunk_iters must be a multiple of 64");
        if (opts->reserved != 0) return fail(RR_EINVAL, "reserved must be 0");
        pl.chunk_iters = opts->chunk_iters;
        if (opts->first_wave % pl.G != 0) return fail(RR_EINVAL, "first_wave must be a multiple of n_groups");
        pl.first_wave = opts->first_wave;
        const bool zoned = opts->zone_bytes || opts->zone_of_window;
        if (opts->reserved2 != 0) return fail(RR_EINVAL, "reserved2 must be 0");
        if (opts->phase_ticks && (!zoned || opts->mode != RR_MODE_FLAT))
            return fail(RR_EINVAL, "phase_ticks needs zones and a flat launch");
        if (zoned) {
            if (opts->zone_bytes && opts->zone_of_window)
                return fail(RR_EINVAL, "give either zone_bytes or zone_of_window, not both");
            if (wm) return fail(RR_EINVAL, "zone-phased reads cannot be combined with a window map");
            if (opts->chunk_iters) return fail(RR_EINVAL, "zone-phased reads do not take chunk_iters");
            if (opts->placement_out || opts->cu_waves_out)
                return fail(RR_EINVAL, "zone-phased reads do not record placement");
            u64 window_lines;  // a power of two; the region has at most 64 such windows
            if (opts->zone_bytes) {
                if (opts->zone_bytes % line_bytes != 0) return fail(RR_EINVAL, "zone_bytes must be a multiple of line_bytes");
                const u64 zone_lines = opts->zone_bytes / line_bytes;
                const u64 nz = (pl.n_lines + zone_lines - 1) / zone_lines;
                if (nz > 16) return fail(RR_EINVAL, "zone_bytes gives %llu zones; at most 16 are supported", nz);
                window_lines = zone_lines & (~zone_lines + 1);  // largest power of two dividing the zone
                const u64 n_win = (pl.n_lines + window_lines - 1) / window_lines;
                if (n_win > 64) return fail(RR_EINVAL, "zone_bytes would need %llu windows; at most 64 are supported", n_win);
                pl.n_zones = (u32)nz;
                for (u64 v = 0; v < n_win; ++v) pl.zone_mask[v * window_lines / zone_lines] |= 1ull << v;
            } else {
                const u32 n_win = opts->n_zone_windows;
                if (n_win == 0 || n_win > 64) return fail(RR_EINVAL, "n_zone_windows must be in [1, 64]");
                if (pl.n_lines % n_win != 0) return fail(RR_EINVAL, "n_zone_windows must divide the number of lines");
                window_lines = pl.n_lines / n_win;
                if (window_lines & (window_lines - 1))
                    return fail(RR_EINVAL, "a zone window must hold a power-of-two number of lines");
                for (u32 v = 0; v < n_win; ++v) {
                    const u32 z = opts->zone_of_window[v];
                    if (z >= 16) return fail(RR_EINVAL, "zone_of_window[%u] = %u is not below 16", v, z);
                    pl.zone_mask[z] |= 1ull << v;
                    if (z + 1 > pl.n_zones) pl.n_zones = z + 1;
                }
            }
            while ((1ull << pl.zone_shift) < window_lines) pl.zone_shift++;
        }
    }
    pl.kernel = pl.family->find(pl.unroll, pl.bcast, pl.nt);
    if (!pl.kernel) return fail(RR_EINVAL, "unroll %u is not built for this line shape", pl.unroll);
    if (pl.n_zones) {
        pl.kernel = find_phased_kernel(pl.lanes, pl.wdw, pl.nt);
        if (!pl.kernel) return fail(RR_EINVAL, "no zone-phased kernel for this line shape");
        pl.block = 256;  // its LDS lists are laid out for four waves per workgroup
    }
    bool needs_tickets = false;
    if (wm) {
        if (wm->n_groups > 1) needs_tickets = true;
        for (u32 c = 0; c < wm->n_cus; ++c)
            if (wm->group_of_cu[c] == RR_CU_EXCLUDED) {
                needs_tickets = true;
                pl.pinned = true;  // most workgroups will land on idle CUs and leave: launch many more
            }
    }
    if (pl.mode == RR_MODE_FLAT && needs_tickets)
        return fail(RR_EINVAL, "flat mode cannot honour a window map with several groups or excluded CUs");
    // zone-phased reads line their phases up only when the work is handed out zone-major by tickets
    if (pl.mode == RR_MODE_AUTO) pl.mode = (needs_tickets || pl.n_zones) ? RR_MODE_TICKET : RR_MODE_FLAT;
    return RR_OK;
}

Reducer make_reducer(u64 L) {
    Reducer r;
    r.L = L;
    r.pow2 = (L & (L - 1)) == 0 ? 1u : 0u;
    r.M = r.pow2 ? 0 : (~0ull) / L;  // floor((2^64-1)/L) == floor(2^64/L) when L is not a power of two
    return r;
}

// Lookup tables of one call: CU key -> group and dense id, group -> window, group -> its CUs, and each
// CU's share of its group's units.  Built in the pinned staging copy and uploaded only if they differ
// from what the device already holds.
int prepare_tables(DeviceState &st, const Plan &pl, const rr_window_map_t *wm, u64 units, u64 L_win,
                   hipStream_t stream) {
    const u32 n_cus = (u32)st.cus.size();
    Tables &tb = *st.tables_host;
    memset(&tb, 0, sizeof tb);
    for (u32 k = 0; k < kNumKeys; ++k) {
        tb.group_of_key[k] = kExcluded;
        tb.dense_of_key[k] = st.dense_of_key_host[k];
    }
    std::vector<u32> cus_in_group(pl.G, 0);
    for (u32 c = 0; c < n_cus; ++c) {
        const u16 g = wm ? wm->group_of_cu[c] : 0;
        tb.group_of_key[key_of(st.cus[c])] = g;
        if (g != kExcluded) cus_in_group[g]++;
    }
    for (u32 g = 0; g < pl.G; ++g) {
        if (cus_in_group[g] == 0) return fail(RR_EPLACE, "group %u has no compute unit", g);
        tb.window_base[g] = wm ? (u32)(wm->window_of_group[g] * L_win) : 0u;
        tb.group_begin[g + 1] = tb.group_begin[g] + cus_in_group[g];
    }
    std::vector<u32> fill_pos(pl.G, 0);
    for (u32 c = 0; c < n_cus; ++c) {  // ascending dense id within each group
        const u16 g = wm ? wm->group_of_cu[c] : 0;
        if (g == kExcluded) continue;
        const u32 k = fill_pos[g]++, n = cus_in_group[g];
        tb.group_cus[tb.group_begin[g] + k] = (u16)c;
        tb.cu_pos[c] = (u16)k;
        const u64 b0 = units * k / n, b1 = units * (k + 1) / n;  // even split of the group's units
        tb.cu_unit_begin[c] = (u32)b0;
        tb.cu_unit_count[c] = (u32)(b1 - b0);
    }
    if (!st.tables_valid || memcmp(st.tables_last, st.tables_host, sizeof(Tables)) != 0) {
        st.tables_valid = false;  // trusted again once a later synchronisation has succeeded
        st.flat_tables_ready = false;
        HIP_TRY(hipMemcpyAsync(st.tables, st.tables_host, sizeof(Tables), hipMemcpyHostToDevice, stream));
        memcpy(st.tables_last, st.tables_host, sizeof(Tables));
    }
    return RR_OK;
}

int run_plan(const Plan &pl, const void *region, uint32_t iters, const rr_window_map_t *wm,
             uint64_t read_seed, hipStream_t stream, const rr_launch_opts_t *opts, rr_result_t *out) {
    rr_result_t res;
    memset(&res, 0, sizeof res);
    if (pl.W == 0) {  // nothing to read
        *out = res;
        return RR_OK;
    }
    std::lock_guard<std::mutex> lock(g_mutex);
    DeviceState *stp = nullptr;
    int rc = get_state(stream, &stp);
    if (rc != RR_OK) return rc;
    DeviceState &st = *stp;
    const u32 n_cus = (u32)st.cus.size();
    if (wm && wm->n_cus != n_cus)
        return fail(RR_EINVAL, "window map describes %u compute units, the device has %u", wm->n_cus, n_cus);

    const u32 lpw = 64 / pl.lanes;
    const u64 L_win = pl.n_lines / pl.n_windows;
    const u64 quota = pl.W / pl.G;
    const u64 units = (quota + lpw - 1) / lpw;  // per group
    // a flat launch without a map reads none of the per-call table fields: reuse what is there
    const bool flat_no_map = !wm && pl.mode == RR_MODE_FLAT;
    if (!(flat_no_map && st.flat_tables_ready)) {
        rc = prepare_tables(st, pl, wm, units, L_win, stream);
        if (rc != RR_OK) return rc;
    }
    const bool want_placement = opts && opts->placement_out;
    if (want_placement && st.placement_cap < pl.W) {
        HIP_TRY(hipStreamSynchronize(stream));
        if (st.placement) HIP_TRY(hipFree(st.placement));
        st.placement = nullptr;
        st.placement_cap = 0;
        HIP_TRY(hipMalloc((void **)&st.placement, pl.W * sizeof(u16)));
        st.placement_cap = pl.W;
    }
    if (want_placement) HIP_TRY(hipMemsetAsync(st.placement, 0xFF, pl.W * sizeof(u16), stream));

    ReadParams p;
    memset(&p, 0, sizeof p);
    p.region = (const char *)region;
    p.read_seed = read_seed;
    p.first_wave = pl.first_wave;
    p.quota = quota;
    p.iters = iters;
    // flat launches default to one hardware wave per whole logical wave (pair); ticketed ones to
    // chunks of 512 iterations so that resident waves finish together
    const bool phased = pl.n_zones > 0;  // its chunks are what one pass through the LDS lists holds
    u32 chunk = phased ? kPhaseChunk : pl.chunk_iters ? pl.chunk_iters : (pl.mode == RR_MODE_TICKET ? 512u : iters);
    if (chunk > iters) chunk = iters;
    p.chunk_iters = chunk;
    p.chunks_per_wave = (iters + chunk - 1) / chunk;
    p.n_groups = pl.G;
    p.n_zones = pl.n_zones;
    p.zone_shift = pl.zone_shift;
    memcpy(p.zone_mask, pl.zone_mask, sizeof p.zone_mask);
    p.ticket_mode = pl.mode == RR_MODE_TICKET ? 1u : 0u;
    p.log2_line = pl.log2_line;
    p.red = make_reducer(L_win);
    p.scratch = st.scratch;
    p.tables = st.tables;
    p.placement = want_placement ? st.placement : nullptr;
    const bool want_cu_waves = opts && opts->cu_waves_out;
    p.locate = (want_placement || want_cu_waves) ? 1u : 0u;
    p.phase_ticks = (opts && pl.n_zones) ? (u64 *)opts->phase_ticks : nullptr;

    const u32 waves_per_block = pl.block / 64;
    // a CU holds at most 32 waves (8 per SIMD); workgroups beyond what really fits queue up,
    // find every share claimed and leave at once
    const u32 blocks_per_cu = 32 / waves_per_block;
    u64 grid;
    if (p.ticket_mode) {
        grid = pl.grid_blocks ? pl.grid_blocks : (u64)blocks_per_cu * n_cus * (pl.pinned ? 64u : 1u);
    } else {
        const u64 hw_waves = (pl.W + lpw - 1) / lpw * (phased ? 1u : p.chunks_per_wave);
        grid = (hw_waves + waves_per_block - 1) / waves_per_block;
    }
    if (grid == 0 || grid > 0x7FFFFFFFull) return fail(RR_EINVAL, "launch of %llu workgroups is out of range", grid);

    const u64 tickets_per_unit = (u64)p.chunks_per_wave * (phased ? pl.n_zones : 1u);
    if (units * tickets_per_unit >= (1ull << 31))
        return fail(RR_EINVAL, "too many tickets per group (%llu)", units * tickets_per_unit);
    // the finish kernel leaves the result cells cleared; counters are needed by ticketed launches only
    const u32 what = (st.cells_clean ? 0u : 1u) | (p.ticket_mode ? 2u : 0u) |
                     ((p.ticket_mode || p.locate) ? 4u : 0u);
    if (what) {
        hipLaunchKernelGGL(reset_kernel, dim3(1), dim3(256), 0, stream, st.scratch, what);
        HIP_TRY(hipGetLastError());
    }
    st.cells_clean = false;
    const int max_launches = p.ticket_mode ? 32 : 1;
    void *args[] = {(void *)&p};
    for (int launch = 0;; ++launch) {
        HIP_TRY(hipEventRecord(st.ev0, stream));
        HIP_TRY(hipLaunchKernel(pl.kernel, dim3((u32)grid), dim3(pl.block), args, 0, stream));
        HIP_TRY(hipEventRecord(st.ev1, stream));
        hipLaunchKernelGGL(finish_kernel, dim3(1), dim3(kNumCells), 0, stream, st.scratch, st.head_dev, st.tables,
                           n_cus, (u32)tickets_per_unit, p.ticket_mode);
        HIP_TRY(hipGetLastError());
        HIP_TRY(hipStreamSynchronize(stream));
        st.cells_clean = true;
        st.tables_valid = true;
        if (flat_no_map) st.flat_tables_ready = true;
        float ms = 0.f;
        HIP_TRY(hipEventElapsedTime(&ms, st.ev0, st.ev1));
        res.launches++;
        res.kernel_ms_event += ms;
        res.checksum += st.head->checksum;
        res.waves_run += st.head->waves_run;
        if (st.head->waves_run && st.head->t_max >= st.head->t_min)
            res.kernel_ms_device += (double)(st.head->t_max - st.head->t_min) / (double)st.wall_khz;
        if (!p.ticket_mode || st.head->unfinished == 0) break;
        if (launch + 1 >= max_launches)
            return fail(RR_EPLACE, "after %d launches %u compute units' shares still have unclaimed tickets",
                        max_launches, st.head->unfinished);
    }
    if (want_placement) {
        HIP_TRY(hipMemcpyAsync(opts->placement_out, st.placement, pl.W * sizeof(u16), hipMemcpyDeviceToHost, stream));
        HIP_TRY(hipStreamSynchronize(stream));
    }
    if (want_cu_waves) {
        HIP_TRY(hipMemcpyAsync(st.cu_waves_host, st.scratch->cu_waves, n_cus * sizeof(u32), hipMemcpyDeviceToHost, stream));
        HIP_TRY(hipStreamSynchronize(stream));
        memcpy(opts->cu_waves_out, st.cu_waves_host, n_cus * sizeof(u32));
    }
    *out = res;
    return RR_OK;
}

}  // namespace

// ------------------------------------------------------------------ C ABI

extern "C" int rr_enumerate_cus(rr_cu_t *out, uint32_t cap, uint32_t *n_cus, void *hip_stream) {
    if (!n_cus) return fail(RR_EINVAL, "n_cus is NULL");
    if (cap > 0 && !out) return fail(RR_EINVAL, "out is NULL but cap > 0");
    std::lock_guard<std::mutex> lock(g_mutex);
    DeviceState *st = nullptr;
    int rc = get_state((hipStream_t)hip_stream, &st);
    if (rc != RR_OK) return rc;
    const u32 n = (u32)st->cus.size();
    for (u32 i = 0; i < n && i < cap; ++i) out[i] = st->cus[i];
    *n_cus = n;
    return RR_OK;
}

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
    const u64 cap = (u64)n_cu * 16;  // grid-stride beyond this
    if (blocks > cap) blocks = cap;
    hipLaunchKernelGGL(fill_kernel, dim3((u32)blocks), dim3(256), 0, stream, (u64x2 *)region, n_pairs,
                       (u64)fill_seed);
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipStreamSynchronize(stream));
    return RR_OK;
}

extern "C" int rr_rand_read(const void *region, uint64_t region_bytes, uint32_t line_bytes,
                            uint32_t lanes_per_line, uint64_t n_reads, uint32_t iters_per_wave,
                            const rr_window_map_t *wm, uint64_t read_seed, void *hip_stream,
                            const rr_launch_opts_t *opts, rr_result_t *out) {
    Plan pl;
    int rc = make_plan(region, region_bytes, line_bytes, lanes_per_line, n_reads, iters_per_wave, wm, opts, out, pl);
    if (rc != RR_OK) return rc;
    return run_plan(pl, region, iters_per_wave, wm, read_seed, (hipStream_t)hip_stream, opts, out);
}

extern "C" int rr_probe_cus(const void *region, uint64_t region_bytes, const uint32_t *cus, uint32_t n_target,
                            uint64_t n_reads, uint32_t iters_per_wave, uint64_t read_seed, void *hip_stream,
                            const rr_launch_opts_t *opts, rr_result_t *out) {
    if (!cus || n_target == 0) return fail(RR_EINVAL, "the target set is empty");
    if (n_target > RR_MAX_CUS) return fail(RR_EINVAL, "too many target compute units");
    for (u32 a = 0; a < n_target; ++a)
        for (u32 b = a + 1; b < n_target; ++b)
            if (cus[a] == cus[b]) return fail(RR_EINVAL, "compute unit %u is named twice", cus[a]);
    if (opts && opts->mode == RR_MODE_FLAT) return fail(RR_EINVAL, "a pinned run cannot use flat mode");
    // validate everything else before touching the device (map filled in below)
    Plan pl;
    int rc = make_plan(region, region_bytes, 128, 32, n_reads, iters_per_wave, nullptr, opts, out, pl);
    if (rc != RR_OK) return rc;
    u32 n_cus = 0;
    {
        std::lock_guard<std::mutex> lock(g_mutex);
        DeviceState *st = nullptr;
        rc = get_state((hipStream_t)hip_stream, &st);
        if (rc != RR_OK) return rc;
        n_cus = (u32)st->cus.size();
    }
    std::vector<uint16_t> group_of_cu(n_cus, RR_CU_EXCLUDED);
    for (u32 a = 0; a < n_target; ++a) {
        if (cus[a] >= n_cus) return fail(RR_EINVAL, "compute unit id %u is not below %u", cus[a], n_cus);
        group_of_cu[cus[a]] = 0;
    }
    const uint16_t window_of_group[1] = {0};
    rr_window_map_t wm = {1, 1, n_cus, group_of_cu.data(), window_of_group};
    pl.mode = RR_MODE_TICKET;
    pl.pinned = true;
    return run_plan(pl, region, iters_per_wave, &wm, read_seed, (hipStream_t)hip_stream, opts, out);
}

extern "C" int rr_probe_pair(const void *region, uint64_t region_bytes, uint32_t cu_a, uint32_t cu_b,
                             uint64_t n_reads, uint32_t iters_per_wave, uint64_t read_seed, void *hip_stream,
                             const rr_launch_opts_t *opts, rr_result_t *out) {
    if (cu_a == cu_b) return fail(RR_EINVAL, "cu_a and cu_b must differ");
    const uint32_t cus[2] = {cu_a, cu_b};
    return rr_probe_cus(region, region_bytes, cus, 2, n_reads, iters_per_wave, read_seed, hip_stream, opts, out);
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
    const u64 cap = 16ull * st->cus.size();  // two rounds of resident workgroups; each wave loops over its chunks
    if (blocks > cap) blocks = cap;
    if (!st->cells_clean) {
        hipLaunchKernelGGL(reset_kernel, dim3(1), dim3(256), 0, stream, st->scratch, 1u);
        HIP_TRY(hipGetLastError());
    }
    st->cells_clean = false;
    HIP_TRY(hipEventRecord(st->ev0, stream));
    hipLaunchKernelGGL(seq_read_kernel, dim3((u32)blocks), dim3(256), 0, stream, (const u32x4 *)region, n_vec,
                       st->scratch);
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipEventRecord(st->ev1, stream));
    hipLaunchKernelGGL(finish_kernel, dim3(1), dim3(kNumCells), 0, stream, st->scratch, st->head_dev, st->tables, 0u,
                       1u, 0u);
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipStreamSynchronize(stream));
    st->cells_clean = true;
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

extern "C" int rr_rand_update(void *region, uint64_t region_bytes, uint32_t line_bytes, uint32_t lanes_per_line,
                              uint64_t n_updates, uint32_t iters_per_wave, uint64_t draw_seed, uint32_t op,
                              uint64_t value_seed, void *hip_stream, rr_result_t *out) {
    Plan pl;
    int rc = make_plan(region, region_bytes, line_bytes, lanes_per_line, n_updates, iters_per_wave, nullptr, nullptr,
                       out, pl);
    if (rc != RR_OK) return rc;
    if (op != RR_OP_WRITE && op != RR_OP_ADD) return fail(RR_EINVAL, "op must be RR_OP_WRITE or RR_OP_ADD");
    kernel_handle kernel = find_update_kernel(pl.lanes, pl.wdw, op);
    if (!kernel) return fail(RR_EINVAL, "no update kernel for this line shape");
    rr_result_t res;
    memset(&res, 0, sizeof res);
    if (pl.W == 0) {
        *out = res;
        return RR_OK;
    }
    const u64 hw_waves = (pl.W + 64 / pl.lanes - 1) / (64 / pl.lanes);
    const u64 grid = (hw_waves + 3) / 4;
    if (grid > 0x7FFFFFFFull) return fail(RR_EINVAL, "launch of %llu workgroups is out of range", grid);
    hipStream_t stream = (hipStream_t)hip_stream;
    std::lock_guard<std::mutex> lock(g_mutex);
    DeviceState *st = nullptr;
    rc = get_state(stream, &st);
    if (rc != RR_OK) return rc;
    UpdateParams p;
    memset(&p, 0, sizeof p);
    p.region = (char *)region;
    p.draw_seed = draw_seed;
    p.value_seed = value_seed;
    p.n_waves = pl.W;
    p.iters = iters_per_wave;
    p.log2_line = pl.log2_line;
    p.red = make_reducer(pl.n_lines);
    p.scratch = st->scratch;
    if (!st->cells_clean) {
        hipLaunchKernelGGL(reset_kernel, dim3(1), dim3(256), 0, stream, st->scratch, 1u);
        HIP_TRY(hipGetLastError());
    }
    st->cells_clean = false;
    void *args[] = {(void *)&p};
    HIP_TRY(hipEventRecord(st->ev0, stream));
    HIP_TRY(hipLaunchKernel(kernel, dim3((u32)grid), dim3(256), args, 0, stream));
    HIP_TRY(hipEventRecord(st->ev1, stream));
    hipLaunchKernelGGL(finish_kernel, dim3(1), dim3(kNumCells), 0, stream, st->scratch, st->head_dev, st->tables, 0u,
                       1u, 0u);
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipStreamSynchronize(stream));
    st->cells_clean = true;
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

extern "C" int rr_chase(const void *region, uint64_t region_bytes, uint32_t line_bytes, uint64_t start,
                        uint64_t stride, uint32_t mask, uint64_t hops, void *hip_stream, rr_chase_result_t *out) {
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
    // the walk's three result words go through the (otherwise idle) key-mark area of the scratch
    ChaseOut *dev_out = (ChaseOut *)st->scratch->key_seen;
    const u32 log2_line = line_bytes == 128 ? 7 : line_bytes == 256 ? 8 : 9;
    HIP_TRY(hipEventRecord(st->ev0, stream));
    hipLaunchKernelGGL(chase_kernel, dim3(1), dim3(64), 0, stream, (const char *)region, make_reducer(n_lines),
                       log2_line, (u64)start, (u64)(stride % n_lines), mask, (u64)hops, dev_out);
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipEventRecord(st->ev1, stream));
    ChaseOut host;
    HIP_TRY(hipMemcpyAsync(&host, dev_out, sizeof host, hipMemcpyDeviceToHost, stream));
    HIP_TRY(hipStreamSynchronize(stream));
    float ms = 0.f;
    HIP_TRY(hipEventElapsedTime(&ms, st->ev0, st->ev1));
    out->final_line = host.final_line;
    out->word_sum = host.word_sum;
    out->kernel_ms_event = ms;
    out->ns_per_hop = (double)host.ticks * 1e6 / (double)st->wall_khz / (double)hops;
    return RR_OK;
}

extern "C" int rr_copy(void *dst, const void *src, uint64_t bytes, void *hip_stream, double *kernel_ms) {
    if (!dst || !src) return fail(RR_EINVAL, "dst or src is NULL");
    if ((uintptr_t)dst % 16 != 0 || (uintptr_t)src % 16 != 0 || bytes % 16 != 0)
        return fail(RR_EINVAL, "dst, src and bytes must be multiples of 16");
    const uintptr_t d = (uintptr_t)dst, c = (uintptr_t)src;
    if (d < c + bytes && c < d + bytes && bytes > 0) return fail(RR_EINVAL, "dst and src overlap");
    if (kernel_ms) *kernel_ms = 0.0;
    if (bytes == 0) return RR_OK;
    hipStream_t stream = (hipStream_t)hip_stream;
    std::lock_guard<std::mutex> lock(g_mutex);
    DeviceState *st = nullptr;
    int rc = get_state(stream, &st);
    if (rc != RR_OK) return rc;
    const u64 n_vec = bytes / 16;
    u64 blocks = (n_vec + 255) / 256;
    const u64 cap = (u64)st->cus.size() * 8;
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

// ------------------------------------------------------------------ regions mapped in pieces

namespace {

struct PiecewiseRegion {
    int device = 0;
    u64 bytes = 0, piece = 0;
    u64 mapped = 0;  // bytes of the reservation that have a piece mapped
    std::vector<hipMemGenericAllocationHandle_t> handles;
};
std::map<void *, PiecewiseRegion> g_regions;  // guarded by g_mutex

// Undo a (possibly partial) piecewise mapping; errors are ignored, this runs on failure paths and at shutdown.
void release_region(void *base, PiecewiseRegion &r) {
    for (u64 off = 0; off < r.mapped; off += r.piece) (void)hipMemUnmap((char *)base + off, r.piece);
    for (auto h : r.handles) (void)hipMemRelease(h);
    (void)hipMemAddressFree(base, r.bytes);
    r.handles.clear();
    r.mapped = 0;
}

hipMemAllocationProp device_memory_prop(int dev) {
    hipMemAllocationProp prop = {};
    prop.type = hipMemAllocationTypePinned;
    prop.location.type = hipMemLocationTypeDevice;
    prop.location.id = dev;
    return prop;
}

}  // namespace

extern "C" int rr_region_granularity(uint64_t *minimum, uint64_t *recommended) {
    if (!minimum && !recommended) return fail(RR_EINVAL, "both outputs are NULL");
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    hipMemAllocationProp prop = device_memory_prop(dev);
    size_t g = 0;
    if (minimum) {
        HIP_TRY(hipMemGetAllocationGranularity(&g, &prop, hipMemAllocationGranularityMinimum));
        *minimum = g;
    }
    if (recommended) {
        HIP_TRY(hipMemGetAllocationGranularity(&g, &prop, hipMemAllocationGranularityRecommended));
        *recommended = g;
    }
    return RR_OK;
}

extern "C" int rr_region_create(uint64_t bytes, uint64_t piece_bytes, void **region_out) {
    if (!region_out) return fail(RR_EINVAL, "region_out is NULL");
    if (bytes == 0 || piece_bytes == 0 || bytes % piece_bytes != 0)
        return fail(RR_EINVAL, "bytes must be a positive multiple of piece_bytes");
    if (piece_bytes % 4096 != 0) return fail(RR_EINVAL, "piece_bytes must be a multiple of 4096");
    // the driver gives a process about 65 500 handles and a mapped piece takes two: 32 752 pieces was the last to map
    if (bytes / piece_bytes > 30000) return fail(RR_EINVAL, "more than 30000 pieces");
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    hipMemAllocationProp prop = device_memory_prop(dev);
    size_t minimum = 0;
    HIP_TRY(hipMemGetAllocationGranularity(&minimum, &prop, hipMemAllocationGranularityMinimum));
    if (minimum == 0 || piece_bytes % minimum != 0)
        return fail(RR_EINVAL, "piece_bytes must be a multiple of the device's allocation granularity (%zu)", minimum);
    u64 align = piece_bytes & (~piece_bytes + 1);  // largest power of two dividing the piece size
    if (align > (1ull << 30)) align = 1ull << 30;
    void *base = nullptr;
    HIP_TRY(hipMemAddressReserve(&base, bytes, align, nullptr, 0));
    PiecewiseRegion r;
    r.device = dev;
    r.bytes = bytes;
    r.piece = piece_bytes;
    r.handles.reserve(bytes / piece_bytes);
    hipError_t e = hipSuccess;
    const char *what = "";
    hipMemAccessDesc access = {};
    access.location = prop.location;
    access.flags = hipMemAccessFlagsProtReadWrite;
    for (u64 off = 0; off < bytes; off += piece_bytes) {
        hipMemGenericAllocationHandle_t h;
        e = hipMemCreate(&h, piece_bytes, &prop, 0);
        what = "hipMemCreate";
        if (e != hipSuccess) break;
        r.handles.push_back(h);
        e = hipMemMap((char *)base + off, piece_bytes, 0, h, 0);
        what = "hipMemMap";
        if (e != hipSuccess) break;
        r.mapped = off + piece_bytes;
        // access is granted piece by piece (one call over the whole range was refused for 32768 pieces)
        e = hipMemSetAccess((char *)base + off, piece_bytes, &access, 1);
        what = "hipMemSetAccess";
        if (e != hipSuccess) break;
    }
    if (e != hipSuccess) {
        const u64 done = r.mapped;
        release_region(base, r);
        return fail(RR_EHIP, "%s failed after %llu of %llu bytes: %s", what, (unsigned long long)done,
                    (unsigned long long)bytes, hipGetErrorString(e));
    }
    std::lock_guard<std::mutex> lock(g_mutex);
    g_regions[base] = std::move(r);
    *region_out = base;
    return RR_OK;
}

extern "C" int rr_region_destroy(void *region) {
    std::lock_guard<std::mutex> lock(g_mutex);
    auto it = g_regions.find(region);
    if (it == g_regions.end()) return fail(RR_EINVAL, "not a region made by rr_region_create");
    int current = 0;
    HIP_TRY(hipGetDevice(&current));
    HIP_TRY(hipSetDevice(it->second.device));
    HIP_TRY(hipDeviceSynchronize());
    release_region(region, it->second);
    g_regions.erase(it);
    HIP_TRY(hipSetDevice(current));
    return RR_OK;
}

extern "C" int rr_shutdown(void) {
    std::lock_guard<std::mutex> lock(g_mutex);
    int current = 0;
    bool have_current = hipGetDevice(&current) == hipSuccess;
    for (int d = 0; d < kMaxDevices; ++d) {
        DeviceState &st = g_state[d];
        if (!st.scratch && !st.head && !st.ev0) continue;
        if (hipSetDevice(d) != hipSuccess) continue;
        (void)hipDeviceSynchronize();
        if (st.scratch) (void)hipFree(st.scratch);
        if (st.tables) (void)hipFree(st.tables);
        if (st.tables_host) (void)hipHostFree(st.tables_host);
        delete st.tables_last;
        if (st.placement) (void)hipFree(st.placement);
        if (st.head) (void)hipHostFree(st.head);
        if (st.cu_waves_host) (void)hipHostFree(st.cu_waves_host);
        if (st.ev0) (void)hipEventDestroy(st.ev0);
        if (st.ev1) (void)hipEventDestroy(st.ev1);
        st = DeviceState();
    }
    for (auto &kv : g_regions) {
        if (hipSetDevice(kv.second.device) != hipSuccess) continue;
        (void)hipDeviceSynchronize();
        release_region(kv.first, kv.second);
    }
    g_regions.clear();
    if (have_current) (void)hipSetDevice(current);
    return RR_OK;
}
