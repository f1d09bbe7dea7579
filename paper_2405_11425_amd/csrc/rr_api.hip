// The random read behind the C ABI declared in include/randline.h: the launch loop (run_plan) and the entry points
// built on it (rr_rand_read, rr_rand_read_noalloc, rr_rand_read_batch, rr_probe_cus, rr_probe_pair, rr_detect_zones,
// rr_rand_update).  Validation, tables and launch parameters of a call are made in rr_plan.hip.  The kernels are in rr_read_kernel.hpp,
// rr_phased_kernel.hpp and rr_update_kernel.hpp and are instantiated in the rr_inst_*.hip files.
#include <algorithm>
#include <chrono>
#include <cstdio>
#include <cstring>
#include <vector>

#include <hip/hip_ext.h>

#include "rr_host.hpp"
#include "rr_plan.hpp"
#include "rr_phased_kernel.hpp"
#include "rr_update_kernel.hpp"
#include "rr_zones.hpp"

using namespace rr;

namespace {

// ------------------------------------------------------------------ the state that allocates nothing

// Device data of the entry point that allocates nothing (rr_rand_read_noalloc): what the other entry points keep
// in hipMalloc'ed and pinned memory -- result cells, counters, lookup tables, the result head -- plus a placement
// log of fixed capacity.  One copy of this array exists on every GPU the library's code object is loaded on, at an
// address of its own; host code gets that address from hipGetSymbolAddress (never from the array's name, which in
// host code is only a stand-in for the symbol).
struct FixedArea {
    Scratch scratch;
    Tables tables;
    ResultHead head;
    u16 placement[RR_NOALLOC_MAX_PLACEMENT];
};
static __device__ __align__(256) unsigned char scratch[sizeof(FixedArea)];

// Host-side companions of that array (plain static memory): table staging, the last upload, per-CU counts.
struct FixedHost {
    Tables staging, last;
    u32 cu_waves[kMaxCus];
};
FixedHost g_fixed_host[kMaxDevices];
DeviceState g_fixed_state[kMaxDevices];

// Set-up of the current device's fixed state, once per device: the address of this device's copy of the
// array, the clock rate, the CU list (enumeration kernel on `stream`).  Allocates nothing.  g_mutex held.
int get_fixed_state(hipStream_t stream, DeviceState **out) {
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(RR_EHIP, "device index %d not supported", dev);
    DeviceState &st = g_fixed_state[dev];
    if (!st.ready) {
        unsigned char *ptr = nullptr;
        HIP_TRY(hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) return fail(RR_EHIP, "the device array has no address on device %d", dev);
        FixedArea *area = (FixedArea *)ptr;  // a device address: host code only does arithmetic on it
        st.fixed = true;
        st.scratch = &area->scratch;
        st.tables = &area->tables;
        st.head_dev = &area->head;
        st.head = &st.head_copy;
        st.placement = area->placement;
        st.placement_cap = RR_NOALLOC_MAX_PLACEMENT;
        st.tables_host = &g_fixed_host[dev].staging;
        st.tables_last = &g_fixed_host[dev].last;
        st.cu_waves_host = g_fixed_host[dev].cu_waves;
        st.tables_valid = false;
        st.cells_clean = false;  // the array holds whatever was there: the first launch clears the cells
        HIP_TRY(hipDeviceGetAttribute(&st.wall_khz, hipDeviceAttributeWallClockRate, dev));
        if (st.wall_khz <= 0) st.wall_khz = 100000;  // s_memrealtime: 100 MHz
        int rc = enumerate(st, stream);
        if (rc != RR_OK) return rc;
        st.ready = true;
    }
    *out = &st;
    return RR_OK;
}

// ------------------------------------------------------------------ the launch loop

int run_plan_locked(DeviceState &st, const Plan &pl, const void *region, uint32_t iters, const rr_window_map_t *wm,
                    uint64_t read_seed, hipStream_t stream, const rr_launch_opts_t *opts, rr_result_t *out) {
    rr_result_t res;
    memset(&res, 0, sizeof res);
    int rc;
    const u32 n_cus = st.n_cus;
    if (wm && wm->n_cus != n_cus)
        return fail(RR_EINVAL, "window map describes %u compute units, the device has %u", wm->n_cus, n_cus);

    const u32 lpw = 64 / pl.lanes;
    const u64 L_win = pl.n_lines / pl.n_windows;
    const u64 quota = pl.W / pl.G;
    const u64 units = (quota + lpw - 1) / lpw;  // per group
    // a flat launch without a map reads none of the per-call table fields: reuse what is there
    const bool flat_no_map = !wm && (pl.mode == RR_MODE_FLAT || pl.mode == RR_MODE_STREAM);
    if (!(flat_no_map && st.flat_tables_ready)) {
        rc = prepare_tables(st, pl, wm, units, L_win, stream);
        if (rc != RR_OK) return rc;
    }
    const bool want_placement = opts && opts->placement_out;
    if (want_placement && st.placement_cap < pl.W) {
        if (st.fixed)
            return fail(RR_EINVAL, "placement_out for %llu logical waves is beyond the %u this entry point has room for",
                        pl.W, (u32)RR_NOALLOC_MAX_PLACEMENT);
        HIP_TRY(hipStreamSynchronize(stream));
        if (st.placement) HIP_TRY(hipFree(st.placement));
        st.placement = nullptr;
        st.placement_cap = 0;
        HIP_TRY(hipMalloc((void **)&st.placement, pl.W * sizeof(u16)));
        st.placement_cap = pl.W;
    }
    if (want_placement) {  // every entry "not executed" (a fill kernel: a memset node is not safe to capture)
        rc = launch_fill_u16(st.placement, pl.W, 0xFFFFu, stream);
        if (rc != RR_OK) return rc;
    }

    Launch ln;
    rc = make_launch(pl, st, region, iters, wm, read_seed, opts, want_placement ? st.placement : nullptr, ln);
    if (rc != RR_OK) return rc;
    const ReadParams &p = ln.p;
    const bool want_cu_waves = opts && opts->cu_waves_out;
    // the finish kernel leaves the result cells cleared
    const u32 what = (st.cells_clean ? 0u : 1u) | ln.reset_bits;
    if (what) {
        rc = launch_reset(st, what, stream);
        if (rc != RR_OK) return rc;
    }
    st.cells_clean = false;
    const int max_launches = p.ticket_mode ? 32 : 1;
    void *args[] = {(void *)&ln.p};
    for (int launch = 0;; ++launch) {
        // (events attached to the dispatch, as in a batch, cost a single call 17 us more on the host)
        if (st.ev0) HIP_TRY(hipEventRecord(st.ev0, stream));
        HIP_TRY(hipLaunchKernel(ln.kernel, dim3(ln.grid), dim3(pl.block), args, 0, stream));
        if (st.ev1) HIP_TRY(hipEventRecord(st.ev1, stream));
        rc = finish_and_wait(st, n_cus, ln.tickets_per_unit, p.ticket_mode, stream);
        if (rc != RR_OK) return rc;
        st.tables_valid = true;
        if (flat_no_map) st.flat_tables_ready = true;
        float ms = 0.f;
        if (st.ev0 && st.ev1) HIP_TRY(hipEventElapsedTime(&ms, st.ev0, st.ev1));
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
    if (want_cu_waves || pl.pinned) {
        HIP_TRY(hipMemcpyAsync(st.cu_waves_host, st.scratch->cu_waves, n_cus * sizeof(u32), hipMemcpyDeviceToHost, stream));
        HIP_TRY(hipStreamSynchronize(stream));
        if (want_cu_waves) memcpy(opts->cu_waves_out, st.cu_waves_host, n_cus * sizeof(u32));
    }
    if (pl.pinned && wm) {
        // A pinned run measures its target compute units together: if one of them executed nothing (the others
        // stole its share) the figure would be that of a smaller set.  Only shares of at least one ticket per wave
        // slot of a CU are checked: the others' waves start to steal when their own share is drained, which takes
        // them at least one whole ticket then, far longer than the dispatcher needs to reach every CU; a smaller
        // share can be gone before its CU's first wave arrives without anything being wrong.
        const Tables &tb = *st.tables_host;
        for (u32 c = 0; c < n_cus; ++c)
            if (wm->group_of_cu[c] != RR_CU_EXCLUDED && (u64)tb.cu_unit_count[c] * ln.tickets_per_unit >= 32 &&
                st.cu_waves_host[c] == 0)
                return fail(RR_EPLACE, "target compute unit %u executed none of the work (no resident wave in time)", c);
    }
    *out = res;
    return RR_OK;
}

// fixed: use the state that allocates nothing (rr_rand_read_noalloc) instead of the hipMalloc'ed one.
int run_plan(const Plan &pl, const void *region, uint32_t iters, const rr_window_map_t *wm, uint64_t read_seed,
             hipStream_t stream, const rr_launch_opts_t *opts, rr_result_t *out, bool fixed = false) {
    if (pl.W == 0) {  // nothing to read
        memset(out, 0, sizeof *out);
        return RR_OK;
    }
    std::lock_guard<std::mutex> lock(g_mutex);
    DeviceState *st = nullptr;
    int rc = fixed ? get_fixed_state(stream, &st) : get_state(stream, &st);
    if (rc != RR_OK) return rc;
    rc = run_plan_locked(*st, pl, region, iters, wm, read_seed, stream, opts, out);
    // A fixed state stages its tables in plain static memory: nothing of this call may still be in flight
    // when the next one rewrites them.
    if (rc != RR_OK && fixed) (void)hipStreamSynchronize(stream);
    return rc;
}

// ------------------------------------------------------------------ zone probe

// What the measuring rate function of rr_detect_zones works with.  g_mutex is held for the whole probe.
struct ZoneProbe {
    DeviceState *st;
    const void *region;
    u64 region_bytes;
    u32 n_windows, iters, launches, unroll;
    hipStream_t stream;
    u64 next_seed;
    u32 launches_made;
    uint16_t parity[kMaxCus];  // group of a compute unit: its dense id modulo 2
};

// One launch of the probe: even compute units read window a, odd ones window b; every wave slot is occupied.
int zone_probe_launch(ZoneProbe &zp, u32 a, u32 b, double *gbps) {
    const uint16_t window_of_group[2] = {(uint16_t)a, (uint16_t)b};
    const rr_window_map_t wm = {2, zp.n_windows, zp.st->n_cus, zp.parity, window_of_group};
    rr_launch_opts_t opts;
    memset(&opts, 0, sizeof opts);
    opts.unroll = zp.unroll;
    const u64 W = (u64)zp.st->n_cus * 64;  // 32 wave slots per compute unit, two logical waves per wavefront
    const u64 n_reads = W * zp.iters;
    rr_result_t res;
    Plan pl;
    int rc = make_plan(zp.region, zp.region_bytes, 128, 32, n_reads, zp.iters, &wm, &opts, &res, pl);
    if (rc != RR_OK) return rc;
    rc = run_plan_locked(*zp.st, pl, zp.region, zp.iters, &wm, zp.next_seed++, zp.stream, &opts, &res);
    if (rc != RR_OK) return rc;
    zp.launches_made += res.launches;
    if (!(res.kernel_ms_event > 0.0)) return fail(RR_EHIP, "a probe launch reported no time");
    if (gbps) *gbps = (double)n_reads * 128.0 / res.kernel_ms_event / 1e6;
    return RR_OK;
}

// rate(a, b): the fastest of the pair's launches (what disturbs a launch only ever makes it slower).
int zone_probe_rate(uint32_t a, uint32_t b, int again, void *user, double *rate_out) {
    ZoneProbe &zp = *(ZoneProbe *)user;
    const u32 n = again ? 2 * zp.launches : zp.launches;
    double best = 0.0;
    for (u32 i = 0; i < n; ++i) {
        double r = 0.0;
        int rc = zone_probe_launch(zp, a, b, &r);
        if (rc != RR_OK) return rc;
        best = std::max(best, r);
    }
    *rate_out = best;
    return RR_OK;
}

}  // namespace

// ------------------------------------------------------------------ C ABI

extern "C" int rr_detect_zones(const void *region, uint64_t region_bytes, uint32_t n_windows,
                               const rr_zone_probe_opts_t *opts, void *hip_stream, uint8_t *zone_of_window_out,
                               rr_zone_probe_t *details_out) {
    const auto t_begin = std::chrono::steady_clock::now();
    rr_zone_probe_opts_t o;
    memset(&o, 0, sizeof o);
    if (opts) o = *opts;
    if (o.min_gap == 0.0) o.min_gap = 0.02;
    if (o.max_zones == 0) o.max_zones = RR_MAX_ZONES;
    if (o.launches == 0) o.launches = 3;
    if (o.iters_per_wave == 0) o.iters_per_wave = 2048;
    if (o.warmup == 0) o.warmup = 8;
    if (o.warmup == RR_ZONE_NO_WARMUP) o.warmup = 0;
    if (o.unroll == 0) o.unroll = 16;
    if (!region) return fail(RR_EINVAL, "region is NULL");
    int rc = check_zone_rule_args(n_windows, o.min_gap, o.max_zones, zone_of_window_out);
    if (rc != RR_OK) return rc;
    if (o.reserved != 0) return fail(RR_EINVAL, "reserved must be 0");
    if (o.launches > 64) return fail(RR_EINVAL, "at most 64 launches per rate");
    if (o.warmup > 4096) return fail(RR_EINVAL, "at most 4096 warm-up launches");
    if ((uintptr_t)region % 128 != 0) return fail(RR_EINVAL, "region is not aligned to 128 bytes");
    if (region_bytes == 0 || region_bytes % ((u64)n_windows * 128) != 0)
        return fail(RR_EINVAL, "region_bytes must be a positive multiple of n_windows lines of 128 bytes");
    if (region_bytes / 128 > (1ull << 32)) return fail(RR_EINVAL, "region has more than 2^32 lines");
    if (!find_read_kernel_32_1(o.unroll, RR_BCAST_DPP, 1))
        return fail(RR_EINVAL, "unroll %u is not built for 128-byte lines", o.unroll);

    hipStream_t stream = (hipStream_t)hip_stream;
    std::lock_guard<std::mutex> lock(g_mutex);
    static ZoneProbe zp;  // guarded by g_mutex; static so that the call does not put 2 KB of table on the stack
    rc = get_state(stream, &zp.st);
    if (rc != RR_OK) return rc;
    if (zp.st->n_cus < 2) return fail(RR_EPLACE, "the probe needs at least two compute units");
    zp.region = region;
    zp.region_bytes = region_bytes;
    zp.n_windows = n_windows;
    zp.iters = o.iters_per_wave;
    zp.launches = o.launches;
    zp.unroll = o.unroll;
    zp.stream = stream;
    zp.next_seed = 1000;
    zp.launches_made = 0;
    for (u32 c = 0; c < zp.st->n_cus; ++c) zp.parity[c] = (uint16_t)(c & 1u);
    for (u32 i = 0; i < o.warmup; ++i) {
        rc = zone_probe_launch(zp, 0, 0, nullptr);
        if (rc != RR_OK) return rc;
    }
    // A process' first launches can run a few per cent slow, for some tens of milliseconds (seen after a fill: 80
    // launches).  Unless the caller asked for no warm-up, go on in groups of eight until the best of a group is no
    // longer more than 0.5 % above the best of the group before it (at most 64 groups).
    if (o.warmup) {
        double before = 0.0;
        for (u32 g = 0; g < 64; ++g) {
            double best = 0.0, r = 0.0;
            for (u32 i = 0; i < 8; ++i) {
                rc = zone_probe_launch(zp, 0, 0, &r);
                if (rc != RR_OK) return rc;
                best = std::max(best, r);
            }
            if (g > 0 && best <= before * 1.005) break;
            before = best;
        }
    }
    uint8_t zone[RR_MAX_ZONE_WINDOWS];
    rr_zone_probe_t d;
    rc = zones_rule(zone_probe_rate, &zp, n_windows, o.min_gap, o.max_zones, zone, &d);
    if (rc != RR_OK) return rc;
    memcpy(zone_of_window_out, zone, n_windows);
    if (details_out) {
        d.launches = zp.launches_made;
        d.seconds = std::chrono::duration<double>(std::chrono::steady_clock::now() - t_begin).count();
        *details_out = d;
    }
    return RR_OK;
}

extern "C" const char *rr_last_kernel(void) { return g_last_kernel; }

extern "C" int rr_describe_read(const void *region, uint64_t region_bytes, uint32_t line_bytes, uint32_t lanes_per_line,
                                uint64_t n_reads, uint32_t iters_per_wave, const rr_window_map_t *wm,
                                const rr_launch_opts_t *opts, rr_read_plan_t *out) {
    Plan pl;
    const int rc = make_plan(region, region_bytes, line_bytes, lanes_per_line, n_reads, iters_per_wave, wm, opts, out, pl);
    if (rc != RR_OK) return rc;
    rr_read_plan_t d;
    memset(&d, 0, sizeof d);
    d.mode = pl.mode;
    d.zone_kernel = pl.n_zones ? 1u : 0u;
    d.n_zones = pl.n_zones;
    if (pl.n_zones) {
        d.n_zone_windows = (u32)((pl.n_lines + ((u64)1 << pl.zone_shift) - 1) >> pl.zone_shift);
        d.zone_window_bytes = ((u64)1 << pl.zone_shift) * line_bytes;
        memcpy(d.zone_windows, pl.zone_mask, sizeof d.zone_windows);
    }
    d.xcd_split = pl.split != RR_SPLIT_OFF ? 1u : 0u;
    d.split_windows[0] = pl.split_incl[0];
    d.split_windows[1] = pl.split_incl[1];
    d.chunk_iters = pl.mode == RR_MODE_STREAM ? pl.chunk_iters : pl.n_zones ? kPhaseChunk : pl.chunk_iters ? pl.chunk_iters : pl.mode == RR_MODE_TICKET ? 1024u : iters_per_wave;
    if (d.chunk_iters > iters_per_wave) d.chunk_iters = iters_per_wave;
    d.block_threads = pl.block;
    d.unroll = pl.n_zones ? (pl.mode == RR_MODE_STREAM ? (pl.wdw == 4 ? 8u : 16u) : 32u / pl.wdw) : pl.unroll;
    d.bcast = pl.bcast;
    d.nontemporal = pl.nt ? RR_NT_ON : RR_NT_OFF;
    *out = d;
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

extern "C" int rr_rand_read_noalloc(const void *region, uint64_t region_bytes, uint32_t line_bytes,
                                    uint32_t lanes_per_line, uint64_t n_reads, uint32_t iters_per_wave,
                                    const rr_window_map_t *wm, uint64_t read_seed, void *hip_stream,
                                    const rr_launch_opts_t *opts, rr_result_t *out) {
    Plan pl;
    int rc = make_plan(region, region_bytes, line_bytes, lanes_per_line, n_reads, iters_per_wave, wm, opts, out, pl);
    if (rc != RR_OK) return rc;
    if (opts && opts->placement_out && pl.W > RR_NOALLOC_MAX_PLACEMENT)
        return fail(RR_EINVAL, "placement_out for %llu logical waves is beyond the %u this entry point has room for",
                    pl.W, (u32)RR_NOALLOC_MAX_PLACEMENT);
    return run_plan(pl, region, iters_per_wave, wm, read_seed, (hipStream_t)hip_stream, opts, out, true);
}

extern "C" int rr_rand_read_batch(const void *region, const rr_read_item_t *items, uint32_t n_items,
                                  uint32_t line_bytes, uint32_t lanes_per_line, uint64_t n_reads,
                                  uint32_t iters_per_wave, void *hip_stream, rr_result_t *out) {
    if (n_items == 0) return RR_OK;
    if (!items) return fail(RR_EINVAL, "items is NULL");
    if (!out) return fail(RR_EINVAL, "out is NULL");
    if (n_items > kMaxBatch) return fail(RR_EINVAL, "a batch holds at most %u calls (got %u)", kMaxBatch, n_items);
    std::vector<Plan> plans(n_items);
    for (u32 i = 0; i < n_items; ++i) {
        const rr_launch_opts_t *o = items[i].opts;
        if (o && (o->placement_out || o->cu_waves_out || o->phase_ticks))
            return fail(RR_EINVAL, "item %u: per-wave outputs are not available in a batch", i);
        int rc = make_plan(region, items[i].region_bytes, line_bytes, lanes_per_line, n_reads, iters_per_wave, nullptr,
                           o, out, plans[i]);
        if (rc != RR_OK) return rc;
    }
    std::vector<rr_result_t> results(n_items);  // out is written on success only
    memset(results.data(), 0, n_items * sizeof(rr_result_t));
    if (plans[0].W == 0) {  // nothing to read, in any item
        memcpy(out, results.data(), n_items * sizeof(rr_result_t));
        return RR_OK;
    }

    hipStream_t stream = (hipStream_t)hip_stream;
    std::lock_guard<std::mutex> lock(g_mutex);
    DeviceState *stp = nullptr;
    int rc = get_state(stream, &stp);
    if (rc != RR_OK) return rc;
    DeviceState &st = *stp;
    while (st.batch_ev.size() < 2 * (size_t)n_items) {
        hipEvent_t e = nullptr;
        HIP_TRY(hipEventCreate(&e));
        st.batch_ev.push_back(e);
    }
    // Without a window map the tables depend on the number of logical waves only, which the items share:
    // one upload (if any) before the first launch serves them all.
    const u32 lpw = 64 / plans[0].lanes;
    const u64 units = (plans[0].W + lpw - 1) / lpw;
    rc = prepare_tables(st, plans[0], nullptr, units, plans[0].n_lines, stream);
    if (rc != RR_OK) return rc;
    std::vector<Launch> launches(n_items);
    for (u32 i = 0; i < n_items; ++i) {
        rc = make_launch(plans[i], st, region, iters_per_wave, nullptr, items[i].read_seed, items[i].opts, nullptr,
                         launches[i]);
        if (rc != RR_OK) return rc;
    }
    // Every launch has a scratch slot of its own, so the stream holds one reset (if anything needs one), the
    // read kernels back to back, and one finish for all of them; then the host waits once.
    std::vector<u32> tickets_per_unit(n_items), ticket_mode(n_items), reset_bits(n_items);
    for (u32 i = 0; i < n_items; ++i) {
        tickets_per_unit[i] = launches[i].tickets_per_unit;
        ticket_mode[i] = launches[i].p.ticket_mode;
        reset_bits[i] = launches[i].reset_bits;
    }
    BatchSlots slots;
    rc = prepare_batch(st, n_items, tickets_per_unit.data(), ticket_mode.data(), reset_bits.data(), stream, slots);
    if (rc != RR_OK) return rc;
    auto queue_all = [&]() -> int {
        for (u32 i = 0; i < n_items; ++i) {
            Launch &ln = launches[i];
            ln.p.scratch = st.batch_scratch + i;
            void *args[] = {(void *)&ln.p};
            // the two events take the start and the end time of this dispatch itself: no marker packets between
            // one read kernel and the next (the host work this costs, 17 us a launch, runs ahead of the device here)
            HIP_TRY(hipExtLaunchKernel(ln.kernel, dim3(ln.grid), dim3(plans[i].block), args, 0, stream,
                                       st.batch_ev[2 * i], st.batch_ev[2 * i + 1], 0));
        }
        return finish_batch(st, n_items, slots, stream);
    };
    rc = queue_all();
    if (rc != RR_OK) {
        (void)hipStreamSynchronize(stream);  // the slots stay marked dirty
        return rc;
    }
    st.tables_valid = true;
    st.flat_tables_ready = true;
    for (u32 i = 0; i < n_items; ++i) {
        const ResultHead &h = st.head[i];
        float ms = 0.f;
        HIP_TRY(hipEventElapsedTime(&ms, st.batch_ev[2 * i], st.batch_ev[2 * i + 1]));
        rr_result_t &r = results[i];
        r.launches = 1;
        r.kernel_ms_event = ms;
        r.checksum = h.checksum;
        r.waves_run = h.waves_run;
        if (h.waves_run && h.t_max >= h.t_min) r.kernel_ms_device = (double)(h.t_max - h.t_min) / (double)st.wall_khz;
        if (launches[i].p.ticket_mode && h.unfinished)
            return fail(RR_EPLACE, "item %u: %u compute units' shares still have unclaimed tickets after its one launch",
                        i, h.unfinished);
    }
    memcpy(out, results.data(), n_items * sizeof(rr_result_t));
    return RR_OK;
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
    // the zone-phased kernel knows no excluded compute units: its waves would run everywhere and steal the targets' work
    if (opts && (opts->zone_bytes || opts->zone_of_window || opts->phase_ticks))
        return fail(RR_EINVAL, "a pinned run cannot be zone-phased");
    // validate everything else before touching the device (map filled in below); a pinned run is a ticketed one
    rr_launch_opts_t ticketed;
    memset(&ticketed, 0, sizeof ticketed);
    if (opts) ticketed = *opts;
    ticketed.mode = RR_MODE_TICKET;
    if (opts && opts->mode == RR_MODE_STREAM) return fail(RR_EINVAL, "a pinned run cannot use stream mode");
    opts = &ticketed;
    Plan pl;
    int rc = make_plan(region, region_bytes, 128, 32, n_reads, iters_per_wave, nullptr, opts, out, pl);
    if (rc != RR_OK) return rc;
    u32 n_cus = 0;
    {
        std::lock_guard<std::mutex> lock(g_mutex);
        DeviceState *st = nullptr;
        rc = get_state((hipStream_t)hip_stream, &st);
        if (rc != RR_OK) return rc;
        n_cus = st->n_cus;
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
    // A region of more than the second-level translation reach plus one window: divided between the halves of the XCDs
    // like a plain read (RR_SPLIT_*), the region as up to 64 windows of a power-of-two number of lines.
    {
        u32 shift = 0;
        while ((64ull << shift) < pl.n_lines) shift++;
        const u64 window_bytes = ((u64)1 << shift) * line_bytes;
        const u32 n_win = (u32)((pl.n_lines + ((u64)1 << shift) - 1) >> shift);
        const u32 n_xcds = count_xcds(*st), half = n_xcds / 2;
        u64 incl[2];
        if (region_bytes >= kSecondLevelReachBytes + window_bytes && n_xcds % 2 == 0 && (half & (half - 1)) == 0 &&
            grid % n_xcds == 0 && divide_windows(n_win, (u32)std::min<u64>(64, kSecondLevelReachBytes / window_bytes), true, incl)) {
            p.split_half = half;
            p.window_shift = shift;
            p.split_incl[0] = incl[0];
            p.split_incl[1] = incl[1];
        }
    }
    rc = begin_cells(*st, stream);
    if (rc != RR_OK) return rc;
    void *args[] = {(void *)&p};
    HIP_TRY(hipEventRecord(st->ev0, stream));
    HIP_TRY(hipLaunchKernel(kernel, dim3((u32)grid), dim3(256), args, 0, stream));
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
