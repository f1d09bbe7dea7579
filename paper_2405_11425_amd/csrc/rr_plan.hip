// Planning of a read call: validation of the arguments (make_plan: everything that can be rejected without the
// device), the per-call lookup tables (prepare_tables) and the launch itself -- kernel, grid, parameters
// (make_launch).  Used by the entry points in rr_api.hip.
#include <algorithm>
#include <cstdio>
#include <cstring>

#include "rr_plan.hpp"
#include "rr_phased_kernel.hpp"

namespace rr {


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

constexpr u32 kTicketWavesPerCu = 8;   // default grid of the plain ticketed kernel, in wavefronts per compute unit
constexpr u32 kStreamBytesPerCu = 32768;  // default grid of the stream kernels: workgroups per compute unit so that this much is in flight

thread_local char g_last_kernel[96] = "";

bool divide_windows(u32 n_win, u32 reach, bool in_turn, u64 incl[2]) {
    if (!(n_win > reach && reach >= 1 && n_win <= 2 * reach && n_win <= 64)) return false;
    const u64 all = n_win == 64 ? ~0ull : ((1ull << n_win) - 1);
    incl[0] = incl[1] = all;
    for (u32 k = 0; k + reach < n_win; ++k) {
        // In turn: both halves get the same extra work.  Otherwise one half gives up all the upper windows, the other
        // all the lower ones -- with several zones the extra work of a half then lies in one zone instead of two, and
        // every draw is evaluated four times instead of five (measured over 280 GiB in three zones: 6.5 TB/s against 6.0).
        const u32 h = in_turn ? (k & 1u) : 0u;
        incl[h] &= ~(1ull << (k + reach));
        incl[h ^ 1u] &= ~(1ull << k);
    }
    return true;
}

u32 count_xcds(const DeviceState &st) {
    u32 n = 1;
    for (u32 c = 0; c < st.n_cus; ++c) n = std::max(n, st.cus[c].xcc + 1u);
    return n;
}

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
        if (opts->mode > RR_MODE_STREAM) return fail(RR_EINVAL, "unknown mode value");
        pl.mode = opts->mode;
        pl.grid_blocks = opts->grid_blocks;
        if (opts->chunk_iters % 64 != 0) return fail(RR_EINVAL, "chunk_iters must be a multiple of 64");
        if (opts->xcd_split > RR_SPLIT_OFF) return fail(RR_EINVAL, "xcd_split must be 0, 1 or 2");
        pl.chunk_iters = opts->chunk_iters;
        if (opts->first_wave % pl.G != 0) return fail(RR_EINVAL, "first_wave must be a multiple of n_groups");
        pl.first_wave = opts->first_wave;
        const bool zoned = opts->zone_bytes || opts->zone_of_window;
        if (opts->zone_descending > 1) return fail(RR_EINVAL, "zone_descending must be 0 or 1");
        if (opts->zone_descending && !zoned) return fail(RR_EINVAL, "zone_descending needs zone_bytes or zone_of_window");
        if (opts->phase_ticks && (!zoned || opts->mode != RR_MODE_FLAT))
            return fail(RR_EINVAL, "phase_ticks needs zones and a flat launch");
        if (zoned) {
            if (opts->zone_bytes && opts->zone_of_window)
                return fail(RR_EINVAL, "give either zone_bytes or zone_of_window, not both");
            if (wm) return fail(RR_EINVAL, "zone-phased reads cannot be combined with a window map");
            if (opts->chunk_iters && opts->mode != RR_MODE_STREAM)
                return fail(RR_EINVAL, "zone-phased reads take chunk_iters in stream mode only");
            if (opts->placement_out || (opts->cu_waves_out && opts->mode != RR_MODE_AUTO && opts->mode != RR_MODE_STREAM))
                return fail(RR_EINVAL, "zone-phased reads do not record placement (per-CU counts: in stream mode)");
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
            if (opts->zone_descending) std::reverse(pl.zone_mask, pl.zone_mask + pl.n_zones);
        }
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
    // A plain read over more than the second-level translation cache of an XCD covers: look at the region as one zone
    // of up to 64 windows, so that the zone stream kernel can divide it between the halves of the XCDs (see
    // RR_SPLIT_*).  Where that kernel does not apply, the read stays what it was.
    // By default only from one whole window beyond the reach on: up to there the division costs more than the few
    // displaced pages do (measured with 8 GiB windows: 5.8-5.9 TB/s against 6.2-6.1 at 258 and 260 GiB, 6.23 against
    // 5.56 at 264 GiB).
    const u32 want_split = opts ? opts->xcd_split : RR_SPLIT_DEFAULT;
    bool implicit_zone = false;
    u32 window_shift = 0;
    while ((64ull << window_shift) < pl.n_lines) window_shift++;
    const u64 implicit_window_bytes = ((u64)1 << window_shift) * line_bytes;
    if (!pl.n_zones && !wm && (pl.mode == RR_MODE_AUTO || pl.mode == RR_MODE_STREAM) && !(opts && opts->block_threads && opts->block_threads != 256) &&
        (want_split == RR_SPLIT_ON ||
         (want_split == RR_SPLIT_DEFAULT && region_bytes >= kSecondLevelReachBytes + implicit_window_bytes))) {
        pl.zone_shift = window_shift;
        const u32 n_win = (u32)((pl.n_lines + ((u64)1 << pl.zone_shift) - 1) >> pl.zone_shift);
        pl.zone_mask[0] = n_win == 64 ? ~0ull : ((1ull << n_win) - 1);
        pl.n_zones = 1;
        implicit_zone = true;
    }
    // The stream kernel serves launches without a map, in whole units, whose chunks are a multiple of 16 iterations
    // that divides the iterations of a wave.
    // (zone by zone: a multiple of 64, since a producer step evaluates 64 iterations of one logical wave).
    const u32 lpw = 64 / pl.lanes;
    const char *no_stream = nullptr;
    u32 stream_chunk = 0;
    kernel_handle stream_kernel = nullptr;
    for (;;) {
        const u32 chunk_unit = pl.n_zones ? 64u : 16u;
        const u32 block = pl.n_zones ? 256u : pl.block;  // the zone kernels are laid out for four waves per workgroup
        no_stream = nullptr;
        stream_chunk = pl.chunk_iters;
        if (!stream_chunk)
            for (stream_chunk = 256; stream_chunk > chunk_unit && iters % stream_chunk != 0;) stream_chunk /= 2;
        stream_kernel = pl.n_zones ? find_zone_stream_kernel(pl.lanes, pl.wdw, pl.nt)
                                   : find_stream_kernel(pl.lanes, pl.wdw, pl.unroll, pl.nt);
        if (wm) no_stream = "a window map";
        else if (opts && opts->phase_ticks) no_stream = "phase_ticks";
        else if (opts && opts->placement_out) no_stream = "a placement log";
        else if (pl.bcast != RR_BCAST_DPP) no_stream = "a broadcast other than DPP";
        else if (pl.W % lpw != 0) no_stream = "an odd number of 32-lane logical waves";
        else if (iters % stream_chunk != 0 || stream_chunk % chunk_unit != 0)
            no_stream = pl.n_zones ? "chunks that are not a multiple of 64 iterations dividing iters_per_wave"
                                   : "chunks that are not a multiple of 16 iterations dividing iters_per_wave";
        else if (block != 256) no_stream = "workgroups of other than 256 threads";
        else if (!stream_kernel) no_stream = "this ring depth";
        else if ((pl.W / lpw) * (u64)(iters / stream_chunk) * (pl.n_zones ? pl.n_zones : 1u) >= (1ull << 31))
            no_stream = "2^31 tickets or more";
        if (!(implicit_zone && no_stream)) break;
        implicit_zone = false;  // not for the zone stream kernel: a plain read after all
        pl.n_zones = 0;
        pl.zone_shift = 0;
        pl.zone_mask[0] = 0;
    }
    if (pl.n_zones) pl.block = 256;
    if (pl.mode == RR_MODE_STREAM && no_stream) return fail(RR_EINVAL, "stream mode does not work with %s", no_stream);
    // without the stream kernel, zone-phased reads line their phases up only when the work is handed out zone-major
    // by tickets
    if (pl.mode == RR_MODE_AUTO)
        pl.mode = needs_tickets ? RR_MODE_TICKET : !no_stream ? RR_MODE_STREAM : pl.n_zones ? RR_MODE_TICKET : RR_MODE_FLAT;
    if (pl.n_zones && pl.mode != RR_MODE_STREAM && opts && opts->cu_waves_out)
        return fail(RR_EINVAL, "per-CU counts of a zone-phased read need stream mode, which does not work with %s", no_stream);
    // The split between the halves of the XCDs: windows k and k + reach (in windows) displace each other in an XCD's
    // second-level translation cache; half (k mod 2) leaves out the upper one, the other half the lower one.  By
    // default for a single zone only: with several zones the further evaluations of every draw cost about what the
    // translations they save do (measured over 280 GiB: 6.5 TB/s with the split, 6.1 without, 6.6 without and the
    // direction of the zones alternating; a single zone: 6.25 with it, 4.0 without).
    if (pl.n_zones && pl.mode == RR_MODE_STREAM && (want_split == RR_SPLIT_ON || (want_split == RR_SPLIT_DEFAULT && pl.n_zones == 1))) {
        const u64 window_bytes = ((u64)1 << pl.zone_shift) * line_bytes;
        const u32 n_win = (u32)((pl.n_lines + ((u64)1 << pl.zone_shift) - 1) >> pl.zone_shift);
        u32 reach = (u32)std::min<u64>(64, kSecondLevelReachBytes / window_bytes);  // in windows; window sizes are powers of two
        if (want_split == RR_SPLIT_ON && n_win <= reach && n_win >= 2) reach = n_win - std::max(1u, n_win / 8);  // for tests
        if (divide_windows(n_win, reach, pl.n_zones == 1, pl.split_incl)) {
            pl.split = want_split;
        } else if (want_split == RR_SPLIT_ON) {
            return fail(RR_EINVAL, "xcd_split needs a region of 2 to 64 zone windows");
        }
    } else if (want_split == RR_SPLIT_ON) {
        return fail(RR_EINVAL, "xcd_split is for reads that the zone stream kernel can take (stream mode: %s)", no_stream ? no_stream : "not chosen");
    }
    if (pl.mode == RR_MODE_STREAM) {
        pl.chunk_iters = stream_chunk;
        pl.kernel = stream_kernel;
    } else if (pl.n_zones) {
        if (!pl.family->find(pl.unroll, pl.bcast, pl.nt)) return fail(RR_EINVAL, "unroll %u is not built for this line shape", pl.unroll);
        pl.kernel = find_phased_kernel(pl.lanes, pl.wdw, pl.nt);
        if (!pl.kernel) return fail(RR_EINVAL, "no zone-phased kernel for this line shape");
    } else {
        pl.kernel = pl.family->find(pl.unroll, pl.bcast, pl.nt);
        if (!pl.kernel) return fail(RR_EINVAL, "unroll %u is not built for this line shape", pl.unroll);
    }
    return RR_OK;
}

// Workgroups of `block` threads of this kernel that one CU holds at a time, as the runtime computes it from the
// kernel's registers and LDS (the 8-per-SIMD wave limit if it cannot say).  Cached per (kernel, block).
u32 resident_blocks_per_cu(kernel_handle kernel, u32 block) {
    struct Entry {
        kernel_handle kernel;
        u32 block, blocks;
    };
    static Entry cache[256];  // guarded by g_mutex (run_plan holds it); a fixed table, so that a lookup allocates nothing
    static u32 n_cached = 0;
    for (u32 i = 0; i < n_cached; ++i)
        if (cache[i].kernel == kernel && cache[i].block == block) return cache[i].blocks;
    int n = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, kernel, (int)block, 0) != hipSuccess || n <= 0) {
        (void)hipGetLastError();
        n = (int)(32 / (block / 64));
    }
    if (n_cached < 256) cache[n_cached++] = Entry{kernel, block, (u32)n};
    return (u32)n;
}

// Lookup tables of one call: CU key -> group and dense id, group -> window, group -> its CUs, and each
// CU's share of its group's units.  Built in the pinned staging copy and uploaded only if they differ
// from what the device already holds.
int prepare_tables(DeviceState &st, const Plan &pl, const rr_window_map_t *wm, u64 units, u64 L_win,
                   hipStream_t stream) {
    const u32 n_cus = st.n_cus;
    Tables &tb = *st.tables_host;
    memset(&tb, 0, sizeof tb);
    for (u32 k = 0; k < kNumKeys; ++k) {
        tb.group_of_key[k] = kExcluded;
        tb.dense_of_key[k] = st.dense_of_key_host[k];
    }
    u32 cus_in_group[kMaxGroups] = {}, fill_pos[kMaxGroups] = {};
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


int make_launch(const Plan &pl, DeviceState &st, const void *region, uint32_t iters, const rr_window_map_t *wm,
                uint64_t read_seed, const rr_launch_opts_t *opts, u16 *placement, Launch &ln) {
    const bool has_map = wm != nullptr;
    const u32 n_cus = st.n_cus;
    const u32 lpw = 64 / pl.lanes;
    const u64 L_win = pl.n_lines / pl.n_windows;
    const u64 quota = pl.W / pl.G;
    const u64 units = (quota + lpw - 1) / lpw;  // per group
    ReadParams &p = ln.p;
    memset(&p, 0, sizeof p);
    p.region = (const char *)region;
    p.read_seed = read_seed;
    p.first_wave = pl.first_wave;
    p.quota = quota;
    p.iters = iters;
    // flat launches default to one hardware wave per whole logical wave (pair); ticketed ones to
    // chunks of 1024 iterations (shorter ones pay for draining the load ring at every chunk end)
    const bool phased = pl.n_zones > 0 && pl.mode != RR_MODE_STREAM;  // its chunks are what one pass through the LDS lists holds
    u32 chunk = phased ? kPhaseChunk : pl.chunk_iters ? pl.chunk_iters : (pl.mode == RR_MODE_TICKET ? 1024u : iters);
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
    p.placement = placement;
    const bool want_cu_waves = opts && opts->cu_waves_out;
    p.locate = (placement || want_cu_waves) ? 1u : 0u;
    p.phase_ticks = (opts && pl.n_zones) ? (u64 *)opts->phase_ticks : nullptr;

    const u32 waves_per_block = pl.block / 64;
    u64 grid;
    if (pl.mode == RR_MODE_STREAM) {
        // a few wavefronts per SIMD that never stop keep the memory system as busy as a full house (measured)
        // What counts is the data in flight: 32 KB per compute unit -- for 128-byte lines two workgroups of four
        // waves with 16 loads of two lines each -- is enough to keep the memory busy, and zone by zone more than that
        // only blurs the zones (256- and 512-byte lines over 256 GiB: 6.86 TB/s with one workgroup per CU, 6.72 with
        // two, 6.5-6.6 with four).
        const u32 ring = pl.n_zones ? (pl.wdw == 4 ? 8u : 16u) : pl.unroll;
        const u32 bytes_per_block = 4u * ring * lpw * (pl.lanes * pl.wdw * 4u);
        const u32 blocks_per_cu = std::max(1u, kStreamBytesPerCu / bytes_per_block);
        grid = pl.grid_blocks ? pl.grid_blocks : (u64)blocks_per_cu * n_cus;
    } else if (p.ticket_mode) {
        // As many workgroups as are resident at once: work-stealing finishes the job whatever the placement, and
        // every workgroup beyond that only starts when the work is done, scans all shares and leaves -- which
        // lengthens the kernel (measured 1-2 %).  Pinned runs need many more, most land on CUs that take no part.
        u32 blocks_per_cu = resident_blocks_per_cu(pl.kernel, pl.block);
        // The plain ticketed kernel does best with few waves: eight per compute unit keep the memory system as busy
        // as thirty-two do and finish more evenly (measured at 64 GiB: 6.85 TB/s with 8 waves per CU, 6.81 with 16,
        // 6.72 with 32; windowed launches at 256 GiB +2 %).  The zone-phased kernel drains its loads at every
        // item's end and needs what fits (16 waves per CU; with 8 it loses 6 %).
        if (!phased) blocks_per_cu = std::min(blocks_per_cu, std::max(1u, kTicketWavesPerCu / waves_per_block));
        if (pl.pinned) blocks_per_cu = (32 / waves_per_block) * 64u;
        grid = pl.grid_blocks ? pl.grid_blocks : (u64)blocks_per_cu * n_cus;
    } else {
        const u64 hw_waves = (pl.W + lpw - 1) / lpw * (phased ? 1u : p.chunks_per_wave);
        grid = (hw_waves + waves_per_block - 1) / waves_per_block;
    }
    if (grid == 0 || grid > 0x7FFFFFFFull) return fail(RR_EINVAL, "launch of %llu workgroups is out of range", grid);
    ln.grid = (u32)grid;
    u32 passes = 1;  // times a zone-phased stream launch goes through every unit
    if (pl.split != RR_SPLIT_OFF) {
        const u32 n_xcds = count_xcds(st);
        const u32 half = n_xcds / 2;
        const bool can = n_xcds >= 2 && n_xcds % 2 == 0 && (half & (half - 1)) == 0 && ln.grid % n_xcds == 0;
        if (can) {
            p.split_half = half;
            p.split_incl[0] = pl.split_incl[0];
            p.split_incl[1] = pl.split_incl[1];
            passes = 2;
        } else if (pl.split == RR_SPLIT_ON) {
            return fail(RR_EINVAL, "xcd_split needs a grid that is a multiple of the %u XCDs (an even number, half of it a power of two)", n_xcds);
        }
    }

    const u64 tickets_per_unit = (u64)p.chunks_per_wave * (phased ? pl.n_zones : 1u);
    if (passes > 1 && units * (u64)p.chunks_per_wave * pl.n_zones * passes >= (1ull << 31))
        return fail(RR_EINVAL, "too many tickets for a split launch");
    if (units * tickets_per_unit >= (1ull << 31))
        return fail(RR_EINVAL, "too many tickets per group (%llu)", units * tickets_per_unit);
    ln.tickets_per_unit = (u32)tickets_per_unit;
    // counters are needed by ticketed launches only
    ln.reset_bits = (p.ticket_mode ? 2u : 0u) | ((p.ticket_mode || p.locate) ? 4u : 0u);
    // the plain flat launch has a kernel of its own (fewer registers, 8 resident waves per SIMD instead of 7)
    ln.kernel = pl.kernel;
    const char *name = pl.mode == RR_MODE_STREAM ? (pl.n_zones ? "rand_read_zone_stream_kernel" : "rand_read_stream_kernel")
                       : phased                   ? "rand_read_phased_kernel"
                                                  : "rand_read_kernel";
    if (pl.mode == RR_MODE_FLAT && !phased && !has_map && !p.locate) {
        kernel_handle flat = find_flat_kernel(pl.lanes, pl.wdw, pl.unroll, pl.bcast, pl.nt);
        if (flat) {
            ln.kernel = flat;
            name = "rand_read_flat_kernel";
        }
    }
    // template arguments as the kernels declare them: lanes per line, dwords per lane, ring depth, [broadcast,] cache hint
    const u32 ring = pl.n_zones ? (pl.mode == RR_MODE_STREAM ? (pl.wdw == 4 ? 8u : 16u) : 32u / pl.wdw) : pl.unroll;
    if (pl.mode == RR_MODE_STREAM || phased)
        snprintf(g_last_kernel, sizeof g_last_kernel, "%s<%u, %u, %u, %u>", name, pl.lanes, pl.wdw, ring, pl.nt);
    else
        snprintf(g_last_kernel, sizeof g_last_kernel, "%s<%u, %u, %u, %u, %u>", name, pl.lanes, pl.wdw, ring, pl.bcast, pl.nt);
    return RR_OK;
}

}  // namespace rr
