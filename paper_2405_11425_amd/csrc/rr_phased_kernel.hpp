// Zone-phased variant of the random line read.
//
// On the MI355X the read rate drops when lines from different 96 GiB thirds of
// the memory are in flight at the same time, whoever issues them; a window per
// compute group (the paper's remedy, Sec. 2.4) does not help, a window per
// *phase* does.  This kernel reads exactly the lines of rand_read_kernel (same
// draws, same checksum) in a different order: the region is cut into at most
// 64 windows of a power-of-two number of lines, every window belongs to one
// zone (the zones need not be contiguous: how the physical zones appear in an
// allocation differs from one allocation to the next), and the work is done
// zone by zone.
//
// A work item is (zone, unit, chunk): of the chunk's iterations only those whose
// line lies in the zone are read.  The wave regenerates the chunk's line
// indices lane-parallel, keeps those inside the zone and appends them to a list
// in LDS (ballot + mbcnt give each kept lane its slot), then walks the dense
// list with the usual ring of U loads in flight.  Lists of the two logical
// waves of a wavefront differ in length; the shorter one pads with loads of the
// region's first line (an L2 hit) whose data is discarded, so that every wave
// issues a branch-free, countable load stream.
//
// Order of the work items:
//   flat launch   : each wave owns one unit and runs zone 0 of all its chunks,
//                   then zone 1, ...  Waves are not synchronised, and since the
//                   hardware serves the oldest workgroups of a CU first (they
//                   run several times faster than the youngest, see
//                   phase_ticks), the phases of different waves overlap widely.
//   ticket launch : every CU hands out the items of its share zone-major --
//                   ticket = (zone * units + unit) * chunks + chunk -- so that
//                   whatever the speed of the individual waves, the items in
//                   progress at any time lie around one point of that order:
//                   the whole device works on one zone, then on the next.
#pragma once
#include "rr_read_kernel.hpp"

namespace rr {

// Iterations binned per work item.  An item ends with the load ring drained, so small items are expensive
// (512: 6.40 TB/s over three zones, 1024: 6.59); 1024 is what fits: 16 waves per CU x 2 lists x 4 KB = 132 KB of LDS.
constexpr u32 kPhaseChunk = 1024;
constexpr u32 kPhasePad = 32;     // list slack so that the last group of the ring may read past the end

// One work item: the lines of iterations [it0, it0 + n_it) of this lane's logical wave that fall into the
// windows named by zone_mask.  Adds the words read to acc.
template <int LANES, int WDW, int U, int NT>
__device__ __forceinline__ void read_chunk_in_zone(const ReadParams &p, u32 *my_list, u64 wave_seed, u64 lane_base,
                                                   u32 it0, u32 n_it, u64 zone_mask, u32 lane, Acc &acc) {
    typedef typename Vec<WDW>::type V;
    const u32 half = (LANES == 32) ? (lane >> 5) : 0;
    const u32 sub = lane & (LANES - 1);
    // (1) bin: keep the iterations of this chunk whose line lies in the zone
    u32 count = 0;
    for (u32 r = 0; r < n_it; r += LANES) {
        const u32 it = it0 + r + sub;
        const u64 h = mix64(wave_seed + ((u64)it + 1) * kGamma);
        const u32 line = reduce_to_line(h, p.red);
        const bool keep = (r + sub < n_it) && ((zone_mask >> (line >> p.zone_shift)) & 1ull);
        const unsigned long long m = __ballot(keep);
        const u32 m_lo = (u32)m, m_hi = (u32)(m >> 32);
        u32 below, kept;
        if (LANES == 32) {
            below = half ? __builtin_amdgcn_mbcnt_hi(m_hi, 0u) : __builtin_amdgcn_mbcnt_lo(m_lo, 0u);
            kept = __builtin_popcount(half ? m_hi : m_lo);
        } else {
            below = __builtin_amdgcn_mbcnt_hi(m_hi, __builtin_amdgcn_mbcnt_lo(m_lo, 0u));
            kept = __builtin_popcountll(m);
        }
        if (keep) my_list[count + below] = line;
        count += kept;
    }
    // (2) read the listed lines, U loads in flight
    u32 n_max = count;
    if (LANES == 32)
        n_max = max(__builtin_amdgcn_readlane(count, 0), __builtin_amdgcn_readlane(count, 32));
    else
        n_max = __builtin_amdgcn_readfirstlane(count);
    if (n_max == 0) return;
    V ring[U];
    // slot Q of the ring holds list entry k0 + Q of the group issued last
    auto issue = [&](auto qc, u32 k0) {
        constexpr int Q = decltype(qc)::value;
        const u32 k = k0 + Q;
        const u32 listed = my_list[k];               // k < kPhaseChunk + kPhasePad always
        const u32 line = (k < count) ? listed : 0u;  // padding reads the region's first line
        ring[Q] = load_line_part<NT, V>(lane_base + ((u64)line << p.log2_line));
    };
    auto consume = [&](auto qc, u32 k0) {
        constexpr int Q = decltype(qc)::value;
        if (k0 + Q < count) acc.add(ring[Q]);  // data of padding loads is dropped
    };
    static_for<0, U>([&](auto qc) { issue(qc, 0u); });
    __builtin_amdgcn_sched_barrier(0);
    u32 k0 = U;
    for (; k0 < n_max; k0 += U) {
        static_for<0, U>([&](auto qc) {
            consume(qc, k0 - U);
            issue(qc, k0);
            __builtin_amdgcn_sched_barrier(0);  // keep issue order: consume slot, refill slot
        });
    }
    static_for<0, U>([&](auto qc) { consume(qc, k0 - U); });
}

template <int LANES, int WDW, int U, int NT>
__global__ void __launch_bounds__(256) rand_read_phased_kernel(const ReadParams p) {
    constexpr u32 LPW = 64 / LANES;
    constexpr u32 kNone = 0xFFFFFFFFu;
    __shared__ u32 lists[4][LPW][kPhaseChunk + kPhasePad];
    const u32 lane = threadIdx.x & 63;
    const u32 half = (LANES == 32) ? (lane >> 5) : 0;
    const u32 sub = lane & (LANES - 1);
    Scratch *s = p.scratch;
    const Tables *tb = p.tables;
    const u32 launch_index = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    u32 *my_list = lists[threadIdx.x >> 6][half];
    const u64 lane_base = (u64)p.region + sub * (WDW * 4);
    const u32 cpw = p.chunks_per_wave;

    // seed of the logical wave this lane works for in `unit`; an odd quota leaves the last upper half idle
    auto lane_seed = [&](u32 unit, bool &valid) -> u64 {
        const u64 j0 = (u64)unit * LPW;
        u64 j = j0 + half;
        valid = j < p.quota;
        if (!valid) j = j0;
        return mix64(p.read_seed + (p.first_wave + j + 1) * kGamma);
    };
    auto zone_item = [&](u32 z, u64 wave_seed, u32 chunk, Acc &acc) {
        const u32 it0 = chunk * p.chunk_iters;
        const u32 n_it = min(p.chunk_iters, p.iters - it0);
        read_chunk_in_zone<LANES, WDW, U, NT>(p, my_list, wave_seed, lane_base, it0, n_it, p.zone_mask[z], lane, acc);
    };

    Acc acc{0u, 0u}, part{0u, 0u};
    u64 total_lane = 0;
    u64 t0 = 0;
    bool worked = false;
    if (!p.ticket_mode) {
        if ((u64)launch_index * LPW >= p.quota) return;
        worked = true;
        t0 = clock_ticks();
        bool valid;
        const u64 wave_seed = lane_seed(launch_index, valid);
        for (u32 z = 0; z < p.n_zones; ++z) {
            for (u32 chunk = 0; chunk < cpw; ++chunk) zone_item(z, wave_seed, chunk, acc);
            if (p.phase_ticks && lane == 0) p.phase_ticks[(u64)launch_index * p.n_zones + z] = clock_ticks();
        }
        total_lane = valid ? acc.value() : 0;
    } else {
        // zone-major tickets from this CU's share, then from the other CUs' shares (as in rand_read_kernel)
        const u32 dense = tb->dense_of_key[cu_key()];
        auto claim = [&](u32 cu) -> u32 {
            u32 t = 0;
            if (lane == 0) t = atomicAdd(&s->tickets[cu * kTicketStride], 1u);
            return __builtin_amdgcn_readfirstlane(t);
        };
        const u32 g_count = tb->group_begin[1];  // one group: all CUs
        const u32 my_pos = tb->cu_pos[dense];
        u32 scan_base = 0, cand = 0;
        unsigned long long open_mask = 0;
        auto next_victim = [&]() -> u32 {
            for (;;) {
                if (open_mask) {
                    const u32 l = (u32)__builtin_ctzll(open_mask);
                    open_mask &= open_mask - 1;
                    return __builtin_amdgcn_readlane(cand, l);
                }
                if (scan_base + 1 >= g_count) return kNone;
                const u32 pos = scan_base + lane;
                bool open = false;
                if (pos + 1 < g_count) {
                    u32 ring_pos = my_pos + 1 + pos;
                    if (ring_pos >= g_count) ring_pos -= g_count;
                    cand = tb->group_cus[ring_pos];
                    const u32 taken = __hip_atomic_load(&s->tickets[cand * kTicketStride], __ATOMIC_RELAXED,
                                                        __HIP_MEMORY_SCOPE_AGENT);
                    open = taken < tb->cu_unit_count[cand] * cpw * p.n_zones;
                }
                open_mask = __ballot(open);
                scan_base += 64;
            }
        };
        u32 cur = dense;
        u32 units = tb->cu_unit_count[cur], unit_begin = tb->cu_unit_begin[cur];
        u32 ticket = claim(cur);
        for (;;) {
            if (ticket >= units * cpw * p.n_zones) {
                cur = next_victim();
                if (cur == kNone) break;
                units = tb->cu_unit_count[cur];
                unit_begin = tb->cu_unit_begin[cur];
                ticket = claim(cur);
                continue;
            }
            const u32 this_ticket = ticket;
            ticket = claim(cur);  // next ticket: its latency hides behind this item's loads
            if (!worked) {
                worked = true;
                t0 = clock_ticks();
            }
            const u32 z = this_ticket / (units * cpw);
            const u32 rest = this_ticket - z * (units * cpw);
            const u32 unit = rest / cpw;
            const u32 chunk = rest - unit * cpw;
            bool valid;
            const u64 wave_seed = lane_seed(unit_begin + unit, valid);
            part = Acc{0u, 0u};
            zone_item(z, wave_seed, chunk, part);
            total_lane += valid ? part.value() : 0;
        }
    }
    if (!worked) return;
    const u64 total = wave_sum(total_lane);
    const u64 t1 = clock_ticks();
    if (lane == 0) {
        Cell *c = &s->cells[launch_index & (kNumCells - 1)];
        atomicAdd(&c->sum, total);
        atomicMin(&c->t_min, t0);
        atomicMax(&c->t_max, t1);
        atomicAdd(&c->waves, 1u);
    }
}

// Host-side handle of the phased kernel for a line shape, or null.
kernel_handle find_phased_kernel(u32 lanes, u32 wdw, u32 nt);

}  // namespace rr
