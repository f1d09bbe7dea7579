// Zone-phased variants of the random line read: rand_read_phased_kernel (items
// binned into LDS lists, handed out by tickets or walked through flat) and, at
// the end of this file, rand_read_zone_stream_kernel (the default: the stream
// kernel's way of working with a filter in front of the loads).
//
// On the MI355X the read rate drops when lines from different 96 GiB thirds of
// the memory are in flight at the same time, whoever issues them; a window per
// compute group (the paper's remedy, Sec. 2.4) does not help, a window per
// *phase* does.  These kernels read exactly the lines of rand_read_kernel (same
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

// Zone by zone as one uninterrupted stream of loads per wave (the stream kernel's way of working, see
// rand_read_stream_kernel, applied to the zone order).
//
// Every workgroup owns a contiguous range of units and goes through its tickets zone-major -- ticket = (zone *
// units + unit) * chunks + chunk, handed to its waves from a counter in LDS.  The workgroups have equal ranges and
// are not synchronised; they advance through the zones together because their work is statistically the same.
// A wave is a producer and a consumer in one loop:
//   * producing: 64 lanes evaluate 64 iterations of one logical wave of the ticket, those whose line lies in the
//     ticket's zone are appended (ballot, mbcnt) to the wave's own circular queue in LDS;
//   * consuming: as soon as the queue holds a batch (16 load instructions' worth: 32 lines when two logical
//     waves share a wavefront), each lane pops the entry its 16-lane row will broadcast, and the usual 16 steps
//     "add the oldest slot of the ring, refill it with a new load" follow.
// Which logical wave a line came from does not matter once it is in the queue -- the checksum is a plain sum -- so
// the two halves of a wavefront simply take alternate entries, and nothing is padded.  The ring is never drained
// between tickets or zones.  At the very end a wave fills its last batch up with entries for line 0 and
// afterwards subtracts what those extra reads added (every lane knows its own words of line 0).
// Needs whole units and chunks of a multiple of 64 iterations that divide the iterations of a wave.
constexpr u32 kZoneQueue = 128;  // queue entries per wave: a batch (32) plus one producer step (64), rounded up

template <int LANES, int WDW, int U, int NT>
__global__ void __launch_bounds__(256) rand_read_zone_stream_kernel(const ReadParams p) {
    typedef typename Vec<WDW>::type V;
    constexpr u32 LPW = 64 / LANES;
    constexpr int ITB = 16;                 // load instructions per batch: DPP row broadcast
    constexpr u32 kBatch = ITB * LPW;       // queue entries a batch consumes
    static_assert(ITB % U == 0, "ring must divide the batch");
    static_assert(kBatch + 64 <= kZoneQueue, "queue too small");
    __shared__ u32 next_ticket;
    __shared__ u32 queues[4][kZoneQueue];
    const u32 lane = threadIdx.x & 63;
    const u32 half = (LANES == 32) ? (lane >> 5) : 0;
    const u32 sub_bytes = (lane & (LANES - 1)) * (WDW * 4);
    const u32 launch_index = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    u32 *queue = queues[threadIdx.x >> 6];
    const u32 cpw = p.chunks_per_wave;
    const u64 units_total = p.quota / LPW;
    const u32 u_begin = (u32)(units_total * blockIdx.x / gridDim.x);
    const u32 n_units = (u32)(units_total * (blockIdx.x + 1) / gridDim.x) - u_begin;
    // With the split on, the workgroup also goes through the units of its partner in the other half of the XCDs, and
    // reads of its own units only what its half may read, of the partner's only what the partner's half may not.
    u32 pu_begin = 0, pn_units = 0;
    u64 incl = ~0ull, partner_incl = ~0ull;
    if (p.split_half) {
        const u32 partner = blockIdx.x ^ p.split_half;
        pu_begin = (u32)(units_total * partner / gridDim.x);
        pn_units = (u32)(units_total * (partner + 1) / gridDim.x) - pu_begin;
        const u32 half = (blockIdx.x / p.split_half) & 1u;
        incl = p.split_incl[half];
        partner_incl = p.split_incl[half ^ 1u];  // what the partner leaves out lies inside incl
    }
    const u32 own_tickets = n_units * cpw;
    const u32 per_zone = own_tickets + pn_units * cpw;  // tickets of this workgroup per zone
    const u32 n_tickets = per_zone * p.n_zones;
    if (threadIdx.x == 0) next_ticket = 0;
    __syncthreads();
    auto claim = [&]() -> u32 {
        u32 t = 0;
        if (lane == 0) t = atomicAdd(&next_ticket, 1u);
        return __builtin_amdgcn_readfirstlane(t);
    };
    if (n_tickets == 0) return;
    const u32 steps_per_wave = p.chunk_iters / 64;   // producer steps per logical wave of a ticket
    const u32 steps_per_ticket = steps_per_wave * LPW;
    const u64 t0 = clock_ticks();

    // producer state (all wave-uniform): the ticket's zone, the seeds of its logical waves, its first iteration
    u64 zone_mask = 0, seed_lo = 0, seed_hi = 0;
    u32 it_base = 0;
    u32 step = steps_per_ticket;  // "ticket used up": the first refill claims one
    u32 head = 0, tail = 0;       // queue positions (not wrapped)
    bool more = true, worked = false;

    V ring[U];
#pragma unroll
    for (int j = 0; j < U; ++j) ring[j] = V(0);
    Acc acc{0u, 0u};
    u32 pads = 0;  // entries for line 0 that this lane's half of the wavefront read at the end

    for (;;) {
        while (tail - head < kBatch && more) {
            if (step == steps_per_ticket) {
                const u32 t = claim();
                if (t >= n_tickets) {
                    more = false;
                    break;
                }
                worked = true;
                const u32 z = t / per_zone;
                u32 rest = t - z * per_zone;
                u32 first_unit = u_begin;
                zone_mask = p.zone_mask[z];
                // own tickets and the partner's in turn while both last: a partner's ticket yields few lines per
                // draw, and the waves of a workgroup should not all be busy with such tickets at the same time
                const u32 paired = 2 * (own_tickets < per_zone - own_tickets ? own_tickets : per_zone - own_tickets);
                bool partners;
                if (rest < paired) {
                    partners = rest & 1u;
                    rest >>= 1;
                } else {
                    partners = own_tickets < per_zone - own_tickets;
                    rest -= paired / 2;
                }
                if (partners) {  // a ticket of the partner's units: what the partner leaves out
                    first_unit = pu_begin;
                    zone_mask &= ~partner_incl;
                } else {
                    zone_mask &= incl;
                }
                if (zone_mask == 0) continue;  // nothing of this zone is for this ticket: take the next one
                const u32 unit = rest / cpw;
                const u32 chunk = rest - unit * cpw;
                const u64 w = p.first_wave + (u64)(first_unit + unit) * LPW;
                seed_lo = mix64(p.read_seed + (w + 1) * kGamma);
                if (LPW == 2) seed_hi = mix64(p.read_seed + (w + 2) * kGamma);
                it_base = chunk * p.chunk_iters;
                step = 0;
            }
            // one producer step: 64 iterations of one logical wave
            const bool upper = (LPW == 2) && step >= steps_per_wave;
            const u64 seed = upper ? seed_hi : seed_lo;
            const u32 it = it_base + (upper ? step - steps_per_wave : step) * 64 + lane;
            const u32 line = reduce_to_line(mix64(seed + ((u64)it + 1) * kGamma), p.red);
            const bool keep = (zone_mask >> (line >> p.zone_shift)) & 1ull;
            const unsigned long long m = __ballot(keep);
            const u32 below = __builtin_amdgcn_mbcnt_hi((u32)(m >> 32), __builtin_amdgcn_mbcnt_lo((u32)m, 0u));
            if (keep) queue[(tail + below) & (kZoneQueue - 1)] = line;
            tail += (u32)__builtin_popcountll(m);
            ++step;
        }
        const u32 avail = tail - head;
        if (avail < kBatch) {  // nothing more will come: fill the last batch up, or stop
            if (avail == 0) break;
            if (lane < kBatch - avail) queue[(tail + lane) & (kZoneQueue - 1)] = 0u;
            // entry k of a batch is read by half k % LPW: count this lane's half among positions avail .. kBatch-1
            const u32 upto = (kBatch + LPW - 1 - half) / LPW, before = (avail + LPW - 1 - half) / LPW;
            pads += upto - before;
            tail = head + kBatch;
        }
        __builtin_amdgcn_wave_barrier();
        // pop a batch: the lane takes the entry that its row broadcasts from it
        const u32 entry = queue[(head + LPW * (lane & (ITB - 1)) + half) & (kZoneQueue - 1)];
        head += kBatch;
        const u64 cur = (u64)p.region + ((u64)entry << p.log2_line);
        const u32 clo = (u32)cur, chi = (u32)(cur >> 32);
        __builtin_amdgcn_sched_barrier(0);
        static_for<0, ITB>([&](auto kc) {
            constexpr int K = decltype(kc)::value;
            acc.add(ring[K % U]);  // oldest load of the ring: waits until only U-1 are outstanding
            const u64 line_addr = bcast_addr<LANES, BC_DPP, K>(clo, chi, lane, 0u);
            ring[K % U] = load_line_part<NT, V>(line_addr | sub_bytes);
            __builtin_amdgcn_sched_barrier(0);  // keep issue order: consume slot, refill slot
        });
    }
    if (!worked) return;
#pragma unroll
    for (int j = 0; j < U; ++j) acc.add(ring[j]);
    u64 mine = acc.value();
    if (pads) {  // take the extra reads of line 0 out again
        Acc one{0u, 0u};
        one.add(load_line_part<0, V>((u64)p.region + sub_bytes));
        mine -= (u64)pads * one.value();
    }
    const u64 total = wave_sum(mine);
    const u64 t1 = clock_ticks();
    if (lane == 0) {
        Cell *c = &p.scratch->cells[launch_index & (kNumCells - 1)];
        atomicAdd(&c->sum, total);
        atomicMin(&c->t_min, t0);
        atomicMax(&c->t_max, t1);
        atomicAdd(&c->waves, 1u);
        if (p.locate) atomicAdd(&p.scratch->cu_waves[p.tables->dense_of_key[cu_key()]], 1u);  // per-CU counts wanted
    }
}

// Host-side handle of the phased kernel for a line shape, or null.
kernel_handle find_phased_kernel(u32 lanes, u32 wdw, u32 nt);
// The same for the zone-by-zone stream kernel (ring depth 16, or 8 for 16-byte lanes).
kernel_handle find_zone_stream_kernel(u32 lanes, u32 wdw, u32 nt);

}  // namespace rr
