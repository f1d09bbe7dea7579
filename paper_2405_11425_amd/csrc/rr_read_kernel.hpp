// The random cache-line read kernel (paper Sec. 2.1: every warp reads random
// coalesced lines in a memory region; Sec. 2.4: per-group windows; Sec. 2.2:
// pinned to chosen compute units), written for 64-lane CDNA4 wavefronts.
//
// Layout of the work inside one hardware wave
//   LANES = 32 : the wave carries two logical waves (lanes 0-31 and 32-63), each
//                reading its own line per iteration, so one global_load touches
//                two independent lines.
//   LANES = 64 : the wave is one logical wave and the line address is uniform.
// Line indices are generated lane-parallel: in a batch lane l evaluates the
// draw for iteration it0 + (l mod ITB) of its logical wave, so one evaluation
// of the 64-bit hash serves ITB iterations.  For iteration k the address held
// by lane k of the half is broadcast to the half's lanes (LDS permute, DPP row
// broadcast or v_readlane) and every lane loads its WDW dwords of that line.
// U loads stay in flight per wave: a ring of U result registers is consumed one
// slot at a time, each slot refilled by the next load, across batch boundaries.
//
// Three kernels share this: rand_read_stream_kernel (the default without a
// window map: few waves, tickets from LDS, the ring never drained),
// rand_read_flat_kernel (one wave per pair of logical waves) and
// rand_read_kernel (tickets from per-CU counters: window maps, pinned runs,
// placement log).
#pragma once
#include <utility>
#include "rr_common.hpp"

namespace rr {

enum { BC_LDS = 1, BC_DPP = 2, BC_READLANE = 3 };

template <int WDW> struct Vec;
template <> struct Vec<1> { typedef u32 type; };
typedef u32 u32x2 __attribute__((ext_vector_type(2)));
typedef u32 u32x4 __attribute__((ext_vector_type(4)));
template <> struct Vec<2> { typedef u32x2 type; };
template <> struct Vec<4> { typedef u32x4 type; };

// 64-bit wrapping accumulator kept as two 32-bit halves: adding a zero-extended
// word is an add with carry-out plus an add of the carry (no 64-bit register pair
// has to be formed around every loaded word).
struct Acc {
    u32 lo, hi;
    __device__ __forceinline__ void add(u32 w) {
        u32 s = lo + w;
        hi += (s < w) ? 1u : 0u;
        lo = s;
    }
    __device__ __forceinline__ void add(u32x2 v) { add(v.x); add(v.y); }
    __device__ __forceinline__ void add(u32x4 v) { add(v.x); add(v.y); add(v.z); add(v.w); }
    __device__ __forceinline__ u64 value() const { return ((u64)hi << 32) | lo; }
};

// Loads go through a global-address-space pointer so that the compiler emits
// global_load (not flat_load, which also ties up the LDS counter).
template <int NT, typename T>
__device__ __forceinline__ T load_line_part(u64 addr) {
    typedef const T __attribute__((address_space(1))) *gptr;
    gptr p = (gptr)addr;
    if constexpr (NT != 0) return __builtin_nontemporal_load(p);
    else return *p;
}

template <int K, int N, typename F>
__device__ __forceinline__ void static_for(F &&f) {
    if constexpr (K < N) {
        f(std::integral_constant<int, K>());
        static_for<K + 1, N>(f);
    }
}

// Address of the line of iteration K (compile-time) for this lane's logical
// wave, taken from the lane that generated it.
template <int LANES, int BC, int K>
__device__ __forceinline__ u64 bcast_addr(u32 alo, u32 ahi, u32 lane, u32 sel4) {
    if constexpr (BC == BC_LDS) {
        u32 lo = __builtin_amdgcn_ds_bpermute(sel4 + 4 * K, alo);
        u32 hi = __builtin_amdgcn_ds_bpermute(sel4 + 4 * K, ahi);
        return ((u64)hi << 32) | lo;
    } else if constexpr (BC == BC_DPP) {
        // row_newbcast:K -- lane K of every 16-lane row to the whole row
        // (every lane has a valid source, so bound_ctrl only spares the compiler a zeroed "old" operand)
        u32 lo = __builtin_amdgcn_update_dpp(0u, alo, 0x150 + K, 0xF, 0xF, true);
        u32 hi = __builtin_amdgcn_update_dpp(0u, ahi, 0x150 + K, 0xF, 0xF, true);
        return ((u64)hi << 32) | lo;
    } else {
        u32 lo = __builtin_amdgcn_readlane(alo, K);
        u32 hi = __builtin_amdgcn_readlane(ahi, K);
        if constexpr (LANES == 32) {
            u32 lo1 = __builtin_amdgcn_readlane(alo, 32 + K);
            u32 hi1 = __builtin_amdgcn_readlane(ahi, 32 + K);
            bool upper = lane >= 32;
            lo = upper ? lo1 : lo;
            hi = upper ? hi1 : hi;
        }
        return ((u64)hi << 32) | lo;
    }
}

// Iterations [it0, it0 + iters) of one logical wave per LANES lanes.  wave_seed =
// sm(read_seed, w) and win_base are per lane (equal within a logical wave).
// Returns this lane's share of the word sum.
template <int LANES, int WDW, int U, int BC, int NT>
__device__ __forceinline__ u64 read_logical_wave(const char *region, u64 wave_seed, u32 win_base,
                                                 u32 it0, u32 iters, u32 log2_line, const Reducer red,
                                                 u32 lane) {
    typedef typename Vec<WDW>::type V;
    constexpr int ITB = (BC == BC_DPP) ? 16 : LANES;  // iterations generated per batch
    static_assert(ITB % U == 0, "ring must divide the batch");
    const u32 itl = lane & (ITB - 1);              // iteration of the batch this lane generates
    const u32 sub_bytes = (lane & (LANES - 1)) * (WDW * 4);  // this lane's slice of a line
    const u32 sel4 = (lane & ~(u32)(LANES - 1)) * 4;         // LDS-permute byte index of lane 0 of the half
    u64 ctr = wave_seed + ((u64)it0 + itl + 1) * kGamma;     // SplitMix64 state of iteration it0 + itl
    const u64 step = (u64)ITB * kGamma;

    auto gen = [&]() -> u64 {
        u32 idx = reduce_to_line(mix64(ctr), red);
        ctr += step;
        return (u64)region + (((u64)win_base + idx) << log2_line);
    };

    V ring[U];
#pragma unroll
    for (int j = 0; j < U; ++j) ring[j] = V(0);
    Acc acc{0u, 0u};
    u64 cur = gen();
    const u32 n_batches = iters / ITB;
    for (u32 b = 0; b < n_batches; ++b) {
        u64 nxt = gen();
        const u32 clo = (u32)cur, chi = (u32)(cur >> 32);
        __builtin_amdgcn_sched_barrier(0);
        static_for<0, ITB>([&](auto kc) {
            constexpr int K = decltype(kc)::value;
            acc.add(ring[K % U]);  // oldest load of the ring: waits until only U-1 are outstanding
            u64 line = bcast_addr<LANES, BC, K>(clo, chi, lane, sel4);
            ring[K % U] = load_line_part<NT, V>(line | sub_bytes);
            __builtin_amdgcn_sched_barrier(0);  // keep issue order: consume slot, refill slot
        });
        cur = nxt;
    }
#pragma unroll
    for (int j = 0; j < U; ++j) acc.add(ring[j]);
    // ragged tail: fewer than ITB iterations left, addresses already in `cur`
    const u32 rem = iters - n_batches * ITB;
    for (u32 k = 0; k < rem; ++k) {
        u32 lo = __builtin_amdgcn_ds_bpermute(sel4 + 4 * k, (u32)cur);
        u32 hi = __builtin_amdgcn_ds_bpermute(sel4 + 4 * k, (u32)(cur >> 32));
        u64 line = ((u64)hi << 32) | lo;
        acc.add(load_line_part<NT, V>(line | sub_bytes));
    }
    return acc.value();
}

// Work distribution.  A "unit" is what one hardware wave carries: a pair of
// logical waves (LANES = 32) or one (LANES = 64) of one group; a ticket is one
// chunk of a unit's iterations: ticket = unit * chunks_per_wave + chunk.
//   flat mode   : the ticket is the wave's launch index; no counters.
//   ticket mode : the wave reads which CU it is on; the CU's group decides which
//                 logical waves it may execute and which window they read.
//                 Each CU owns a contiguous share of its group's units and a
//                 ticket counter of its own, so claims from different CUs never
//                 meet on one address.  A wave first drains its own CU's share,
//                 then scans the other CUs of the group (64 at a time, one lane
//                 per CU, ballot) and drains whatever shares are still open, so
//                 every ticket is executed even if some CU received no wave.
template <int LANES, int WDW, int U, int BC, int NT>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_num_sgpr(80))) rand_read_kernel(const ReadParams p) {
    constexpr u32 LPW = 64 / LANES;  // logical waves per hardware wave
    constexpr u32 kNone = 0xFFFFFFFFu;
    const u32 lane = threadIdx.x & 63;
    const u32 half = (LANES == 32) ? (lane >> 5) : 0;
    Scratch *s = p.scratch;
    const Tables *tb = p.tables;
    const u32 launch_index = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);

    u32 group = 0, dense = 0;
    if (p.ticket_mode || p.locate) {
        u32 key = cu_key();
        group = tb->group_of_key[key];
        dense = tb->dense_of_key[key];
        if (group == kExcluded) return;  // a CU that takes no part (pinned runs)
    }
    const u32 win_base = tb->window_base[group];
    const u32 cpw = p.chunks_per_wave;

    auto claim = [&](u32 cu) -> u32 {
        u32 t = 0;
        if (lane == 0) t = atomicAdd(&s->tickets[cu * kTicketStride], 1u);
        return __builtin_amdgcn_readfirstlane(t);
    };
    // stealing: scan the group's other CUs, 64 at a time (one per lane), starting behind this CU
    auto next_victim = [&]() -> u32 {
        const u32 g_begin = tb->group_begin[group];
        const u32 g_count = tb->group_begin[group + 1] - g_begin;
        const u32 my_pos = tb->cu_pos[dense];
        for (u32 scan_base = 0; scan_base + 1 < g_count; scan_base += 64) {  // the ring minus this CU has g_count-1 entries
            const u32 pos = scan_base + lane;
            bool open = false;
            u32 cand = 0;
            if (pos + 1 < g_count) {
                u32 ring = my_pos + 1 + pos;
                if (ring >= g_count) ring -= g_count;
                cand = tb->group_cus[g_begin + ring];
                const u32 taken = __hip_atomic_load(&s->tickets[cand * kTicketStride], __ATOMIC_RELAXED,
                                                    __HIP_MEMORY_SCOPE_AGENT);
                open = taken < tb->cu_unit_count[cand] * cpw;
            }
            const unsigned long long open_mask = __ballot(open);
            if (open_mask) return __builtin_amdgcn_readlane(cand, (u32)__builtin_ctzll(open_mask));
        }
        return kNone;
    };

    u32 cur = dense;          // CU whose share is being drained
    u32 unit_begin = 0, limit;
    u32 ticket;
    if (p.ticket_mode) {
        unit_begin = tb->cu_unit_begin[cur];
        limit = tb->cu_unit_count[cur] * cpw;
        ticket = claim(cur);
    } else {
        limit = (u32)((p.quota + LPW - 1) / LPW) * cpw;
        ticket = launch_index;
    }
    u64 acc = 0;
    bool worked = false;
    for (;;) {
        if (ticket >= limit) {
            if (!p.ticket_mode) break;
            cur = next_victim();
            if (cur == kNone) break;
            unit_begin = tb->cu_unit_begin[cur];
            limit = tb->cu_unit_count[cur] * cpw;
            ticket = claim(cur);
            continue;
        }
        const u32 this_ticket = ticket;
        if (p.ticket_mode) ticket = claim(cur);  // next ticket: its latency hides behind this chunk's loads
        else ticket = kNone;
        const u32 unit = this_ticket / cpw;
        const u32 chunk = this_ticket - unit * cpw;
        if (!worked) {  // the start time goes to the wave's cell at once, so that it need not be kept
            worked = true;
            const u64 t0 = clock_ticks();
            if (lane == 0) atomicMin(&s->cells[launch_index & (kNumCells - 1)].t_min, t0);
        }
        const u64 j0 = (u64)(unit_begin + unit) * LPW;  // index, within the group, of the lower logical wave
        u64 j = j0 + half;
        const bool valid = j < p.quota;  // odd quota: the upper half shadows the lower one
        if (!valid) j = j0;
        const u64 w = p.first_wave + group + (u64)p.n_groups * j;
        const u64 wave_seed = mix64(p.read_seed + (w + 1) * kGamma);
        const u32 it0 = chunk * p.chunk_iters;
        const u32 n_it = min(p.chunk_iters, p.iters - it0);
        u64 part = read_logical_wave<LANES, WDW, U, BC, NT>(p.region, wave_seed, win_base, it0, n_it,
                                                            p.log2_line, p.red, lane);
        acc += valid ? part : 0;
        if (p.placement && valid && (lane & (LANES - 1)) == 0) p.placement[w - p.first_wave] = (u16)dense;
    }
    if (!worked) return;
    const u64 total = wave_sum(acc);
    const u64 t1 = clock_ticks();
    if (lane == 0) {
        Cell *c = &s->cells[launch_index & (kNumCells - 1)];
        atomicAdd(&c->sum, total);
        atomicMax(&c->t_max, t1);
        atomicAdd(&c->waves, 1u);
        if (p.ticket_mode || p.locate) atomicAdd(&s->cu_waves[dense], 1u);
    }
}

// The flat launch without a window map, on its own: no tickets, no tables, no CU lookup.  It needs 34 scalar and
// 36-78 vector registers where the general kernel needs 85 and 64+, so that a SIMD really holds 8 waves of it (the
// general kernel: 7, the scalar registers being the limit) and all 8192 hardware waves of the sweep's launches are
// resident from the start.  Ticket = launch index = unit * chunks_per_wave + chunk.
template <int LANES, int WDW, int U, int BC, int NT>
__global__ void __launch_bounds__(256) rand_read_flat_kernel(const ReadParams p) {
    constexpr u32 LPW = 64 / LANES;
    const u32 lane = threadIdx.x & 63;
    const u32 half = (LANES == 32) ? (lane >> 5) : 0;
    const u32 launch_index = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const u32 cpw = p.chunks_per_wave;
    const u32 unit = launch_index / cpw;
    const u32 chunk = launch_index - unit * cpw;
    const u64 j0 = (u64)unit * LPW;  // the lower logical wave of the unit
    if (j0 >= p.quota) return;
    const u64 t0 = clock_ticks();
    u64 j = j0 + half;
    const bool valid = j < p.quota;  // odd quota: the upper half shadows the lower one
    if (!valid) j = j0;
    const u64 w = p.first_wave + j;
    const u64 wave_seed = mix64(p.read_seed + (w + 1) * kGamma);
    const u32 it0 = chunk * p.chunk_iters;
    const u32 n_it = min(p.chunk_iters, p.iters - it0);
    const u64 part = read_logical_wave<LANES, WDW, U, BC, NT>(p.region, wave_seed, 0u, it0, n_it, p.log2_line, p.red, lane);
    const u64 total = wave_sum(valid ? part : 0);
    const u64 t1 = clock_ticks();
    if (lane == 0) {
        Cell *c = &p.scratch->cells[launch_index & (kNumCells - 1)];
        atomicAdd(&c->sum, total);
        atomicMin(&c->t_min, t0);
        atomicMax(&c->t_max, t1);
        atomicAdd(&c->waves, 1u);
    }
}

// The launch without a window map as one uninterrupted stream of loads per wave.
//
// Measured on the MI355X: a few wavefronts per SIMD keep the memory system as busy as a full house does (two
// per SIMD with 16 loads each in flight reach the rate of eight), provided that they never stop -- and a launch
// that gives every wave slot one unit and lets it run loses a few per cent at its end, because the hardware
// serves the oldest waves first and the slots of those that have finished stay empty.  So this kernel starts few
// workgroups (a multiple of the number of compute units) and lets their waves take work in small pieces:
//   * every workgroup owns a contiguous range of tickets (ticket = unit * chunks_per_wave + chunk) and hands them
//     out to its waves from a counter in LDS.  An LDS atomic returns through the LDS counter of the wave, not
//     through the one the global loads use, so that asking for the next ticket does not wait for the loads in
//     flight;
//   * the ring of U loads is never drained between tickets: the batch loop is one loop, in which the addresses
//     of the next batch come either from the same ticket or, at a ticket's end, from the next one.
// A ticket therefore costs a few dozen instructions and can be short (256 iterations), which makes the waves of
// a workgroup finish within microseconds of each other; the workgroups have equal ranges.  Needs whole units
// (an even number of logical waves when two share a wavefront) and chunks of a multiple of 16 iterations that
// divide the iterations of a wave; the host falls back to rand_read_flat_kernel otherwise.
template <int LANES, int WDW, int U, int NT>
__global__ void __launch_bounds__(256) rand_read_stream_kernel(const ReadParams p) {
    typedef typename Vec<WDW>::type V;
    constexpr u32 LPW = 64 / LANES;
    constexpr int ITB = 16;  // iterations per batch: DPP row broadcast
    static_assert(ITB % U == 0, "ring must divide the batch");
    __shared__ u32 next_ticket;
    const u32 lane = threadIdx.x & 63;
    const u32 half = (LANES == 32) ? (lane >> 5) : 0;
    const u32 itl = lane & (ITB - 1);
    const u32 sub_bytes = (lane & (LANES - 1)) * (WDW * 4);
    const u32 launch_index = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const u32 cpw = p.chunks_per_wave;
    const u64 total = (p.quota / LPW) * cpw;  // tickets of the launch (the host keeps this below 2^31)
    const u32 t_begin = (u32)(total * blockIdx.x / gridDim.x);
    const u32 t_end = (u32)(total * (blockIdx.x + 1) / gridDim.x);
    if (threadIdx.x == 0) next_ticket = t_begin;
    __syncthreads();
    auto claim = [&]() -> u32 {
        u32 t = 0;
        if (lane == 0) t = atomicAdd(&next_ticket, 1u);
        return __builtin_amdgcn_readfirstlane(t);
    };
    u32 ticket = claim();
    if (ticket >= t_end) return;
    const u64 t0 = clock_ticks();
    // SplitMix64 state of this lane's first iteration of a ticket: iteration chunk * chunk_iters + itl of the
    // logical wave unit * LPW + half
    auto ticket_ctr = [&](u32 t) -> u64 {
        const u32 unit = t / cpw;
        const u32 chunk = t - unit * cpw;
        const u64 w = p.first_wave + (u64)unit * LPW + half;
        const u64 wave_seed = mix64(p.read_seed + (w + 1) * kGamma);
        return wave_seed + ((u64)chunk * p.chunk_iters + itl + 1) * kGamma;
    };
    u64 ctr = ticket_ctr(ticket);
    const u64 step = (u64)ITB * kGamma;
    auto gen = [&]() -> u64 {
        const u32 idx = reduce_to_line(mix64(ctr), p.red);
        ctr += step;
        return (u64)p.region + ((u64)idx << p.log2_line);
    };
    V ring[U];
#pragma unroll
    for (int j = 0; j < U; ++j) ring[j] = V(0);
    Acc acc{0u, 0u};
    const u32 batches_per_ticket = p.chunk_iters / ITB;
    u32 left = batches_per_ticket;  // batches of the current ticket whose loads are still to be issued
    u64 cur = gen();
    bool more = true;
    while (more) {
        // the batch after this one: same ticket, the next ticket, or none
        if (--left == 0) {
            ticket = claim();
            if (ticket >= t_end) {
                more = false;
            } else {
                ctr = ticket_ctr(ticket);
                left = batches_per_ticket;
            }
        }
        const u64 nxt = gen();
        const u32 clo = (u32)cur, chi = (u32)(cur >> 32);
        __builtin_amdgcn_sched_barrier(0);
        static_for<0, ITB>([&](auto kc) {
            constexpr int K = decltype(kc)::value;
            acc.add(ring[K % U]);  // oldest load of the ring: waits until only U-1 are outstanding
            const u64 line = bcast_addr<LANES, BC_DPP, K>(clo, chi, lane, 0u);
            ring[K % U] = load_line_part<NT, V>(line | sub_bytes);
            __builtin_amdgcn_sched_barrier(0);  // keep issue order: consume slot, refill slot
        });
        cur = nxt;
    }
#pragma unroll
    for (int j = 0; j < U; ++j) acc.add(ring[j]);
    const u64 total_sum = wave_sum(acc.value());
    const u64 t1 = clock_ticks();
    if (lane == 0) {
        Cell *c = &p.scratch->cells[launch_index & (kNumCells - 1)];
        atomicAdd(&c->sum, total_sum);
        atomicMin(&c->t_min, t0);
        atomicMax(&c->t_max, t1);
        atomicAdd(&c->waves, 1u);
        if (p.locate) atomicAdd(&p.scratch->cu_waves[p.tables->dense_of_key[cu_key()]], 1u);  // per-CU counts wanted
    }
}

// Each (LANES, WDW) family lives in its own translation unit and exposes a
// finder that returns the kernel's host-side handle for (unroll, bcast,
// nontemporal), or null if that combination is not built.
kernel_handle find_read_kernel_32_1(u32 unroll, u32 bcast, u32 nt);
kernel_handle find_read_kernel_32_2(u32 unroll, u32 bcast, u32 nt);
kernel_handle find_read_kernel_32_4(u32 unroll, u32 bcast, u32 nt);
kernel_handle find_read_kernel_64_1(u32 unroll, u32 bcast, u32 nt);
kernel_handle find_read_kernel_64_2(u32 unroll, u32 bcast, u32 nt);
// The flat-only kernel is built for the DPP broadcast and each family's default ring depth; null otherwise.
kernel_handle find_flat_kernel(u32 lanes, u32 wdw, u32 unroll, u32 bcast, u32 nt);
// The stream kernel (DPP broadcast) for a line shape and ring depth; null if not built.
kernel_handle find_stream_kernel(u32 lanes, u32 wdw, u32 unroll, u32 nt);

}  // namespace rr
