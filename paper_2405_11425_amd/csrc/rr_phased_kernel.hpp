// Zone-phased variant of the random line read.
//
// On the MI355X the read rate drops when lines from different 96 GiB thirds of
// the memory are in flight at the same time, whoever issues them; a window per
// compute group (the paper's remedy, Sec. 2.4) does not help, a window per
// *phase* does.  This kernel reads exactly the lines of rand_read_kernel (same
// draws, same checksum) but in a different order: the region is cut into zones
// of zone_lines lines, and every wave first reads all of its lines that fall
// in zone 0, then those in zone 1, and so on.  There is no synchronisation
// between waves: measured with phase_ticks, the workgroups of a CU advance in
// launch order (the oldest several times faster than the youngest), so the
// phases of different waves overlap only partly and the gain is small; a
// device-wide barrier between phases was tried and is slower still, because the
// youngest waves then finish each phase alone and cannot fill the memory pipes.
//
// Per phase and per chunk of kChunk iterations a wave (1) regenerates the
// chunk's line indices lane-parallel, keeps those inside the zone and appends
// them to a list in LDS (ballot + mbcnt give each kept lane its slot), then
// (2) walks the dense list with the usual ring of U loads in flight.  Lists
// of the two logical waves of a wavefront differ in length; the shorter one
// pads with loads of the window's first line (an L2 hit) whose data is
// discarded, so that every wave issues a branch-free, countable load stream.
#pragma once
#include "rr_read_kernel.hpp"

namespace rr {

constexpr u32 kPhaseChunk = 512;  // iterations binned per pass through LDS
constexpr u32 kPhasePad = 32;     // list slack so that the last group of the ring may read past the end

template <int LANES, int WDW, int U, int NT>
__global__ void __launch_bounds__(256) rand_read_phased_kernel(const ReadParams p) {
    typedef typename Vec<WDW>::type V;
    constexpr u32 LPW = 64 / LANES;
    __shared__ u32 lists[4][LPW][kPhaseChunk + kPhasePad];
    const u32 lane = threadIdx.x & 63;
    const u32 half = (LANES == 32) ? (lane >> 5) : 0;
    const u32 sub = lane & (LANES - 1);
    Scratch *s = p.scratch;
    const u32 launch_index = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    u32 *my_list = lists[threadIdx.x >> 6][half];

    const u64 j0 = (u64)launch_index * LPW;
    if (j0 >= p.quota) return;
    u64 j = j0 + half;
    const bool valid = j < p.quota;  // odd number of logical waves: the upper half shadows the lower one
    if (!valid) j = j0;
    const u64 w = p.first_wave + j;
    const u64 wave_seed = mix64(p.read_seed + (w + 1) * kGamma);
    const u64 lane_base = (u64)p.region + sub * (WDW * 4);
    const u64 t0 = clock_ticks();

    Acc acc{0u, 0u};
    for (u32 z = 0; z < p.n_zones; ++z) {
        const u64 z_lo = (u64)z * p.zone_lines, z_hi = z_lo + p.zone_lines;
        for (u32 it0 = 0; it0 < p.iters; it0 += kPhaseChunk) {
            const u32 n_it = min(kPhaseChunk, p.iters - it0);
            // (1) bin: keep the iterations of this chunk whose line lies in zone z
            u32 count = 0;
            for (u32 r = 0; r < n_it; r += LANES) {
                const u32 it = it0 + r + sub;
                const u64 h = mix64(wave_seed + ((u64)it + 1) * kGamma);
                const u32 line = reduce_to_line(h, p.red);
                const bool keep = (r + sub < n_it) && line >= z_lo && line < z_hi;
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
            if (n_max == 0) continue;
            V ring[U];
            // slot Q of the ring holds list entry k0 + Q of the group issued last
            auto issue = [&](auto qc, u32 k0) {
                constexpr int Q = decltype(qc)::value;
                const u32 k = k0 + Q;
                const u32 listed = my_list[k];              // k < kPhaseChunk + kPhasePad always
                const u32 line = (k < count) ? listed : 0u;  // padding reads the region's first line
                ring[Q] = load_line_part<NT, V>(lane_base + ((u64)line << p.log2_line));
            };
            auto consume = [&](auto qc, u32 k0) {
                constexpr int Q = decltype(qc)::value;
                if (k0 + Q < count) acc.add(ring[Q]);        // data of padding loads is dropped
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
        if (p.phase_ticks && lane == 0) p.phase_ticks[(u64)launch_index * p.n_zones + z] = clock_ticks();
    }
    const u64 total = wave_sum(valid ? acc.value() : 0);
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
