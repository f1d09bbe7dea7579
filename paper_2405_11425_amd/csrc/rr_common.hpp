// Shared declarations of the random cache-line read library: kernel parameter
// block, device scratch layout, device-side integer helpers.  gfx950 only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rr {

typedef unsigned long long u64;
typedef unsigned int u32;
typedef unsigned short u16;

constexpr u64 kGamma = 0x9E3779B97F4A7C15ull;  // SplitMix64 increment
constexpr u32 kMaxGroups = 1024;
constexpr u32 kMaxCus = 1024;
constexpr u32 kKeyBits = 12;  // xcc[11:8] se[7:5] sh[4] cu[3:0]
constexpr u32 kNumKeys = 1u << kKeyBits;
constexpr u16 kExcluded = 0xFFFFu;

constexpr u32 kNumCells = 1024;     // result cells, one 128-byte line each
constexpr u32 kTicketStride = 32;   // u32 slots between two CUs' ticket counters (one 128-byte line each)

// Same-address device atomics retire at roughly one per 12 ns on this GPU, so
// nothing that every wave touches may live at one address: results go to one
// of kNumCells cells chosen by the wave's launch index, ticket counters are per
// compute unit and each sits in a cache line of its own.
struct Cell {
    u64 sum;     // wrapping sum of the words read by the waves that hashed here
    u64 t_min;   // earliest start of a working wave (constant-rate clock ticks)
    u64 t_max;   // latest end of a working wave
    u32 waves;   // working hardware waves
    u32 pad[25];
};
static_assert(sizeof(Cell) == 128, "one cell per 128-byte line");

// Result of one launch, written by finish_kernel straight into pinned host memory.
struct ResultHead {
    u64 checksum;              // wrapping sum over all result cells
    u64 t_min;
    u64 t_max;
    u32 waves_run;
    u32 unfinished;            // ticket mode: compute units whose share is not yet fully claimed
};

// Device scratch, one per GPU.
struct Scratch {
    u32 cu_waves[kMaxCus];     // working hardware waves per dense CU id
    u32 tickets[kMaxCus * kTicketStride];  // next unclaimed ticket of each CU's share
    u32 key_seen[kNumKeys];    // CU enumeration: 1 if a workgroup ran on the CU with this key
    Cell cells[kNumCells];
};

// Per-call lookup tables, built on the host and uploaded in one copy.
struct Tables {
    u16 group_of_key[kNumKeys];   // group of the CU with that hardware key, or kExcluded
    u16 dense_of_key[kNumKeys];   // dense CU id of that key
    u32 window_base[kMaxGroups];  // first line of each group's window
    u32 group_begin[kMaxGroups + 1];  // group g's CUs are group_cus[group_begin[g] .. group_begin[g+1])
    u16 group_cus[kMaxCus];       // dense CU ids sorted by group
    u16 cu_pos[kMaxCus];          // position of a CU inside its group's list
    u32 cu_unit_begin[kMaxCus];   // the CU's share of its group's work units: first unit ...
    u32 cu_unit_count[kMaxCus];   // ... and how many
};

// Exact h mod L for L <= 2^32: mask when L is a power of two, else a
// host-computed reciprocal M = floor((2^64-1)/L) and one correction step.
struct Reducer {
    u64 L;
    u64 M;
    u32 pow2;
};

// A kernel as the host launches it (the address of its host-side stub).
typedef const void *kernel_handle;

// Everything a read kernel needs, passed by value.
struct ReadParams {
    const char *region;       // device base, aligned to the line size
    u64 read_seed;
    u64 first_wave;           // id of the first logical wave of this call
    u64 quota;                // logical waves per group (flat mode: all of them)
    u32 iters;                // iterations (lines read) per logical wave
    u32 chunk_iters;          // iterations per ticket (a multiple of 64, or all of them)
    u32 chunks_per_wave;      // ceil(iters / chunk_iters)
    u32 n_groups;             // G
    u32 ticket_mode;          // 0 flat, 1 ticketed
    u32 locate;               // 1: look up the CU even in flat mode (placement log or per-CU counts wanted)
    u32 log2_line;            // 7, 8 or 9
    u32 n_zones;              // phased variant: number of zones; the region is cut into at most 64 windows of
    u32 zone_shift;           // 2^zone_shift lines, and bit v of zone_mask[z] says that window v belongs to zone z
    u64 zone_mask[16];
    u32 split_half;           // zone stream kernel: 0, or half the number of XCDs: workgroup b belongs to half
    u64 split_incl[2];        // (b / split_half) & 1, reads only windows in split_incl[that half] of its own units and
                              // the other windows of the units of workgroup b ^ split_half
    Reducer red;              // L = lines per window
    Scratch *scratch;
    const Tables *tables;
    u16 *placement;           // [W] or null: dense CU id that executed each logical wave
    u64 *phase_ticks;         // [hardware waves x zones] or null: clock at the end of each zone phase
};

__device__ __forceinline__ u64 mix64(u64 z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

__device__ __forceinline__ u32 reduce_to_line(u64 h, const Reducer &r) {
    if (r.pow2) return (u32)(h & (r.L - 1));
    u64 q = __umul64hi(h, r.M);  // floor(h/L) or one less
    u64 rem = h - q * r.L;
    if (rem >= r.L) rem -= r.L;
    return (u32)rem;
}

// 12-bit key of the CU this wave runs on: XCC_ID[3:0], then SE_ID, SH_ID and
// CU_ID of HW_ID (bits 15:13, 12, 11:8).
__device__ __forceinline__ u32 cu_key() {
    // s_getreg operand: id | offset << 6 | (size-1) << 11
    u32 hw = __builtin_amdgcn_s_getreg(4 | (8 << 6) | (7 << 11));    // HW_ID bits 15:8
    u32 xcc = __builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11));  // XCC_ID bits 3:0
    return (xcc << 8) | hw;
}

// Constant-rate device clock (s_memrealtime).
__device__ __forceinline__ u64 clock_ticks() { return wall_clock64(); }

// Sum of a 64-bit value over the 64 lanes of the wave, result valid in every
// lane.  Within each row of 16 lanes a DPP butterfly (quad permutes, then the
// half-row and row mirrors); the four row totals are combined through
// v_readlane.
template <int CTRL>
__device__ __forceinline__ u64 dpp_add(u64 v) {
    u32 lo = __builtin_amdgcn_update_dpp(0u, (u32)v, CTRL, 0xF, 0xF, false);
    u32 hi = __builtin_amdgcn_update_dpp(0u, (u32)(v >> 32), CTRL, 0xF, 0xF, false);
    return v + (((u64)hi << 32) | lo);
}

__device__ __forceinline__ u64 wave_sum(u64 v) {
    v = dpp_add<0xB1>(v);   // quad_perm [1,0,3,2]
    v = dpp_add<0x4E>(v);   // quad_perm [2,3,0,1]
    v = dpp_add<0x141>(v);  // row_half_mirror
    v = dpp_add<0x140>(v);  // row_mirror
    u64 total = 0;
#pragma unroll
    for (int row = 0; row < 4; ++row) {
        u32 lo = __builtin_amdgcn_readlane((u32)v, row * 16);
        u32 hi = __builtin_amdgcn_readlane((u32)(v >> 32), row * 16);
        total += ((u64)hi << 32) | lo;
    }
    return total;
}

}  // namespace rr
