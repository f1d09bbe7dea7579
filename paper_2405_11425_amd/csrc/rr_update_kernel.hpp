// Random line write and read-modify-write: the same draw stream as the read
// kernel (logical wave w, iteration it -> line), but every lane stores to, or
// atomically adds to, its words of the line instead of loading them.  The paper
// motivates its benchmark with an application that wants random access to a
// large part of the memory (Sec. 1.3); reads are all it measures, these are the
// two other access kinds such an application has.
//
// Value of 32-bit word i (64-bit word index):  v(i) = low 32 bits of (value_seed + i * 0x9E3779B1).
//   write : word i <- v(i)            -- the same value whoever writes it, so repeated hits are harmless
//   add   : word i <- word i + v(i)   -- one device-scope atomic per word, so concurrent hits all count
// Checksum: wrapping 64-bit sum of v(i) over all words of all lines hit, repeats included.
// Over more memory than the second-level translation cache of an XCD covers the launch is divided between the two halves
// of the XCDs like a read (see rand_read_zone_stream_kernel): every wave goes through its own logical waves and keeps the
// lines its half may touch, then through those of its partner in the other half and keeps what the partner may not.
#pragma once
#include "rr_read_kernel.hpp"

namespace rr {

enum { OP_WRITE = 1, OP_ADD = 2 };
constexpr u64 kValueMul = 0x9E3779B1ull;

struct UpdateParams {
    char *region;        // device base, aligned to the line size
    u64 draw_seed;
    u64 value_seed;
    u64 n_waves;         // logical waves
    u32 iters;
    u32 log2_line;
    Reducer red;         // L = lines of the region
    Scratch *scratch;
    u32 split_half;      // 0, or half the number of XCDs: the region is divided between the halves of the XCDs as in the
    u32 window_shift;    // zone stream read kernel (windows of 2^window_shift lines; half (b / split_half) & 1 of workgroup
    u64 split_incl[2];   // b may touch the windows in split_incl[half]; the rest of its work workgroup b ^ split_half does)
};

template <int LANES, int WDW, int OP>
__global__ void __launch_bounds__(256) rand_update_kernel(const UpdateParams p) {
    constexpr u32 LPW = 64 / LANES;
    constexpr int ITB = 16;  // iterations generated per batch (DPP row broadcast)
    const u32 lane = threadIdx.x & 63;
    const u32 half = (LANES == 32) ? (lane >> 5) : 0;
    const u32 sub = lane & (LANES - 1);
    const u32 itl = lane & (ITB - 1);
    const u32 launch_index = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const u32 words_per_line_log2 = p.log2_line - 2;
    const u64 t0 = clock_ticks();
    u64 acc = 0;
    bool worked = false;
    // this lane's words of `line`: stored, or added to
    auto touch = [&](u32 line) {
        const u64 first_word = ((u64)line << words_per_line_log2) + sub * WDW;
        u32 *dst = (u32 *)p.region + first_word;
        u32 v[WDW];
#pragma unroll
        for (int q = 0; q < WDW; ++q) {
            v[q] = (u32)(p.value_seed + (first_word + q) * kValueMul);
            acc += v[q];
        }
        if constexpr (OP == OP_WRITE) {
            if constexpr (WDW == 1) {
                __builtin_nontemporal_store(v[0], dst);
            } else if constexpr (WDW == 2) {
                __builtin_nontemporal_store(u32x2{v[0], v[1]}, (u32x2 *)dst);
            } else {
                __builtin_nontemporal_store(u32x4{v[0], v[1], v[2], v[3]}, (u32x4 *)dst);
            }
        } else {
#pragma unroll
            for (int q = 0; q < WDW; ++q) atomicAdd(dst + q, v[q]);
        }
    };
    // The logical waves of hardware wave `li` of the launch, as far as their lines lie in the windows of `keep` (most
    // of them): every 16-lane row evaluates a batch of 16 iterations and broadcasts them one by one.
    auto pass = [&](u32 li, u64 keep) {
        const u64 j0 = (u64)li * LPW;
        if (j0 >= p.n_waves) return;
        worked = true;
        const u64 j = j0 + half;
        const bool valid = j < p.n_waves;  // odd number of logical waves: the upper half stays idle
        const u64 wave_seed = mix64(p.draw_seed + ((valid ? j : j0) + 1) * kGamma);
        const bool all = keep == ~0ull;
        for (u32 it0 = 0; it0 < p.iters; it0 += ITB) {
            const u32 mine = reduce_to_line(mix64(wave_seed + ((u64)it0 + itl + 1) * kGamma), p.red);
            static_for<0, ITB>([&](auto kc) {
                constexpr int K = decltype(kc)::value;
                const u32 line = __builtin_amdgcn_update_dpp(0u, mine, 0x150 + K, 0xF, 0xF, true);  // row_newbcast:K
                if (it0 + K < p.iters && valid && (all || ((keep >> (line >> p.window_shift)) & 1ull))) touch(line);
            });
        }
    };
    // The same for windows that hold few of the lines (what a partner leaves over): the 64 lanes evaluate 64 different
    // iterations of one logical wave at a time, and the few lines that are kept are handed to the lanes one by one
    // (two at a time where a line takes 32 lanes) -- a fifth of the instructions of the pass above per draw.
    auto sparse_pass = [&](u32 li, u64 keep) {
        for (u32 w = 0; w < LPW; ++w) {
            const u64 j = (u64)li * LPW + w;
            if (j >= p.n_waves) break;
            worked = true;
            const u64 wave_seed = mix64(p.draw_seed + (j + 1) * kGamma);
            for (u32 it0 = 0; it0 < p.iters; it0 += 64) {
                const u32 it = it0 + lane;
                const u32 line = reduce_to_line(mix64(wave_seed + ((u64)it + 1) * kGamma), p.red);
                unsigned long long m = __ballot(it < p.iters && ((keep >> (line >> p.window_shift)) & 1ull));
                while (m) {
                    const u32 b0 = (u32)__builtin_ctzll(m);
                    m &= m - 1;
                    u32 b1 = b0;
                    bool two = false;
                    if (LANES == 32 && m) {
                        b1 = (u32)__builtin_ctzll(m);
                        m &= m - 1;
                        two = true;
                    }
                    const u32 l0 = __builtin_amdgcn_readlane(line, b0), l1 = __builtin_amdgcn_readlane(line, b1);
                    if (half == 0 || two) touch(half ? l1 : l0);
                }
            }
        }
    };
    if (!p.split_half) {
        pass(launch_index, ~0ull);
    } else {  // own logical waves where this half of the XCDs may write, the partner's where the partner's half may not
        const u32 h = (blockIdx.x / p.split_half) & 1u;
        pass(launch_index, p.split_incl[h]);
        sparse_pass((blockIdx.x ^ p.split_half) * (blockDim.x >> 6) + (threadIdx.x >> 6), ~p.split_incl[h ^ 1u]);
    }
    if (!worked) return;
    const u64 total = wave_sum(acc);  // idle lanes hold 0
    const u64 t1 = clock_ticks();
    if (lane == 0) {
        Cell *c = &p.scratch->cells[launch_index & (kNumCells - 1)];
        atomicAdd(&c->sum, total);
        atomicMin(&c->t_min, t0);
        atomicMax(&c->t_max, t1);
        atomicAdd(&c->waves, 1u);
    }
}

kernel_handle find_update_kernel(u32 lanes, u32 wdw, u32 op);

}  // namespace rr
