// Instantiations of the flat-only read kernel: DPP broadcast, each line shape's default ring depth, both cache hints.
#include "rr_read_kernel.hpp"
namespace rr {
kernel_handle find_flat_kernel(u32 lanes, u32 wdw, u32 unroll, u32 bcast, u32 nt) {
    if (bcast != BC_DPP) return nullptr;
#define RR_FLAT(L, W, U)                                                                              \
    if (lanes == L && wdw == W && unroll == U)                                                        \
        return nt ? (kernel_handle)&rand_read_flat_kernel<L, W, U, BC_DPP, 1> : (kernel_handle)&rand_read_flat_kernel<L, W, U, BC_DPP, 0>;
    RR_FLAT(32, 1, 16)
    RR_FLAT(32, 2, 16)
    RR_FLAT(32, 4, 8)
    RR_FLAT(64, 1, 16)
    RR_FLAT(64, 2, 16)
#undef RR_FLAT
    return nullptr;
}
}  // namespace rr
