// Instantiations of the random line write / add kernel.
#include "rr_update_kernel.hpp"
namespace rr {
kernel_handle find_update_kernel(u32 lanes, u32 wdw, u32 op) {
#define RR_UPD(L, W)                                                                          \
    if (lanes == L && wdw == W)                                                               \
        return op == OP_WRITE ? (kernel_handle)&rand_update_kernel<L, W, OP_WRITE>            \
                              : (kernel_handle)&rand_update_kernel<L, W, OP_ADD>;
    RR_UPD(32, 1)
    RR_UPD(32, 2)
    RR_UPD(32, 4)
    RR_UPD(64, 1)
    RR_UPD(64, 2)
#undef RR_UPD
    return nullptr;
}
}  // namespace rr
