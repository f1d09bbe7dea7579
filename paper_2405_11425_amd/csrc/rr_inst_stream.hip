// Instantiations of the stream read kernel: each line shape with ring depths 8 and 16, both cache hints.
#include "rr_read_kernel.hpp"
namespace rr {
kernel_handle find_stream_kernel(u32 lanes, u32 wdw, u32 unroll, u32 nt) {
#define RR_STREAM(L, W, U)                                                                                  \
    if (lanes == L && wdw == W && unroll == U)                                                              \
        return nt ? (kernel_handle)&rand_read_stream_kernel<L, W, U, 1> : (kernel_handle)&rand_read_stream_kernel<L, W, U, 0>;
    RR_STREAM(32, 1, 16)
    RR_STREAM(32, 1, 8)
    RR_STREAM(32, 2, 16)
    RR_STREAM(32, 2, 8)
    RR_STREAM(32, 4, 16)
    RR_STREAM(32, 4, 8)
    RR_STREAM(64, 1, 16)
    RR_STREAM(64, 1, 8)
    RR_STREAM(64, 2, 16)
    RR_STREAM(64, 2, 8)
#undef RR_STREAM
    return nullptr;
}
}  // namespace rr
