// Instantiations of the read kernel for 32 lanes per line, 4 dword(s) per lane.
#include "rr_read_kernel.hpp"
namespace rr {
kernel_handle find_read_kernel_32_4(u32 unroll, u32 bcast, u32 nt) {
    if (unroll == 2 && bcast == 1 && nt == 0) return (kernel_handle)&rand_read_kernel<32, 4, 2, 1, 0>;
    if (unroll == 2 && bcast == 1 && nt == 1) return (kernel_handle)&rand_read_kernel<32, 4, 2, 1, 1>;
    if (unroll == 2 && bcast == 2 && nt == 0) return (kernel_handle)&rand_read_kernel<32, 4, 2, 2, 0>;
    if (unroll == 2 && bcast == 2 && nt == 1) return (kernel_handle)&rand_read_kernel<32, 4, 2, 2, 1>;
    if (unroll == 2 && bcast == 3 && nt == 0) return (kernel_handle)&rand_read_kernel<32, 4, 2, 3, 0>;
    if (unroll == 2 && bcast == 3 && nt == 1) return (kernel_handle)&rand_read_kernel<32, 4, 2, 3, 1>;
    if (unroll == 4 && bcast == 1 && nt == 0) return (kernel_handle)&rand_read_kernel<32, 4, 4, 1, 0>;
    if (unroll == 4 && bcast == 1 && nt == 1) return (kernel_handle)&rand_read_kernel<32, 4, 4, 1, 1>;
    if (unroll == 4 && bcast == 2 && nt == 0) return (kernel_handle)&rand_read_kernel<32, 4, 4, 2, 0>;
    if (unroll == 4 && bcast == 2 && nt == 1) return (kernel_handle)&rand_read_kernel<32, 4, 4, 2, 1>;
    if (unroll == 4 && bcast == 3 && nt == 0) return (kernel_handle)&rand_read_kernel<32, 4, 4, 3, 0>;
    if (unroll == 4 && bcast == 3 && nt == 1) return (kernel_handle)&rand_read_kernel<32, 4, 4, 3, 1>;
    if (unroll == 8 && bcast == 1 && nt == 0) return (kernel_handle)&rand_read_kernel<32, 4, 8, 1, 0>;
    if (unroll == 8 && bcast == 1 && nt == 1) return (kernel_handle)&rand_read_kernel<32, 4, 8, 1, 1>;
    if (unroll == 8 && bcast == 2 && nt == 0) return (kernel_handle)&rand_read_kernel<32, 4, 8, 2, 0>;
    if (unroll == 8 && bcast == 2 && nt == 1) return (kernel_handle)&rand_read_kernel<32, 4, 8, 2, 1>;
    if (unroll == 8 && bcast == 3 && nt == 0) return (kernel_handle)&rand_read_kernel<32, 4, 8, 3, 0>;
    if (unroll == 8 && bcast == 3 && nt == 1) return (kernel_handle)&rand_read_kernel<32, 4, 8, 3, 1>;
    return nullptr;
}
}  // namespace rr
