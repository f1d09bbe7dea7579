// Instantiations of the zone-phased read kernel, one per line shape and cache hint.
#include "rr_phased_kernel.hpp"
namespace rr {
kernel_handle find_phased_kernel(u32 lanes, u32 wdw, u32 nt) {
    if (lanes == 32 && wdw == 1) return nt ? (kernel_handle)&rand_read_phased_kernel<32, 1, 32, 1> : (kernel_handle)&rand_read_phased_kernel<32, 1, 32, 0>;
    if (lanes == 32 && wdw == 2) return nt ? (kernel_handle)&rand_read_phased_kernel<32, 2, 16, 1> : (kernel_handle)&rand_read_phased_kernel<32, 2, 16, 0>;
    if (lanes == 32 && wdw == 4) return nt ? (kernel_handle)&rand_read_phased_kernel<32, 4, 8, 1> : (kernel_handle)&rand_read_phased_kernel<32, 4, 8, 0>;
    if (lanes == 64 && wdw == 1) return nt ? (kernel_handle)&rand_read_phased_kernel<64, 1, 32, 1> : (kernel_handle)&rand_read_phased_kernel<64, 1, 32, 0>;
    if (lanes == 64 && wdw == 2) return nt ? (kernel_handle)&rand_read_phased_kernel<64, 2, 16, 1> : (kernel_handle)&rand_read_phased_kernel<64, 2, 16, 0>;
    return nullptr;
}
kernel_handle find_zone_stream_kernel(u32 lanes, u32 wdw, u32 nt) {
    if (lanes == 32 && wdw == 1) return nt ? (kernel_handle)&rand_read_zone_stream_kernel<32, 1, 16, 1> : (kernel_handle)&rand_read_zone_stream_kernel<32, 1, 16, 0>;
    if (lanes == 32 && wdw == 2) return nt ? (kernel_handle)&rand_read_zone_stream_kernel<32, 2, 16, 1> : (kernel_handle)&rand_read_zone_stream_kernel<32, 2, 16, 0>;
    if (lanes == 32 && wdw == 4) return nt ? (kernel_handle)&rand_read_zone_stream_kernel<32, 4, 8, 1> : (kernel_handle)&rand_read_zone_stream_kernel<32, 4, 8, 0>;
    if (lanes == 64 && wdw == 1) return nt ? (kernel_handle)&rand_read_zone_stream_kernel<64, 1, 16, 1> : (kernel_handle)&rand_read_zone_stream_kernel<64, 1, 16, 0>;
    if (lanes == 64 && wdw == 2) return nt ? (kernel_handle)&rand_read_zone_stream_kernel<64, 2, 16, 1> : (kernel_handle)&rand_read_zone_stream_kernel<64, 2, 16, 0>;
    return nullptr;
}
}  // namespace rr
