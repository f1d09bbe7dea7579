// Device regions mapped in separately allocated pieces (HIP virtual memory management).
#include <map>
#include <vector>

#include "rr_host.hpp"

using namespace rr;

namespace {

struct PiecewiseRegion {
    int device = 0;
    u64 bytes = 0, piece = 0;
    u64 mapped = 0;  // bytes of the reservation that have a piece mapped
    std::vector<hipMemGenericAllocationHandle_t> handles;
};
std::map<void *, PiecewiseRegion> g_regions;  // guarded by g_mutex

// Undo a (possibly partial) piecewise mapping; errors are ignored, this runs on failure paths and at shutdown.
void release_region(void *base, PiecewiseRegion &r) {
    for (u64 off = 0; off < r.mapped; off += r.piece) (void)hipMemUnmap((char *)base + off, r.piece);
    for (auto h : r.handles) (void)hipMemRelease(h);
    (void)hipMemAddressFree(base, r.bytes);
    r.handles.clear();
    r.mapped = 0;
}

hipMemAllocationProp device_memory_prop(int dev) {
    hipMemAllocationProp prop = {};
    prop.type = hipMemAllocationTypePinned;
    prop.location.type = hipMemLocationTypeDevice;
    prop.location.id = dev;
    return prop;
}

}  // namespace

extern "C" int rr_region_granularity(uint64_t *minimum, uint64_t *recommended) {
    if (!minimum && !recommended) return fail(RR_EINVAL, "both outputs are NULL");
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    hipMemAllocationProp prop = device_memory_prop(dev);
    size_t g = 0;
    if (minimum) {
        HIP_TRY(hipMemGetAllocationGranularity(&g, &prop, hipMemAllocationGranularityMinimum));
        *minimum = g;
    }
    if (recommended) {
        HIP_TRY(hipMemGetAllocationGranularity(&g, &prop, hipMemAllocationGranularityRecommended));
        *recommended = g;
    }
    return RR_OK;
}

extern "C" int rr_region_create(uint64_t bytes, uint64_t piece_bytes, void **region_out) {
    if (!region_out) return fail(RR_EINVAL, "region_out is NULL");
    if (bytes == 0 || piece_bytes == 0 || bytes % piece_bytes != 0)
        return fail(RR_EINVAL, "bytes must be a positive multiple of piece_bytes");
    if (piece_bytes % 4096 != 0) return fail(RR_EINVAL, "piece_bytes must be a multiple of 4096");
    // the driver gives a process about 65 500 handles and a mapped piece takes two: 32 752 pieces was the last to map
    if (bytes / piece_bytes > 30000) return fail(RR_EINVAL, "more than 30000 pieces");
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    hipMemAllocationProp prop = device_memory_prop(dev);
    size_t minimum = 0;
    HIP_TRY(hipMemGetAllocationGranularity(&minimum, &prop, hipMemAllocationGranularityMinimum));
    if (minimum == 0 || piece_bytes % minimum != 0)
        return fail(RR_EINVAL, "piece_bytes must be a multiple of the device's allocation granularity (%zu)", minimum);
    u64 align = piece_bytes & (~piece_bytes + 1);  // largest power of two dividing the piece size
    if (align > (1ull << 30)) align = 1ull << 30;
    void *base = nullptr;
    HIP_TRY(hipMemAddressReserve(&base, bytes, align, nullptr, 0));
    PiecewiseRegion r;
    r.device = dev;
    r.bytes = bytes;
    r.piece = piece_bytes;
    r.handles.reserve(bytes / piece_bytes);
    hipError_t e = hipSuccess;
    const char *what = "";
    hipMemAccessDesc access = {};
    access.location = prop.location;
    access.flags = hipMemAccessFlagsProtReadWrite;
    for (u64 off = 0; off < bytes; off += piece_bytes) {
        hipMemGenericAllocationHandle_t h;
        e = hipMemCreate(&h, piece_bytes, &prop, 0);
        what = "hipMemCreate";
        if (e != hipSuccess) break;
        r.handles.push_back(h);
        e = hipMemMap((char *)base + off, piece_bytes, 0, h, 0);
        what = "hipMemMap";
        if (e != hipSuccess) break;
        r.mapped = off + piece_bytes;
        // access is granted piece by piece (one call over the whole range was refused for 32768 pieces)
        e = hipMemSetAccess((char *)base + off, piece_bytes, &access, 1);
        what = "hipMemSetAccess";
        if (e != hipSuccess) break;
    }
    if (e != hipSuccess) {
        const u64 done = r.mapped;
        release_region(base, r);
        return fail(RR_EHIP, "%s failed after %llu of %llu bytes: %s", what, (unsigned long long)done,
                    (unsigned long long)bytes, hipGetErrorString(e));
    }
    std::lock_guard<std::mutex> lock(g_mutex);
    g_regions[base] = std::move(r);
    *region_out = base;
    return RR_OK;
}

extern "C" int rr_region_destroy(void *region) {
    std::lock_guard<std::mutex> lock(g_mutex);
    auto it = g_regions.find(region);
    if (it == g_regions.end()) return fail(RR_EINVAL, "not a region made by rr_region_create");
    int current = 0;
    HIP_TRY(hipGetDevice(&current));
    HIP_TRY(hipSetDevice(it->second.device));
    HIP_TRY(hipDeviceSynchronize());
    release_region(region, it->second);
    g_regions.erase(it);
    HIP_TRY(hipSetDevice(current));
    return RR_OK;
}

void rr::release_all_regions() {
    for (auto &kv : g_regions) {
        if (hipSetDevice(kv.second.device) != hipSuccess) continue;
        (void)hipDeviceSynchronize();
        release_region(kv.first, kv.second);
    }
    g_regions.clear();
}
