// Host-side internals shared by the library's translation units: error reporting, the per-device
// state (scratch, tables, result head, events, CU list) and the launches of the two housekeeping
// kernels.  Nothing here is part of the C ABI.
#pragma once
#include <mutex>
#include <vector>

#include "../../include/randline.h"
#include "rr_common.hpp"

namespace rr {

// Records the message for rr_last_error (per thread) and returns code.
int fail(int code, const char *fmt, ...);

#define HIP_TRY(expr)                                                                          \
    do {                                                                                       \
        hipError_t e_ = (expr);                                                                \
        if (e_ != hipSuccess)                                                                  \
            return rr::fail(RR_EHIP, "%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_), __FILE__, \
                            __LINE__);                                                         \
    } while (0)

struct DeviceState {
    bool ready = false;
    Scratch *scratch = nullptr;
    Scratch *batch_scratch = nullptr;  // [kMaxBatch], allocated by the first batched call
    bool batch_dirty = false;          // a batch did not reach its finish: clear every slot's cells before the next
    Tables *tables = nullptr;       // device
    Tables *tables_host = nullptr;  // pinned staging copy
    Tables *tables_last = nullptr;  // what the device copy holds (plain host memory), to skip equal uploads
    bool tables_valid = false;
    bool cells_clean = false;       // result cells are in their cleared state
    u16 *placement = nullptr;
    size_t placement_cap = 0;
    ResultHead *head = nullptr;      // [kMaxBatch] pinned host memory, mapped ...
    ResultHead *head_dev = nullptr;  // ... and its address as the device sees it; single calls use entry 0
    // The state behind the entry point that allocates nothing keeps its device data in a file-scope device
    // array: head_dev is then plain device memory, head points at head_copy below, and finish_and_wait copies
    // the one into the other before it waits.  Such a state has no events and a placement buffer of fixed size.
    bool fixed = false;
    ResultHead head_copy = {};
    u32 *cu_waves_host = nullptr;    // pinned staging for the per-CU wave counts
    bool flat_tables_ready = false;  // the device tables are those of a call without a window map
    hipEvent_t ev0 = nullptr, ev1 = nullptr;
    std::vector<hipEvent_t> batch_ev;     // two per launch of a batch, created when first needed
    int wall_khz = 0;
    u32 n_cus = 0;
    rr_cu_t cus[kMaxCus];                 // dense id -> coordinates
    u16 dense_of_key_host[kNumKeys];      // kExcluded if no such CU
};

constexpr int kMaxDevices = 16;
constexpr u32 kMaxBatch = 64;  // launches one batched call may queue before it waits

// What the launches of a batch differ in, as far as their reset and finish are concerned (a kernel argument).
struct BatchSlots {
    u32 tickets_per_unit[kMaxBatch];
    unsigned char ticket_mode[kMaxBatch];
    unsigned char what[kMaxBatch];  // reset_kernel's bits
};

// One lock for everything below: device states, the piecewise regions, and every launch that uses the
// per-device scratch (calls on one device are serialised).
extern std::mutex g_mutex;

// The state of the current device, created on first use (scratch, tables, events, CU enumeration on
// `stream`).  g_mutex must be held.
int get_state(hipStream_t stream, DeviceState **out);
// Lists the device's compute units into st (needs st.scratch); used by get_state and by the state that
// allocates nothing.
int enumerate(DeviceState &st, hipStream_t stream);

inline u32 key_of(const rr_cu_t &c) { return (c.xcc << 8) | (c.se << 5) | (c.sh << 4) | c.cu; }

inline Reducer make_reducer(u64 L) {
    Reducer r;
    r.L = L;
    r.pow2 = (L & (L - 1)) == 0 ? 1u : 0u;
    r.M = r.pow2 ? 0 : (~0ull) / L;  // floor((2^64-1)/L) == floor(2^64/L) when L is not a power of two
    return r;
}

// reset_kernel on `stream`; what: bit 0 result cells, bit 1 ticket counters, bit 2 per-CU wave counts, bit 3 key marks
int launch_reset(DeviceState &st, u32 what, hipStream_t stream);
// p[0 .. n) = v on `stream` (device memory)
int launch_fill_u16(u16 *p, u64 n, u16 v, hipStream_t stream);
// Make sure the result cells are cleared before a kernel that adds into them (marks them used).
int begin_cells(DeviceState &st, hipStream_t stream);
// finish_kernel (cells -> result head 0 in mapped host memory, cells left cleared), then wait for the stream.
int finish_and_wait(DeviceState &st, u32 n_cus, u32 tickets_per_unit, u32 ticket_mode, hipStream_t stream);

// A batch of n launches (n <= kMaxBatch): launch i works on st.batch_scratch[i] and reports into st.head[i].
// prepare_batch allocates the slots when first needed and clears in them what the launches need cleared
// (reset_bits[i]: bit 1 ticket counters, bit 2 per-CU wave counts; result cells as far as they are not clear
// already); finish_batch folds every slot into its result head and waits for the stream.
int prepare_batch(DeviceState &st, u32 n, const u32 *tickets_per_unit, const u32 *ticket_mode, const u32 *reset_bits,
                  hipStream_t stream, BatchSlots &b);
int finish_batch(DeviceState &st, u32 n, const BatchSlots &b, hipStream_t stream);

// Piecewise regions still alive (rr_region.hip); for rr_shutdown, g_mutex held.
void release_all_regions();

}  // namespace rr
