// Errors, the per-device state and its housekeeping kernels (CU enumeration, scratch reset, result
// fold), rr_enumerate_cus and rr_shutdown.
#include <cstdarg>
#include <cstdio>
#include <cstring>

#include "rr_host.hpp"

namespace rr {

// ------------------------------------------------------------------ kernels

// Marks the key of the CU each workgroup runs on; a short sleep keeps the
// workgroup resident so that the dispatcher has to use the other CUs too.
__global__ void __launch_bounds__(64) enumerate_kernel(Scratch *s, u32 naps) {
    if (threadIdx.x == 0) s->key_seen[cu_key()] = 1u;
    for (u32 i = 0; i < naps; ++i) __builtin_amdgcn_s_sleep(100);
}

// what: bit 0 result cells; bit 1 ticket counters; bit 2 per-CU wave counts; bit 3 key marks
__device__ __forceinline__ void reset_scratch(Scratch *s, u32 what) {
    const u32 t = threadIdx.x;
    if (what & 1u) {
        for (u32 i = t; i < kNumCells; i += blockDim.x) {
            s->cells[i].sum = 0;
            s->cells[i].t_min = ~0ull;
            s->cells[i].t_max = 0;
            s->cells[i].waves = 0;
        }
    }
    if (what & 2u)
        for (u32 i = t; i < kMaxCus; i += blockDim.x) s->tickets[i * kTicketStride] = 0;
    if (what & 4u)
        for (u32 i = t; i < kMaxCus; i += blockDim.x) s->cu_waves[i] = 0;
    if (what & 8u)
        for (u32 i = t; i < kNumKeys; i += blockDim.x) s->key_seen[i] = 0;
}

__global__ void __launch_bounds__(256) reset_kernel(Scratch *s, u32 what) { reset_scratch(s, what); }

// p[0 .. n) = v, grid-stride (used where a memset node would otherwise end up in a caller's captured graph).
__global__ void __launch_bounds__(256) fill_u16_kernel(u16 *p, u64 n, u16 v) {
    const u64 stride = (u64)gridDim.x * blockDim.x;
    for (u64 i = (u64)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) p[i] = v;
}

// One workgroup per slot of a batch: slot b has its own scratch, slots[b].
__global__ void __launch_bounds__(256) reset_batch_kernel(Scratch *slots, BatchSlots b) {
    reset_scratch(&slots[blockIdx.x], b.what[blockIdx.x]);
}

// After a read launch (one block of kNumCells threads, one result cell each):
// fold the cells into the result head (pinned host memory mapped into the
// device, so no copy follows), leave them cleared for the next launch, and count
// the compute units whose share of tickets has not been fully claimed.
__device__ __forceinline__ void fold_cells(Scratch *s, ResultHead *head, const Tables *tb, u32 n_cus, u32 cpw,
                                           u32 ticket_mode) {
    __shared__ u64 sh_sum[kNumCells], sh_min[kNumCells], sh_max[kNumCells];
    __shared__ u32 sh_waves[kNumCells], sh_open[kNumCells];
    const u32 t = threadIdx.x;
    Cell *c = &s->cells[t];
    sh_sum[t] = c->sum;
    sh_min[t] = c->t_min;
    sh_max[t] = c->t_max;
    sh_waves[t] = c->waves;
    c->sum = 0;
    c->t_min = ~0ull;
    c->t_max = 0;
    c->waves = 0;
    u32 open = 0;
    if (ticket_mode && t < n_cus && s->tickets[t * kTicketStride] < tb->cu_unit_count[t] * cpw) open = 1;
    sh_open[t] = open;
    __syncthreads();
    for (u32 step = kNumCells / 2; step > 0; step >>= 1) {
        if (t < step) {
            sh_sum[t] += sh_sum[t + step];
            sh_min[t] = sh_min[t + step] < sh_min[t] ? sh_min[t + step] : sh_min[t];
            sh_max[t] = sh_max[t + step] > sh_max[t] ? sh_max[t + step] : sh_max[t];
            sh_waves[t] += sh_waves[t + step];
            sh_open[t] += sh_open[t + step];
        }
        __syncthreads();
    }
    if (t == 0) {
        head->checksum = sh_sum[0];
        head->t_min = sh_min[0];
        head->t_max = sh_max[0];
        head->waves_run = sh_waves[0];
        head->unfinished = sh_open[0];
    }
}

__global__ void __launch_bounds__(kNumCells) finish_kernel(Scratch *s, ResultHead *head, const Tables *tb,
                                                           u32 n_cus, u32 cpw, u32 ticket_mode) {
    fold_cells(s, head, tb, n_cus, cpw, ticket_mode);
}

// The same for every slot of a batch at once: workgroup b folds slots[b] into heads[b].
__global__ void __launch_bounds__(kNumCells) finish_batch_kernel(Scratch *slots, ResultHead *heads, const Tables *tb,
                                                                 u32 n_cus, BatchSlots b) {
    const u32 i = blockIdx.x;
    fold_cells(&slots[i], &heads[i], tb, n_cus, b.tickets_per_unit[i], b.ticket_mode[i]);
}
static_assert(kMaxCus <= kNumCells, "finish_kernel checks one compute unit per thread");

// ------------------------------------------------------------------ errors

static thread_local char g_last_error[512] = "";  // a fixed buffer: reporting a failure allocates nothing

int fail(int code, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_last_error, sizeof g_last_error, fmt, ap);
    va_end(ap);
    return code;
}

// ------------------------------------------------------------------ per-device state

std::mutex g_mutex;

namespace {

DeviceState g_state[kMaxDevices];

}  // namespace

int enumerate(DeviceState &st, hipStream_t stream) {
    int dev = 0, n_expected = 0;
    HIP_TRY(hipGetDevice(&dev));
    HIP_TRY(hipDeviceGetAttribute(&n_expected, hipDeviceAttributeMultiprocessorCount, dev));
    u32 seen[kNumKeys];
    u32 found = 0;
    for (int attempt = 0; attempt < 4 && (int)found < n_expected; ++attempt) {
        int rc = launch_reset(st, 8u, stream);
        if (rc != RR_OK) return rc;
        const u32 blocks = (u32)n_expected * 64u << attempt;
        hipLaunchKernelGGL(enumerate_kernel, dim3(blocks), dim3(64), 0, stream, st.scratch, 4u << attempt);
        HIP_TRY(hipGetLastError());
        HIP_TRY(hipMemcpyAsync(seen, st.scratch->key_seen, kNumKeys * sizeof(u32),
                               hipMemcpyDeviceToHost, stream));
        HIP_TRY(hipStreamSynchronize(stream));
        found = 0;
        for (u32 k = 0; k < kNumKeys; ++k) found += seen[k] ? 1u : 0u;
    }
    if (found == 0 || found > kMaxCus)
        return fail(RR_EPLACE, "CU enumeration found %u compute units (device reports %d)", found, n_expected);
    if ((int)found != n_expected)
        return fail(RR_EPLACE, "CU enumeration found %u of %d compute units", found, n_expected);
    st.n_cus = 0;
    for (u32 k = 0; k < kNumKeys; ++k) {  // ascending key == sorted (xcc, se, sh, cu)
        st.dense_of_key_host[k] = kExcluded;
        if (!seen[k]) continue;
        rr_cu_t c;
        c.xcc = k >> 8;
        c.se = (k >> 5) & 7u;
        c.sh = (k >> 4) & 1u;
        c.cu = k & 15u;
        st.dense_of_key_host[k] = (u16)st.n_cus;
        st.cus[st.n_cus++] = c;
    }
    return RR_OK;
}

// Create (once per device) the scratch, tables, events and the CU list.
int get_state(hipStream_t stream, DeviceState **out) {
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(RR_EHIP, "device index %d not supported", dev);
    DeviceState &st = g_state[dev];
    if (!st.ready) {
        if (!st.scratch) HIP_TRY(hipMalloc((void **)&st.scratch, sizeof(Scratch)));
        if (!st.tables) HIP_TRY(hipMalloc((void **)&st.tables, sizeof(Tables)));
        if (!st.tables_host) HIP_TRY(hipHostMalloc((void **)&st.tables_host, sizeof(Tables), hipHostMallocDefault));
        if (!st.tables_last) st.tables_last = new Tables;
        if (!st.head) {
            HIP_TRY(hipHostMalloc((void **)&st.head, kMaxBatch * sizeof(ResultHead), hipHostMallocMapped));
            HIP_TRY(hipHostGetDevicePointer((void **)&st.head_dev, st.head, 0));
        }
        if (!st.cu_waves_host) HIP_TRY(hipHostMalloc((void **)&st.cu_waves_host, kMaxCus * sizeof(u32), hipHostMallocDefault));
        if (!st.ev0) HIP_TRY(hipEventCreate(&st.ev0));
        if (!st.ev1) HIP_TRY(hipEventCreate(&st.ev1));
        HIP_TRY(hipDeviceGetAttribute(&st.wall_khz, hipDeviceAttributeWallClockRate, dev));
        if (st.wall_khz <= 0) st.wall_khz = 100000;  // s_memrealtime: 100 MHz
        int rc = enumerate(st, stream);
        if (rc != RR_OK) return rc;
        st.ready = true;
    }
    *out = &st;
    return RR_OK;
}

int launch_reset(DeviceState &st, u32 what, hipStream_t stream) {
    hipLaunchKernelGGL(reset_kernel, dim3(1), dim3(256), 0, stream, st.scratch, what);
    HIP_TRY(hipGetLastError());
    return RR_OK;
}

int launch_fill_u16(u16 *p, u64 n, u16 v, hipStream_t stream) {
    if (n == 0) return RR_OK;
    u64 blocks = (n + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(fill_u16_kernel, dim3((u32)blocks), dim3(256), 0, stream, p, n, v);
    HIP_TRY(hipGetLastError());
    return RR_OK;
}

int begin_cells(DeviceState &st, hipStream_t stream) {
    if (!st.cells_clean) {
        int rc = launch_reset(st, 1u, stream);
        if (rc != RR_OK) return rc;
    }
    st.cells_clean = false;
    return RR_OK;
}

// Scratch for the launches of a batch, one per slot, so that nothing has to run between two read kernels;
// allocated when the first batch arrives, cleared once, and left with clear cells by every finish.
int prepare_batch(DeviceState &st, u32 n, const u32 *tickets_per_unit, const u32 *ticket_mode, const u32 *reset_bits,
                  hipStream_t stream, BatchSlots &b) {
    if (n == 0 || n > kMaxBatch) return fail(RR_EINVAL, "batch of %u launches is out of range", n);
    bool fresh = false;
    if (!st.batch_scratch) {
        HIP_TRY(hipMalloc((void **)&st.batch_scratch, kMaxBatch * sizeof(Scratch)));
        fresh = true;
    }
    memset(&b, 0, sizeof b);
    bool any = false;
    for (u32 i = 0; i < n; ++i) {
        b.tickets_per_unit[i] = tickets_per_unit[i];
        b.ticket_mode[i] = (unsigned char)ticket_mode[i];
        b.what[i] = (unsigned char)(reset_bits[i] | ((fresh || st.batch_dirty) ? 1u : 0u));
        any = any || b.what[i];
    }
    if (fresh || st.batch_dirty) {  // every slot, not only the ones of this batch
        BatchSlots all = b;
        for (u32 i = n; i < kMaxBatch; ++i) all.what[i] = 1u;
        hipLaunchKernelGGL(reset_batch_kernel, dim3(kMaxBatch), dim3(256), 0, stream, st.batch_scratch, all);
        HIP_TRY(hipGetLastError());
    } else if (any) {
        hipLaunchKernelGGL(reset_batch_kernel, dim3(n), dim3(256), 0, stream, st.batch_scratch, b);
        HIP_TRY(hipGetLastError());
    }
    st.batch_dirty = true;  // until finish_batch has run and the stream has been waited for
    return RR_OK;
}

int finish_batch(DeviceState &st, u32 n, const BatchSlots &b, hipStream_t stream) {
    hipLaunchKernelGGL(finish_batch_kernel, dim3(n), dim3(kNumCells), 0, stream, st.batch_scratch, st.head_dev, st.tables,
                       st.n_cus, b);
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipStreamSynchronize(stream));
    st.batch_dirty = false;
    return RR_OK;
}

int finish_and_wait(DeviceState &st, u32 n_cus, u32 tickets_per_unit, u32 ticket_mode, hipStream_t stream) {
    hipLaunchKernelGGL(finish_kernel, dim3(1), dim3(kNumCells), 0, stream, st.scratch, st.head_dev, st.tables, n_cus,
                       tickets_per_unit, ticket_mode);
    HIP_TRY(hipGetLastError());
    if (st.fixed)  // the head is in device memory: fetch it (the wait below covers the copy)
        HIP_TRY(hipMemcpyAsync(st.head, st.head_dev, sizeof(ResultHead), hipMemcpyDeviceToHost, stream));
    HIP_TRY(hipStreamSynchronize(stream));
    st.cells_clean = true;
    return RR_OK;
}

}  // namespace rr

using namespace rr;

// ------------------------------------------------------------------ C ABI

extern "C" const char *rr_strerror(int code) {
    switch (code) {
        case RR_OK: return "success";
        case RR_EINVAL: return "invalid argument";
        case RR_EHIP: return "HIP runtime error";
        case RR_EPLACE: return "a group or target compute unit received no resident wave";
        default: return "unknown error code";
    }
}

extern "C" const char *rr_last_error(void) { return g_last_error; }

extern "C" int rr_enumerate_cus(rr_cu_t *out, uint32_t cap, uint32_t *n_cus, void *hip_stream) {
    if (!n_cus) return fail(RR_EINVAL, "n_cus is NULL");
    if (cap > 0 && !out) return fail(RR_EINVAL, "out is NULL but cap > 0");
    std::lock_guard<std::mutex> lock(g_mutex);
    DeviceState *st = nullptr;
    int rc = get_state((hipStream_t)hip_stream, &st);
    if (rc != RR_OK) return rc;
    const u32 n = st->n_cus;
    for (u32 i = 0; i < n && i < cap; ++i) out[i] = st->cus[i];
    *n_cus = n;
    return RR_OK;
}

extern "C" int rr_shutdown(void) {
    std::lock_guard<std::mutex> lock(g_mutex);
    int current = 0;
    bool have_current = hipGetDevice(&current) == hipSuccess;
    for (int d = 0; d < kMaxDevices; ++d) {
        DeviceState &st = g_state[d];
        if (!st.scratch && !st.head && !st.ev0) continue;
        if (hipSetDevice(d) != hipSuccess) continue;
        (void)hipDeviceSynchronize();
        if (st.scratch) (void)hipFree(st.scratch);
        if (st.batch_scratch) (void)hipFree(st.batch_scratch);
        if (st.tables) (void)hipFree(st.tables);
        if (st.tables_host) (void)hipHostFree(st.tables_host);
        delete st.tables_last;
        if (st.placement) (void)hipFree(st.placement);
        if (st.head) (void)hipHostFree(st.head);
        if (st.cu_waves_host) (void)hipHostFree(st.cu_waves_host);
        if (st.ev0) (void)hipEventDestroy(st.ev0);
        if (st.ev1) (void)hipEventDestroy(st.ev1);
        for (hipEvent_t e : st.batch_ev) (void)hipEventDestroy(e);
        st = DeviceState();
    }
    release_all_regions();
    if (have_current) (void)hipSetDevice(current);
    return RR_OK;
}
