// Device-touching part of the C ABI (include/rar.h): argument checks on the host, then
// launches.  Every shape the kernels assume is verified here before anything is enqueued.
#include <hip/hip_runtime.h>

#include <cstring>
#include <mutex>

#include "launch.hpp"

using rar::Geometry;
using rar::RankPtrs;
using rar::Tuning;

// The scratch of rar_allreduce_static: part of the library's image on every GPU it runs on, so a
// caller that cannot allocate has somewhere to exchange partials.  Host code never uses this name
// as an address: static_scratch() below asks the runtime where the array lives on the current
// device and everything else goes through that pointer.
static __device__ __align__(256) unsigned char scratch[RAR_STATIC_SCRATCH_BYTES];

namespace {

std::mutex g_static_guard;
unsigned char *g_static_ptr[16];   // device address of `scratch` per device (each GPU has its own copy)
// Time-outs found in a device's array so far (by rar_plan_status of whichever plan looked first):
// the array's status word is shared by all plans, so a plan compares this count with the one it saw
// at its first call since its last status query.
unsigned long g_static_epoch[16];

int static_scratch(int *device, unsigned char **out) {
    int dev = 0;
    if (rar::note_hip(hipGetDevice(&dev)) != hipSuccess || dev < 0 || dev >= 16) return RAR_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_static_guard);
    if (!g_static_ptr[dev]) {
        void *ptr = nullptr;
        if (rar::note_hip(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch))) != hipSuccess || !ptr) return RAR_ERR_HIP;
        g_static_ptr[dev] = static_cast<unsigned char *>(ptr);
    }
    if (device) *device = dev;
    *out = g_static_ptr[dev];
    return RAR_OK;
}

inline hipStream_t as_stream(void *s) { return static_cast<hipStream_t>(s); }

int ensure_scratch(const rar_plan_t *plan) {
    if (!plan->scratch || plan->scratch_size < plan->geo.scratch_bytes) return RAR_ERR_SCRATCH;
    return RAR_OK;
}

// Is `stream` being captured into a graph?  *id (may be NULL) receives the capture's identity.
bool capturing(hipStream_t stream, unsigned long long *id = nullptr) {
    hipStreamCaptureStatus status = hipStreamCaptureStatusNone;
    unsigned long long got = 0;
    if (hipStreamGetCaptureInfo(stream, &status, &got) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    if (id) *id = got;
    return status != hipStreamCaptureStatusNone;
}

void release_pinned(volatile uint32_t *word) { (void)hipHostFree(const_cast<uint32_t *>(word)); }

int ensure_ordering_event(int device);

// A step-barrier wait of this plan has given up and rar_plan_status has not been asked since.
inline bool poisoned(const rar_plan_t *plan) { return plan->host_status && *plan->host_status != 0u; }

// Remember the device and ask how many workgroups of each fused kernel it holds at once.
// Allocates nothing.
int ensure_occupancy(rar_plan_t *plan) {
    if (plan->have_occupancy) return RAR_OK;
    rar::DeviceInfo info;
    int got = rar::device_info(&info);
    if (got != RAR_OK) return got;
    plan->compute_units = info.compute_units;
    if (rar::note_hip(hipGetDevice(&plan->device)) != hipSuccess) return RAR_ERR_HIP;
    for (int i = 0; i < 4; ++i) {
        int rc = rar::fused_max_resident(plan->geo.dtype, plan->geo.G, 1 << i, false, plan->geo.fold != 0, false, &plan->resident[i]);
        if (rc != RAR_OK) return rc;
        rc = rar::fused_max_resident(plan->geo.dtype, plan->geo.G, 1 << i, true, plan->geo.fold != 0, false, &plan->resident_packed[i]);
        if (rc != RAR_OK) return rc;
    }
    plan->have_occupancy = true;
    return RAR_OK;
}

// First launch of a plan on its own scratch: the above, plus the pinned word through which a
// kernel reports a time-out and the device's event for ordering launches of different streams.
int ensure_residency(rar_plan_t *plan) {
    if (plan->have_resident) return RAR_OK;
    int rc = ensure_occupancy(plan);
    if (rc != RAR_OK) return rc;
    rc = ensure_ordering_event(plan->device);
    if (rc != RAR_OK) return rc;
    if (!plan->host_status) {
        void *word = nullptr;
        void *on_device = nullptr;
        if (rar::note_hip(hipHostMalloc(&word, 64, hipHostMallocMapped)) != hipSuccess) return RAR_ERR_HIP;
        if (rar::note_hip(hipHostGetDevicePointer(&on_device, word, 0)) != hipSuccess) {
            (void)hipHostFree(word);
            return RAR_ERR_HIP;
        }
        *static_cast<volatile uint32_t *>(word) = 0u;
        plan->host_status = static_cast<volatile uint32_t *>(word);
        plan->host_status_dev = static_cast<uint32_t *>(on_device);
        plan->release_host_status = release_pinned;
    }
    plan->have_resident = true;
    return RAR_OK;
}

int ensure_chain_residency(rar_plan_t *plan) {
    if (plan->have_resident_chain) return RAR_OK;
    for (int i = 0; i < 4; ++i) {
        int rc = rar::fused_max_resident(plan->geo.dtype, plan->geo.G, 1 << i, false, plan->geo.fold != 0, true, &plan->resident_chain[i]);
        if (rc != RAR_OK) return rc;
        rc = rar::fused_max_resident(plan->geo.dtype, plan->geo.G, 1 << i, true, plan->geo.fold != 0, true,
                                     &plan->resident_chain_packed[i]);
        if (rc != RAR_OK) return rc;
    }
    plan->have_resident_chain = true;
    return RAR_OK;
}

inline int unroll_index(const Tuning &t) { return t.unroll == 1 ? 0 : t.unroll == 2 ? 1 : t.unroll == 4 ? 2 : 3; }

// The fused kernel's step barriers need every workgroup of the grid resident at once.
int fused_tuning(rar_plan_t *plan, bool packed, Tuning *t) {
    const long *resident = packed ? plan->resident_packed : plan->resident;
    *t = rar::resolve_tuning(*plan, resident);
    const long grid = static_cast<long>(plan->geo.P) * t->B_s;
    if (grid > resident[unroll_index(*t)] || grid > static_cast<long>(rar::kMaxWorkgroupsPerCU) * plan->compute_units)
        return RAR_ERR_LIMIT;
    return RAR_OK;
}

// What a fused launch needs before it may be enqueued.  Set-up work (the first launch, the first
// after a time-out) cannot become part of a captured graph: a fill kernel recorded there would
// clear the flags again on every replay.
int prepare_fused(rar_plan_t *plan, bool packed, hipStream_t stream) {
    if (poisoned(plan)) return RAR_ERR_TIMEOUT;
    const bool setup = !plan->have_resident || !plan->flags_clean || (packed && !plan->packed_clean);
    if (!setup) return RAR_OK;
    if (capturing(stream)) return RAR_ERR_CAPTURE;
    int rc = ensure_residency(plan);
    if (rc != RAR_OK) return rc;
    if (!plan->flags_clean) {  // header and barrier flags
        rc = rar::launch_fill_zero(plan->scratch, plan->geo.data_offset, plan->host_status_dev, stream);
        if (rc != RAR_OK) return rc;
        plan->flags_clean = true;
    }
    // the data+flag buffers (both sets, and the second set of partial buffers between them) must
    // not hold a word whose upper half could equal a sequence number
    if (packed && !plan->packed_clean && plan->geo.packed_offset != 0) {
        const Geometry &g = plan->geo;
        rc = rar::launch_fill_zero(static_cast<unsigned char *>(plan->scratch) + g.packed_offset, g.scratch_bytes - g.packed_offset,
                                   nullptr, stream);
        if (rc != RAR_OK) return rc;
        plan->packed_clean = true;
    }
    return RAR_OK;
}

// ---- keeping fused kernels of different streams apart -------------------------------------------
//
// Two fused kernels that share the device can each hold workgroup slots that the other one's
// waiting workgroups need.  Unless the caller has said that its plans share the device
// (rar_plan_set_concurrency), a fused launch therefore first waits for the fused launches made on
// other streams: an event is recorded on that other stream now (it covers the earlier launch,
// which was enqueued there before) and the new launch's stream waits for it.  Launches on one
// stream cost nothing extra.  "Exclusive" = a launch of a plan with concurrency 1.
struct Ordering {
    std::mutex guard;
    hipEvent_t event = nullptr;
    hipStream_t exclusive = nullptr;   // stream of the last exclusive launch
    bool have_exclusive = false;
    hipStream_t shared[8];             // streams of the sharing launches made since
    int shared_count = 0;
};
Ordering g_ordering[16];

void wait_for_stream(Ordering &o, hipStream_t stream, hipStream_t other) {
    if (other == stream) return;
    unsigned long long mine = 0, theirs = 0;
    const bool cap_mine = capturing(stream, &mine);
    // the legacy default stream cannot belong to a capture, and merely asking about it while a
    // blocking stream is being captured would invalidate that capture
    if (cap_mine && other == nullptr) return;
    const bool cap_theirs = capturing(other, &theirs);
    // a dependency cannot cross the boundary of a capture: inside capture only streams of the same capture are ordered
    if (cap_mine != cap_theirs || (cap_mine && mine != theirs)) return;
    if (!o.event) return;
    // `other` may have been destroyed since: then the record fails, and there is nothing left to wait for
    if (hipEventRecord(o.event, other) != hipSuccess || hipStreamWaitEvent(stream, o.event, 0) != hipSuccess) (void)hipGetLastError();
}

// Created at a plan's first launch on the device, which is never inside stream capture.
int ensure_ordering_event(int device) {
    if (device < 0 || device >= 16) return RAR_OK;  // such a device gets no ordering
    Ordering &o = g_ordering[device];
    std::lock_guard<std::mutex> lock(o.guard);
    if (o.event) return RAR_OK;
    if (rar::note_hip(hipEventCreateWithFlags(&o.event, hipEventDisableTiming)) != hipSuccess) {
        o.event = nullptr;
        return RAR_ERR_HIP;
    }
    return RAR_OK;
}

void order_fused_launch(const rar_plan_t *plan, hipStream_t stream) {
    const int dev = plan->device;
    if (dev < 0 || dev >= 16) return;
    Ordering &o = g_ordering[dev];
    std::lock_guard<std::mutex> lock(o.guard);
    if (plan->concurrency == 1) {
        if (o.have_exclusive) wait_for_stream(o, stream, o.exclusive);
        for (int i = 0; i < o.shared_count; ++i) wait_for_stream(o, stream, o.shared[i]);
        o.shared_count = 0;
        o.exclusive = stream;
        o.have_exclusive = true;
    } else {
        bool known = false;  // a stream in the list has already been ordered after the last exclusive launch
        for (int i = 0; i < o.shared_count; ++i) known = known || o.shared[i] == stream;
        if (!known) {
            if (o.have_exclusive) wait_for_stream(o, stream, o.exclusive);
            if (o.shared_count == 8) {  // more streams than slots: forget the oldest (its plans share the device anyway)
                for (int i = 1; i < 8; ++i) o.shared[i - 1] = o.shared[i];
                o.shared_count = 7;
            }
            o.shared[o.shared_count++] = stream;
        }
    }
}

int check_bufs(void *const *bufs, const Geometry &g, RankPtrs *ptrs) {
    std::memset(ptrs, 0, sizeof *ptrs);
    for (int p = 0; p < g.P; ++p) {
        if (!bufs[p]) return RAR_ERR_ARG;
        if (reinterpret_cast<uintptr_t>(bufs[p]) % 16 != 0) return RAR_ERR_ALIGN;
        ptrs->p[p] = bufs[p];
    }
    return RAR_OK;
}

// Discard a time-out that the caller has dealt with: the next launch clears flags and words.
void rearm(rar_plan_t *plan) {
    if (plan->host_status) *plan->host_status = 0u;
    plan->flags_clean = false;
    plan->packed_clean = false;
}

}  // namespace

extern "C" {

int rar_plan_status(rar_plan_t *plan, void *stream) {
    if (!plan) return RAR_ERR_ARG;
    if (rar::note_hip(hipStreamSynchronize(as_stream(stream))) != hipSuccess) return RAR_ERR_HIP;
    bool timed_out = poisoned(plan);
    if (plan->scratch && plan->flags_clean) {  // the header of the plan's own scratch says the same
        uint32_t word = 0;
        if (rar::note_hip(hipMemcpy(&word, plan->scratch, sizeof word, hipMemcpyDeviceToHost)) != hipSuccess) return RAR_ERR_HIP;
        timed_out = timed_out || word != 0;
    }
    if (plan->ran_static) {  // calls on the library's array report through its header alone
        unsigned char *array = nullptr;
        int device = 0;
        int rc = static_scratch(&device, &array);
        if (rc != RAR_OK) return rc;
        std::lock_guard<std::mutex> lock(g_static_guard);
        uint32_t word = 0;
        if (rar::note_hip(hipMemcpy(&word, array, sizeof word, hipMemcpyDeviceToHost)) != hipSuccess) return RAR_ERR_HIP;
        if (word != 0) {
            ++g_static_epoch[device];
            word = 0;
            if (rar::note_hip(hipMemcpy(array, &word, sizeof word, hipMemcpyHostToDevice)) != hipSuccess) return RAR_ERR_HIP;
        }
        // a time-out found since this plan's first call on the array, by this query or by another
        // plan's: this plan's calls ran beside it on the same flags
        timed_out = timed_out || g_static_epoch[device] != plan->static_epoch;
        plan->ran_static = false;
    }
    if (!timed_out) return RAR_OK;
    rearm(plan);  // counters of different slots may now disagree: start over
    return RAR_ERR_TIMEOUT;
}

int rar_step_combine(void *dst, const void *src, size_t chunk, size_t n, int dtype, void *stream) {
    if (!dst || !src) return RAR_ERR_ARG;
    if (dtype != RAR_BF16 && dtype != RAR_F32) return RAR_ERR_DTYPE;
    if (n == 0) return RAR_OK;
    const size_t es = dtype == RAR_BF16 ? 2 : 4;
    if (chunk != 0 && n > SIZE_MAX / es / chunk) return RAR_ERR_LIMIT;
    const size_t offset = chunk * n * es;
    if ((reinterpret_cast<uintptr_t>(dst) | reinterpret_cast<uintptr_t>(src) | offset) % 16 != 0) return RAR_ERR_ALIGN;
    const size_t per_vec = 16 / es;
    unsigned char *d = static_cast<unsigned char *>(dst) + offset;
    const unsigned char *s = static_cast<const unsigned char *>(src) + offset;
    const size_t bytes = n * es;
    if ((d < s + bytes) && (s < d + bytes)) return RAR_ERR_ARG;  // overlapping ranges
    return rar::launch_combine(d, s, n / per_vec, static_cast<unsigned>(n % per_vec), dtype, as_stream(stream));
}

int rar_allreduce(void *const *bufs, rar_plan_t *plan, void *stream) {
    if (!bufs || !plan) return RAR_ERR_ARG;
    const Geometry &g = plan->geo;
    int rc = ensure_scratch(plan);
    if (rc != RAR_OK) return rc;
    RankPtrs ptrs;
    rc = check_bufs(bufs, g, &ptrs);
    if (rc != RAR_OK) return rc;
    hipStream_t st = as_stream(stream);
    if (plan->mode == RAR_MODE_STEPWISE) return rar::launch_stepwise(*plan, ptrs, st);
    const bool packed = rar::effective_mode(*plan) == RAR_MODE_FUSED_PACKED && g.L > 0;
    rc = prepare_fused(plan, packed, st);
    if (rc != RAR_OK) return rc;
    Tuning t;
    rc = fused_tuning(plan, packed, &t);
    if (rc != RAR_OK) return rc;
    order_fused_launch(plan, st);
    if (!packed) return rar::launch_fused(*plan, plan->scratch, ptrs, t, true, 0, st);
    return rar::launch_fused_packed(*plan, ptrs, t, 0, st);
}

int rar_allreduce_chain(void *const *bufs, rar_plan_t *plan, int K, void *stream) {
    if (!bufs || !plan || K < 1 || K > rar::kMaxChainCalls) return RAR_ERR_ARG;
    if (plan->mode == RAR_MODE_STEPWISE) return RAR_ERR_ARG;
    const Geometry &g = plan->geo;
    int rc = ensure_scratch(plan);
    if (rc != RAR_OK) return rc;
    RankPtrs ptrs;
    rc = check_bufs(bufs, g, &ptrs);
    if (rc != RAR_OK) return rc;
    hipStream_t st = as_stream(stream);
    const bool packed = rar::effective_mode(*plan) == RAR_MODE_FUSED_PACKED && g.L > 0;
    if (!plan->have_resident_chain && capturing(st)) return RAR_ERR_CAPTURE;
    rc = prepare_fused(plan, packed, st);
    if (rc != RAR_OK) return rc;
    rc = ensure_chain_residency(plan);
    if (rc != RAR_OK) return rc;
    const long *resident = packed ? plan->resident_chain_packed : plan->resident_chain;
    const Tuning t = rar::resolve_chain_tuning(*plan, resident);
    const long grid = static_cast<long>(g.P) * t.B_s;
    if (grid > resident[unroll_index(t)] || grid > static_cast<long>(rar::kMaxWorkgroupsPerCU) * plan->compute_units)
        return RAR_ERR_LIMIT;
    // the flag tickets count the trips of all calls and are compared as signed 32-bit differences
    if (static_cast<unsigned long long>(K) * static_cast<unsigned long long>(t.iters) >= (1ull << 31)) return RAR_ERR_LIMIT;
    // without a second set of buffers the trips alternate between two places inside a partial buffer
    if (g.L > 0 && g.alt_offset == 0 &&
        2ull * t.B_s * rar::kThreads * t.unroll * 16ull > static_cast<unsigned long long>(g.chunk_stride))
        return RAR_ERR_LIMIT;
    order_fused_launch(plan, st);
    if (!packed) return rar::launch_fused(*plan, plan->scratch, ptrs, t, true, K, st);
    return rar::launch_fused_packed(*plan, ptrs, t, K, st);
}

int rar_allreduce_static(void *const *bufs, rar_plan_t *plan, void *stream) {
    if (!bufs || !plan) return RAR_ERR_ARG;
    const Geometry &g = plan->geo;
    if (g.fused_bytes > RAR_STATIC_SCRATCH_BYTES) return RAR_ERR_LIMIT;
    RankPtrs ptrs;
    int rc = check_bufs(bufs, g, &ptrs);
    if (rc != RAR_OK) return rc;
    unsigned char *array = nullptr;
    int device = 0;
    rc = static_scratch(&device, &array);
    if (rc != RAR_OK) return rc;
    rc = ensure_occupancy(plan);
    if (rc != RAR_OK) return rc;
    if (plan->device != device) return RAR_ERR_ARG;  // the plan belongs to another device
    Tuning t;
    rc = fused_tuning(plan, false, &t);
    if (rc != RAR_OK) return rc;
    hipStream_t st = as_stream(stream);
    if (!plan->ran_static) {
        std::lock_guard<std::mutex> lock(g_static_guard);
        plan->static_epoch = g_static_epoch[device];
        plan->ran_static = true;
    }
    order_fused_launch(plan, st);  // behind fused launches of other streams, like any fused launch
    // whatever the last call on this GPU left behind: the flags and the rest of the header start
    // at zero (a fill kernel, which a captured graph can replay; no pointer to host memory in the
    // header).  The status word in front stays as it is: a wait that gave up is not forgotten
    // before rar_plan_status has reported it.
    rc = rar::launch_fill_zero(array + 4, g.data_offset - 4, nullptr, st);
    if (rc != RAR_OK) return rc;
    return rar::launch_fused(*plan, array, ptrs, t, true, 0, st);
}

int rar_autotune(void *const *bufs, rar_plan_t *plan, void *stream, int calls, double *best_us) {
    if (!bufs || !plan || calls < 1) return RAR_ERR_ARG;
    if (plan->mode == RAR_MODE_STEPWISE) return RAR_ERR_ARG;
    hipStream_t st = as_stream(stream);
    if (capturing(st)) return RAR_ERR_CAPTURE;
    if (poisoned(plan)) return RAR_ERR_TIMEOUT;
    int rc = ensure_residency(plan);
    if (rc != RAR_OK) return rc;
    const bool packed = rar::effective_mode(*plan) == RAR_MODE_FUSED_PACKED && plan->geo.L > 0;
    const long *resident = packed ? plan->resident_packed : plan->resident;
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return RAR_ERR_HIP;
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return RAR_ERR_HIP; }

    const int keep_B = plan->user_B_s;
    const size_t keep_C = plan->user_C_s;
    int best_B = keep_B;
    size_t best_C = keep_C;
    double best = -1.0;
    bool any_timeout = false;
    rc = RAR_OK;
    for (int i = 0; i < 4 && rc == RAR_OK; ++i) {
        const size_t C_s = static_cast<size_t>(rar::kThreads) * 16 * (1u << i);
        plan->user_C_s = C_s;
        plan->user_B_s = 0;
        // the widest grid the planner allows (four workgroups per compute unit at most), then
        // halves of it while a rank keeps at least one workgroup
        const Tuning widest = rar::resolve_tuning(*plan, resident);
        int last = -1;
        for (int B_s = widest.B_s; B_s >= 1 && rc == RAR_OK; B_s /= 2) {
            plan->user_B_s = B_s;
            const Tuning t = rar::resolve_tuning(*plan, resident);
            if (t.B_s == last) continue;
            last = t.B_s;
            for (int k = 0; k < 2 && rc == RAR_OK; ++k) rc = rar_allreduce(bufs, plan, stream);
            if (rc != RAR_OK) break;
            if (hipEventRecord(e0, st) != hipSuccess) { rc = RAR_ERR_HIP; break; }
            for (int k = 0; k < calls && rc == RAR_OK; ++k) rc = rar_allreduce(bufs, plan, stream);
            if (rc != RAR_OK) break;
            float ms = 0.f;
            if (hipEventRecord(e1, st) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
                hipEventElapsedTime(&ms, e0, e1) != hipSuccess) { rc = RAR_ERR_HIP; break; }
            // a candidate during which a wait gave up did not do the work: its time means nothing
            const int status = rar_plan_status(plan, stream);
            if (status == RAR_ERR_TIMEOUT) { any_timeout = true; continue; }
            if (status != RAR_OK) { rc = status; break; }
            const double us = static_cast<double>(ms) * 1000.0 / calls;
            if (best < 0.0 || us < best) { best = us; best_B = t.B_s; best_C = C_s; }
            if (static_cast<long>(t.B_s) * plan->geo.P <= 64) break;  // narrower grids only get slower
        }
        // a time-out reported by a launch itself (the plan was poisoned between two calls)
        if (rc == RAR_ERR_TIMEOUT) {
            any_timeout = true;
            if (hipStreamSynchronize(st) != hipSuccess) { rc = RAR_ERR_HIP; break; }
            rearm(plan);
            rc = RAR_OK;
        }
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc != RAR_OK || best < 0.0) {
        plan->user_B_s = keep_B;
        plan->user_C_s = keep_C;
        return rc != RAR_OK ? rc : any_timeout ? RAR_ERR_TIMEOUT : RAR_ERR_HIP;
    }
    plan->user_B_s = best_B;
    plan->user_C_s = best_C;
    if (best_us) *best_us = best;
    return RAR_OK;
}

int rar_launch_floor(rar_plan_t *plan, void *stream) {
    if (!plan) return RAR_ERR_ARG;
    if (!plan->have_resident && capturing(as_stream(stream))) return RAR_ERR_CAPTURE;
    int rc = ensure_residency(plan);
    if (rc != RAR_OK) return rc;
    Tuning t;
    rc = fused_tuning(plan, rar::effective_mode(*plan) == RAR_MODE_FUSED_PACKED && plan->geo.L > 0, &t);
    if (rc != RAR_OK) return rc;
    return rar::launch_empty(static_cast<unsigned>(plan->geo.P) * t.B_s, as_stream(stream));
}

int rar_barrier_only(rar_plan_t *plan, void *stream) {
    if (!plan) return RAR_ERR_ARG;
    int rc = ensure_scratch(plan);
    if (rc != RAR_OK) return rc;
    hipStream_t st = as_stream(stream);
    rc = prepare_fused(plan, false, st);
    if (rc != RAR_OK) return rc;
    Tuning t;
    rc = fused_tuning(plan, false, &t);
    if (rc != RAR_OK) return rc;
    order_fused_launch(plan, st);
    RankPtrs ptrs;
    std::memset(&ptrs, 0, sizeof ptrs);
    return rar::launch_fused(*plan, plan->scratch, ptrs, t, false, 0, st);
}

const char *rar_last_hip_error(void) { return rar::last_hip_error_string(); }

int rar_copy_probe(void *dst, const void *src, size_t bytes, void *stream) {
    if (!dst || !src) return RAR_ERR_ARG;
    if ((reinterpret_cast<uintptr_t>(dst) | reinterpret_cast<uintptr_t>(src) | bytes) % 16 != 0) return RAR_ERR_ALIGN;
    return rar::launch_copy(dst, src, bytes / 16, as_stream(stream));
}

int rar_read_probe(void *sink, const void *src, size_t bytes, void *stream) {
    if (!sink || !src) return RAR_ERR_ARG;
    if ((reinterpret_cast<uintptr_t>(sink) | reinterpret_cast<uintptr_t>(src) | bytes) % 16 != 0) return RAR_ERR_ALIGN;
    return rar::launch_read(sink, src, bytes / 16, as_stream(stream));
}

}  // extern "C"
