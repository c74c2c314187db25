// Device-touching part of the C ABI (include/rar.h): argument checks on the host, then
// launches.  Every shape the kernels assume is verified here before anything is enqueued.
#include <hip/hip_runtime.h>

#include <cstring>

#include "launch.hpp"

using rar::Geometry;
using rar::RankPtrs;
using rar::Tuning;

namespace {

inline hipStream_t as_stream(void *s) { return static_cast<hipStream_t>(s); }

int ensure_scratch(const rar_plan_t *plan) {
    if (!plan->scratch || plan->scratch_size < plan->geo.scratch_bytes) return RAR_ERR_SCRATCH;
    return RAR_OK;
}

// Zero the header and the barrier flags on the stream if they are not known to be clean.
int ensure_flags(rar_plan_t *plan, hipStream_t stream) {
    if (plan->flags_clean) return RAR_OK;
    int rc = rar::launch_fill_zero(plan->scratch, plan->geo.data_offset, stream);
    if (rc == RAR_OK) plan->flags_clean = true;
    return rc;
}

int ensure_residency(rar_plan_t *plan) {
    if (plan->have_resident) return RAR_OK;
    rar::DeviceInfo info;
    int got = rar::device_info(&info);
    if (got != RAR_OK) return got;
    plan->compute_units = info.compute_units;
    for (int i = 0; i < 4; ++i) {
        int rc = rar::fused_max_resident(plan->geo.dtype, plan->geo.G, 1 << i, false, plan->geo.fold != 0, &plan->resident[i]);
        if (rc != RAR_OK) return rc;
        rc = rar::fused_max_resident(plan->geo.dtype, plan->geo.G, 1 << i, true, plan->geo.fold != 0, &plan->resident_packed[i]);
        if (rc != RAR_OK) return rc;
    }
    plan->have_resident = true;
    return RAR_OK;
}

// The fused kernel's step barriers need every workgroup of the grid resident at once.
int fused_tuning(rar_plan_t *plan, bool packed, Tuning *t) {
    int rc = ensure_residency(plan);
    if (rc != RAR_OK) return rc;
    const long *resident = packed ? plan->resident_packed : plan->resident;
    *t = rar::resolve_tuning(*plan, resident);
    const int index = t->unroll == 1 ? 0 : t->unroll == 2 ? 1 : t->unroll == 4 ? 2 : 3;
    if (static_cast<long>(plan->geo.P) * t->B_s > resident[index]) return RAR_ERR_LIMIT;
    return RAR_OK;
}

// The data+flag buffers must not hold a word whose upper half could equal a sequence number.
int ensure_packed(rar_plan_t *plan, hipStream_t stream) {
    if (plan->packed_clean || plan->geo.packed_offset == 0) return RAR_OK;
    const Geometry &g = plan->geo;
    int rc = rar::launch_fill_zero(static_cast<unsigned char *>(plan->scratch) + g.packed_offset,
                                   g.scratch_bytes - g.packed_offset, stream);
    if (rc == RAR_OK) plan->packed_clean = true;
    return rc;
}

}  // namespace

extern "C" {

int rar_plan_status(rar_plan_t *plan, void *stream) {
    if (!plan) return RAR_ERR_ARG;
    if (ensure_scratch(plan) != RAR_OK) return RAR_ERR_SCRATCH;
    if (rar::note_hip(hipStreamSynchronize(as_stream(stream))) != hipSuccess) return RAR_ERR_HIP;
    if (!plan->flags_clean) return RAR_OK;  // header never initialised: nothing has run
    uint32_t word = 0;
    if (rar::note_hip(hipMemcpy(&word, plan->scratch, sizeof word, hipMemcpyDeviceToHost)) != hipSuccess) return RAR_ERR_HIP;
    if (word == 0) return RAR_OK;
    plan->flags_clean = false;  // counters of different slots may now disagree: start over
    plan->packed_clean = false;
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
    std::memset(&ptrs, 0, sizeof ptrs);
    for (int p = 0; p < g.P; ++p) {
        if (!bufs[p]) return RAR_ERR_ARG;
        if (reinterpret_cast<uintptr_t>(bufs[p]) % 16 != 0) return RAR_ERR_ALIGN;
        ptrs.p[p] = bufs[p];
    }
    hipStream_t st = as_stream(stream);
    if (plan->mode == RAR_MODE_STEPWISE) return rar::launch_stepwise(*plan, ptrs, st);
    const bool packed = rar::effective_mode(*plan) == RAR_MODE_FUSED_PACKED && g.L > 0;
    Tuning t;
    rc = fused_tuning(plan, packed, &t);
    if (rc != RAR_OK) return rc;
    rc = ensure_flags(plan, st);
    if (rc != RAR_OK) return rc;
    if (!packed) return rar::launch_fused(*plan, ptrs, t, true, st);
    rc = ensure_packed(plan, st);
    if (rc != RAR_OK) return rc;
    return rar::launch_fused_packed(*plan, ptrs, t, st);
}

int rar_autotune(void *const *bufs, rar_plan_t *plan, void *stream, int calls, double *best_us) {
    if (!bufs || !plan || calls < 1) return RAR_ERR_ARG;
    if (plan->mode == RAR_MODE_STEPWISE) return RAR_ERR_ARG;
    int rc = ensure_residency(plan);
    if (rc != RAR_OK) return rc;
    const bool packed = rar::effective_mode(*plan) == RAR_MODE_FUSED_PACKED && plan->geo.L > 0;
    const long *resident = packed ? plan->resident_packed : plan->resident;
    hipStream_t st = as_stream(stream);
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return RAR_ERR_HIP;
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return RAR_ERR_HIP; }

    const int keep_B = plan->user_B_s;
    const size_t keep_C = plan->user_C_s;
    int best_B = keep_B;
    size_t best_C = keep_C;
    double best = -1.0;
    rc = RAR_OK;
    for (int i = 0; i < 4 && rc == RAR_OK; ++i) {
        const size_t C_s = static_cast<size_t>(rar::kThreads) * 16 * (1u << i);
        plan->user_C_s = C_s;
        plan->user_B_s = 0;
        const Tuning widest = rar::resolve_tuning(*plan, resident);
        int last = -1;
        // the widest grid that fits, then halves of it while a rank keeps at least one workgroup
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
            const double us = static_cast<double>(ms) * 1000.0 / calls;
            if (best < 0.0 || us < best) { best = us; best_B = t.B_s; best_C = C_s; }
            if (static_cast<long>(t.B_s) * plan->geo.P <= 64) break;  // narrower grids only get slower
        }
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc != RAR_OK || best < 0.0) {
        plan->user_B_s = keep_B;
        plan->user_C_s = keep_C;
        return rc != RAR_OK ? rc : RAR_ERR_HIP;
    }
    plan->user_B_s = best_B;
    plan->user_C_s = best_C;
    if (best_us) *best_us = best;
    return RAR_OK;
}

int rar_launch_floor(rar_plan_t *plan, void *stream) {
    if (!plan) return RAR_ERR_ARG;
    Tuning t;
    int rc = fused_tuning(plan, rar::effective_mode(*plan) == RAR_MODE_FUSED_PACKED && plan->geo.L > 0, &t);
    if (rc != RAR_OK) return rc;
    return rar::launch_empty(static_cast<unsigned>(plan->geo.P) * t.B_s, as_stream(stream));
}

int rar_barrier_only(rar_plan_t *plan, void *stream) {
    if (!plan) return RAR_ERR_ARG;
    int rc = ensure_scratch(plan);
    if (rc != RAR_OK) return rc;
    Tuning t;
    rc = fused_tuning(plan, false, &t);
    if (rc != RAR_OK) return rc;
    hipStream_t st = as_stream(stream);
    rc = ensure_flags(plan, st);
    if (rc != RAR_OK) return rc;
    RankPtrs ptrs;
    std::memset(&ptrs, 0, sizeof ptrs);
    return rar::launch_fused(*plan, ptrs, t, false, st);
}

const char *rar_last_hip_error(void) { return rar::last_hip_error_string(); }

int rar_copy_probe(void *dst, const void *src, size_t bytes, void *stream) {
    if (!dst || !src) return RAR_ERR_ARG;
    if ((reinterpret_cast<uintptr_t>(dst) | reinterpret_cast<uintptr_t>(src) | bytes) % 16 != 0) return RAR_ERR_ALIGN;
    return rar::launch_copy(dst, src, bytes / 16, as_stream(stream));
}

}  // extern "C"
