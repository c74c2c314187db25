// Internal interface between the C ABI (api.hip) and the kernels (kernels.hip).
#pragma once

#include <hip/hip_runtime_api.h>

#include "plan.hpp"

namespace rar {

// Device pointers of all ranks' messages, passed to kernels by value (kernel arguments), so
// that a call needs no device-side table and no host-to-device copy.
struct RankPtrs {
    void *p[RAR_MAX_RANKS];
};

struct DeviceInfo {
    int compute_units;
};

int device_info(DeviceInfo *out);

// Remember a failing HIP status (returns its argument); text of the last one remembered.
hipError_t note_hip(hipError_t e);
const char *last_hip_error_string();

// Workgroups of the fused kernel (dtype, G, unroll; fold = the variant for N that is not a power
// of two) the current device can hold at once.
int fused_max_resident(int dtype, int G, int unroll, bool packed, bool fold, long *out);

int launch_fill_zero(void *words, size_t bytes, hipStream_t stream);
int launch_fused(const rar_plan_t &plan, const RankPtrs &bufs, const Tuning &t, bool data, hipStream_t stream);
int launch_fused_packed(const rar_plan_t &plan, const RankPtrs &bufs, const Tuning &t, hipStream_t stream);
int launch_stepwise(const rar_plan_t &plan, const RankPtrs &bufs, hipStream_t stream);
int launch_empty(unsigned grid, hipStream_t stream);
int launch_combine(void *dst, const void *src, size_t full_vecs, unsigned tail, int dtype, hipStream_t stream);
int launch_copy(void *dst, const void *src, size_t vecs, hipStream_t stream);

}  // namespace rar
