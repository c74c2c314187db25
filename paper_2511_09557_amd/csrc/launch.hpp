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
// of two; chain = the variant that runs several calls in one launch) the current device can
// hold at once.
int fused_max_resident(int dtype, int G, int unroll, bool packed, bool fold, bool chain, long *out);

// Zero `bytes` bytes at `words`; the 8 bytes at offset 8 receive the address `at_word_2` (the
// scratch header's pointer to the host's time-out word; nullptr for a plain zero fill).
int launch_fill_zero(void *words, size_t bytes, const void *at_word_2, hipStream_t stream);
// scratch: the memory the launch works on (the plan's, or the library's static array);
// calls = 0: one all-reduce; calls >= 1: a chain of that many in one launch.
int launch_fused(const rar_plan_t &plan, void *scratch, const RankPtrs &bufs, const Tuning &t, bool data, int calls,
                 hipStream_t stream);
int launch_fused_packed(const rar_plan_t &plan, const RankPtrs &bufs, const Tuning &t, int calls, hipStream_t stream);
int launch_stepwise(const rar_plan_t &plan, const RankPtrs &bufs, hipStream_t stream);
int launch_empty(unsigned grid, hipStream_t stream);
int launch_combine(void *dst, const void *src, size_t full_vecs, unsigned tail, int dtype, hipStream_t stream);
int launch_copy(void *dst, const void *src, size_t vecs, hipStream_t stream);
int launch_read(void *sink, const void *src, size_t vecs, hipStream_t stream);

}  // namespace rar
