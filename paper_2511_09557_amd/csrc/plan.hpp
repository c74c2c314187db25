// Host-side schedule of the hierarchical recursive-doubling all-reduce (Algorithm 1 of the
// paper): who is whose peer at which step, which elements form which chunk, where every
// per-step partial buffer and barrier flag lives in the scratch.  Pure integer logic; no HIP.
#pragma once

#include <cstddef>
#include <cstdint>

#include "rar.h"

namespace rar {

constexpr int kThreads = 256;           // threads per workgroup of every kernel
constexpr int kMaxWorkgroupsPerRank = 256;
// No fused launch is wider than this many workgroups per compute unit, whatever the occupancy
// query says.  The step barriers spin, so the whole grid has to be resident at once, and the
// query's figure is arithmetic on register counts with no margin: launches sized exactly to it
// (7 per compute unit, a figure set by scalar registers) once ended in step-barrier time-outs on
// one machine.  Four per compute unit is also where the measured optimum lies: more workgroups
// only add step barriers.
constexpr int kMaxWorkgroupsPerCU = 4;
constexpr int kMaxChainCalls = 1 << 16; // calls in one rar_allreduce_chain launch
constexpr size_t kHeaderBytes = 256;    // scratch header: status word at offset 0
constexpr size_t kAlign = 256;
// The fused data+flag exchange doubles the exchanged bytes, so it is offered for small messages
// only: chunks of at most this many bytes (a 1 MiB message at G = 4).
constexpr size_t kPackedMaxChunkBytes = 256 * 1024;

inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

struct Geometry {
    int P = 0, G = 0, N = 0, L = 0;
    int fold = 0;            // r in N = 2^L + r: the first 2r nodes are folded pairwise (0 = N is a power of two)
    int dtype = RAR_BF16;
    size_t n = 0;            // elements per rank
    size_t elem_bytes = 0;   // 2 or 4
    size_t per_vec = 0;      // elements per 16-byte vector (8 or 4)
    size_t chunk_len = 0;    // elements per full chunk (multiple of per_vec)
    size_t chunk_vecs = 0;   // 16-byte vectors per full chunk
    size_t chunk_stride = 0; // bytes between consecutive S buffers in the scratch
    size_t flags_offset = 0; // byte offset of the barrier flags in the scratch
    size_t flags_bytes = 0;
    size_t data_offset = 0;  // byte offset of S_0(rank 0)
    size_t packed_offset = 0;  // byte offset of the data+flag buffers (0 = the plan has none)
    size_t packed_stride = 0;  // bytes of one data+flag buffer: 2 * chunk bytes, rounded
    int packed_levels = 0;     // data+flag buffers per rank: L, or L + 1 if N is not a power of two
    // A second set of exchange buffers, used by the odd calls of a chained launch (0 = none: the
    // plan's chunks are too long for it, and a chain then alternates between two places inside
    // the first set).  Same shape as the first set.
    size_t alt_offset = 0;         // second set of partial buffers S_0..S_L
    size_t packed_alt_offset = 0;  // second set of data+flag buffers
    size_t fused_bytes = 0;        // header + flags + first set of partial buffers: what the flag exchange needs
    size_t scratch_bytes = 0;
};

}  // namespace rar

struct rar_plan_s {
    rar::Geometry geo;
    int mode = RAR_MODE_AUTO;
    int user_B_s = 0;          // 0 = built-in choice
    size_t user_C_s = 0;       // 0 = built-in choice
    uint64_t wait_limit_us = 5000000;
    int concurrency = 1;       // fused kernels of different plans the caller runs at the same time
    void *scratch = nullptr;   // device, borrowed
    size_t scratch_size = 0;
    bool flags_clean = false;  // header + flags zeroed since the last event that invalidated them
    bool packed_clean = false; // data+flag buffers zeroed (no stale word can match a sequence number)
    long resident[4] = {0, 0, 0, 0};  // cached residency of the fused kernel per unroll 1,2,4,8
    long resident_packed[4] = {0, 0, 0, 0};  // same for the packed fused kernel
    bool have_occupancy = false;   // the four figures above are known
    bool have_resident = false;    // ... and the plan's host-side set-up (time-out word, ordering event) is done
    long resident_chain[4] = {0, 0, 0, 0};         // same for the kernels that run a chain of calls
    long resident_chain_packed[4] = {0, 0, 0, 0};
    bool have_resident_chain = false;
    int compute_units = 256;   // of the device the residency was measured on (MI355X until then)
    int device = -1;           // the device of the first launch
    bool ran_static = false;   // rar_allreduce_static has run on this plan (its time-outs sit in the library's array)
    unsigned long static_epoch = 0;  // time-outs found in that array, by any plan, when this plan first ran on it
    // One word of pinned host memory that a kernel sets when a step-barrier wait gives up, so that
    // the next call can refuse to run without synchronising anything.  Allocated at the first
    // launch by the part of the library that may call HIP, released through `release_host_status`.
    volatile uint32_t *host_status = nullptr;
    uint32_t *host_status_dev = nullptr;  // the same word as the device addresses it
    void (*release_host_status)(volatile uint32_t *) = nullptr;
};

namespace rar {

// Fill geo from (P, G, n, dtype); returns a rar_status.
int make_geometry(int P, int G, size_t n, int dtype, Geometry *geo);

// N = 2^L + r that is not a power of two (outside the paper, whose Algorithm 1 assumes 2^L
// nodes): the customary extension of recursive doubling.  Nodes (2i, 2i+1), i < r, pair up; the
// even one hands its reduce-scatter result to the odd one and sits out; the 2^L nodes that
// remain are renumbered (node 2i+1 -> i, node j >= 2r -> j - r) and run the L steps on those
// numbers; the odd node finally hands the result back to its even partner.
inline bool sits_out(int r_n, int fold) { return r_n < 2 * fold && (r_n % 2) == 0; }
inline bool folds_in(int r_n, int fold) { return r_n < 2 * fold && (r_n % 2) == 1; }
inline int step_number(int r_n, int fold) { return r_n < 2 * fold ? r_n / 2 : r_n - fold; }
inline int node_of_number(int v, int fold) { return v < fold ? 2 * v + 1 : v + fold; }

inline size_t chunk_begin(const Geometry &g, int c) {
    size_t b = static_cast<size_t>(c) * g.chunk_len;
    return b < g.n ? b : g.n;
}

// Byte offset of S_l(rank) in the scratch (set 0, or set 1 for the odd calls of a chain).
inline size_t partial_offset(const Geometry &g, int level, int rank, int set = 0) {
    return (set ? g.alt_offset : g.data_offset) + (static_cast<size_t>(level) * g.P + rank) * g.chunk_stride;
}

struct Tuning {
    int B_s;      // workgroups per rank
    int unroll;   // 16-byte vectors per thread per trip (C_s = kThreads * 16 * unroll)
    int iters;    // trips per workgroup: ceil(chunk_vecs / (B_s * kThreads * unroll))
};

// The mode a call runs in: RAR_MODE_AUTO takes the data+flag exchange while all ranks together
// exchange at most 1 MiB per step (measured on MI355X: 8 KiB..1 MiB messages, P = 8..128: up to
// there it is 5-25 % faster than the flag exchange, beyond it doubling the bytes costs more than
// the flags), the flag exchange otherwise.
constexpr size_t kAutoPackedMaxStepBytes = 1u << 20;
inline int effective_mode(const rar_plan_t &plan) {
    if (plan.mode != RAR_MODE_AUTO) return plan.mode;
    const Geometry &g = plan.geo;
    const bool small = static_cast<size_t>(g.P) * g.chunk_vecs * 16 <= kAutoPackedMaxStepBytes;
    return g.L > 0 && g.packed_offset != 0 && small ? RAR_MODE_FUSED_PACKED : RAR_MODE_FUSED;
}

// Resolve the plan's tuning.  max_resident[i] = workgroups the device can hold at once for
// the fused kernel with unroll 1 << i (nullptr or 0 = no residency limit, for host-only use).
Tuning resolve_tuning(const rar_plan_t &plan, const long *max_resident);

// The tuning of a chained launch (rar_allreduce_chain): the plan's tuning, narrowed where needed
// so that a workgroup has two places of its own in every partial buffer when the plan has no
// second set of buffers (its trips then alternate between the two places across calls).
Tuning resolve_chain_tuning(const rar_plan_t &plan, const long *max_resident);

}  // namespace rar
