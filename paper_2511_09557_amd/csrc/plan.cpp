// Planner and the host-only part of the C ABI (Algorithm 1's inputs and peer rule; the chunk
// partition; scratch layout).  No HIP calls in this file.
#include "plan.hpp"

#include <new>

namespace rar {

static int floor_log2(int v) {  // largest l with 2^l <= v, v >= 1
    int l = 0;
    while ((2 << l) <= v) ++l;
    return l;
}

int make_geometry(int P, int G, size_t n, int dtype, Geometry *geo) {
    if (!geo || P < 1 || G < 1 || n == 0) return RAR_ERR_ARG;
    if (dtype != RAR_BF16 && dtype != RAR_F32) return RAR_ERR_DTYPE;
    if (P > RAR_MAX_RANKS) return RAR_ERR_LIMIT;
    if (P % G != 0) return RAR_ERR_SHAPE;
    const int N = P / G;
    const int L = floor_log2(N);

    Geometry g;
    g.P = P; g.G = G; g.N = N; g.L = L; g.dtype = dtype; g.n = n;
    g.fold = N - (1 << L);
    g.elem_bytes = dtype == RAR_BF16 ? 2 : 4;
    g.per_vec = 16 / g.elem_bytes;
    const size_t per_rank = (n + static_cast<size_t>(G) - 1) / static_cast<size_t>(G);
    g.chunk_len = round_up(per_rank, g.per_vec);
    g.chunk_vecs = g.chunk_len / g.per_vec;
    // Vector indices inside a chunk, and G*chunk_vecs over a message, are 32-bit in the kernels.
    if (g.chunk_vecs * static_cast<size_t>(G) >= (static_cast<size_t>(1) << 31)) return RAR_ERR_LIMIT;
    g.chunk_stride = round_up(g.chunk_vecs * 16, kAlign);
    // A partial buffer is addressed through a buffer descriptor with 32-bit byte offsets.
    if (g.chunk_stride >= (static_cast<size_t>(1) << 32)) return RAR_ERR_LIMIT;
    g.flags_offset = kHeaderBytes;
    // One flag per (buffer S_l, rank, workgroup slot).  S_L is exchanged only when N is not a
    // power of two (it carries the result back to the nodes that sat out).
    g.flags_bytes = round_up(static_cast<size_t>(L + 1) * P * kMaxWorkgroupsPerRank * 4, kAlign);
    g.data_offset = g.flags_offset + g.flags_bytes;
    g.fused_bytes = g.data_offset + static_cast<size_t>(L + 1) * P * g.chunk_stride;
    g.scratch_bytes = g.fused_bytes;
    // Data+flag buffers for the packed exchange: one per (step l < L, rank), twice a chunk; one
    // more per rank if N is not a power of two (the last partial goes back to a node that sat out).
    if (L > 0 && g.chunk_vecs * 16 <= kPackedMaxChunkBytes) {
        g.packed_offset = g.scratch_bytes;
        g.packed_levels = L + (g.fold ? 1 : 0);
        // whole slices of the largest trip (8 vectors per thread): the word layout inside a
        // slice is strided by thread, so a ragged last slice still spans its full extent
        g.packed_stride = round_up(g.chunk_vecs, static_cast<size_t>(kThreads) * 8) * 32;
        g.scratch_bytes = g.packed_offset + static_cast<size_t>(g.packed_levels) * P * g.packed_stride;
        // Chained calls (rar_allreduce_chain) reuse an exchange buffer two calls later: a second
        // set of both kinds of buffers for the odd calls.  Only for these short chunks; longer
        // ones alternate between two places inside the first set instead.
        g.alt_offset = g.scratch_bytes;
        g.packed_alt_offset = g.alt_offset + static_cast<size_t>(L + 1) * P * g.chunk_stride;
        g.scratch_bytes = g.packed_alt_offset + static_cast<size_t>(g.packed_levels) * P * g.packed_stride;
    }
    *geo = g;
    return RAR_OK;
}

Tuning resolve_tuning(const rar_plan_t &plan, const long *max_resident) {
    const Geometry &g = plan.geo;
    const long units = plan.compute_units > 0 ? plan.compute_units : 256;
    auto cap_for = [&](int unroll_index) {
        long cap = kMaxWorkgroupsPerRank;
        // never wider than kMaxWorkgroupsPerCU per compute unit, nor than what the device holds at once
        long whole = kMaxWorkgroupsPerCU * units;
        if (max_resident && max_resident[unroll_index] > 0 && max_resident[unroll_index] < whole)
            whole = max_resident[unroll_index];
        long fit = whole / plan.concurrency / g.P;
        if (fit < 1) fit = 1;
        if (fit < cap) cap = fit;
        return cap;
    };
    const size_t V = g.chunk_vecs;
    auto slices = [&](int unroll) {
        return static_cast<long>((V + static_cast<size_t>(kThreads) * unroll - 1) /
                                 (static_cast<size_t>(kThreads) * unroll));
    };

    // Built-in choice, from a scan of all (B_s, C_s) on MI355X over P = 8..128, G = 1..8, 16 KiB to
    // 16 MiB, both types.  Four workgroups per compute unit keep the memory system busy, and
    // more of them only add step barriers (two per compute unit already do with four or more
    // steps, where barriers weigh more).  So: the smallest trip whose slices fit in that many
    // workgroups, one slice each.  A message too long for that runs 16 KiB trips on four
    // workgroups per compute unit (32 KiB trips when a rank reads at most two buffers per
    // element, so that a thread still has 16 loads in flight; half the workgroups when it
    // reads eight or more).
    const long target = 4L * units / plan.concurrency;
    const long small_target = g.L >= 4 ? target / 2 : target;
    long grid_cap = kMaxWorkgroupsPerRank;  // workgroups per rank beyond which the built-in choice does not go
    Tuning t{};
    int index = 3;
    if (plan.user_C_s) {
        t.unroll = static_cast<int>(plan.user_C_s / (static_cast<size_t>(kThreads) * 16));
        index = t.unroll == 1 ? 0 : t.unroll == 2 ? 1 : t.unroll == 4 ? 2 : 3;
    } else {
        index = 0;
        while (index < 2 && slices(1 << index) * g.P > small_target) ++index;
        if (slices(1 << index) * g.P > small_target) {
            if (g.G > 2 && slices(4) * g.P <= target) {
                index = 2;
            } else {  // the long-message regime
                index = g.G <= 2 ? 3 : 2;
                grid_cap = (g.G >= 8 ? target / 2 : target) / g.P;
                if (grid_cap < 1) grid_cap = 1;
                // Exactly two trips per workgroup leave every slice its own place in the partial
                // buffers, so their whole footprint is live; from three trips on a workgroup reuses
                // two places and the footprint halves with every halving of the trip.  Where the
                // messages plus that footprint exceed the 256 MiB memory-side cache, half-sized
                // trips (four per workgroup) measured up to 25 % faster (P = 128, 1 MiB per rank).
                const long all = slices(1 << index);
                const long width = all < grid_cap ? all : grid_cap;
                const size_t live = static_cast<size_t>(g.P) * g.n * g.elem_bytes + static_cast<size_t>(g.L) * g.P * g.chunk_stride;
                if (index > 0 && (all + width - 1) / width == 2 && live > (static_cast<size_t>(256) << 20)) --index;
            }
        }
        t.unroll = 1 << index;
    }
    const long cap = cap_for(index);
    const long all = slices(t.unroll);
    long want;
    if (plan.user_B_s) {
        want = plan.user_B_s < cap ? plan.user_B_s : cap;
        if (want > all) want = all;
    } else {
        want = all < cap ? all : cap;  // one slice per workgroup if the device can hold them all
        if (want > grid_cap) want = grid_cap;
    }
    if (want < 1) want = 1;
    t.B_s = static_cast<int>(want);
    t.iters = static_cast<int>((all + want - 1) / want);
    if (t.iters < 1) t.iters = 1;
    return t;
}

Tuning resolve_chain_tuning(const rar_plan_t &plan, const long *max_resident) {
    Tuning t = resolve_tuning(plan, max_resident);
    const Geometry &g = plan.geo;
    if (g.L == 0 || g.alt_offset != 0) return t;  // nothing is exchanged, or the odd calls have their own buffers
    // Two places per workgroup inside one partial buffer: 2 * B_s slices must fit in a chunk.
    const size_t slice = static_cast<size_t>(kThreads) * t.unroll;
    const size_t all = (g.chunk_vecs + slice - 1) / slice;
    size_t fit = g.chunk_stride / 16 / slice / 2;
    if (fit < 1) fit = 1;  // cannot happen: a plan without a second set has chunks of more than 256 KiB
    if (static_cast<size_t>(t.B_s) > fit) t.B_s = static_cast<int>(fit);
    t.iters = static_cast<int>((all + t.B_s - 1) / t.B_s);
    if (t.iters < 1) t.iters = 1;
    return t;
}

}  // namespace rar

using rar::Geometry;

extern "C" {

int rar_version(void) { return 200; }

const char *rar_strerror(int status) {
    switch (status) {
        case RAR_OK: return "ok";
        case RAR_ERR_ARG: return "invalid argument";
        case RAR_ERR_SHAPE: return "G must divide P";
        case RAR_ERR_DTYPE: return "unknown dtype";
        case RAR_ERR_LIMIT: return "size beyond the library's limits";
        case RAR_ERR_SCRATCH: return "scratch not set, too small or misaligned";
        case RAR_ERR_ALIGN: return "data pointer not 16-byte aligned";
        case RAR_ERR_HIP: return "HIP call failed";
        case RAR_ERR_TIMEOUT: return "step barrier wait timed out";
        case RAR_ERR_TUNING: return "unsupported B_s / C_s";
        case RAR_ERR_CAPTURE: return "first call of a plan (or first after a time-out) made during stream capture";
        default: return "unknown status";
    }
}

int rar_plan(int P, int G, size_t n, int dtype, rar_plan_t **out) {
    if (!out) return RAR_ERR_ARG;
    *out = nullptr;
    Geometry geo;
    int rc = rar::make_geometry(P, G, n, dtype, &geo);
    if (rc != RAR_OK) return rc;
    rar_plan_t *p = new (std::nothrow) rar_plan_t();
    if (!p) return RAR_ERR_ARG;
    p->geo = geo;
    *out = p;
    return RAR_OK;
}

int rar_plan_free(rar_plan_t *plan) {
    if (plan && plan->host_status && plan->release_host_status) plan->release_host_status(plan->host_status);
    delete plan;
    return RAR_OK;
}

int rar_plan_ranks(const rar_plan_t *plan) { return plan ? plan->geo.P : RAR_ERR_ARG; }
int rar_plan_nodes(const rar_plan_t *plan) { return plan ? plan->geo.N : RAR_ERR_ARG; }
int rar_plan_steps(const rar_plan_t *plan) { return plan ? plan->geo.L : RAR_ERR_ARG; }

int rar_plan_peer(const rar_plan_t *plan, int rank, int step) {
    if (!plan) return RAR_ERR_ARG;
    const Geometry &g = plan->geo;
    if (rank < 0 || rank >= g.P || step < 0 || step >= g.L) return RAR_ERR_ARG;
    const int r_n = rank / g.G, r_g = rank % g.G;
    if (rar::sits_out(r_n, g.fold)) return rank;
    return rar::node_of_number(rar::step_number(r_n, g.fold) ^ (1 << step), g.fold) * g.G + r_g;
}

int rar_plan_fold_partner(const rar_plan_t *plan, int rank) {
    if (!plan) return RAR_ERR_ARG;
    const Geometry &g = plan->geo;
    if (rank < 0 || rank >= g.P) return RAR_ERR_ARG;
    const int r_n = rank / g.G;
    if (rar::sits_out(r_n, g.fold)) return rank + g.G;
    if (rar::folds_in(r_n, g.fold)) return rank - g.G;
    return rank;
}

int rar_plan_chunk(const rar_plan_t *plan, int c, size_t *offset, size_t *length) {
    if (!plan || !offset || !length) return RAR_ERR_ARG;
    const Geometry &g = plan->geo;
    if (c < 0 || c >= g.G) return RAR_ERR_ARG;
    *offset = rar::chunk_begin(g, c);
    *length = rar::chunk_begin(g, c + 1) - *offset;
    return RAR_OK;
}

size_t rar_plan_scratch_bytes(const rar_plan_t *plan) { return plan ? plan->geo.scratch_bytes : 0; }

size_t rar_plan_static_bytes(const rar_plan_t *plan) { return plan ? plan->geo.fused_bytes : 0; }

int rar_plan_scratch_layout(const rar_plan_t *plan, size_t *flags_offset, size_t *flags_bytes,
                            size_t *packed_offset, size_t *packed_bytes) {
    if (!plan) return RAR_ERR_ARG;
    const Geometry &g = plan->geo;
    if (flags_offset) *flags_offset = g.flags_offset;
    if (flags_bytes) *flags_bytes = g.flags_bytes;
    if (packed_offset) *packed_offset = g.packed_offset;
    if (packed_bytes) *packed_bytes = g.packed_offset ? g.scratch_bytes - g.packed_offset : 0;
    return RAR_OK;
}

int rar_plan_set_scratch(rar_plan_t *plan, void *scratch, size_t bytes) {
    if (!plan) return RAR_ERR_ARG;
    if (!scratch || bytes < plan->geo.scratch_bytes ||
        reinterpret_cast<uintptr_t>(scratch) % rar::kAlign != 0)
        return RAR_ERR_SCRATCH;
    plan->scratch = scratch;
    plan->scratch_size = bytes;
    plan->flags_clean = false;
    plan->packed_clean = false;
    return RAR_OK;
}

int rar_plan_set_mode(rar_plan_t *plan, int mode) {
    if (!plan) return RAR_ERR_ARG;
    if (mode != RAR_MODE_STEPWISE && mode != RAR_MODE_FUSED && mode != RAR_MODE_FUSED_PACKED && mode != RAR_MODE_AUTO)
        return RAR_ERR_ARG;
    // N = 1 has no exchange at all: the packed mode is then the plain fused kernel.
    if (mode == RAR_MODE_FUSED_PACKED && plan->geo.L > 0 && plan->geo.packed_offset == 0) return RAR_ERR_LIMIT;
    plan->mode = mode;
    return RAR_OK;
}

int rar_plan_get_mode(const rar_plan_t *plan) { return plan ? plan->mode : RAR_ERR_ARG; }

int rar_plan_effective_mode(const rar_plan_t *plan) { return plan ? rar::effective_mode(*plan) : RAR_ERR_ARG; }

int rar_plan_set_tuning(rar_plan_t *plan, int B_s, size_t C_s) {
    if (!plan) return RAR_ERR_ARG;
    if (B_s < 0 || B_s > rar::kMaxWorkgroupsPerRank) return RAR_ERR_TUNING;
    if (C_s != 0 && C_s != 4096 && C_s != 8192 && C_s != 16384 && C_s != 32768) return RAR_ERR_TUNING;
    plan->user_B_s = B_s;
    plan->user_C_s = C_s;
    return RAR_OK;
}

int rar_plan_get_tuning(const rar_plan_t *plan, int *B_s, size_t *C_s) {
    if (!plan || !B_s || !C_s) return RAR_ERR_ARG;
    const long *resident = !plan->have_occupancy ? nullptr
                           : rar::effective_mode(*plan) == RAR_MODE_FUSED_PACKED ? plan->resident_packed : plan->resident;
    rar::Tuning t = rar::resolve_tuning(*plan, resident);
    *B_s = t.B_s;
    *C_s = static_cast<size_t>(rar::kThreads) * 16 * t.unroll;
    return RAR_OK;
}

int rar_plan_set_concurrency(rar_plan_t *plan, int k) {
    if (!plan || k < 1 || k > 8) return RAR_ERR_ARG;
    plan->concurrency = k;
    return RAR_OK;
}

int rar_plan_set_wait_limit_us(rar_plan_t *plan, uint64_t microseconds) {
    if (!plan) return RAR_ERR_ARG;
    plan->wait_limit_us = microseconds;
    return RAR_OK;
}

}  // extern "C"
