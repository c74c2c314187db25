// gfx950 kernels of the hierarchical recursive-doubling all-reduce (Algorithm 1 and Section
// 4.1 of the paper) and their launchers.  HBM-bound streaming work: 16-byte vector loads and
// stores, binary32 accumulation, no matrix cores.
//
// Vocabulary: a rank's message is cut into G chunks; chunk c belongs to local rank c.  A
// chunk is cut into slices of kThreads*U 16-byte vectors; a workgroup moves one slice per
// trip (the paper's C_s), and B_s workgroups serve a rank (Section 4.2.1).  S_l(p) is rank
// p's partial after l inter-node steps, one scratch buffer per step so that a rank may run
// ahead of its peer (Section 4.2.1, per-step send/receive buffers).
#include <hip/hip_runtime.h>

#include <cstdint>
#include <mutex>

#include "launch.hpp"

namespace rar {

typedef uint32_t u32;
typedef uint64_t u64;

// ---- element arithmetic -----------------------------------------------------------------------

__device__ __forceinline__ float bits_f(u32 u) { return __uint_as_float(u); }
__device__ __forceinline__ u32 f_bits(float f) { return __float_as_uint(f); }

// binary32 -> bf16 bits, round to nearest, ties to even; NaN stays NaN (quiet).
__device__ __forceinline__ u32 narrow_bf16(float f) {
    const u32 u = f_bits(f);
    const u32 r = (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
    return (u & 0x7fffffffu) > 0x7f800000u ? ((u >> 16) | 0x40u) : r;
}

// A 16-byte vector as binary32 lanes: 8 for bf16, 4 for fp32.
template <int DT> struct Lanes;
template <> struct Lanes<RAR_BF16> {
    static constexpr int kCount = 8;
    float f[8];
    __device__ __forceinline__ void widen(const uint4 &v) {
        f[0] = bits_f(v.x << 16); f[1] = bits_f(v.x & 0xffff0000u);
        f[2] = bits_f(v.y << 16); f[3] = bits_f(v.y & 0xffff0000u);
        f[4] = bits_f(v.z << 16); f[5] = bits_f(v.z & 0xffff0000u);
        f[6] = bits_f(v.w << 16); f[7] = bits_f(v.w & 0xffff0000u);
    }
    __device__ __forceinline__ uint4 narrow() const {
        uint4 v;
        v.x = narrow_bf16(f[0]) | (narrow_bf16(f[1]) << 16);
        v.y = narrow_bf16(f[2]) | (narrow_bf16(f[3]) << 16);
        v.z = narrow_bf16(f[4]) | (narrow_bf16(f[5]) << 16);
        v.w = narrow_bf16(f[6]) | (narrow_bf16(f[7]) << 16);
        return v;
    }
};
template <> struct Lanes<RAR_F32> {
    static constexpr int kCount = 4;
    float f[4];
    __device__ __forceinline__ void widen(const uint4 &v) {
        f[0] = bits_f(v.x); f[1] = bits_f(v.y); f[2] = bits_f(v.z); f[3] = bits_f(v.w);
    }
    __device__ __forceinline__ uint4 narrow() const {
        return make_uint4(f_bits(f[0]), f_bits(f[1]), f_bits(f[2]), f_bits(f[3]));
    }
};

template <int DT>
__device__ __forceinline__ void add_into(Lanes<DT> &acc, const uint4 &v) {
    Lanes<DT> t;
    t.widen(v);
#pragma unroll
    for (int i = 0; i < Lanes<DT>::kCount; ++i) acc.f[i] = acc.f[i] + t.f[i];
}

// narrow( widen(a) + widen(b) ): one exchange-and-sum on a vector.
template <int DT>
__device__ __forceinline__ uint4 combine(const uint4 &a, const uint4 &b) {
    Lanes<DT> acc;
    acc.widen(a);
    add_into<DT>(acc, b);
    return acc.narrow();
}

__device__ __forceinline__ uint4 ld16(const void *base, u64 vec) {
    return reinterpret_cast<const uint4 *>(base)[vec];
}
__device__ __forceinline__ void st16(void *base, u64 vec, const uint4 &v) {
    reinterpret_cast<uint4 *>(base)[vec] = v;
}

// The one vector of a message that is only partly inside it (n not a multiple of the vector
// width): element-wise access, padding with zeros.
template <int DT>
__device__ __forceinline__ uint4 ld_partial(const void *base, u64 vec, u32 count) {
    u32 w[4] = {0u, 0u, 0u, 0u};
    if (DT == RAR_BF16) {
        const uint16_t *e = reinterpret_cast<const uint16_t *>(base) + vec * 8;
        for (u32 i = 0; i < count; ++i) w[i >> 1] |= static_cast<u32>(e[i]) << ((i & 1u) * 16);
    } else {
        const u32 *e = reinterpret_cast<const u32 *>(base) + vec * 4;
        for (u32 i = 0; i < count; ++i) w[i] = e[i];
    }
    return make_uint4(w[0], w[1], w[2], w[3]);
}
template <int DT>
__device__ __forceinline__ void st_partial(void *base, u64 vec, u32 count, const uint4 &v) {
    const u32 w[4] = {v.x, v.y, v.z, v.w};
    if (DT == RAR_BF16) {
        uint16_t *e = reinterpret_cast<uint16_t *>(base) + vec * 8;
        for (u32 i = 0; i < count; ++i) e[i] = static_cast<uint16_t>(w[i >> 1] >> ((i & 1u) * 16));
    } else {
        u32 *e = reinterpret_cast<u32 *>(base) + vec * 4;
        for (u32 i = 0; i < count; ++i) e[i] = w[i];
    }
}

// Message vector `m` of a rank's buffer: whole, partial (the last one) or outside.
template <int DT>
__device__ __forceinline__ uint4 ld_message(const void *base, u32 m, u32 full_vecs, u32 tail) {
    if (m < full_vecs) return ld16(base, m);
    if (m == full_vecs && tail) return ld_partial<DT>(base, m, tail);
    return make_uint4(0u, 0u, 0u, 0u);
}
template <int DT>
__device__ __forceinline__ void st_message(void *base, u32 m, u32 full_vecs, u32 tail, const uint4 &v) {
    if (m < full_vecs) st16(base, m, v);
    else if (m == full_vecs && tail) st_partial<DT>(base, m, tail, v);
}

// ---- the three phases on one slice ---------------------------------------------------------

struct Shape {
    unsigned char *scratch;  // device
    u64 chunk_stride;        // bytes between S buffers
    u64 flags_offset;
    u64 data_offset;
    u64 alt_offset;          // second set of S buffers for the odd calls of a chain (0 = none)
    u64 packed_offset;       // data+flag buffers of the packed exchange
    u64 packed_alt_offset;   // their second set
    u64 packed_stride;
    u64 wait_ticks;          // step-barrier time limit in 100 MHz ticks
    u32 P, G, N, L;
    u32 fold;                // r in N = 2^L + r (0 when N is a power of two)
    u32 chunk_vecs;          // vectors per full chunk
    u32 full_vecs;           // whole vectors in a message
    u32 tail;                // elements in the partial last vector (0 = none)
    u32 flag_stride;         // 32-bit words between the flags of consecutive workgroup slots
    u32 B_s;                 // workgroups per rank
    u32 iters;               // trips per workgroup and call
    u32 calls;               // all-reduces in this launch (1 unless it is a chain)
};

// S_l(rank); set 1 is the second set that the odd calls of a chain use.
__device__ __forceinline__ unsigned char *partial_buf(const Shape &s, u32 level, u32 rank, u32 set = 0u) {
    return s.scratch + (set ? s.alt_offset : s.data_offset) + (static_cast<u64>(level) * s.P + rank) * s.chunk_stride;
}

// Vectors of chunk c that lie inside the message (the last chunks may be short or empty).
__device__ __forceinline__ u32 chunk_valid_vecs(const Shape &s, u32 c) {
    const u32 total = s.full_vecs + (s.tail ? 1u : 0u);
    const u64 begin = static_cast<u64>(c) * s.chunk_vecs;
    if (begin >= total) return 0u;
    const u64 left = total - begin;
    return left < s.chunk_vecs ? static_cast<u32>(left) : s.chunk_vecs;
}

// Phase 1 on one slice: part[u] = narrow( x(r_n,0) + x(r_n,1) + .. + x(r_n,G-1) ), binary32,
// local rank order (Section 4.1, reduce-scatter).  GT = compile-time G, 0 = run-time G.
template <int DT, int GT, int U>
__device__ __forceinline__ void reduce_scatter_slice(const RankPtrs &bufs, const Shape &s, u32 r_n,
                                                     u32 c, u32 v0, u32 valid, bool whole,
                                                     uint4 (&part)[U]) {
    const u32 G = GT ? GT : s.G;
    const u32 mbase = c * s.chunk_vecs;
    Lanes<DT> acc[U];
    if (whole) {
        // every vector of the slice is a whole vector inside the message: no checks
        // buffers loaded per batch: all of them when G is known and small, else four at a time
        constexpr int GB = GT == 0 ? 4 : (GT * U <= 32 ? GT : (32 / U > 0 ? 32 / U : 1));
        uint4 in[GB][U];
#pragma unroll
        for (int u = 0; u < U; ++u) acc[u].widen(ld16(bufs.p[r_n * G], mbase + v0 + u * kThreads));
        for (u32 g0 = 1; g0 < G; g0 += GB) {
#pragma unroll
            for (int gb = 0; gb < GB; ++gb) {
                if (g0 + gb < G) {
                    const void *x = bufs.p[r_n * G + g0 + gb];
#pragma unroll
                    for (int u = 0; u < U; ++u) in[gb][u] = ld16(x, mbase + v0 + u * kThreads);
                }
            }
#pragma unroll
            for (int gb = 0; gb < GB; ++gb) {
                if (g0 + gb < G) {
#pragma unroll
                    for (int u = 0; u < U; ++u) add_into<DT>(acc[u], in[gb][u]);
                }
            }
        }
    } else {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const u32 v = v0 + u * kThreads;
            if (v < valid) {
                acc[u].widen(ld_message<DT>(bufs.p[r_n * G], mbase + v, s.full_vecs, s.tail));
                for (u32 g = 1; g < G; ++g)
                    add_into<DT>(acc[u], ld_message<DT>(bufs.p[r_n * G + g], mbase + v, s.full_vecs, s.tail));
            } else {
                acc[u].widen(make_uint4(0u, 0u, 0u, 0u));
            }
        }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) part[u] = acc[u].narrow();
}

// Phase 3 on one slice: put the reduced slice into chunk c of all G buffers of the node
// (Section 4.1, all-gather).
template <int DT, int GT, int U>
__device__ __forceinline__ void all_gather_slice(const RankPtrs &bufs, const Shape &s, u32 r_n, u32 c,
                                                 u32 v0, u32 valid, bool whole, const uint4 (&part)[U]) {
    const u32 G = GT ? GT : s.G;
    const u32 mbase = c * s.chunk_vecs;
    for (u32 g = 0; g < G; ++g) {
        void *x = bufs.p[r_n * G + g];
        if (whole) {
#pragma unroll
            for (int u = 0; u < U; ++u) st16(x, mbase + v0 + u * kThreads, part[u]);
        } else {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const u32 v = v0 + u * kThreads;
                if (v < valid) st_message<DT>(x, mbase + v, s.full_vecs, s.tail, part[u]);
            }
        }
    }
}

template <int U>
__device__ __forceinline__ void store_slice(unsigned char *S, u32 v0, u32 valid, bool whole,
                                            const uint4 (&part)[U]) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const u32 v = v0 + u * kThreads;
        if (whole || v < valid) st16(S, v, part[u]);
    }
}

template <int U>
__device__ __forceinline__ void load_slice(const unsigned char *S, u32 v0, u32 valid, bool whole,
                                           uint4 (&out)[U]) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const u32 v = v0 + u * kThreads;
        out[u] = (whole || v < valid) ? ld16(S, v) : make_uint4(0u, 0u, 0u, 0u);
    }
}

// Device-coherent access to a partial buffer that another workgroup (possibly on another XCD,
// behind another L2) produces or consumes inside the same launch.  The "sc1" cache policy
// makes each 16-byte store write through to device scope and each load fetch from device
// scope, so no cache-wide write-back or invalidate is needed around the step barrier.  The
// buffer descriptor bounds every access to the partial buffer (out-of-range lanes are
// dropped by the hardware).
typedef u32 u32x4 __attribute__((ext_vector_type(4)));
constexpr int kDeviceScope = 16;            // cache-policy bit "sc1"
constexpr u32 kRawBufferFlags = 0x00020000; // 32-bit raw buffer, no swizzle

__device__ __forceinline__ __amdgpu_buffer_rsrc_t partial_rsrc(const Shape &s, u32 level, u32 rank, u32 set = 0u) {
    return __builtin_amdgcn_make_buffer_rsrc(partial_buf(s, level, rank, set), 0, static_cast<u32>(s.chunk_stride),
                                             kRawBufferFlags);
}

// s0 = where in the partial buffer this thread's first vector lives (the slice's own place, or
// the workgroup's ring slot); v0 / valid / whole say which of the thread's vectors exist.
template <int U>
__device__ __forceinline__ void store_slice_coherent(__amdgpu_buffer_rsrc_t S, u32 s0, u32 v0, u32 valid, bool whole,
                                                     const uint4 (&part)[U]) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const u32 v = v0 + u * kThreads;
        if (whole || v < valid) {
            u32x4 t = {part[u].x, part[u].y, part[u].z, part[u].w};
            __builtin_amdgcn_raw_buffer_store_b128(t, S, (s0 + u * kThreads) * 16u, 0, kDeviceScope);
        }
    }
}

template <int U>
__device__ __forceinline__ void load_slice_coherent(__amdgpu_buffer_rsrc_t S, u32 s0, u32 v0, u32 valid, bool whole,
                                                    uint4 (&out)[U]) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const u32 v = v0 + u * kThreads;
        if (whole || v < valid) {
            const u32x4 t = __builtin_amdgcn_raw_buffer_load_b128(S, (s0 + u * kThreads) * 16u, 0, kDeviceScope);
            out[u] = make_uint4(t.x, t.y, t.z, t.w);
        } else {
            out[u] = make_uint4(0u, 0u, 0u, 0u);
        }
    }
}

// ---- step barrier (Algorithm 1: "wait until flag(dst_q) == seq") ---------------------------
//
// One 32-bit flag per (step buffer, rank, workgroup slot).  The value is a trip counter that
// only ever grows (the paper's sequence number: flags are never cleared between calls), so a
// consumer waits for "at least the value of my own trip", compared as a signed difference.

// A (buffer, rank) owns kMaxWorkgroupsPerRank words, and a launch spreads its B_s flags over them
// (flags that share a cache line serialise their stores and polls).  The spacing may change from
// call to call: whichever word a launch uses, it uses for every buffer and every rank and stamps
// with the same tickets, so all copies of one word index always hold the same count.
__device__ __forceinline__ u32 *flag_ptr(const Shape &s, u32 level, u32 rank, u32 slot) {
    u32 *flags = reinterpret_cast<u32 *>(s.scratch + s.flags_offset);
    return flags + (static_cast<u64>(level) * s.P + rank) * kMaxWorkgroupsPerRank + slot * s.flag_stride;
}

// The workgroup's stores to S were issued at device scope; once every wave has seen them
// complete, thread 0 raises the flag (also at device scope).
__device__ __forceinline__ void publish(u32 *flag, u32 value) {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0);  // this wave's write-through stores have completed
    __syncthreads();
    if (threadIdx.x == 0) __hip_atomic_store(flag, value, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// A launch in which a wait ran out of time tells the host before it ends: the scratch header
// (words 2 and 3) holds the device address of a word of pinned host memory (0 = none) that the
// host reads, without any synchronisation, before it enqueues the plan's next launch.  (Word 0 of
// the header is the status word that makes all other waits on the device give up quickly.)
__device__ __forceinline__ void tell_host(const Shape &s, bool gave_up) {
    if (gave_up) {
        const u32 *header = reinterpret_cast<const u32 *>(s.scratch);
        const u64 lo = __hip_atomic_load(header + 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const u64 hi = __hip_atomic_load(header + 3, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        u32 *host_word = reinterpret_cast<u32 *>(lo | (hi << 32));
        if (host_word) __hip_atomic_store(host_word, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    }
}

// Thread 0 polls; the wait is bounded by wall-clock time and by the shared status word, so
// every workgroup leaves the kernel even if a peer never arrives.  The loads of S that follow
// are device-scope loads, so nothing has to be invalidated here.
__device__ __forceinline__ void wait_for(const Shape &s, const u32 *flag, u32 expect, bool &gave_up) {
    if (threadIdx.x == 0) {
        if (!gave_up) {
            u32 *status = reinterpret_cast<u32 *>(s.scratch);
            const u64 t0 = wall_clock64();
            u32 spins = 0;
            for (;;) {
                const u32 seen = __hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (static_cast<int>(seen - expect) >= 0) break;
                __builtin_amdgcn_s_sleep(1);
                if ((++spins & 31u) == 0u || s.wait_ticks == 0u) {  // a limit of 0: give up after the first look (tests)
                    const bool late = wall_clock64() - t0 > s.wait_ticks;
                    if (late) __hip_atomic_store(status, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    if (late || __hip_atomic_load(status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) {
                        gave_up = true;
                        break;
                    }
                }
            }
        }
    }
    __syncthreads();
}

// N = 2^L + r nodes with r > 0 (outside the paper, whose Algorithm 1 assumes N = 2^L): the
// customary extension of recursive doubling.  Nodes (2i, 2i+1), i < r, pair up; the even one
// hands its reduce-scatter result to the odd one and sits out; the 2^L nodes that remain take
// the numbers (node 2i+1 -> i, node j >= 2r -> j - r) on which the XOR peer rule acts; the odd
// node finally hands the result back.  With r = 0 every node keeps its own number.
__device__ __forceinline__ bool sits_out(u32 r_n, u32 fold) { return r_n < 2u * fold && (r_n & 1u) == 0u; }
__device__ __forceinline__ bool folds_in(u32 r_n, u32 fold) { return r_n < 2u * fold && (r_n & 1u) == 1u; }
__device__ __forceinline__ u32 peer_node(u32 r_n, u32 l, u32 fold) {
    const u32 number = r_n < 2u * fold ? r_n >> 1 : r_n - fold;
    const u32 v = number ^ (1u << l);
    return v < fold ? 2u * v + 1u : v + fold;
}

// Workgroup index -> (node, chunk, slot): the N workgroups (one per node) that exchange one
// (chunk, slot) get consecutive indices.  They are dispatched together, and since workgroups
// are dealt to the 8 XCDs round-robin by index they sit on different XCDs.  Measured against a
// mapping that puts all N on one XCD: the exchange is device-scope traffic either way, and
// spreading it over the XCDs is 2-8 % faster (c2 6.6 vs 7.2 us, c3 20.3 vs 21.8 us).
__device__ __forceinline__ void locate(const Shape &s, u32 block, u32 &r_n, u32 &c, u32 &slot) {
    const u32 pair = block / s.N;
    r_n = block % s.N;
    c = pair % s.G;
    slot = pair / s.G;
}

// ---- the fused schedule: phases 1-3 of Algorithm 1 in one persistent launch -----------------
//
// Workgroup (rank p = (r_n, c), slot w) owns slices w, w + B_s, .. of chunk c.  Per slice:
// reduce-scatter into registers, publish S_0, then for each step wait for the peer's S_l,
// add it to the partial held in registers, publish S_{l+1} (the last step's result is not
// exchanged, so it is not written to scratch), finally all-gather from registers.  If N is not
// a power of two, a rank that sits out publishes S_0 and all-gathers its partner's S_L, and the
// partner adds that S_0 to its own before the steps and publishes S_L after them.
// DATA = false leaves all data movement out (barrier traffic only, for measurement).
// FOLD = false compiles the hand-over for N that is not a power of two out (Algorithm 1 as it
// stands); ONE = true is the launch in which every workgroup makes a single trip (no loop, no
// reuse of places); FULL = true the launch whose slices are all whole slices inside the message
// (the host checks it: no ragged chunk, no tail, no trip past the chunk).  Each measured 1-5 %
// faster than the run-time branches.
//
// CHAIN = true runs s.calls all-reduces one after the other, each on the result of the one
// before (Section 4.2.1 and 4.2.3: a rank goes on to its next call without waiting for the
// others to finish this one).  A workgroup's slices are the same in every call, and chunk c of
// the G buffers of a node is read (reduce-scatter) and written (all-gather) by rank (r_n, c)
// alone, so what a workgroup reads in call k+1 is what the same threads wrote in call k: no
// barrier between calls.  The trips of all calls form one sequence T = 0, 1, ..: the flag
// tickets just keep counting, and an exchange buffer is written again only two trips (or two
// calls) later, in the other of two places: the odd calls use the second set of buffers if the
// plan has one, else trip T uses place T mod 2 of the workgroup's two places in the first set
// (the host narrows B_s so that they fit).  By then the reader of the old contents is done:
// the writer has since waited, at the same step of the trip in between, for a flag that this
// reader raises only after the trip in which it read.
template <int DT, int GT, int U, bool DATA, bool FOLD, bool ONE, bool FULL, bool CHAIN>
__global__ __launch_bounds__(kThreads) void fused_kernel(RankPtrs bufs, Shape s) {
    static_assert(!(CHAIN && ONE), "a chain makes several trips");
    u32 r_n, c, w;
    locate(s, blockIdx.x, r_n, c, w);
    const u32 G = GT ? GT : s.G;
    const u32 p = r_n * G + c;
    const u32 valid_vecs = chunk_valid_vecs(s, c);
    // vectors of this chunk that are whole vectors of the message
    const u64 cbegin = static_cast<u64>(c) * s.chunk_vecs;
    const u32 whole_vecs = s.full_vecs > cbegin
                               ? (s.full_vecs - cbegin < valid_vecs ? static_cast<u32>(s.full_vecs - cbegin) : valid_vecs)
                               : 0u;
    // this slot's counter as the previous call left it (all ranks' slot w hold the same value)
    const u32 base = s.L ? __hip_atomic_load(flag_ptr(s, 0, p, w), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0u;
    bool gave_up = false;
    const u32 fold = FOLD ? s.fold : 0u;
    const bool idle = sits_out(r_n, fold), takes_in = folds_in(r_n, fold);

    const u32 trips = ONE ? 1u : s.iters;
    const u32 calls = CHAIN ? s.calls : 1u;
    const bool two_sets = CHAIN && s.alt_offset != 0;
    u32 T = 0u;  // trips made so far, over all calls of the launch
    for (u32 k = 0; k < calls; ++k) {
    for (u32 it = 0; it < trips; ++it, ++T) {
        const u32 slice = w + it * s.B_s;
        const u64 first = static_cast<u64>(slice) * (kThreads * U);
        const u32 v0 = static_cast<u32>(first) + threadIdx.x;  // first < 2^31 by construction
        const bool whole = FULL || first + kThreads * U <= whole_vecs;
        const u32 valid = FULL ? s.chunk_vecs : (first < valid_vecs ? valid_vecs : 0u);  // slices past the chunk do nothing
        const u32 ticket = base + T + 1u;
        // Where the slice lives in a partial buffer.  With one or two trips every slice has its
        // own place.  With three or more, a workgroup alternates between two places of its own
        // (2*B_s*C_s bytes per buffer, which is less than a chunk then): a place is rewritten
        // two trips later, and by then its reader is done with it, because this workgroup has
        // since waited for that reader's next trip at the same step, which the reader starts
        // only after finishing the trip in which it read the place.  The smaller footprint keeps
        // the exchange inside the memory-side cache however long the message is.  A chain does
        // the same across its calls (see above).
        const u32 ring = (w * 2u + (T & 1u)) * (kThreads * U) + threadIdx.x;
        const u32 s0 = CHAIN ? (two_sets ? v0 : ring) : (!ONE && s.iters >= 3u ? ring : v0);
        const u32 set = two_sets ? (k & 1u) : 0u;

        uint4 part[U];
        if (DATA) reduce_scatter_slice<DT, GT, U>(bufs, s, r_n, c, v0, valid, whole, part);
        if (s.L) {
            if (takes_in) {  // the even partner's reduce-scatter result joins before the steps
                wait_for(s, flag_ptr(s, 0, p - G, w), ticket, gave_up);
                if (DATA) {
                    uint4 got[U];
                    load_slice_coherent<U>(partial_rsrc(s, 0, p - G, set), s0, v0, valid, whole, got);
#pragma unroll
                    for (int u = 0; u < U; ++u) part[u] = combine<DT>(got[u], part[u]);
                }
            }
            if (DATA) store_slice_coherent<U>(partial_rsrc(s, 0, p, set), s0, v0, valid, whole, part);
            publish(flag_ptr(s, 0, p, w), ticket);
        }
        if (idle) {  // no steps: the odd partner's S_L is the result
            wait_for(s, flag_ptr(s, s.L, p + G, w), ticket, gave_up);
            if (DATA) load_slice_coherent<U>(partial_rsrc(s, s.L, p + G, set), s0, v0, valid, whole, part);
        } else {
            for (u32 l = 0; l < s.L; ++l) {
                const u32 peer = peer_node(r_n, l, fold) * G + c;
                wait_for(s, flag_ptr(s, l, peer, w), ticket, gave_up);
                if (DATA) {
                    uint4 got[U];
                    load_slice_coherent<U>(partial_rsrc(s, l, peer, set), s0, v0, valid, whole, got);
#pragma unroll
                    for (int u = 0; u < U; ++u) part[u] = combine<DT>(got[u], part[u]);
                }
                // the last step's result is exchanged only if a partner that sat out needs it
                if (l + 1 < s.L || takes_in) {
                    if (DATA) store_slice_coherent<U>(partial_rsrc(s, l + 1, p, set), s0, v0, valid, whole, part);
                    publish(flag_ptr(s, l + 1, p, w), ticket);
                }
            }
        }
        if (DATA) all_gather_slice<DT, GT, U>(bufs, s, r_n, c, v0, valid, whole, part);
    }
    }
    tell_host(s, gave_up);
}

// ---- the fused schedule with data+flag words (Section 4.2.2, the low-latency payload) -------
//
// Every 8-byte word that crosses between ranks carries 4 bytes of data and the 4-byte sequence
// number of the call, written and read with single 64-bit device-scope accesses, so a word is
// either old (previous sequence number) or complete.  The receiver polls the data words
// themselves: no separate flag, no wait for the stores to complete, no workgroup barrier; each
// wavefront moves on as soon as its own 64 lanes have their words.  Twice the exchanged bytes.
//
// Where the sequence number comes from: every call makes every rank write every word position
// of its buffers exactly once (the position of a word does not depend on B_s or C_s), so all
// ranks' words at one position carry the same number after any history of calls (if N is not a
// power of two, a rank that sits out the steps writes only its first buffer and one that takes
// a partner in also writes a last one, every call alike, and only those are read).  A thread
// therefore reads the number the previous call left in the first word it is about to
// overwrite, adds one, and both stamps its own words with it and expects it in its peers'
// words at the same positions.  No counter shared between workgroups, nothing to update when
// the kernel ends, and a captured graph can replay the call.  Buffers start zero-filled; zero
// is never used as a number.

__device__ __forceinline__ u64 *packed_buf(const Shape &s, u32 level, u32 rank, u32 set = 0u) {
    return reinterpret_cast<u64 *>(s.scratch + (set ? s.packed_alt_offset : s.packed_offset) +
                                   (static_cast<u64>(level) * s.P + rank) * s.packed_stride);
}

// Word layout inside a slice: [vector-in-thread u][word k of the vector][thread], so that one
// store or load instruction of a wavefront covers 512 contiguous bytes.
template <int U>
__device__ __forceinline__ void store_slice_packed(u64 *buf, u32 slice, u32 v0, u32 valid, bool whole, u32 seq,
                                                   const uint4 (&part)[U]) {
    u64 *base = buf + static_cast<u64>(slice) * (kThreads * U * 4) + threadIdx.x;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        if (whole || v0 + u * kThreads < valid) {
            const u32 d[4] = {part[u].x, part[u].y, part[u].z, part[u].w};
#pragma unroll
            for (int k = 0; k < 4; ++k)
                __hip_atomic_store(base + (u * 4 + k) * kThreads, (static_cast<u64>(seq) << 32) | d[k],
                                   __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

template <int U>
__device__ __forceinline__ void load_slice_packed(const Shape &s, const u64 *buf, u32 slice, u32 v0, u32 valid,
                                                  bool whole, u32 seq, bool &gave_up, uint4 (&out)[U]) {
    const u64 *base = buf + static_cast<u64>(slice) * (kThreads * U * 4) + threadIdx.x;
    u32 *status = reinterpret_cast<u32 *>(s.scratch);
    const u64 t0 = wall_clock64();
    u32 spins = 0;
    for (;;) {
        bool ready = true;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            u32 d[4] = {0u, 0u, 0u, 0u};
            if (whole || v0 + u * kThreads < valid) {
                u64 w[4];
#pragma unroll
                for (int k = 0; k < 4; ++k)
                    w[k] = __hip_atomic_load(base + (u * 4 + k) * kThreads, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    ready = ready && static_cast<u32>(w[k] >> 32) == seq;
                    d[k] = static_cast<u32>(w[k]);
                }
            }
            out[u] = make_uint4(d[0], d[1], d[2], d[3]);
        }
        if (__all(ready) || gave_up) break;
        __builtin_amdgcn_s_sleep(1);
        if ((++spins & 31u) == 0u || s.wait_ticks == 0u) {  // a limit of 0: give up after the first look (tests)
            const bool late = wall_clock64() - t0 > s.wait_ticks;  // wave-uniform
            if (late) __hip_atomic_store(status, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (late || __hip_atomic_load(status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) gave_up = true;
        }
    }
}

// CHAIN = true: s.calls all-reduces in one launch, as in fused_kernel.  The even calls use the
// first set of data+flag buffers and the odd calls the second, each set with its own sequence
// numbers (a set advances by one per call that uses it, on every rank alike).  A word is
// overwritten two calls later; the thread that read its old contents is done by then, because the
// writing thread has meanwhile, in the call in between, consumed a word that this reader
// wrote after it was done reading (the exchange pairs thread t of one rank with thread t of the
// other, in both directions).
template <int DT, int GT, int U, bool FOLD, bool ONE, bool FULL, bool CHAIN>
__global__ __launch_bounds__(kThreads) void fused_packed_kernel(RankPtrs bufs, Shape s) {
    static_assert(!(CHAIN && ONE), "a chain makes several trips");
    u32 r_n, c, w;
    locate(s, blockIdx.x, r_n, c, w);
    const u32 G = GT ? GT : s.G;
    const u32 p = r_n * G + c;
    const u32 valid_vecs = chunk_valid_vecs(s, c);
    const u64 cbegin = static_cast<u64>(c) * s.chunk_vecs;
    const u32 whole_vecs = s.full_vecs > cbegin
                               ? (s.full_vecs - cbegin < valid_vecs ? static_cast<u32>(s.full_vecs - cbegin) : valid_vecs)
                               : 0u;
    bool gave_up = false;
    const u32 fold = FOLD ? s.fold : 0u;
    const bool idle = sits_out(r_n, fold), takes_in = folds_in(r_n, fold);

    const u32 trips = ONE ? 1u : s.iters;
    const u32 calls = CHAIN ? s.calls : 1u;
    for (u32 k = 0; k < calls; ++k) {
    const u32 set = CHAIN ? (k & 1u) : 0u;
    for (u32 it = 0; it < trips; ++it) {
        const u32 slice = w + it * s.B_s;
        const u64 first = static_cast<u64>(slice) * (kThreads * U);
        const u32 v0 = static_cast<u32>(first) + threadIdx.x;
        const bool whole = FULL || first + kThreads * U <= whole_vecs;
        const u32 valid = FULL ? s.chunk_vecs : (first < valid_vecs ? valid_vecs : 0u);
        // the number of the previous call, from this thread's own first word of the slice (a
        // thread without a word in this slice neither writes nor waits)
        u32 seq = 0u;
        if (s.L && (whole || v0 < valid)) {
            const u64 *own = packed_buf(s, 0, p, set) + static_cast<u64>(slice) * (kThreads * U * 4) + threadIdx.x;
            seq = static_cast<u32>(__hip_atomic_load(own, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >> 32);
        }
        seq += 1u;
        if (seq == 0u) seq = 1u;  // zero marks a word that was never written

        uint4 part[U];
        reduce_scatter_slice<DT, GT, U>(bufs, s, r_n, c, v0, valid, whole, part);
        if (valid != 0u && s.L) {  // uniform over the workgroup; a slice past the chunk exchanges nothing
            if (takes_in) {  // the even partner's reduce-scatter result joins before the steps
                uint4 got[U];
                load_slice_packed<U>(s, packed_buf(s, 0, p - G, set), slice, v0, valid, whole, seq, gave_up, got);
#pragma unroll
                for (int u = 0; u < U; ++u) part[u] = combine<DT>(got[u], part[u]);
            }
            store_slice_packed<U>(packed_buf(s, 0, p, set), slice, v0, valid, whole, seq, part);
            if (idle) {  // no steps: the odd partner's last partial is the result
                load_slice_packed<U>(s, packed_buf(s, s.L, p + G, set), slice, v0, valid, whole, seq, gave_up, part);
            } else {
                for (u32 l = 0; l < s.L; ++l) {
                    const u32 peer = peer_node(r_n, l, fold) * G + c;
                    uint4 got[U];
                    load_slice_packed<U>(s, packed_buf(s, l, peer, set), slice, v0, valid, whole, seq, gave_up, got);
#pragma unroll
                    for (int u = 0; u < U; ++u) part[u] = combine<DT>(got[u], part[u]);
                    if (l + 1 < s.L || takes_in)
                        store_slice_packed<U>(packed_buf(s, l + 1, p, set), slice, v0, valid, whole, seq, part);
                }
            }
        }
        all_gather_slice<DT, GT, U>(bufs, s, r_n, c, v0, valid, whole, part);
    }
    }
    tell_host(s, gave_up);
}

// ---- stepwise kernels: one launch per phase, one slice per workgroup -------------------------

struct StepShape {
    Shape s;
    u32 slices;  // slices per rank; grid = P * slices
};

template <int DT, int U>
__device__ __forceinline__ void step_locate(const StepShape &a, u32 &p, u32 &r_n, u32 &c, u32 &v0,
                                            u32 &valid, bool &whole) {
    p = blockIdx.x / a.slices;
    const u32 slice = blockIdx.x % a.slices;
    r_n = p / a.s.G;
    c = p % a.s.G;
    const u32 valid_vecs = chunk_valid_vecs(a.s, c);
    const u64 cbegin = static_cast<u64>(c) * a.s.chunk_vecs;
    const u32 whole_vecs = a.s.full_vecs > cbegin
                               ? (a.s.full_vecs - cbegin < valid_vecs ? static_cast<u32>(a.s.full_vecs - cbegin) : valid_vecs)
                               : 0u;
    const u64 first = static_cast<u64>(slice) * (kThreads * U);
    v0 = static_cast<u32>(first) + threadIdx.x;
    whole = first + kThreads * U <= whole_vecs;
    valid = first < valid_vecs ? valid_vecs : 0u;
}

template <int DT, int U>
__global__ __launch_bounds__(kThreads) void reduce_scatter_kernel(RankPtrs bufs, StepShape a) {
    u32 p, r_n, c, v0, valid;
    bool whole;
    step_locate<DT, U>(a, p, r_n, c, v0, valid, whole);
    uint4 part[U];
    reduce_scatter_slice<DT, 0, U>(bufs, a.s, r_n, c, v0, valid, whole, part);
    store_slice<U>(partial_buf(a.s, 0, p), v0, valid, whole, part);
}

// N not a power of two only: S_0(p) = narrow( S_0(p - G) + S_0(p) ) for the ranks of the odd
// nodes among the first 2r.  In place: a rank's slice of S_0 is read and written by one thread.
template <int DT, int U>
__global__ __launch_bounds__(kThreads) void fold_in_kernel(StepShape a) {
    u32 p, r_n, c, v0, valid;
    bool whole;
    step_locate<DT, U>(a, p, r_n, c, v0, valid, whole);
    if (!folds_in(r_n, a.s.fold)) return;
    uint4 own[U], got[U];
    load_slice<U>(partial_buf(a.s, 0, p), v0, valid, whole, own);
    load_slice<U>(partial_buf(a.s, 0, p - a.s.G), v0, valid, whole, got);
#pragma unroll
    for (int u = 0; u < U; ++u) own[u] = combine<DT>(got[u], own[u]);
    store_slice<U>(partial_buf(a.s, 0, p), v0, valid, whole, own);
}

// S_{l+1}(p) = narrow( S_l(peer) + S_l(p) )  (Algorithm 1, RD_inter, one step for all ranks)
template <int DT, int U>
__global__ __launch_bounds__(kThreads) void exchange_sum_kernel(StepShape a, u32 l) {
    u32 p, r_n, c, v0, valid;
    bool whole;
    step_locate<DT, U>(a, p, r_n, c, v0, valid, whole);
    if (sits_out(r_n, a.s.fold)) return;
    const u32 peer = peer_node(r_n, l, a.s.fold) * a.s.G + c;
    uint4 own[U], got[U];
    load_slice<U>(partial_buf(a.s, l, p), v0, valid, whole, own);
    load_slice<U>(partial_buf(a.s, l, peer), v0, valid, whole, got);
#pragma unroll
    for (int u = 0; u < U; ++u) own[u] = combine<DT>(got[u], own[u]);
    store_slice<U>(partial_buf(a.s, l + 1, p), v0, valid, whole, own);
}

template <int DT, int U>
__global__ __launch_bounds__(kThreads) void all_gather_kernel(RankPtrs bufs, StepShape a) {
    u32 p, r_n, c, v0, valid;
    bool whole;
    step_locate<DT, U>(a, p, r_n, c, v0, valid, whole);
    uint4 part[U];
    // a rank that sat out the steps takes the result from its partner on the next node
    const u32 from = sits_out(r_n, a.s.fold) ? p + a.s.G : p;
    load_slice<U>(partial_buf(a.s, a.s.L, from), v0, valid, whole, part);
    all_gather_slice<DT, 0, U>(bufs, a.s, r_n, c, v0, valid, whole, part);
}

// ---- single-rank exchange-and-sum, in place on dst ------------------------------------------

template <int DT>
__global__ __launch_bounds__(kThreads) void combine_kernel(unsigned char *dst, const unsigned char *src,
                                                           u64 full_vecs, u32 tail) {
    const u64 stride = static_cast<u64>(gridDim.x) * kThreads;
    for (u64 v = static_cast<u64>(blockIdx.x) * kThreads + threadIdx.x; v < full_vecs; v += stride)
        st16(dst, v, combine<DT>(ld16(dst, v), ld16(src, v)));
    if (tail && blockIdx.x == 0 && threadIdx.x == 0) {
        const uint4 r = combine<DT>(ld_partial<DT>(dst, full_vecs, tail), ld_partial<DT>(src, full_vecs, tail));
        st_partial<DT>(dst, full_vecs, tail, r);
    }
}

// ---- small utilities ---------------------------------------------------------------------------

// Zero `count` words; words 2 and 3 receive `at_word_2` instead (the scratch header keeps the
// device address of the host's time-out word there; 0 when a plain zero fill is wanted).
__global__ __launch_bounds__(kThreads) void fill_zero_kernel(u32 *words, u64 count, u64 at_word_2) {
    const u64 stride = static_cast<u64>(gridDim.x) * kThreads;
    for (u64 i = static_cast<u64>(blockIdx.x) * kThreads + threadIdx.x; i < count; i += stride)
        words[i] = i == 2 ? static_cast<u32>(at_word_2) : i == 3 ? static_cast<u32>(at_word_2 >> 32) : 0u;
}

__global__ __launch_bounds__(kThreads) void empty_kernel() {}

__global__ __launch_bounds__(kThreads) void copy_kernel(uint4 *dst, const uint4 *src, u64 vecs) {
    const u64 stride = static_cast<u64>(gridDim.x) * kThreads;
    for (u64 v = static_cast<u64>(blockIdx.x) * kThreads + threadIdx.x; v < vecs; v += stride) dst[v] = src[v];
}

// Reads only: every thread folds the vectors it loads into one value, and one thread per
// workgroup whose value happens to be all ones stores it (so the loads cannot be dropped, and in
// practice nothing is written).
__global__ __launch_bounds__(kThreads) void read_kernel(uint4 *sink, const uint4 *src, u64 vecs) {
    const u64 stride = static_cast<u64>(gridDim.x) * kThreads;
    uint4 acc = make_uint4(0u, 0u, 0u, 0u);
    for (u64 v = static_cast<u64>(blockIdx.x) * kThreads + threadIdx.x; v < vecs; v += stride) {
        const uint4 t = src[v];
        acc.x ^= t.x; acc.y ^= t.y; acc.z ^= t.z; acc.w ^= t.w;
    }
    if ((acc.x & acc.y & acc.z & acc.w) == 0xffffffffu) *sink = acc;
}

// ---- launchers ---------------------------------------------------------------------------------

static Shape make_shape(const rar_plan_t &plan, const Tuning &t) {
    const Geometry &g = plan.geo;
    Shape s{};
    s.scratch = static_cast<unsigned char *>(plan.scratch);
    s.chunk_stride = g.chunk_stride;
    s.flags_offset = g.flags_offset;
    s.data_offset = g.data_offset;
    s.alt_offset = g.alt_offset;
    s.packed_offset = g.packed_offset;
    s.packed_alt_offset = g.packed_alt_offset;
    s.packed_stride = g.packed_stride;
    s.wait_ticks = plan.wait_limit_us * 100ull;  // the wall clock counts at 100 MHz
    s.P = g.P; s.G = g.G; s.N = g.N; s.L = g.L;
    s.fold = static_cast<u32>(g.fold);
    s.chunk_vecs = static_cast<u32>(g.chunk_vecs);
    s.full_vecs = static_cast<u32>(g.n / g.per_vec);
    s.tail = static_cast<u32>(g.n % g.per_vec);
    s.B_s = t.B_s;
    s.iters = t.iters;
    s.calls = 1;
    // One flag per 64 bytes where the words allow it (measured: barrier time -15..25 %, whole call
    // -1..3 % from 256 workgroups up; small grids are better off with 32 bytes).
    const u32 widest = static_cast<u32>(g.P) * t.B_s >= 256u ? 16u : 8u;
    u32 stride = 1;
    while (stride < widest && stride * 2u * t.B_s <= static_cast<u32>(kMaxWorkgroupsPerRank)) stride *= 2u;
    s.flag_stride = stride;
    return s;
}

typedef void (*FusedFn)(RankPtrs, Shape);

// Which instance serves a launch.  The special cases (single trip, all slices whole) exist for
// G = 1, 2, 4, 8 and power-of-two N; run-time G and the hand-over for other N take the generic one.
struct Variant {
    int dtype, G, unroll;
    bool data;   // false: the barrier-only kernel (no data movement)
    bool fold;   // N is not a power of two
    bool one;    // every workgroup makes a single trip
    bool full;   // every slice of the launch is a whole slice inside the message
    bool chain;  // several all-reduces in one launch
};

template <int DT, int GT, bool DATA, bool FOLD, bool ONE, bool FULL, bool CHAIN>
static FusedFn pick_unroll(int unroll) {
    switch (unroll) {
        case 1: return fused_kernel<DT, GT, 1, DATA, FOLD, ONE, FULL, CHAIN>;
        case 2: return fused_kernel<DT, GT, 2, DATA, FOLD, ONE, FULL, CHAIN>;
        case 4: return fused_kernel<DT, GT, 4, DATA, FOLD, ONE, FULL, CHAIN>;
        default: return fused_kernel<DT, GT, 8, DATA, FOLD, ONE, FULL, CHAIN>;
    }
}
template <int DT, bool DATA, bool ONE, bool FULL, bool CHAIN>
static FusedFn pick_group(int G, int unroll) {
    switch (G) {
        case 1: return pick_unroll<DT, 1, DATA, false, ONE, FULL, CHAIN>(unroll);
        case 2: return pick_unroll<DT, 2, DATA, false, ONE, FULL, CHAIN>(unroll);
        case 4: return pick_unroll<DT, 4, DATA, false, ONE, FULL, CHAIN>(unroll);
        case 8: return pick_unroll<DT, 8, DATA, false, ONE, FULL, CHAIN>(unroll);
        default: return pick_unroll<DT, 0, DATA, false, false, false, CHAIN>(unroll);
    }
}
template <int DT>
static FusedFn pick_special(const Variant &v) {
    if (v.chain) {
        if (v.fold) return pick_unroll<DT, 0, true, true, false, false, true>(v.unroll);
        return v.full ? pick_group<DT, true, false, true, true>(v.G, v.unroll) : pick_group<DT, true, false, false, true>(v.G, v.unroll);
    }
    if (v.fold) return pick_unroll<DT, 0, true, true, false, false, false>(v.unroll);
    if (v.one)
        return v.full ? pick_group<DT, true, true, true, false>(v.G, v.unroll) : pick_group<DT, true, true, false, false>(v.G, v.unroll);
    return v.full ? pick_group<DT, true, false, true, false>(v.G, v.unroll) : pick_group<DT, true, false, false, false>(v.G, v.unroll);
}
template <int DT>
static FusedFn pick_barrier_only(const Variant &v) {  // a measurement aid: the generic instances are enough
    if (v.fold) return pick_unroll<DT, 0, false, true, false, false, false>(v.unroll);
    return pick_group<DT, false, false, false, false>(v.G, v.unroll);
}
static FusedFn pick_fused(const Variant &v) {
    if (v.dtype == RAR_BF16) return v.data ? pick_special<RAR_BF16>(v) : pick_barrier_only<RAR_BF16>(v);
    return v.data ? pick_special<RAR_F32>(v) : pick_barrier_only<RAR_F32>(v);
}

template <int DT, int GT, bool FOLD, bool ONE, bool FULL, bool CHAIN>
static FusedFn pick_packed_unroll(int unroll) {
    switch (unroll) {
        case 1: return fused_packed_kernel<DT, GT, 1, FOLD, ONE, FULL, CHAIN>;
        case 2: return fused_packed_kernel<DT, GT, 2, FOLD, ONE, FULL, CHAIN>;
        case 4: return fused_packed_kernel<DT, GT, 4, FOLD, ONE, FULL, CHAIN>;
        default: return fused_packed_kernel<DT, GT, 8, FOLD, ONE, FULL, CHAIN>;
    }
}
template <int DT, bool ONE, bool FULL, bool CHAIN>
static FusedFn pick_packed_group(int G, int unroll) {
    switch (G) {
        case 1: return pick_packed_unroll<DT, 1, false, ONE, FULL, CHAIN>(unroll);
        case 2: return pick_packed_unroll<DT, 2, false, ONE, FULL, CHAIN>(unroll);
        case 4: return pick_packed_unroll<DT, 4, false, ONE, FULL, CHAIN>(unroll);
        case 8: return pick_packed_unroll<DT, 8, false, ONE, FULL, CHAIN>(unroll);
        default: return pick_packed_unroll<DT, 0, false, false, false, CHAIN>(unroll);
    }
}
template <int DT>
static FusedFn pick_packed_special(const Variant &v) {
    if (v.chain) {
        if (v.fold) return pick_packed_unroll<DT, 0, true, false, false, true>(v.unroll);
        return v.full ? pick_packed_group<DT, false, true, true>(v.G, v.unroll) : pick_packed_group<DT, false, false, true>(v.G, v.unroll);
    }
    if (v.fold) return pick_packed_unroll<DT, 0, true, false, false, false>(v.unroll);
    if (v.one)
        return v.full ? pick_packed_group<DT, true, true, false>(v.G, v.unroll) : pick_packed_group<DT, true, false, false>(v.G, v.unroll);
    return v.full ? pick_packed_group<DT, false, true, false>(v.G, v.unroll) : pick_packed_group<DT, false, false, false>(v.G, v.unroll);
}
static FusedFn pick_packed(const Variant &v) {
    return v.dtype == RAR_BF16 ? pick_packed_special<RAR_BF16>(v) : pick_packed_special<RAR_F32>(v);
}

// The most recent failing HIP status seen by the library on this thread (for rar_last_hip_error).
static thread_local hipError_t g_last_hip_error = hipSuccess;
hipError_t note_hip(hipError_t e) {
    if (e != hipSuccess) g_last_hip_error = e;
    return e;
}
const char *last_hip_error_string() { return g_last_hip_error == hipSuccess ? "no error" : hipGetErrorString(g_last_hip_error); }

int device_info(DeviceInfo *out) {
    static DeviceInfo cached[16];
    static bool have[16] = {};
    static std::mutex guard;  // plans of different threads may ask at the same time
    int dev = 0;
    if (note_hip(hipGetDevice(&dev)) != hipSuccess) return RAR_ERR_HIP;
    if (dev < 0 || dev >= 16) return RAR_ERR_HIP;
    std::lock_guard<std::mutex> lock(guard);
    if (!have[dev]) {
        int cus = 0;
        if (note_hip(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev)) != hipSuccess || cus < 1)
            return RAR_ERR_HIP;
        cached[dev].compute_units = cus;
        have[dev] = true;
    }
    *out = cached[dev];
    return RAR_OK;
}

int fused_max_resident(int dtype, int G, int unroll, bool packed, bool fold, bool chain, long *out) {
    DeviceInfo info;
    int rc = device_info(&info);
    if (rc != RAR_OK) return rc;
    // the smallest over the special-case instances: the planner asks before it knows how many trips
    // a launch will make
    int fewest = 0;
    for (int k = 0; k < 4; ++k) {
        const bool one = (k & 1) != 0;
        if (chain && one) continue;
        const Variant v{dtype, G, unroll, true, fold, one, (k & 2) != 0, chain};
        FusedFn fn = packed ? pick_packed(v) : pick_fused(v);
        int per_cu = 0;
        if (note_hip(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, reinterpret_cast<const void *>(fn), kThreads, 0)) !=
                hipSuccess || per_cu < 1)
            return RAR_ERR_HIP;
        if (fewest == 0 || per_cu < fewest) fewest = per_cu;
    }
    // The query is arithmetic on the kernel's register counts.  Where vector registers set the
    // figure it is exact; a figure of 7 or 8 per compute unit can be set by scalar registers or
    // wave slots, of which the hardware may keep some for itself, so such a figure is taken one
    // lower.  (The planner never goes beyond kMaxWorkgroupsPerCU anyway.)
    if (fewest >= 7) fewest -= 1;
    *out = static_cast<long>(fewest) * info.compute_units;
    return RAR_OK;
}

// A launch reports failure through the thread's "last error", which an earlier HIP call of the
// application may have left set: clear it first, so that what is read afterwards is the launch's.
static void begin_launch() { (void)hipGetLastError(); }
static int check_launch() { return note_hip(hipGetLastError()) == hipSuccess ? RAR_OK : RAR_ERR_HIP; }

int launch_fill_zero(void *words, size_t bytes, const void *at_word_2, hipStream_t stream) {
    begin_launch();
    const u64 count = bytes / 4;
    u64 blocks = (count + kThreads - 1) / kThreads;
    if (blocks > 1024) blocks = 1024;
    if (blocks == 0) return RAR_OK;
    fill_zero_kernel<<<dim3(static_cast<u32>(blocks)), dim3(kThreads), 0, stream>>>(static_cast<u32 *>(words), count,
                                                                                     reinterpret_cast<u64>(at_word_2));
    return check_launch();
}

// Every slice of every workgroup is a whole slice inside the message: no tail, no ragged or short
// chunk, no trip past the end of a chunk.
static bool all_slices_whole(const Geometry &g, const Tuning &t) {
    const size_t slice = static_cast<size_t>(kThreads) * t.unroll;
    return g.n % g.per_vec == 0 && g.n == static_cast<size_t>(g.G) * g.chunk_len && g.chunk_vecs % slice == 0 &&
           static_cast<size_t>(t.B_s) * t.iters * slice == g.chunk_vecs;
}

// `scratch` is the memory the launch works on: the plan's own, or the library's static array.
// calls = 0: one all-reduce (the plain instances); calls >= 1: a chain of that many.
int launch_fused(const rar_plan_t &plan, void *scratch, const RankPtrs &bufs, const Tuning &t, bool data, int calls,
                 hipStream_t stream) {
    begin_launch();
    const Geometry &g = plan.geo;
    Shape s = make_shape(plan, t);
    s.scratch = static_cast<unsigned char *>(scratch);
    const bool chain = calls > 0;
    if (chain) s.calls = static_cast<u32>(calls);
    const u32 grid = static_cast<u32>(g.P) * t.B_s;
    FusedFn fn = pick_fused(Variant{g.dtype, g.G, t.unroll, data, g.fold != 0, !chain && t.iters == 1, all_slices_whole(g, t), chain});
    fn<<<dim3(grid), dim3(kThreads), 0, stream>>>(bufs, s);
    return check_launch();
}

int launch_fused_packed(const rar_plan_t &plan, const RankPtrs &bufs, const Tuning &t, int calls, hipStream_t stream) {
    begin_launch();
    const Geometry &g = plan.geo;
    Shape s = make_shape(plan, t);
    const bool chain = calls > 0;
    if (chain) s.calls = static_cast<u32>(calls);
    const u32 grid = static_cast<u32>(g.P) * t.B_s;
    FusedFn fn = pick_packed(Variant{g.dtype, g.G, t.unroll, true, g.fold != 0, !chain && t.iters == 1, all_slices_whole(g, t), chain});
    fn<<<dim3(grid), dim3(kThreads), 0, stream>>>(bufs, s);
    return check_launch();
}

int launch_empty(unsigned grid, hipStream_t stream) {
    begin_launch();
    empty_kernel<<<dim3(grid), dim3(kThreads), 0, stream>>>();
    return check_launch();
}

template <int DT>
static int launch_stepwise_t(const rar_plan_t &plan, const RankPtrs &bufs, hipStream_t stream) {
    begin_launch();
    constexpr int U = 4;
    const Geometry &g = plan.geo;
    Tuning t{1, U, 1};
    StepShape a{};
    a.s = make_shape(plan, t);
    a.slices = static_cast<u32>((g.chunk_vecs + kThreads * U - 1) / (kThreads * U));
    const u64 grid64 = static_cast<u64>(g.P) * a.slices;
    if (grid64 >= (1ull << 31)) return RAR_ERR_LIMIT;
    const dim3 grid(static_cast<u32>(grid64)), block(kThreads);
    reduce_scatter_kernel<DT, U><<<grid, block, 0, stream>>>(bufs, a);
    if (check_launch() != RAR_OK) return RAR_ERR_HIP;
    if (g.fold) {
        fold_in_kernel<DT, U><<<grid, block, 0, stream>>>(a);
        if (check_launch() != RAR_OK) return RAR_ERR_HIP;
    }
    for (int l = 0; l < g.L; ++l) {
        exchange_sum_kernel<DT, U><<<grid, block, 0, stream>>>(a, static_cast<u32>(l));
        if (check_launch() != RAR_OK) return RAR_ERR_HIP;
    }
    all_gather_kernel<DT, U><<<grid, block, 0, stream>>>(bufs, a);
    return check_launch();
}

int launch_stepwise(const rar_plan_t &plan, const RankPtrs &bufs, hipStream_t stream) {
    return plan.geo.dtype == RAR_BF16 ? launch_stepwise_t<RAR_BF16>(plan, bufs, stream)
                                      : launch_stepwise_t<RAR_F32>(plan, bufs, stream);
}

int launch_combine(void *dst, const void *src, size_t full_vecs, unsigned tail, int dtype, hipStream_t stream) {
    begin_launch();
    u64 blocks = (full_vecs + kThreads - 1) / kThreads;
    if (blocks == 0) blocks = 1;
    if (blocks > 16384) blocks = 16384;
    const dim3 grid(static_cast<u32>(blocks)), block(kThreads);
    if (dtype == RAR_BF16)
        combine_kernel<RAR_BF16><<<grid, block, 0, stream>>>(static_cast<unsigned char *>(dst),
                                                             static_cast<const unsigned char *>(src), full_vecs, tail);
    else
        combine_kernel<RAR_F32><<<grid, block, 0, stream>>>(static_cast<unsigned char *>(dst),
                                                            static_cast<const unsigned char *>(src), full_vecs, tail);
    return check_launch();
}

int launch_read(void *sink, const void *src, size_t vecs, hipStream_t stream) {
    begin_launch();
    u64 blocks = (vecs + kThreads - 1) / kThreads;
    if (blocks == 0) return RAR_OK;
    if (blocks > 16384) blocks = 16384;
    read_kernel<<<dim3(static_cast<u32>(blocks)), dim3(kThreads), 0, stream>>>(static_cast<uint4 *>(sink),
                                                                               static_cast<const uint4 *>(src), vecs);
    return check_launch();
}

int launch_copy(void *dst, const void *src, size_t vecs, hipStream_t stream) {
    begin_launch();
    u64 blocks = (vecs + kThreads - 1) / kThreads;
    if (blocks == 0) return RAR_OK;
    if (blocks > 16384) blocks = 16384;
    copy_kernel<<<dim3(static_cast<u32>(blocks)), dim3(kThreads), 0, stream>>>(
        static_cast<uint4 *>(dst), static_cast<const uint4 *>(src), vecs);
    return check_launch();
}

}  // namespace rar
