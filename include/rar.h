/*
 * rar.h - C ABI of the MI355X (gfx950) hierarchical recursive-doubling all-reduce.
 *
 * The operation is the three-phase all-reduce of the paper's Algorithm 1 ("NVRAR") and
 * Section 4.1: an intra-node reduce-scatter over the G ranks of a node, log2(N) inter-node
 * recursive-doubling exchange-and-sum steps on each rank's 1/G chunk (step l pairs rank
 * (r_n, r_g) with rank (r_n XOR 2^l, r_g)), then an intra-node all-gather.  All P = G*N
 * ranks are emulated on ONE GPU as P resident device buffers; rank p = r_n*G + r_g.
 *
 * Numerics (fixed, the result is a function of the schedule): elements are widened to
 * binary32, added with round-to-nearest-even and gradual underflow; the reduce-scatter adds
 * local ranks 0..G-1 in that order in binary32 and narrows once to the message type; every
 * inter-node step narrows its sum to the message type; bf16 narrowing rounds to nearest,
 * ties to even.  NaN results are NaN, their payload is unspecified.
 *
 * Conventions
 *   - "host" / "device" is stated for every pointer.  Device pointers are plain addresses in
 *     the current HIP device's memory (e.g. torch.Tensor.data_ptr()).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls that take
 *     a stream only enqueue work and return; results are valid in stream order.
 *   - Every function returns RAR_OK (0) or a negative rar_status.  No exceptions, no aborts.
 *   - Nothing here allocates or frees device memory; scratch is lent by the caller.  A plan's
 *     first launch allocates one word of pinned host memory (the time-out word below).
 *   - A plan is not thread-safe, and two all-reduces on one plan must not overlap in time
 *     (they share the plan's scratch): order them on one stream or use two plans.  A plan
 *     belongs to the device that is current at its first launch (it remembers that device's
 *     size and how many workgroups of each kernel it holds at once).
 *   - The fused modes size their grid so that every workgroup is resident at once on an
 *     otherwise idle device (their step barriers spin): never more than four workgroups per
 *     compute unit, and never more than the device holds of the kernel in question.  Other
 *     work on other streams may run at the same time as long as it finishes by itself.  Fused
 *     all-reduces of different plans on different streams are, by default, ordered one after
 *     the other by the library (an event between the two streams); rar_plan_set_concurrency
 *     lets them overlap.  RAR_MODE_STEPWISE has no residency requirement.
 *   - All waits are bounded (rar_plan_set_wait_limit_us): a call that cannot proceed ends
 *     instead of hanging, its output is then unspecified, and the plan is "poisoned": every
 *     later launch on it returns RAR_ERR_TIMEOUT without enqueuing anything until
 *     rar_plan_status has been called (which reports the time-out and re-arms the plan).
 *   - Stream capture: a plan's first launch, and the first after a time-out, must be made
 *     outside capture (they set up flags and host memory); inside capture they return
 *     RAR_ERR_CAPTURE.  Every later launch may be captured and replayed.
 */
#ifndef RAR_H
#define RAR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum rar_dtype {
    RAR_BF16 = 0, /* 2-byte bfloat16 (upper half of binary32) */
    RAR_F32 = 1   /* 4-byte IEEE binary32 */
} rar_dtype;

typedef enum rar_mode {
    RAR_MODE_STEPWISE = 0, /* one launch per phase: 1 reduce-scatter + L steps + 1 all-gather */
    RAR_MODE_FUSED = 1,    /* one persistent launch; flag-based step barriers                */
    RAR_MODE_FUSED_PACKED = 2, /* one persistent launch; every 8-byte word exchanged carries 4 bytes of
                              data and the call's 4-byte sequence number (Section 4.2.2, the
                              low-latency payload), so a step needs no separate flag and no
                              workgroup barrier; twice the exchanged bytes; small messages only */
    RAR_MODE_AUTO = 3      /* (default) RAR_MODE_FUSED_PACKED where it measured faster on MI355X: at most
                              1 MiB exchanged per step by all ranks together (P * chunk bytes);
                              RAR_MODE_FUSED otherwise                                             */
} rar_mode;

typedef enum rar_status {
    RAR_OK = 0,
    RAR_ERR_ARG = -1,     /* NULL pointer, P < 1, G < 1, n == 0, value out of range        */
    RAR_ERR_SHAPE = -2,   /* G does not divide P                                            */
    RAR_ERR_DTYPE = -3,   /* unknown rar_dtype                                              */
    RAR_ERR_LIMIT = -4,   /* P > RAR_MAX_RANKS or n too large for 32-bit vector indices     */
    RAR_ERR_SCRATCH = -5, /* scratch not set, too small, or misaligned                      */
    RAR_ERR_ALIGN = -6,   /* a data pointer is not 16-byte aligned                          */
    RAR_ERR_HIP = -7,     /* a HIP call failed (no device, launch error, ...)               */
    RAR_ERR_TIMEOUT = -8, /* a step barrier gave up waiting (reported by rar_plan_status)   */
    RAR_ERR_TUNING = -9,  /* rar_plan_set_tuning: unsupported B_s / C_s                     */
    RAR_ERR_CAPTURE = -10 /* a plan's first launch (or the first after a time-out) was made
                             while its stream was being captured                            */
} rar_status;

#define RAR_MAX_RANKS 128

typedef struct rar_plan_s rar_plan_t;

/* Library version, major*10000 + minor*100 + patch. */
int rar_version(void);

/* Static, never-NULL description of a status code. */
const char *rar_strerror(int status);

/* After a call returned RAR_ERR_HIP: the HIP runtime's own text for the failing status that
 * the library saw last on the calling thread ("no error" if none).  Never NULL. */
const char *rar_last_hip_error(void);

/* ---- planner (host only; Algorithm 1's inputs G, N, C_s and its peer rule) ---------------
 *
 * rar_plan: build the schedule for P ranks, G per node, n elements of `dtype` per rank.
 *   N = P/G nodes, L = log2 N steps.  The message is cut into G chunks: chunk length is
 *   ceil(n/G) rounded up to whole 16-byte groups, chunk c covers elements
 *   [min(c*len, n), min((c+1)*len, n)), so trailing chunks may be short or empty (the paper
 *   writes |M|/G and does not treat the ragged case).  N = 1 (no inter-node phase) and G = 1
 *   (phases 1 and 3 reduce to a copy) are valid.  Algorithm 1 assumes N = 2^L.  For any other
 *   N = 2^L + r the customary extension of recursive doubling is applied (not from the paper):
 *   nodes (2i, 2i+1), i < r, pair up, the even one hands its reduce-scatter result to the odd
 *   one and sits out, the 2^L remaining nodes are renumbered (node 2i+1 -> i, node j >= 2r ->
 *   j - r) and run the L steps on those numbers, and the odd node hands the result back.
 *   *out (host) receives a plan owned by the caller; release it with rar_plan_free.
 *   Touches no device.
 */
int rar_plan(int P, int G, size_t n, int dtype, rar_plan_t **out);
int rar_plan_free(rar_plan_t *plan);

/* Shape queries (host only). rar_plan_steps returns L; rar_plan_nodes returns N. */
int rar_plan_ranks(const rar_plan_t *plan);
int rar_plan_nodes(const rar_plan_t *plan);
int rar_plan_steps(const rar_plan_t *plan);

/* Peer of `rank` at inter-node step `step` (0 <= step < L): (r_n XOR 2^step)*G + r_g
 * (Algorithm 1, peer rule of RD_inter).  If N is not a power of two the XOR acts on the
 * renumbered nodes, and a rank that sits out the steps gets itself back.  Negative rar_status
 * on bad arguments. */
int rar_plan_peer(const rar_plan_t *plan, int rank, int step);

/* The rank that `rank` is paired with before and after the steps when N is not a power of two
 * (same local id, neighbouring node), or `rank` itself if it has no such partner. */
int rar_plan_fold_partner(const rar_plan_t *plan, int rank);

/* Element range of chunk c (0 <= c < G): *offset and *length (host, both required). */
int rar_plan_chunk(const rar_plan_t *plan, int c, size_t *offset, size_t *length);

/* Bytes of device scratch rar_allreduce needs: a 256-byte header (status word), the step
 * barrier flags, the per-step partial buffers S_0..S_L of every rank
 * (Section 4.2.1: one buffer per inter-node step, so a rank may run ahead of its peer) and,
 * for chunks of at most 256 KiB, the per-step data+flag buffers of the packed mode plus a
 * second set of both kinds of buffers for the odd calls of rar_allreduce_chain. */
size_t rar_plan_scratch_bytes(const rar_plan_t *plan);

/* Where things live inside the scratch, as byte offsets and sizes (host pointers, each may be
 * NULL): the step-barrier flags (32-bit counters, one per (buffer S_l, rank, workgroup slot))
 * and the data+flag buffers of RAR_MODE_FUSED_PACKED (8-byte words, sequence number in the upper
 * half; size 0 if the plan has none).  For tests and tools that inspect or preset them. */
int rar_plan_scratch_layout(const rar_plan_t *plan, size_t *flags_offset, size_t *flags_bytes,
                            size_t *packed_offset, size_t *packed_bytes);

/* Lend `bytes` of device memory at `scratch` (256-byte aligned, >= rar_plan_scratch_bytes)
 * to the plan.  The plan borrows it until rar_plan_free or the next set_scratch; the caller
 * frees it afterwards.  Contents need no initialisation: the first all-reduce clears the
 * header and flags with a fill kernel on its stream. */
int rar_plan_set_scratch(rar_plan_t *plan, void *scratch, size_t bytes);

/* Execution mode (default RAR_MODE_AUTO).  All modes produce identical bits.
 * RAR_MODE_FUSED_PACKED is accepted only while a chunk is at most 256 KiB (RAR_ERR_LIMIT
 * otherwise); rar_plan_scratch_bytes already includes its buffers for such plans.
 * rar_plan_get_mode returns the mode as set; rar_plan_effective_mode the one a call would run
 * (RAR_MODE_AUTO resolved to RAR_MODE_FUSED or RAR_MODE_FUSED_PACKED). */
int rar_plan_set_mode(rar_plan_t *plan, int mode);
int rar_plan_get_mode(const rar_plan_t *plan);
int rar_plan_effective_mode(const rar_plan_t *plan);

/* The paper's two hyper-parameters (Section 4.2.1, Appendix "Impact of Chunk Size and Block
 * Size"): B_s = workgroups per rank, C_s = bytes of a rank's chunk that one workgroup moves
 * per trip (its "chunk" of the chunked pipeline).  C_s must be 4096, 8192, 16384 or 32768;
 * 1 <= B_s <= 256.  B_s = 0 and/or C_s = 0 restore the built-in choice for that parameter.
 * They change timing only, never a result bit.  In fused mode B_s is clamped at launch so
 * that all P*B_s workgroups are resident at once (the step barriers need that): at most four
 * workgroups per compute unit of the device, fewer if the kernel in question fits fewer. */
int rar_plan_set_tuning(rar_plan_t *plan, int B_s, size_t C_s);
int rar_plan_get_tuning(const rar_plan_t *plan, int *B_s, size_t *C_s);

/* How many fused all-reduces (of different plans, on different streams) the caller lets run on
 * the device at the same time: 1 (default) to 8.
 * k = 1: the library keeps fused launches apart.  A fused launch on another stream than the
 *   library's previous fused launch on the device first waits (hipStreamWaitEvent) for an event
 *   recorded on that previous stream, so the two kernels never share the device.  (Two fused
 *   kernels that together exceed what the device holds can each keep workgroup slots the other
 *   one waits for; the waits are bounded, so such calls would end in RAR_ERR_TIMEOUT rather than
 *   hang, but they would not complete.)  Inside stream capture the dependency is added only if
 *   both streams belong to the same capture; graphs replayed side by side are the caller's to order.
 * k > 1: no such ordering; the built-in B_s and the residency clamp leave the plan 1/k of the
 *   device, so that k such kernels fit at once.
 * Kernels that do not wait for anything (matrix products, copies) may share the device freely. */
int rar_plan_set_concurrency(rar_plan_t *plan, int k);

/* Upper bound on the time one step-barrier wait may take before the kernel gives up, in
 * microseconds (default 5,000,000).  A wait that gives up records RAR_ERR_TIMEOUT in the
 * scratch header, and every workgroup still runs to the end of the kernel (no hang); the
 * output buffers are then unspecified.  The clock is looked at every 32 polls, so a wait that
 * is satisfied within those never gives up.  0 is for tests of the time-out handling: a wait
 * then gives up as soon as it has looked once without finding what it waits for. */
int rar_plan_set_wait_limit_us(rar_plan_t *plan, uint64_t microseconds);

/* Synchronise `stream`, then report whether a step-barrier wait of this plan has given up since
 * the last report: RAR_OK or RAR_ERR_TIMEOUT.  After a time-out the plan is re-armed: the next
 * launch (which must be outside stream capture) clears the flags first. */
int rar_plan_status(rar_plan_t *plan, void *stream);

/* ---- one rank's exchange-and-sum (Algorithm 1, RD_inter: B_send[l+1] <- dst + src) --------
 *
 * For i in [chunk*n, chunk*n + n):  dst[i] <- narrow( widen(dst[i]) + widen(src[i]) ).
 * dst, src: device base pointers of two buffers with identical layout, 16-byte aligned,
 * not overlapping; n = elements per chunk, chunk = chunk index, so the touched byte offset
 * chunk*n*sizeof(element) must itself be a multiple of 16.  dtype is a rar_dtype (the
 * paper's list of arguments has no type because its buffers are typed by the call site).
 * Enqueues one kernel on `stream`; src must not be written while it runs.  n == 0 is a
 * no-op.
 */
int rar_step_combine(void *dst, const void *src, size_t chunk, size_t n, int dtype, void *stream);

/* ---- the whole schedule (Algorithm 1, function NVRAR) --------------------------------------
 *
 * bufs: host array of P device pointers; bufs[p] is rank p's message M of n elements,
 * 16-byte aligned, the P buffers pairwise disjoint and disjoint from the scratch.  The array
 * is read before the call returns.  In place: once the enqueued work has run, every buffer
 * holds the schedule-ordered sum, the same bits on all ranks.  Fused mode is one launch
 * (plus a fill launch on a plan's first use); stepwise mode is L + 2 launches.
 */
int rar_allreduce(void *const *bufs, rar_plan_t *plan, void *stream);

/* K all-reduces of the same buffers, each on the result of the one before, in ONE persistent
 * launch (K >= 1, at most 65536): the same bits as K calls of rar_allreduce.  This is the part
 * of Algorithm 1 that lets a rank start call k+1 before call k has finished everywhere
 * (Section 4.2.1, per-step buffers; Section 4.2.3, sequence numbers instead of a barrier
 * between calls): a workgroup goes on to the next call as soon as its own slices of the current
 * one are gathered; nothing orders the calls but the step flags (or the sequence numbers in the
 * exchanged words).  An exchange buffer is written again two calls later; by then its reader is
 * done with it, because the writer has since waited, in the call in between, for data that the
 * reader produces only after it finished reading.  That takes two buffers per step and rank:
 * plans with chunks of at most 256 KiB have a second set in their scratch, longer chunks
 * alternate between two places inside the first set (B_s is narrowed for that if need be).
 * Runs the plan's fused mode (flag or data+flag exchange); RAR_MODE_STEPWISE: RAR_ERR_ARG. */
int rar_allreduce_chain(void *const *bufs, rar_plan_t *plan, int K, void *stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): rar_allreduce in RAR_MODE_FUSED (flag exchange) on
 * a scratch array that is part of the library (RAR_STATIC_SCRATCH_BYTES of device memory per
 * GPU, held until the process ends) instead of the plan's lent scratch, which need not be
 * set.  Allocates nothing, neither on the device nor on the host.  The plan's flag-exchange
 * footprint (header, flags, partial buffers: rar_plan_static_bytes) must fit the array:
 * RAR_ERR_LIMIT otherwise.  All calls on one GPU share the array: the call clears the header
 * and the flags with a fill kernel on `stream` before the all-reduce, so plans of any shape
 * may alternate, and calls that overlap in time on one GPU race (order them on one stream).
 * Like any fused launch of a plan with concurrency 1, the call is ordered behind the fused
 * launches made on other streams.  A wait that gives up sets the status word in the array's
 * header, which no call clears: until rar_plan_status has been asked, later calls on that GPU
 * give up their waits at once (unspecified results).  rar_plan_status (of any plan that has
 * run on the array since its last query) reports RAR_ERR_TIMEOUT if the word was set, by one
 * of its own calls or by another plan's that ran on the array in the meantime, and clears it;
 * the calls after that work again, since every call starts from cleared flags. */
#define RAR_STATIC_SCRATCH_BYTES (48u << 20)
int rar_allreduce_static(void *const *bufs, rar_plan_t *plan, void *stream);
size_t rar_plan_static_bytes(const rar_plan_t *plan);

/* Pick B_s and C_s by measurement (the paper tunes both once per message size and node count,
 * Section 4.2.1, and leaves heuristics to future work).  Runs the fused all-reduce of the
 * plan's current mode on `bufs` (same contract as rar_allreduce; the buffers are overwritten
 * with repeated sums, so pass buffers whose contents do not matter) with every candidate pair,
 * `calls` timed calls each (>= 1) after two warm-up calls, timed with HIP events on `stream`,
 * and leaves the fastest pair set in the plan as if by rar_plan_set_tuning.  Synchronises the
 * stream.  *best_us (host, may be NULL) receives the winner's mean microseconds per call.
 * A candidate during which a step-barrier wait gave up is discarded (the plan is re-armed and
 * the search goes on); RAR_ERR_TIMEOUT if no candidate survives.  Must be called outside stream
 * capture.  Stepwise mode has nothing to tune: RAR_ERR_ARG. */
int rar_autotune(void *const *bufs, rar_plan_t *plan, void *stream, int calls, double *best_us);

/* ---- measurement aids (used by the benchmark, no effect on results) -----------------------
 *
 * rar_launch_floor: enqueue an empty kernel with the grid and block size the plan's fused
 *   all-reduce would use (the single-launch floor).
 * rar_barrier_only: enqueue the fused kernel with all data movement left out: only the step
 *   barrier traffic (flag stores, waits, fences) of a real call.
 * rar_copy_probe: enqueue a plain 16-byte-vector copy of `bytes` bytes (multiple of 16)
 *   from src to dst (device), the known-size kernel that rocprof counters are scaled by.
 * rar_read_probe: enqueue a kernel that only reads `bytes` bytes (multiple of 16) at src with
 *   16-byte loads (the streaming-read rate of the device); *sink (device, 16 bytes) receives a
 *   value that depends on every vector read.
 */
int rar_launch_floor(rar_plan_t *plan, void *stream);
int rar_barrier_only(rar_plan_t *plan, void *stream);
int rar_copy_probe(void *dst, const void *src, size_t bytes, void *stream);
int rar_read_probe(void *sink, const void *src, size_t bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* RAR_H */
