/*
 * ftar.h - C ABI of the MI355X (gfx950) GPU data path of the Fault Tolerant
 * All Reduce (FTAR): the masked multi-replica gradient reduction.
 *
 * Division of labour (paper section 4.2, "CPU-GPU interaction"): the CPU is the
 * control plane - it decides who is in the group (the paper's reconfig
 * function; here `live_mask`) and the chunk schedule (here `ftar_plan`); the
 * GPU is the data plane - it runs the per-chunk reduce and copy (here the
 * kernels behind the *_step and reduce_* calls).  No call in this header ever
 * takes a membership decision on the device.
 *
 * One GPU, simulated replicas: replica r's gradient is the device buffer
 * bufs[r].  The union of all ranks' send/receive buffers of the paper's ring
 * collapses to one fp32 buffer `acc` holding, for every portion, the partial
 * sum that is in flight.
 *
 * Conventions for every call
 *   - `bufs` is a HOST array of n_replicas DEVICE pointers indexed by replica
 *     id.  Entries of dead replicas are never dereferenced and may be NULL.
 *     The library copies what it needs before returning; the caller may free
 *     the host array at once.  All device memory that holds data is caller-owned;
 *     no compute call allocates or frees memory (only ftar_ctrl_create/destroy do,
 *     at set-up: the control block of the persistent ring).
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).
 *     Compute calls only enqueue work on it and return; they never
 *     synchronise.  Calls on one stream are ordered by the stream.
 *   - Device pointers must be aligned to their element size.  When every
 *     pointer (and every portion or bucket boundary) is 16-byte aligned the
 *     128-bit vector kernels run, otherwise an element-wise kernel of the same
 *     arithmetic runs.
 *   - Errors are return codes; nothing aborts or throws across this boundary.
 *     On any error no work has been enqueued and no state has changed.
 *     Following the paper's split (section 4.2, "Timeout and error handling"):
 *     caller errors and device errors are not retryable; the retryable class
 *     is reserved for a membership change while work is queued.
 *   - Host threads may call at the same time, each on a stream of its own: the library
 *     holds no lock, a plan is only read by the compute calls, the last error is per thread.
 *   - Arithmetic: inputs are widened exactly to fp32; sums are fp32 additions
 *     in a fixed order; the mean is ONE multiplication by
 *     scale = 1.0f/(float)n_live (one correctly rounded fp32 division, done on
 *     the host); bf16 outputs are rounded once, to nearest even.  No fused
 *     multiply-add, no flush of denormals.
 */
#ifndef FTAR_H_
#define FTAR_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FTAR_MAX_REPLICAS 64

typedef struct ftar_plan_s ftar_plan_t; /* opaque, host memory owned by the library */

typedef enum { FTAR_F32 = 0, FTAR_BF16 = 1 } ftar_dtype_t;

typedef enum {
  FTAR_OK = 0,
  /* caller errors */
  FTAR_ERR_INVALID_ARG = 1, /* null pointer, n_replicas outside [1,64], count == 0,
                               chunk_elems == 0, unknown dtype, misaligned pointer */
  FTAR_ERR_NO_LIVE = 2,     /* live_mask has no bit set below n_replicas */
  FTAR_ERR_BAD_MASK = 3,    /* live_mask has a bit set at or above n_replicas */
  FTAR_ERR_BAD_STEP = 4,    /* step outside [0, n_live-2] */
  FTAR_ERR_TOO_LARGE = 5,   /* ftar_ring_persistent_static: more partial sums than the static scratch holds */
  /* retryable: re-plan over the new group and restart the schedule */
  FTAR_ERR_STALE_PLAN = 16, /* the persistent ring was cancelled or timed out before finishing */
  FTAR_ERR_SKIPPED = 17,    /* a queued persistent ring never started: a call before it was cancelled or timed out */
  /* fatal: the HIP runtime reported a failure */
  FTAR_ERR_DEVICE = 32
} ftar_status_t;

/* ---------------------------------------------------------------------------
 * ftar_plan - the CPU side of the ring schedule.
 * Paper: section 4.2 - reconfig decides the group ("CPU-GPU interaction"); the
 * ring has a ReduceScatter and an AllGather phase of N-1 steps each and replica
 * i starts by sending its i-th portion to its right neighbour ("Ring
 * algorithm"); data moves in fixed-size chunks.
 *
 * n_replicas   number of replica slots, 1..64
 * live_mask    bit r set = replica r takes part; N = popcount
 * count        elements per replica buffer (> 0)
 * chunk_elems  chunk size in elements (> 0); portion boundaries fall on chunk
 *              boundaries: portion k = [min(count, floor(k*n_chunks/N)*chunk_elems),
 *              ...next), n_chunks = ceil(count/chunk_elems)
 * Ring position p is the p-th live replica in ascending index order; the right
 * neighbour of p is (p+1) mod N.
 * Returns a plan (default dtype FTAR_BF16) or NULL; ftar_last_error() tells why.
 * The plan holds no device memory and the same arguments always give the same
 * plan; only the ftar_plan_set_* calls below change it (element type, zero-gradient
 * participants, sum or mean, partition size), never a compute call.
 * A membership change is handled by destroying the plan, making a new one and
 * restarting from ReduceScatter step 0; this is sound as long as the last
 * ReduceScatter step of the old plan has not been enqueued, because until then
 * no replica buffer has been written.
 */
ftar_plan_t* ftar_plan(int n_replicas, uint64_t live_mask, size_t count, size_t chunk_elems);
void ftar_plan_destroy(ftar_plan_t* plan);

/* Element type of the replica buffers for the step calls (input and output type are the same). */
ftar_status_t ftar_plan_set_dtype(ftar_plan_t* plan, ftar_dtype_t dtype);

int ftar_plan_n_live(const ftar_plan_t* plan);     /* N; 0 if plan is NULL */
int ftar_plan_n_steps(const ftar_plan_t* plan);    /* N-1, the steps of each phase */
size_t ftar_plan_acc_bytes(const ftar_plan_t* plan); /* size of `acc`: 4 bytes per element of one partition */
float ftar_plan_scale(const ftar_plan_t* plan);    /* 1.0f/(float)N unless changed by set_zero_mask / set_op */
/* Portion k in [0,N): element range [*begin,*end) and the replica that holds its
 * finished value after the ReduceScatter phase (the replica at ring position k-1). */
ftar_status_t ftar_plan_segment(const ftar_plan_t* plan, int k, size_t* begin, size_t* end,
                                int* owner_replica);

/* ---------------------------------------------------------------------------
 * Zero-gradient participants.
 * Paper: section 4.3, "Non-blocking Catch Up" - a replica that has fallen behind fetches a
 * checkpoint while the others train, takes part in the gradient exchange at the end of the step
 * and sends a ZERO gradient; the exchange brings all replicas to the same state.
 * Replicas in zero_mask (a subset of live_mask) are participants: they count among the N ring
 * members, and in the ring calls their buffers RECEIVE the result; but they contribute +0.0 and
 * their buffers are never read (N_zero * E bytes per element are not moved).  The result is
 * bit-identical to running with buffers that hold +0.0 everywhere.
 * The divisor is N (a catching-up replica is a participant); with contributors_only != 0 it is
 * N - N_zero.  FTAR_ERR_BAD_MASK if zero_mask has a bit outside live_mask; FTAR_ERR_NO_LIVE if
 * contributors_only leaves nobody, or (plan only) if the single live replica is a zero participant:
 * a ring of one has no steps that could deliver its +0.0.
 * ftar_plan_set_zero_mask applies to every ring call made with the plan afterwards (step calls,
 * one-pass, persistent); ftar_reduce_masked_zero is the one-shot form, where a zero
 * participant's entry in bufs may be NULL.
 */
ftar_status_t ftar_plan_set_zero_mask(ftar_plan_t* plan, uint64_t zero_mask, int contributors_only);
ftar_status_t ftar_reduce_masked_zero(const void* const* bufs, int n_replicas, uint64_t live_mask,
                                      uint64_t zero_mask, int contributors_only, size_t count,
                                      ftar_dtype_t dtype, void* out, void* stream);

/* ---------------------------------------------------------------------------
 * ftar_plan_set_partition - split the data into partitions for ftar_ring_persistent.
 * Paper: section 4.2 - the send and receive buffers are a fixed S x C bytes; the message is split
 * into partitions of at most S x C x N bytes; each partition runs one whole round of the ring
 * (2N-2 steps), then the next partition starts.
 * Partition p covers elements [p*partition_elems, min((p+1)*partition_elems, count)) of every
 * buffer and is split into N portions by the rule of ftar_plan applied to the partition's own
 * length (so the result differs from the unpartitioned ring only in which rotation of the
 * summation order an element gets).  `acc` then holds ONE partition (ftar_plan_acc_bytes) and is
 * reused by the next one.  A "slot" is one step of one partition; slots run partition-major and
 * are what the CPU releases and what progress counts: ftar_plan_n_slots = partitions * (2N-2).
 * partition_elems == 0 or >= count restores the single partition.  A partitioned plan is only
 * valid for ftar_ring_persistent; the per-step calls reject it (a caller who wants partitions
 * with per-step kernels makes one plan per partition over offset pointers).
 * A cancel or timeout leaves the partitions before the blocked one finished, the later ones
 * untouched, and the blocked one untouched only if its last ReduceScatter slot was not released.
 */
ftar_status_t ftar_plan_set_partition(ftar_plan_t* plan, size_t partition_elems);
int ftar_plan_n_partitions(const ftar_plan_t* plan);
int ftar_plan_n_slots(const ftar_plan_t* plan);
ftar_status_t ftar_plan_partition_segment(const ftar_plan_t* plan, int partition, int k, size_t* begin,
                                          size_t* end, int* owner_replica);

/* ---------------------------------------------------------------------------
 * ftar_reduce_step - one ReduceScatter step, for all N portions at once (each
 * portion stands for the work of a different rank at that step).
 * Paper: section 4.2, "Ring algorithm" (reduce on arrival, forward) and
 * "Optimizations" (intermediate results go to the send buffer only; the last
 * step's result goes to the local data buffer, fused into the same kernel).
 * With x_p = fp32 image of the buffer of the replica at ring position p, for i in portion k:
 *   step 0 (N >= 3)      acc[i] = x_k[i] + x_{k+1}[i]
 *   step s, 1..N-3       acc[i] = acc[i] + x_{k+s+1}[i]
 *   step N-2 (N >= 3)    o = k+N-1:  buf_o[i] = cvt(scale * (acc[i] + x_o[i]))   (in place)
 *   N == 2, step 0       o = k+1:    buf_o[i] = cvt(scale * (x_k[i] + x_o[i]))   (acc unused)
 * (position indices mod N).  N == 1 has no steps.
 * acc: device, ftar_plan_acc_bytes() bytes, 16-byte aligned; contents are
 * defined only between step 0 and step N-2 of one plan.  May be NULL when N == 2.
 */
ftar_status_t ftar_reduce_step(const ftar_plan_t* plan, int step, void* const* bufs, float* acc,
                               void* stream);

/* ---------------------------------------------------------------------------
 * ftar_allgather_step - one AllGather step, for all N portions at once.
 * Paper: section 4.2, "Ring algorithm" (each GPU forwards its finished portion
 * to its right neighbour, receivers forward what they received) and
 * "Optimizations" (received data is stored to the local data buffer).
 *   step t, 0..N-2: for i in portion k: buf_{k+t}[i] = buf_{k+t-1}[i]   (bit copy; positions mod N)
 */
ftar_status_t ftar_allgather_step(const ftar_plan_t* plan, int step, void* const* bufs,
                                  void* stream);

/* ---------------------------------------------------------------------------
 * ftar_reduce_masked - the whole reduction in one pass: what the all-reduce
 * over the live group must deliver (paper section 4.1: the sum of the
 * participants' gradients; the mean by this library's convention).
 *   out[i] = cvt(scale * (((x_a[i] + x_b[i]) + x_c[i]) + ...)),  a < b < c ... the live replicas
 * The sum starts from the first live value, so a single live replica is the
 * bitwise identity.  out: device, count elements of `dtype`; it may be equal to
 * bufs[r] of a live replica (same-thread read then write) but must not
 * partially overlap any input.
 */
ftar_status_t ftar_reduce_masked(const void* const* bufs, int n_replicas, uint64_t live_mask,
                                 size_t count, ftar_dtype_t dtype, void* out, void* stream);

/* ---------------------------------------------------------------------------
 * Delivery variants.
 * Paper: section 4.1 states the exchange as the SUM of the participants' gradients (the mean is
 * this build's default reading); FTAR_SUM gives exactly that: the scale factor is 1.0f, all else
 * is unchanged.  ftar_plan_set_op applies to every ring call made with the plan afterwards;
 * ftar_plan_scale reports the factor in force.
 * ftar_reduce_masked_ex is the one-shot reduce with everything selectable: zero-gradient
 * participants (as ftar_reduce_masked_zero), the operation, and the result type independently of
 * the input type: FTAR_F32 from FTAR_BF16 inputs stores the fp32 sum/mean unrounded (2N read + 4
 * written bytes per element); FTAR_BF16 from FTAR_F32 inputs rounds it once, to nearest even (4N
 * read + 2 written).
 */
typedef enum { FTAR_MEAN = 0, FTAR_SUM = 1 } ftar_op_t;
ftar_status_t ftar_plan_set_op(ftar_plan_t* plan, ftar_op_t op);
ftar_status_t ftar_reduce_masked_ex(const void* const* bufs, int n_replicas, uint64_t live_mask,
                                    uint64_t zero_mask, int contributors_only, size_t count,
                                    ftar_dtype_t in_dtype, ftar_dtype_t out_dtype, ftar_op_t op,
                                    void* out, void* stream);

/* ---------------------------------------------------------------------------
 * Learning-rate intervention factors.
 * Paper: section 6.2 - with fewer healthy replicas a step trains on less data; the "linear"
 * strategy scales the learning rate by healthy/total replicas, the "sqrt" strategy by the
 * square root of that ratio.  Healthy = live and not a zero-gradient participant of the plan;
 * total = n_replicas.  Host-only: *linear = (float)healthy / (float)n_replicas,
 * *root = (float)sqrt((double)healthy / (double)n_replicas).  Either pointer may be NULL.
 */
ftar_status_t ftar_plan_lr_factors(const ftar_plan_t* plan, float* linear, float* root);

/* ---------------------------------------------------------------------------
 * ftar_reduce_masked_bucketed - ftar_reduce_masked with a live mask of its own
 * for every bucket of bucket_elems consecutive elements (the last bucket may be
 * short), in one launch per 256 buckets.  Models replicas that leave and rejoin
 * between the iterations of one all-reduce (paper section 4.2: FTAR may run for
 * several iterations, each exchanging a portion of the gradients; membership is
 * decided by the CPU before each).  Same arithmetic as calling
 * ftar_reduce_masked once per bucket with masks[b]; scale is per bucket.  (Buckets of half a GiB
 * of traffic or more are in fact run that way, one after the other on the stream.)
 * masks: HOST array of ceil(count/bucket_elems) masks, each valid for n_replicas.
 */
ftar_status_t ftar_reduce_masked_bucketed(const void* const* bufs, int n_replicas,
                                          const uint64_t* masks, size_t n_buckets,
                                          size_t bucket_elems, size_t count, ftar_dtype_t dtype,
                                          void* out, void* stream);

/* ---------------------------------------------------------------------------
 * ftar_reduce_scatter_all - what the N-1 ftar_reduce_step calls of the plan leave in the replica
 * buffers, in ONE pass and without `acc`: every element's N contributions are added in a
 * register in the ring's order for its portion (positions k, k+1, ..., k+N-1 mod N; paper
 * section 4.2, "Ring algorithm") and the rounded mean is written into the buffer of the portion's
 * owner (ring position k-1) only; everything else stays as it was.  Bit-identical to the step
 * calls; N*E + E bytes per element.  This is the reduce-scatter a sharded optimizer wants (every
 * replica ends with its own portion); ftar_allgather_all or the ftar_allgather_step calls complete
 * it to the all-reduce.  N == 1: nothing to do.
 */
ftar_status_t ftar_reduce_scatter_all(const ftar_plan_t* plan, void* const* bufs, void* stream);

/* ---------------------------------------------------------------------------
 * ftar_allgather_all - what the N-1 ftar_allgather_step calls of the plan leave in the replica
 * buffers, in ONE pass: every portion is read once from the buffer of the replica that holds its
 * finished value after the ReduceScatter phase (ring position k-1 for portion k; paper section
 * 4.2, "Ring algorithm") and written to the N-1 other live buffers.  The ring hands a portion on
 * one neighbour per step because a network sits between the replicas; with all buffers on one
 * device this moves E + (N-1)E bytes per element instead of 2(N-1)E.  Bit copies: the same result
 * as the step calls.  Call it after the last ftar_reduce_step.  N == 1: nothing to do.
 */
ftar_status_t ftar_allgather_all(const ftar_plan_t* plan, void* const* bufs, void* stream);

/* ---------------------------------------------------------------------------
 * ftar_allreduce_onepass - what the whole schedule of the plan (N-1 ftar_reduce_step calls, then
 * N-1 ftar_allgather_step calls) leaves in the replica buffers, computed in ONE pass: every
 * element's N contributions are added in a register in the ring's order (portion k: ring
 * positions k, k+1, ..., k+N-1 mod N; paper section 4.2, "Ring algorithm") and the rounded mean
 * is written into all N live buffers.  Bit-identical to the step schedule; `acc` is not needed.
 * The ring's steps exist for the network between the replicas; with all replicas' buffers on one
 * device this is the bandwidth-optimal form: 2*N*E bytes per element.
 * Dead replicas' buffers are neither read nor written.  N == 1: nothing to do.
 */
ftar_status_t ftar_allreduce_onepass(const ftar_plan_t* plan, void* const* bufs, void* stream);

/* ---------------------------------------------------------------------------
 * CPU-driven persistent ring: the whole ring all-reduce as ONE kernel whose progress the CPU
 * gates through flags in host-pinned memory.
 * Paper: section 4.2, "Optimizations" (one kernel per AllReduce that busy-polls a flag in
 * host-pinned memory set by a CPU thread; run on few compute units with many loads in flight
 * per thread) and "Timeout and error handling" (the GPU-side wait is a loop with a timeout so
 * the GPU never hangs; a recoverable error returns a retryable work and queued operations are
 * cancelled and marked skipped).
 *
 * The kernel runs the 2N-2 steps of the plan in order (ReduceScatter 0..N-2, then AllGather
 * N-1..2N-3), partition after partition if the plan is partitioned, with the arithmetic of
 * ftar_reduce_step / ftar_allgather_step.  Before gate unit u (by default one step of one
 * partition) every workgroup waits until the CPU has released it (ftar_ctrl_release(ctrl, r) with
 * r > u); after it, it publishes its progress.  A wait ends without the release when the CPU
 * cancels (ftar_ctrl_cancel) or when timeout_us microseconds have passed: the workgroup then
 * records why and exits, so the kernel always terminates.  No user buffer is written before
 * the last ReduceScatter step (s = N-2) is released: a cancel or timeout before that leaves every
 * bufs[r] untouched and the caller re-plans and restarts.
 *
 * ctrl is a control block made by ftar_ctrl_create(): coherent host-pinned memory plus a mirror
 * of 4 KiB in device memory (both allocated at set-up, not on the hot path).
 *
 * Gate units.  What the CPU releases, and what progress counts, is the gate unit.  By default a unit
 * is a slot (one step of one partition): ftar_plan_n_slots units per call.  With
 * FTAR_PERSIST_CHUNKS a unit is one ROW OF CHUNKS of a slot - chunk c of every portion, i.e. the
 * c-th chunk of every rank's work in that step (section 4.2: every step of a partition is pipelined
 * over the chunks of a portion, chunk_elems of ftar_plan being the chunk).  Units are ordered
 * partition, step, row; releasing n lets units [0, n) run; ftar_plan_n_gate_units tells how many a
 * call has (rows per step = the largest number of chunks a portion of that partition has).  A
 * workgroup looks at the gate whenever its next tile lies in a later row and reports when it moves
 * on to one.  Results never depend on the unit.  A tile never crosses a chunk's end: chunk_elems
 * should be a multiple of 8192 elements (fp32: 4096) for full speed.
 *
 * Several calls on one control block.  Calls may be queued one behind the other on ONE stream
 * against one control block (section 4.1: one all-reduce per gradient bucket, overlapped with the
 * backward pass); at most 64 may be in flight.  Every call gets a ticket (ftar_ctrl_last_ticket,
 * right after the call, from the enqueueing thread) and is released, observed and judged by it
 * (ftar_ctrl_*_call); the forms without a ticket mean the call enqueued last.  ftar_ctrl_cancel
 * ends EVERY call enqueued so far at its next wait and lets calls enqueued afterwards run; a
 * timeout inside one call does the same to the calls queued behind it (section 4.2: queued
 * operations are cancelled and marked skipped).  ftar_ctrl_result_call then tells them apart:
 * FTAR_OK (finished before), FTAR_ERR_STALE_PLAN (the call that was stopped: units_done units are
 * complete), FTAR_ERR_SKIPPED (queued behind it: it left at its first wait, nothing was read or
 * written).  After a timeout the caller acknowledges with ftar_ctrl_cancel before re-planning:
 * until then newly enqueued calls count as "queued behind" and are skipped too.
 * With a partitioned plan whose last partition is shorter, the workgroups also wait
 * for each other once (bounded by timeout_us like every wait), before that partition's first slot.
 * Every workgroup must be resident at once: on a stream that is restricted to some of the
 * compute units the caller chooses n_blocks to fit them.
 *   n_blocks    worker workgroups (= compute units used), 1..1024; 0 = one per compute unit
 *               (two with a partitioned plan); one more workgroup relays the CPU's gate word;
 *               clamped to what the GPU can keep resident at once (a waiting workgroup keeps
 *               its place, so all of them must fit)
 *   timeout_us  per-wait limit in microseconds (> 0)
 *   flags       FTAR_PERSIST_PUBLISH: a unit counts as done (ftar_ctrl_progress) only after its
 *               data has been written back from the GPU's L2, as a NIC reading the buffers on
 *               the CPU's signal would need; without it progress means "computed", and the data
 *               is guaranteed visible off the GPU once the stream has been synchronised.  (One
 *               workgroup per XCD writes that XCD's L2 back for all the workgroups that run there.)
 *               FTAR_PERSIST_ALIGN: workgroups that ran ahead wait (bounded) for the others after
 *               every step and, inside a step, after every 256 Mi elements (not with
 *               FTAR_PERSIST_CHUNKS); a performance hint for long steps, never needed for correctness.
 *               The library sets it by itself when the partial sums of one partition exceed
 *               256 MiB (steps of hundreds of microseconds: +5..9 %; below that it costs).
 *               FTAR_PERSIST_CHUNKS: the gate unit is a row of chunks (above).
 * Returns at once like every other compute call; on an error nothing was enqueued and the control
 * block is unchanged (FTAR_ERR_INVALID_ARG also when 64 earlier calls on it are still in flight).
 * After the stream has been synchronised, ftar_ctrl_result tells how it ended; *units_done = units
 * completed by every workgroup.
 */
#define FTAR_PERSIST_PUBLISH 1u
#define FTAR_PERSIST_ALIGN 2u
#define FTAR_PERSIST_CHUNKS 4u
void* ftar_ctrl_create(void);   /* NULL on failure */
void ftar_ctrl_destroy(void* ctrl); /* only when no call on it is in flight */
ftar_status_t ftar_ring_persistent(const ftar_plan_t* plan, void* const* bufs, float* acc, void* ctrl,
                                   int n_blocks, unsigned timeout_us, unsigned flags, void* stream);
int ftar_plan_n_gate_units(const ftar_plan_t* plan, unsigned flags); /* 0: plan or flags not usable */
/* ---------------------------------------------------------------------------
 * ftar_ring_persistent_static - ftar_ring_persistent for callers that cannot allocate device memory
 * and have none to spare for a workspace: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same kernel, same arguments, same results bit for bit, but the
 * partial sums (`acc`) and the device mirror of the control block live in a static device array of
 * the library (16 MiB + 8 KiB per GPU, held from the first use on that GPU until the process ends)
 * instead of caller memory and the mirror made by ftar_ctrl_create.  The call itself allocates and
 * frees nothing and calls no allocating routine; `ctrl` is still a block from ftar_ctrl_create
 * (made at set-up), bufs are the caller's.
 * Limit: one partition - ftar_plan_set_partition's partition_elems, or `count` for an unpartitioned
 * plan - is at most FTAR_STATIC_ACC_ELEMS (4 Mi) elements; beyond that FTAR_ERR_TOO_LARGE and
 * nothing is enqueued.  (Partitions of this size are the intended use: the partial sums then stay in
 * the caches.)  The array's address is looked up once per GPU, at ftar_ctrl_create or else at the
 * first call on that GPU, with that GPU current.
 * All calls on one GPU share the array, and it keeps the last call's contents: the mirror is
 * cleared on `stream` before every launch, the partial sums are always written before they are
 * read.  Two calls that overlap in time on one GPU (different streams, or threads) race on it:
 * keep them on one stream, or use ftar_ring_persistent with buffers of their own.
 */
#define FTAR_STATIC_ACC_ELEMS ((size_t)4 << 20)
ftar_status_t ftar_ring_persistent_static(const ftar_plan_t* plan, void* const* bufs, void* ctrl,
                                          int n_blocks, unsigned timeout_us, unsigned flags, void* stream);
/* CPU side of the handshake (atomic host stores/loads on the control block; release, cancel, progress
 * and result are callable from any thread while kernels run; enqueueing calls on one control block
 * and ftar_ctrl_last_ticket belong to one thread at a time). */
int ftar_ctrl_last_ticket(const void* ctrl);                        /* ticket of the call enqueued last; -1: none */
void ftar_ctrl_release_call(void* ctrl, int ticket, int n_units);   /* units [0, n_units) of that call may run */
void ftar_ctrl_release(void* ctrl, int n_units);                    /* the same for the call enqueued last */
void ftar_ctrl_cancel(void* ctrl);               /* every call enqueued so far stops at its next wait */
int ftar_ctrl_progress_call(const void* ctrl, int ticket);
int ftar_ctrl_progress(const void* ctrl);        /* units completed by EVERY workgroup: a lower bound
                                                    while the kernel runs ahead of it, exact
                                                    whenever the kernel waits for a release */
ftar_status_t ftar_ctrl_result_call(const void* ctrl, int ticket, int* units_done);
ftar_status_t ftar_ctrl_result(const void* ctrl, int* units_done);

/* --------------------------------------------------------------------------- */
ftar_status_t ftar_last_error(void);          /* status of this thread's last failing call */
int ftar_status_is_retryable(ftar_status_t s);
const char* ftar_status_str(ftar_status_t s); /* static string */

#ifdef __cplusplus
}
#endif
#endif /* FTAR_H_ */
