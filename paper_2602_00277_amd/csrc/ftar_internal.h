// Internal interface between the host API (ftar_api.cpp) and the kernel launchers
// (ftar_reduce.hip, ftar_ring.hip, ftar_persistent.hip).  Not installed; the public surface is
// include/ftar.h.
#ifndef FTAR_INTERNAL_H_
#define FTAR_INTERNAL_H_

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "ftar.h"

namespace ftar {

constexpr int kMaxReplicas = FTAR_MAX_REPLICAS;
constexpr int kMaxBucketsPerLaunch = 256;

// Compact pointer table: the live-mask indirection already resolved on the CPU.
// Passed to the kernels by value (kernel-argument segment) and staged in LDS there.
struct PtrTable {
  void* p[kMaxReplicas];
};

// Portion boundaries in elements, N+1 entries used.
struct SegTable {
  unsigned long long begin[kMaxReplicas + 1];
};

struct BucketTable {
  unsigned long long mask[kMaxBucketsPerLaunch];
};

// 1.0f/(float)N for N = 0..64, computed on the host (entry 0 unused).
struct ScaleTable {
  float s[kMaxReplicas + 1];
};

// Control block of the persistent ring.  The CPU side lives in coherent host-pinned memory; words
// that one side writes and the other polls sit on 64-byte lines of their own.  Only ONE workgroup
// (the relay) ever reads it: 256 workgroups polling host memory over PCIe cost tens of microseconds
// per step.  The relay copies the gate into a small mirror in device memory, which the workers poll.
//
// Several calls may be queued on one stream against one control block (paper section 4.1: one
// all-reduce per gradient bucket, overlapped with the backward pass).  Each call gets a ticket and
// a record of its own in the block; a cancel, or a timeout inside any call, ends every call queued
// so far at its first wait (section 4.2, "Timeout and error handling": queued operations are
// cancelled and marked skipped).  This works through epochs: every call carries the epoch it was
// enqueued in; the CPU kills an epoch by storing it into dead_epoch (and opens the next one), a
// workgroup whose wait times out stores it into gpu_dead_epoch; the relay of every later kernel of
// a dead epoch sees that before it passes on anything and tells its workers to leave.
constexpr int kMaxPersistentBlocks = 1024;
constexpr int kMaxXcds = 16;  // the hardware's XCC id has four bits
constexpr int kCtrlCalls = 64;  // records in a control block: calls that may be in flight at once
constexpr unsigned long long kGateCancel = 1ull << 63;  // in the mirror's gate word only

struct DevCtrl {  // device memory, zeroed on the stream before every launch
  unsigned long long gate;      // units released (copy of the call's gate) | kGateCancel, written by the relay
  unsigned int verdict;         // 0 run, 1 a wait timed out, 2 cancelled, 3 skipped: everybody leaves
  unsigned int exited;          // workers that have left the kernel
  unsigned int min_unit;        // gate units finished by EVERY worker, maintained by the relay
  unsigned int align_count;     // arrivals at the soft barriers inside long steps (a performance hint only)
  // FTAR_PERSIST_PUBLISH: one worker per XCD (its "leader") writes the XCD's L2 back
  unsigned int xcd_workers[kMaxXcds];  // workers that run on XCD x (each registers before its first wait)
  unsigned int xcd_min[kMaxXcds];      // gate units finished by every worker of XCD x, maintained by the relay
  unsigned int xcd_done[kMaxXcds];     // ... and written back from that XCD's L2 by its leader
  unsigned char worker_xcd[kMaxPersistentBlocks];  // the XCD worker b runs on
  unsigned int worker_unit[kMaxPersistentBlocks];  // gate units finished by worker b
};

struct alignas(64) CallRec {  // one queued call
  alignas(64) unsigned long long gate;      // CPU -> GPU: gate units released
  alignas(64) unsigned long long status;    // GPU -> CPU: 0 ok so far, 1 a wait timed out, 2 cancelled, 3 skipped
  unsigned long long blocked_unit;          // GPU -> CPU: unit a workgroup gave up at
  unsigned long long progress;              // GPU -> CPU: units finished by EVERY worker
  unsigned long long ended;                 // GPU -> CPU: 1 once the kernel has left
  alignas(64) unsigned long long epoch;     // host only from here on
  long long ticket;                         // -1: never used
  unsigned int n_blocks;                    // workers; 0: nothing was launched (ring of one)
  unsigned int n_units;                     // gate units of the call
};

struct alignas(64) Ctrl {
  alignas(64) unsigned long long dead_epoch;      // CPU -> GPU: calls of epochs <= this are cancelled
  alignas(64) unsigned long long gpu_dead_epoch;  // GPU -> GPU and CPU: a call of this epoch timed out
  alignas(64) unsigned long long cur_epoch;       // host only: epoch of the next call (starts at 1)
  long long next_ticket;                          // host only
  DevCtrl* dev;                                   // the mirror, allocated with the control block
  CallRec call[kCtrlCalls];
};

enum RingMode {
  kRsFirst = 0,  // acc = x_k + x_{k+1}
  kRsMid = 1,    // acc = acc + x_{k+s+1}
  kRsLast = 2,   // buf_o = cvt(scale * (acc + x_o)), o = k+N-1
  kRsOnly = 3,   // N == 2: buf_o = cvt(scale * (x_k + x_o)), o = k+1
};

struct Tuning {
  int blocks_per_cu;  // 0 = default
  int flags;          // 0 = default policy; 0x10 | p = explicit (bit 0 NT loads, bit 1 NT stores)
};

Tuning current_tuning();

// Hands over (and clears) the timing events armed for this thread's next launch; both null if none.
void take_timing_events(hipEvent_t* start, hipEvent_t* stop);
// Arms the pair for this thread's next launch (what the measurement hook does).
void set_timing_events(hipEvent_t start, hipEvent_t stop);
int device_cu_count();  // of the current device; cached

// All launchers enqueue on `stream` and return hipGetLastError().
// `vec` selects the 128-bit vector kernels (caller has checked alignment).
// zero_pos / zpos below: bit p set = the p-th live replica (ring position p) is a zero-gradient
// participant: it contributes +0.0 and its buffer is never read.
// live: the n_src buffers that are read, in summation order (zero-gradient participants already
// left out: zero_participants says whether there were any; n_src may then be 0).
// dtype: element type of the inputs; out_dtype: of the result (any of the four pairs).
// whole_count: elements of the whole output when this call writes one part of it (the store policy
// follows the whole output's size); 0 = this call is the whole.
hipError_t launch_reduce_masked(const PtrTable& live, int n_src, size_t count, ftar_dtype_t dtype,
                                ftar_dtype_t out_dtype, bool vec, void* out, float scale,
                                bool zero_participants, size_t whole_count, hipStream_t stream);

hipError_t launch_reduce_bucketed(const PtrTable& all, int n_replicas, const BucketTable& masks,
                                  int n_buckets, size_t first_elem, size_t bucket_elems,
                                  size_t count, const ScaleTable& scales, ftar_dtype_t dtype,
                                  bool vec, void* out, hipStream_t stream);

// ring: table of the N live buffers in ring order
hipError_t launch_ring_reduce(RingMode mode, const PtrTable& ring, int n_live, int step,
                              const SegTable& seg, ftar_dtype_t dtype, bool vec, float* acc,
                              float scale, unsigned long long zpos, hipStream_t stream);

hipError_t launch_ring_allgather(const PtrTable& ring, int n_live, int step, const SegTable& seg,
                                 ftar_dtype_t dtype, bool vec, hipStream_t stream);

// All N-1 AllGather steps in one pass: each portion from its owner's buffer into the others.
hipError_t launch_ring_allgather_all(const PtrTable& ring, int n_live, const SegTable& seg, ftar_dtype_t dtype,
                                     bool vec, hipStream_t stream);

// The whole ring in one kernel, gated by the control block (ctrl_dev = device view of it).
// What the whole ring schedule leaves in the buffers, in one pass (N reads, N writes per element).
// owner_only: write each portion into its owner's buffer only (the state after the ReduceScatter phase).
hipError_t launch_ring_onepass(const PtrTable& ring, int n_live, const SegTable& seg,
                               ftar_dtype_t dtype, bool vec, float scale, unsigned long long zpos,
                               bool owner_only, hipStream_t stream);

// Geometry of a partitioned ring: n_parts partitions of part_elems elements (the last one may be
// shorter); portion boundaries are relative to the partition's first element.
// chunk_elems != 0: the gate unit is a ROW of chunks - chunk c of every portion - of one step of one
// partition instead of the whole step (paper section 4.2: each step is pipelined over the chunks of
// a portion); rows_full / rows_last = rows per step in a full / in the last partition.
struct PartGeom {
  unsigned n_parts;
  unsigned long long part_elems;
  SegTable seg_full;  // portions of a full partition
  SegTable seg_last;  // portions of the last partition
  unsigned long long chunk_elems;
  unsigned rows_full, rows_last;
};

// n_blocks workers plus one relay workgroup; clears *mirror on the stream first.
// ctrl_dev / rec_dev: device views of the control block and of this call's record.
hipError_t launch_ring_persistent(const PtrTable& ring, int n_live, const PartGeom& geom,
                                  ftar_dtype_t dtype, bool vec, float* acc, float scale, Ctrl* ctrl_dev,
                                  CallRec* rec_dev, unsigned long long epoch, DevCtrl* mirror, unsigned n_blocks,
                                  unsigned long long timeout_ticks, unsigned flags, unsigned long long zpos,
                                  hipStream_t stream);

// Static scratch of the entry point that allocates nothing (ftar_ring_persistent_static): the
// mirror of the control block and room for the partial sums of one partition, in a file-scope
// device array of the library.  Resolves the array's address on the current device (once per
// device, kept afterwards) and hands out the two parts.  Every call on one GPU shares them.
constexpr size_t kStaticAccElems = static_cast<size_t>(4) << 20;  // 4 Mi floats = 16 MiB
hipError_t static_scratch(DevCtrl** mirror, float** acc);

// Measurement only: n_read streams read and n_written streams written, n_vec 16-byte vectors each
// (tab: the read streams first).  Written streams receive the xor of the read ones, or `fill`.
hipError_t launch_probe_stream(const PtrTable& tab, int n_read, int n_written, size_t n_vec, uint32_t fill,
                               hipStream_t stream);

// Measurement only: n_read streams read, one written through the LDS stage in windows of the wall
// clock (period and window in 10 ns ticks, period a power of two).
hipError_t launch_probe_stream_win(const PtrTable& tab, int n_read, size_t n_vec, unsigned period_ticks,
                                   unsigned window_ticks, hipStream_t stream);

// Measurement only: n_read (1 or 2) streams read and one written by n_workgroups workgroups of
// `threads` lanes that move `per_lane` 16-byte vectors per lane and tile.
hipError_t launch_probe_few(const PtrTable& tab, int n_read, size_t n_vec, unsigned n_workgroups, unsigned threads,
                            unsigned per_lane, hipStream_t stream);

}  // namespace ftar

#endif  // FTAR_INTERNAL_H_
