// Host side of the FTAR data path: the planner (the CPU's part of the ring
// schedule), argument validation and the C ABI declared in include/ftar.h.
// Paper section 4.2: the CPU owns membership and control ("CPU-GPU
// interaction"), the ring is N-1 ReduceScatter plus N-1 AllGather steps with
// replica i first sending portion i to its right neighbour ("Ring algorithm"),
// errors are either reported for a retry or fatal ("Timeout and error handling").

#include <atomic>
#include <cstdlib>
#include <cmath>
#include <cstring>
#include <new>

#include "ftar_internal.h"
#include "ftar_measure.h"

namespace ftar {
namespace {

constexpr uint32_t kPlanMagic = 0x46544152u;  // "FTAR"
constexpr unsigned long long kRecLaunchFailed = 255;  // CallRec::status of a call whose launch failed (host only)

thread_local ftar_status_t t_last_error = FTAR_OK;

ftar_status_t fail(ftar_status_t s) {
  t_last_error = s;
  return s;
}

thread_local hipEvent_t t_time_start = nullptr;
thread_local hipEvent_t t_time_stop = nullptr;

// measurement overrides (include/ftar_measure.h); zero = every kernel's own default
std::atomic<int> g_blocks_per_cu{0};
std::atomic<int> g_flags{0};

// Live replicas in ascending index order = ring positions 0..N-1.
ftar_status_t resolve_mask(int n_replicas, uint64_t live_mask, int* ring, int* n_live) {
  if (n_replicas < 1 || n_replicas > kMaxReplicas) return FTAR_ERR_INVALID_ARG;
  if (n_replicas < 64 && (live_mask >> n_replicas) != 0) return FTAR_ERR_BAD_MASK;
  int N = 0;
  for (int r = 0; r < n_replicas; ++r)
    if ((live_mask >> r) & 1ull) ring[N++] = r;
  if (N == 0) return FTAR_ERR_NO_LIVE;
  *n_live = N;
  return FTAR_OK;
}

size_t elem_size(ftar_dtype_t d) { return d == FTAR_F32 ? 4 : 2; }

bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

}  // namespace

Tuning current_tuning() { return Tuning{g_blocks_per_cu.load(), g_flags.load()}; }

void take_timing_events(hipEvent_t* start, hipEvent_t* stop) {
  *start = t_time_start;
  *stop = t_time_stop;
  t_time_start = nullptr;
  t_time_stop = nullptr;
}

void set_timing_events(hipEvent_t start, hipEvent_t stop) {
  t_time_start = start;
  t_time_stop = stop;
}

int device_cu_count() {
  static thread_local int cached_dev = -1;
  static thread_local int cached_cu = 0;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 256;
  if (dev != cached_dev) {
    int cu = 0;
    if (hipDeviceGetAttribute(&cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cu < 1)
      cu = 256;
    cached_dev = dev;
    cached_cu = cu;
  }
  return cached_cu;
}

}  // namespace ftar

using namespace ftar;

struct ftar_plan_s {
  uint32_t magic;
  int n_replicas;
  uint64_t live_mask;
  size_t count;
  size_t chunk_elems;
  int n_live;
  int ring[kMaxReplicas];  // ring position -> replica id
  float scale;             // 1.0f/(float)n_live
  ftar_dtype_t dtype;
  SegTable seg;            // portion boundaries, n_live+1 entries (of the whole buffer)
  // partitioned ring (persistent kernel only); part_elems == 0: one partition = the whole buffer
  unsigned long long zero_pos;  // bit p: ring position p is a zero-gradient participant
  int n_zero;                   // popcount(zero_pos)
  int contributors_only;        // divisor = n_live - n_zero instead of n_live
  ftar_op_t op;
  size_t part_elems;
  size_t n_parts;
  SegTable part_seg_full;  // portions of a full partition, relative to its first element
  SegTable part_seg_last;  // portions of the last partition
};

static void refresh_scale(ftar_plan_s* p) {
  const int divisor = p->contributors_only ? p->n_live - p->n_zero : p->n_live;
  p->scale = p->op == FTAR_SUM ? 1.0f : 1.0f / static_cast<float>(divisor);
}

// Portions are whole chunks, as even as whole chunks allow: portion k starts at chunk
// floor(k * n_chunks / N).  Only the very last chunk can be short.
static void portions(size_t len, size_t chunk_elems, int N, SegTable* seg) {
  const size_t n_chunks = len / chunk_elems + (len % chunk_elems ? 1 : 0);
  for (int k = 0; k < N; ++k) {
    const unsigned __int128 first_chunk = static_cast<unsigned __int128>(n_chunks) * k / N;
    const unsigned __int128 b = first_chunk * chunk_elems;
    seg->begin[k] = b < len ? static_cast<unsigned long long>(b) : len;
  }
  for (int k = N; k <= kMaxReplicas; ++k) seg->begin[k] = len;
}

extern "C" {

ftar_plan_t* ftar_plan(int n_replicas, uint64_t live_mask, size_t count, size_t chunk_elems) {
  int ring[kMaxReplicas];
  int N = 0;
  ftar_status_t s = resolve_mask(n_replicas, live_mask, ring, &N);
  if (s != FTAR_OK) { fail(s); return nullptr; }
  if (count == 0 || chunk_elems == 0) { fail(FTAR_ERR_INVALID_ARG); return nullptr; }
  ftar_plan_t* p = new (std::nothrow) ftar_plan_t;
  if (!p) { fail(FTAR_ERR_INVALID_ARG); return nullptr; }
  std::memset(p, 0, sizeof(*p));
  p->magic = kPlanMagic;
  p->n_replicas = n_replicas;
  p->live_mask = live_mask;
  p->count = count;
  p->chunk_elems = chunk_elems;
  p->n_live = N;
  std::memcpy(p->ring, ring, sizeof(int) * N);
  p->scale = 1.0f / static_cast<float>(N);
  p->dtype = FTAR_BF16;
  portions(count, chunk_elems, N, &p->seg);
  p->part_elems = 0;
  p->n_parts = 1;
  p->part_seg_full = p->seg;
  p->part_seg_last = p->seg;
  return p;
}

void ftar_plan_destroy(ftar_plan_t* plan) {
  if (!plan || plan->magic != kPlanMagic) return;
  plan->magic = 0;
  delete plan;
}

static bool plan_ok(const ftar_plan_t* p) { return p && p->magic == kPlanMagic; }

ftar_status_t ftar_plan_set_dtype(ftar_plan_t* plan, ftar_dtype_t dtype) {
  if (!plan_ok(plan) || (dtype != FTAR_F32 && dtype != FTAR_BF16)) return fail(FTAR_ERR_INVALID_ARG);
  plan->dtype = dtype;
  return FTAR_OK;
}

ftar_status_t ftar_plan_set_zero_mask(ftar_plan_t* plan, uint64_t zero_mask, int contributors_only) {
  if (!plan_ok(plan)) return fail(FTAR_ERR_INVALID_ARG);
  if ((zero_mask & ~plan->live_mask) != 0) return fail(FTAR_ERR_BAD_MASK);
  unsigned long long zpos = 0;
  int Z = 0;
  for (int p = 0; p < plan->n_live; ++p) {
    if ((zero_mask >> plan->ring[p]) & 1ull) {
      zpos |= 1ull << p;
      ++Z;
    }
  }
  const int divisor = contributors_only ? plan->n_live - Z : plan->n_live;
  if (divisor <= 0) return fail(FTAR_ERR_NO_LIVE);
  // a ring of one has no steps, so nothing could write the +0.0 a lone zero participant is owed
  if (plan->n_live == 1 && Z == 1) return fail(FTAR_ERR_NO_LIVE);
  plan->zero_pos = zpos;
  plan->n_zero = Z;
  plan->contributors_only = contributors_only ? 1 : 0;
  refresh_scale(plan);
  return FTAR_OK;
}

ftar_status_t ftar_plan_set_op(ftar_plan_t* plan, ftar_op_t op) {
  if (!plan_ok(plan) || (op != FTAR_MEAN && op != FTAR_SUM)) return fail(FTAR_ERR_INVALID_ARG);
  plan->op = op;
  refresh_scale(plan);
  return FTAR_OK;
}

ftar_status_t ftar_plan_lr_factors(const ftar_plan_t* plan, float* linear, float* root) {
  if (!plan_ok(plan)) return fail(FTAR_ERR_INVALID_ARG);
  const int healthy = plan->n_live - plan->n_zero;
  if (linear) *linear = static_cast<float>(healthy) / static_cast<float>(plan->n_replicas);
  if (root)
    *root = static_cast<float>(std::sqrt(static_cast<double>(healthy) / static_cast<double>(plan->n_replicas)));
  return FTAR_OK;
}

ftar_status_t ftar_plan_set_partition(ftar_plan_t* plan, size_t partition_elems) {
  if (!plan_ok(plan)) return fail(FTAR_ERR_INVALID_ARG);
  if (partition_elems == 0 || partition_elems >= plan->count) {
    plan->part_elems = 0;
    plan->n_parts = 1;
    plan->part_seg_full = plan->seg;
    plan->part_seg_last = plan->seg;
    return FTAR_OK;
  }
  const size_t n_parts = plan->count / partition_elems + (plan->count % partition_elems ? 1 : 0);
  if (n_parts * static_cast<size_t>(2 * plan->n_live - 2) > 0x7fffffffull) return fail(FTAR_ERR_INVALID_ARG);
  plan->part_elems = partition_elems;
  plan->n_parts = n_parts;
  portions(partition_elems, plan->chunk_elems, plan->n_live, &plan->part_seg_full);
  portions(plan->count - (n_parts - 1) * partition_elems, plan->chunk_elems, plan->n_live,
           &plan->part_seg_last);
  return FTAR_OK;
}

int ftar_plan_n_live(const ftar_plan_t* plan) { return plan_ok(plan) ? plan->n_live : 0; }
int ftar_plan_n_steps(const ftar_plan_t* plan) { return plan_ok(plan) ? plan->n_live - 1 : 0; }
int ftar_plan_n_partitions(const ftar_plan_t* plan) {
  return plan_ok(plan) ? static_cast<int>(plan->n_parts) : 0;
}
int ftar_plan_n_slots(const ftar_plan_t* plan) {
  return plan_ok(plan) ? static_cast<int>(plan->n_parts) * (2 * plan->n_live - 2) : 0;
}
size_t ftar_plan_acc_bytes(const ftar_plan_t* plan) {
  if (!plan_ok(plan)) return 0;
  return (plan->part_elems ? plan->part_elems : plan->count) * 4;
}
float ftar_plan_scale(const ftar_plan_t* plan) { return plan_ok(plan) ? plan->scale : 0.0f; }

ftar_status_t ftar_plan_segment(const ftar_plan_t* plan, int k, size_t* begin, size_t* end,
                                int* owner_replica) {
  if (!plan_ok(plan) || k < 0 || k >= plan->n_live || plan->part_elems != 0)
    return fail(FTAR_ERR_INVALID_ARG);
  if (begin) *begin = plan->seg.begin[k];
  if (end) *end = plan->seg.begin[k + 1];
  if (owner_replica) *owner_replica = plan->ring[(k + plan->n_live - 1) % plan->n_live];
  return FTAR_OK;
}

ftar_status_t ftar_plan_partition_segment(const ftar_plan_t* plan, int partition, int k, size_t* begin,
                                          size_t* end, int* owner_replica) {
  if (!plan_ok(plan) || k < 0 || k >= plan->n_live || partition < 0 ||
      static_cast<size_t>(partition) >= plan->n_parts)
    return fail(FTAR_ERR_INVALID_ARG);
  const SegTable& seg = static_cast<size_t>(partition) + 1 == plan->n_parts ? plan->part_seg_last
                                                                             : plan->part_seg_full;
  const size_t base = static_cast<size_t>(partition) * plan->part_elems;
  if (begin) *begin = base + seg.begin[k];
  if (end) *end = base + seg.begin[k + 1];
  if (owner_replica) *owner_replica = plan->ring[(k + plan->n_live - 1) % plan->n_live];
  return FTAR_OK;
}

// Gathers the live buffers in ring order and decides between the vector and the
// element-wise kernels.  Vector kernels need every live pointer 16-byte aligned and
// every portion to start on a multiple of 8 elements.
static ftar_status_t ring_table(const ftar_plan_t* plan, void* const* bufs, PtrTable* tab, bool* vec) {
  const size_t es = elem_size(plan->dtype);
  bool v = true;
  for (int p = 0; p < plan->n_live; ++p) {
    void* b = bufs[plan->ring[p]];
    if (!b || !aligned(b, es)) return FTAR_ERR_INVALID_ARG;
    if (!aligned(b, 16)) v = false;
    tab->p[p] = b;
  }
  for (int k = 1; k < plan->n_live; ++k) {
    if (plan->part_seg_full.begin[k] % 8 != 0 && plan->part_seg_full.begin[k] != plan->part_seg_full.begin[plan->n_live])
      v = false;
    if (plan->part_seg_last.begin[k] % 8 != 0 && plan->part_seg_last.begin[k] != plan->part_seg_last.begin[plan->n_live])
      v = false;
  }
  if (plan->part_elems % 8 != 0) v = false;
  *vec = v;
  return FTAR_OK;
}

ftar_status_t ftar_reduce_step(const ftar_plan_t* plan, int step, void* const* bufs, float* acc,
                               void* stream) {
  if (!plan_ok(plan) || !bufs || plan->part_elems != 0) return fail(FTAR_ERR_INVALID_ARG);
  const int N = plan->n_live;
  if (step < 0 || step > N - 2) return fail(FTAR_ERR_BAD_STEP);
  PtrTable tab;
  std::memset(&tab, 0, sizeof(tab));
  bool vec = true;
  ftar_status_t s = ring_table(plan, bufs, &tab, &vec);
  if (s != FTAR_OK) return fail(s);
  RingMode mode;
  if (N == 2) mode = kRsOnly;
  else if (step == 0) mode = kRsFirst;
  else if (step == N - 2) mode = kRsLast;
  else mode = kRsMid;
  if (mode != kRsOnly) {
    if (!acc || !aligned(acc, 4)) return fail(FTAR_ERR_INVALID_ARG);
    if (!aligned(acc, 16)) vec = false;
  }
  hipError_t e = launch_ring_reduce(mode, tab, N, step, plan->seg, plan->dtype, vec, acc, plan->scale,
                                    plan->zero_pos, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? FTAR_OK : fail(FTAR_ERR_DEVICE);
}

ftar_status_t ftar_allgather_step(const ftar_plan_t* plan, int step, void* const* bufs,
                                  void* stream) {
  if (!plan_ok(plan) || !bufs || plan->part_elems != 0) return fail(FTAR_ERR_INVALID_ARG);
  const int N = plan->n_live;
  if (step < 0 || step > N - 2) return fail(FTAR_ERR_BAD_STEP);
  PtrTable tab;
  std::memset(&tab, 0, sizeof(tab));
  bool vec = true;
  ftar_status_t s = ring_table(plan, bufs, &tab, &vec);
  if (s != FTAR_OK) return fail(s);
  hipError_t e = launch_ring_allgather(tab, N, step, plan->seg, plan->dtype, vec,
                                       static_cast<hipStream_t>(stream));
  return e == hipSuccess ? FTAR_OK : fail(FTAR_ERR_DEVICE);
}

ftar_status_t ftar_allgather_all(const ftar_plan_t* plan, void* const* bufs, void* stream) {
  if (!plan_ok(plan) || !bufs || plan->part_elems != 0) return fail(FTAR_ERR_INVALID_ARG);
  const int N = plan->n_live;
  PtrTable tab;
  std::memset(&tab, 0, sizeof(tab));
  bool vec = true;
  ftar_status_t s = ring_table(plan, bufs, &tab, &vec);
  if (s != FTAR_OK) return fail(s);
  if (N < 2) return FTAR_OK;  // nothing to hand round
  hipError_t e = launch_ring_allgather_all(tab, N, plan->seg, plan->dtype, vec, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? FTAR_OK : fail(FTAR_ERR_DEVICE);
}

static ftar_status_t reduce_masked_common(const void* const* bufs, int n_replicas, uint64_t live_mask,
                                          uint64_t zero_mask, int contributors_only, size_t count,
                                          ftar_dtype_t dtype, ftar_dtype_t out_dtype, ftar_op_t op,
                                          void* out, void* stream) {
  if (!bufs || !out || count == 0 || (dtype != FTAR_F32 && dtype != FTAR_BF16) ||
      (out_dtype != FTAR_F32 && out_dtype != FTAR_BF16) || (op != FTAR_MEAN && op != FTAR_SUM))
    return fail(FTAR_ERR_INVALID_ARG);
  int ring[kMaxReplicas];
  int N = 0;
  ftar_status_t s = resolve_mask(n_replicas, live_mask, ring, &N);
  if (s != FTAR_OK) return fail(s);
  if ((zero_mask & ~live_mask) != 0) return fail(FTAR_ERR_BAD_MASK);
  const size_t es = elem_size(dtype);
  if (!aligned(out, elem_size(out_dtype))) return fail(FTAR_ERR_INVALID_ARG);
  bool vec = aligned(out, 16);
  PtrTable tab;
  std::memset(&tab, 0, sizeof(tab));
  int n_src = 0;
  for (int j = 0; j < N; ++j) {
    if ((zero_mask >> ring[j]) & 1ull) continue;  // takes part, contributes +0.0, is never read
    const void* b = bufs[ring[j]];
    if (!b || !aligned(b, es)) return fail(FTAR_ERR_INVALID_ARG);
    if (!aligned(b, 16)) vec = false;
    tab.p[n_src++] = const_cast<void*>(b);
  }
  const int divisor = contributors_only ? n_src : N;
  if (divisor <= 0) return fail(FTAR_ERR_NO_LIVE);
  const float scale = op == FTAR_SUM ? 1.0f : 1.0f / static_cast<float>(divisor);
  hipError_t e = launch_reduce_masked(tab, n_src, count, dtype, out_dtype, vec, out, scale, n_src != N, 0,
                                      static_cast<hipStream_t>(stream));
  return e == hipSuccess ? FTAR_OK : fail(FTAR_ERR_DEVICE);
}

ftar_status_t ftar_reduce_masked(const void* const* bufs, int n_replicas, uint64_t live_mask,
                                 size_t count, ftar_dtype_t dtype, void* out, void* stream) {
  return reduce_masked_common(bufs, n_replicas, live_mask, 0, 0, count, dtype, dtype, FTAR_MEAN, out,
                              stream);
}

ftar_status_t ftar_reduce_masked_zero(const void* const* bufs, int n_replicas, uint64_t live_mask,
                                      uint64_t zero_mask, int contributors_only, size_t count,
                                      ftar_dtype_t dtype, void* out, void* stream) {
  return reduce_masked_common(bufs, n_replicas, live_mask, zero_mask, contributors_only, count, dtype,
                              dtype, FTAR_MEAN, out, stream);
}

ftar_status_t ftar_reduce_masked_ex(const void* const* bufs, int n_replicas, uint64_t live_mask,
                                    uint64_t zero_mask, int contributors_only, size_t count,
                                    ftar_dtype_t in_dtype, ftar_dtype_t out_dtype, ftar_op_t op,
                                    void* out, void* stream) {
  return reduce_masked_common(bufs, n_replicas, live_mask, zero_mask, contributors_only, count,
                              in_dtype, out_dtype, op, out, stream);
}

ftar_status_t ftar_reduce_masked_bucketed(const void* const* bufs, int n_replicas,
                                          const uint64_t* masks, size_t n_buckets,
                                          size_t bucket_elems, size_t count, ftar_dtype_t dtype,
                                          void* out, void* stream) {
  if (!bufs || !out || !masks || count == 0 || bucket_elems == 0 ||
      (dtype != FTAR_F32 && dtype != FTAR_BF16))
    return fail(FTAR_ERR_INVALID_ARG);
  if (n_replicas < 1 || n_replicas > kMaxReplicas) return fail(FTAR_ERR_INVALID_ARG);
  if (n_buckets != count / bucket_elems + (count % bucket_elems ? 1 : 0))
    return fail(FTAR_ERR_INVALID_ARG);
  const size_t es = elem_size(dtype);
  if (!aligned(out, es)) return fail(FTAR_ERR_INVALID_ARG);
  bool vec = aligned(out, 16) && (bucket_elems % 8 == 0 || n_buckets == 1);
  uint64_t any_live = 0;
  for (size_t b = 0; b < n_buckets; ++b) {
    int ring[kMaxReplicas];
    int N = 0;
    ftar_status_t s = resolve_mask(n_replicas, masks[b], ring, &N);
    if (s != FTAR_OK) return fail(s);
    any_live |= masks[b];
  }
  PtrTable tab;
  std::memset(&tab, 0, sizeof(tab));
  for (int r = 0; r < n_replicas; ++r) {
    if (!((any_live >> r) & 1ull)) continue;  // never live in any bucket: never dereferenced
    const void* b = bufs[r];
    if (!b || !aligned(b, es)) return fail(FTAR_ERR_INVALID_ARG);
    if (!aligned(b, 16)) vec = false;
    tab.p[r] = const_cast<void*>(b);
  }
  ScaleTable scales;
  scales.s[0] = 0.0f;
  for (int n = 1; n <= kMaxReplicas; ++n) scales.s[n] = 1.0f / static_cast<float>(n);
  // Big buckets (half a GiB of traffic or more each) go through the one-shot kernel, one bucket
  // after the other: its loop is compiled for the bucket's own N and a long bucket is cut into
  // launches of about 1 GiB (8 x 512 Mi fp32 in 21 buckets: 5.47 -> 5.58 TB/s).  The kernel with the
  // per-tile bucket lookup is for many small buckets, where a launch per bucket would cost more.
  {
    int n_any = 0;
    for (int r = 0; r < n_replicas; ++r) n_any += static_cast<int>((any_live >> r) & 1ull);
    if (bucket_elems * es * static_cast<size_t>(n_any + 1) >= (static_cast<size_t>(512) << 20) &&
        (current_tuning().flags & 0x40) == 0) {
      const hipEvent_t t_start = t_time_start, t_stop = t_time_stop;  // a timed call brackets the series
      for (size_t b = 0; b < n_buckets; ++b) {
        const size_t first = b * bucket_elems;
        const size_t len = count - first < bucket_elems ? count - first : bucket_elems;
        int ring[kMaxReplicas];
        int N = 0;
        resolve_mask(n_replicas, masks[b], ring, &N);  // checked above
        PtrTable live;
        std::memset(&live, 0, sizeof(live));
        for (int j = 0; j < N; ++j) live.p[j] = static_cast<char*>(tab.p[ring[j]]) + first * es;
        t_time_start = b == 0 ? t_start : nullptr;
        t_time_stop = b + 1 == n_buckets ? t_stop : nullptr;
        hipError_t e = launch_reduce_masked(live, N, len, dtype, dtype, vec, static_cast<char*>(out) + first * es,
                                            scales.s[N], false, count, static_cast<hipStream_t>(stream));
        if (e != hipSuccess) return fail(FTAR_ERR_DEVICE);
      }
      return FTAR_OK;
    }
  }
  const size_t per = kMaxBucketsPerLaunch;
  const hipEvent_t t_start = t_time_start, t_stop = t_time_stop;  // a timed call brackets the whole series
  for (size_t b0 = 0; b0 < n_buckets; b0 += per) {
    const size_t nb = n_buckets - b0 < per ? n_buckets - b0 : per;
    BucketTable bt;
    std::memset(&bt, 0, sizeof(bt));
    for (size_t i = 0; i < nb; ++i) bt.mask[i] = masks[b0 + i];
    t_time_start = b0 == 0 ? t_start : nullptr;
    t_time_stop = b0 + nb >= n_buckets ? t_stop : nullptr;
    hipError_t e = launch_reduce_bucketed(tab, n_replicas, bt, static_cast<int>(nb), b0 * bucket_elems,
                                          bucket_elems, count, scales, dtype, vec, out,
                                          static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail(FTAR_ERR_DEVICE);
  }
  return FTAR_OK;
}

static ftar_status_t onepass_common(const ftar_plan_t* plan, void* const* bufs, bool owner_only, void* stream) {
  if (!plan_ok(plan) || !bufs || plan->part_elems != 0) return fail(FTAR_ERR_INVALID_ARG);
  const int N = plan->n_live;
  PtrTable tab;
  std::memset(&tab, 0, sizeof(tab));
  bool vec = true;
  ftar_status_t s = ring_table(plan, bufs, &tab, &vec);
  if (s != FTAR_OK) return fail(s);
  if (N < 2) return FTAR_OK;  // a ring of one exchanges nothing: the buffer stays as it is
  hipError_t e = launch_ring_onepass(tab, N, plan->seg, plan->dtype, vec, plan->scale, plan->zero_pos,
                                     owner_only, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? FTAR_OK : fail(FTAR_ERR_DEVICE);
}

ftar_status_t ftar_allreduce_onepass(const ftar_plan_t* plan, void* const* bufs, void* stream) {
  return onepass_common(plan, bufs, false, stream);
}

ftar_status_t ftar_reduce_scatter_all(const ftar_plan_t* plan, void* const* bufs, void* stream) {
  return onepass_common(plan, bufs, true, stream);
}

void* ftar_ctrl_create(void) {
  void* p = nullptr;
  if (hipHostMalloc(&p, sizeof(Ctrl), hipHostMallocCoherent | hipHostMallocMapped) != hipSuccess || !p) {
    fail(FTAR_ERR_DEVICE);
    return nullptr;
  }
  std::memset(p, 0, sizeof(Ctrl));
  Ctrl* c = static_cast<Ctrl*>(p);
  c->cur_epoch = 1;
  for (int i = 0; i < kCtrlCalls; ++i) c->call[i].ticket = -1;
  void* mirror = nullptr;
  if (hipMalloc(&mirror, sizeof(DevCtrl)) != hipSuccess || !mirror) {
    (void)hipHostFree(p);
    fail(FTAR_ERR_DEVICE);
    return nullptr;
  }
  c->dev = static_cast<DevCtrl*>(mirror);
  // set-up is also where the static scratch of ftar_ring_persistent_static is located on this
  // device (that entry point looks it up itself if no control block was ever made here)
  DevCtrl* sm = nullptr;
  float* sa = nullptr;
  (void)static_scratch(&sm, &sa);
  return p;
}

void ftar_ctrl_destroy(void* ctrl) {
  if (!ctrl) return;
  (void)hipFree(static_cast<Ctrl*>(ctrl)->dev);
  (void)hipHostFree(ctrl);
}

// Rows of chunks per step for one partition shape (the gate units of a step with
// FTAR_PERSIST_CHUNKS): the largest number of chunks any portion has.  *ok = false if the shape
// is not what the kernel's row tables assume (all rows but the last two hold N full chunks).
static unsigned chunk_rows(const SegTable& seg, int N, size_t chunk, bool* ok) {
  unsigned long long c_min = ~0ull, c_max = 0;
  for (int k = 0; k < N; ++k) {
    const unsigned long long len = seg.begin[k + 1] - seg.begin[k];
    const unsigned long long c = (len + chunk - 1) / chunk;
    c_min = c < c_min ? c : c_min;
    c_max = c > c_max ? c : c_max;
    // every chunk of a portion but its last must be whole
    if (len > 0 && seg.begin[k] % chunk != 0 && k > 0) *ok = false;
  }
  const unsigned long long uni = c_min > 0 ? c_min - 1 : 0;
  if (c_max - uni > 2 || c_max > 0x7fffffffull) *ok = false;
  return static_cast<unsigned>(c_max);
}

// Gate units of a call: slots, or rows of chunks summed over all slots.
static bool gate_units(const ftar_plan_t* plan, unsigned flags, unsigned* rows_full, unsigned* rows_last,
                       unsigned long long* units) {
  const unsigned long long steps = static_cast<unsigned long long>(2 * plan->n_live - 2);
  if ((flags & FTAR_PERSIST_CHUNKS) == 0) {
    *rows_full = *rows_last = 1;
    *units = plan->n_parts * steps;
    return true;
  }
  bool ok = true;
  *rows_full = chunk_rows(plan->part_seg_full, plan->n_live, plan->chunk_elems, &ok);
  *rows_last = chunk_rows(plan->part_seg_last, plan->n_live, plan->chunk_elems, &ok);
  *units = steps * ((plan->n_parts - 1) * static_cast<unsigned long long>(*rows_full) + *rows_last);
  return ok && *units <= 0x7fffffffull;
}

int ftar_plan_n_gate_units(const ftar_plan_t* plan, unsigned flags) {
  if (!plan_ok(plan)) return 0;
  unsigned rf = 0, rl = 0;
  unsigned long long units = 0;
  if (!gate_units(plan, flags, &rf, &rl, &units)) return 0;
  return static_cast<int>(units);
}

static bool call_over(const CallRec& r) {
  return r.ticket < 0 || r.n_blocks == 0 || __atomic_load_n(&r.ended, __ATOMIC_ACQUIRE) != 0;
}

// own_scratch: the partial sums and the mirror of the control block live in the library's static
// device array instead of caller-provided / set-up-allocated memory (acc is then ignored).
static ftar_status_t ring_persistent_common(const ftar_plan_t* plan, void* const* bufs, float* acc, void* ctrl,
                                            int n_blocks, unsigned timeout_us, unsigned flags, bool own_scratch,
                                            void* stream) {
  if (!plan_ok(plan) || !bufs || !ctrl || timeout_us == 0 || n_blocks < 0 || n_blocks > kMaxPersistentBlocks ||
      (flags & ~(FTAR_PERSIST_PUBLISH | FTAR_PERSIST_ALIGN | FTAR_PERSIST_CHUNKS)) != 0)
    return fail(FTAR_ERR_INVALID_ARG);
  const int N = plan->n_live;
  Ctrl* c = static_cast<Ctrl*>(ctrl);
  DevCtrl* mirror = c->dev;
  if (own_scratch) {
    static_assert(kStaticAccElems == FTAR_STATIC_ACC_ELEMS, "the header states the limit");
    if (N >= 3 && (plan->part_elems ? plan->part_elems : plan->count) > kStaticAccElems)
      return fail(FTAR_ERR_TOO_LARGE);  // rings of one or two keep no partial sums
    if (static_scratch(&mirror, &acc) != hipSuccess) return fail(FTAR_ERR_DEVICE);
  }
  if (!mirror) return fail(FTAR_ERR_INVALID_ARG);
  PtrTable tab;
  std::memset(&tab, 0, sizeof(tab));
  bool vec = true;
  ftar_status_t s = ring_table(plan, bufs, &tab, &vec);
  if (s != FTAR_OK) return fail(s);
  if (N >= 3) {
    if (!acc || !aligned(acc, 4)) return fail(FTAR_ERR_INVALID_ARG);
    if (!aligned(acc, 16)) vec = false;
  }
  PartGeom geom;
  unsigned long long units = 0;
  if (!gate_units(plan, flags, &geom.rows_full, &geom.rows_last, &units)) return fail(FTAR_ERR_INVALID_ARG);
  // default: one worker per compute unit; two when the slots are short (partitioned)
  unsigned blocks = n_blocks > 0 ? static_cast<unsigned>(n_blocks)
                                 : static_cast<unsigned>(device_cu_count()) * (plan->n_parts > 1 ? 2u : 1u);
  if (blocks > static_cast<unsigned>(kMaxPersistentBlocks)) blocks = kMaxPersistentBlocks;
  void* dev = nullptr;
  if (N >= 2 && (hipHostGetDevicePointer(&dev, ctrl, 0) != hipSuccess || !dev)) return fail(FTAR_ERR_INVALID_ARG);
  // the call's record: free only if the call that used it last is over (at most kCtrlCalls in flight)
  const long long ticket = c->next_ticket;
  CallRec* rec = &c->call[ticket % kCtrlCalls];
  if (!call_over(*rec)) return fail(FTAR_ERR_INVALID_ARG);
  // everything has been checked: from here on the control block changes
  rec->gate = 0;
  rec->status = 0;
  rec->blocked_unit = 0;
  rec->progress = 0;
  rec->ended = 0;
  rec->epoch = c->cur_epoch;
  rec->n_blocks = N >= 2 ? blocks : 0;
  rec->n_units = N >= 2 ? static_cast<unsigned>(units) : 0;
  rec->ticket = ticket;
  c->next_ticket = ticket + 1;
  std::atomic_thread_fence(std::memory_order_seq_cst);
  if (N < 2) return FTAR_OK;  // a ring of one has no steps: nothing to launch
  geom.n_parts = static_cast<unsigned>(plan->n_parts);
  geom.part_elems = plan->part_elems;
  geom.seg_full = plan->part_seg_full;
  geom.seg_last = plan->part_seg_last;
  geom.chunk_elems = (flags & FTAR_PERSIST_CHUNKS) ? plan->chunk_elems : 0;
  // long slots: keep the workers in step (measured: pays from 128 Mi elements per partition on)
  if ((plan->part_elems ? plan->part_elems : plan->count) * 4 > (static_cast<size_t>(256) << 20))
    flags |= FTAR_PERSIST_ALIGN;
  Ctrl* ctrl_dev = static_cast<Ctrl*>(dev);
  CallRec* rec_dev = &ctrl_dev->call[ticket % kCtrlCalls];
  hipError_t e = launch_ring_persistent(tab, N, geom, plan->dtype, vec, acc, plan->scale, ctrl_dev, rec_dev,
                                        rec->epoch, mirror, blocks,
                                        static_cast<unsigned long long>(timeout_us) * 100ull, flags,
                                        plan->zero_pos, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) {
    rec->n_blocks = 0;  // nothing runs: the record reads as a call that is over, with nothing done
    rec->status = kRecLaunchFailed;
    return fail(FTAR_ERR_DEVICE);
  }
  return FTAR_OK;
}

ftar_status_t ftar_ring_persistent(const ftar_plan_t* plan, void* const* bufs, float* acc, void* ctrl,
                                   int n_blocks, unsigned timeout_us, unsigned flags, void* stream) {
  return ring_persistent_common(plan, bufs, acc, ctrl, n_blocks, timeout_us, flags, false, stream);
}

ftar_status_t ftar_ring_persistent_static(const ftar_plan_t* plan, void* const* bufs, void* ctrl, int n_blocks,
                                          unsigned timeout_us, unsigned flags, void* stream) {
  return ring_persistent_common(plan, bufs, nullptr, ctrl, n_blocks, timeout_us, flags, true, stream);
}

int ftar_ctrl_last_ticket(const void* ctrl) {
  if (!ctrl) return -1;
  return static_cast<int>(static_cast<const Ctrl*>(ctrl)->next_ticket - 1);
}

// The record of a ticket, or null if the ticket was never issued or its record has been reused.
static CallRec* record_of(void* ctrl, int ticket) {
  if (!ctrl || ticket < 0) return nullptr;
  Ctrl* c = static_cast<Ctrl*>(ctrl);
  CallRec* r = &c->call[ticket % kCtrlCalls];
  return r->ticket == ticket ? r : nullptr;
}

void ftar_ctrl_release_call(void* ctrl, int ticket, int n_units) {
  CallRec* r = record_of(ctrl, ticket);
  if (!r || n_units < 0) return;
  // one plain store: the cancel lives in a word of its own, so a release can never undo it
  __atomic_store_n(&r->gate, static_cast<unsigned long long>(n_units), __ATOMIC_RELEASE);
}

void ftar_ctrl_release(void* ctrl, int n_units) { ftar_ctrl_release_call(ctrl, ftar_ctrl_last_ticket(ctrl), n_units); }

void ftar_ctrl_cancel(void* ctrl) {
  if (!ctrl) return;
  Ctrl* c = static_cast<Ctrl*>(ctrl);
  // everything enqueued so far belongs to epochs <= cur_epoch: kill them, open the next epoch
  const unsigned long long e = __atomic_fetch_add(&c->cur_epoch, 1ull, __ATOMIC_ACQ_REL);
  unsigned long long seen = __atomic_load_n(&c->dead_epoch, __ATOMIC_RELAXED);
  while (seen < e && !__atomic_compare_exchange_n(&c->dead_epoch, &seen, e, false, __ATOMIC_RELEASE, __ATOMIC_RELAXED)) {
  }
}

int ftar_ctrl_progress_call(const void* ctrl, int ticket) {
  const CallRec* r = record_of(const_cast<void*>(ctrl), ticket);
  if (!r) return 0;
  if (r->n_blocks == 0) return static_cast<int>(r->n_units);
  return static_cast<int>(__atomic_load_n(&r->progress, __ATOMIC_ACQUIRE));
}

int ftar_ctrl_progress(const void* ctrl) { return ftar_ctrl_progress_call(ctrl, ftar_ctrl_last_ticket(ctrl)); }

ftar_status_t ftar_ctrl_result_call(const void* ctrl, int ticket, int* units_done) {
  const CallRec* r = record_of(const_cast<void*>(ctrl), ticket);
  if (!r) return fail(FTAR_ERR_INVALID_ARG);
  const int done = ftar_ctrl_progress_call(ctrl, ticket);
  if (units_done) *units_done = done;
  const unsigned long long status = __atomic_load_n(&r->status, __ATOMIC_ACQUIRE);
  if (status == kRecLaunchFailed) return fail(FTAR_ERR_DEVICE);
  if (status == 3) return fail(FTAR_ERR_SKIPPED);  // queued behind a cancel or a timeout: nothing ran
  if (status != 0) return fail(FTAR_ERR_STALE_PLAN);  // timed out or cancelled: re-plan and restart
  if (r->n_blocks != 0 && __atomic_load_n(&r->ended, __ATOMIC_ACQUIRE) == 0)
    return fail(FTAR_ERR_INVALID_ARG);  // still running
  if (done != static_cast<int>(r->n_units)) return fail(FTAR_ERR_INVALID_ARG);
  return FTAR_OK;
}

ftar_status_t ftar_ctrl_result(const void* ctrl, int* units_done) {
  return ftar_ctrl_result_call(ctrl, ftar_ctrl_last_ticket(ctrl), units_done);
}

ftar_status_t ftar_last_error(void) { return t_last_error; }

int ftar_status_is_retryable(ftar_status_t s) { return (s == FTAR_ERR_STALE_PLAN || s == FTAR_ERR_SKIPPED) ? 1 : 0; }

const char* ftar_status_str(ftar_status_t s) {
  switch (s) {
    case FTAR_OK: return "ok";
    case FTAR_ERR_INVALID_ARG: return "invalid argument";
    case FTAR_ERR_NO_LIVE: return "live mask selects no replica";
    case FTAR_ERR_BAD_MASK: return "live mask has a bit at or above n_replicas";
    case FTAR_ERR_BAD_STEP: return "step outside [0, n_live-2]";
    case FTAR_ERR_TOO_LARGE: return "partition (or unpartitioned buffer) exceeds the library's static scratch";
    case FTAR_ERR_STALE_PLAN: return "plan is stale: re-plan over the new group and restart";
    case FTAR_ERR_SKIPPED: return "skipped: queued behind a call that was cancelled or timed out; nothing ran";
    case FTAR_ERR_DEVICE: return "HIP runtime error";
  }
  return "unknown status";
}

// ---- measurement hooks (declared in include/ftar_measure.h) ----
void ftar_time_next_launch(void* start_event, void* stop_event) {
  set_timing_events(static_cast<hipEvent_t>(start_event), static_cast<hipEvent_t>(stop_event));
}

void ftar_set_tuning(int blocks_per_cu, int flags) {
  g_blocks_per_cu = blocks_per_cu < 0 ? 0 : blocks_per_cu;
  g_flags = flags;
}

}  // extern "C"
