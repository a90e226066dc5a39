// The whole ring all-reduce as one CPU-gated persistent kernel, and its launcher.

#include <mutex>

#include "ftar_device.h"

// Scratch memory of ftar_ring_persistent_static, for callers that cannot allocate: the mirror of
// the control block (cleared on the stream before every launch) followed by the partial sums of
// one partition.  One copy per GPU, held until the process ends; all calls on a GPU share it.
// In host code this name is only a handle for hipGetSymbolAddress: the device address it stands
// for is looked up once per device (static_scratch below) and used from then on.
namespace ftar {
namespace {
struct StaticScratch {
  DevCtrl mirror;
  alignas(256) float acc[kStaticAccElems];
};
}  // namespace
}  // namespace ftar
static __device__ __align__(256) unsigned char scratch[sizeof(ftar::StaticScratch)];

namespace ftar {
namespace {

// ---- the whole ring as one CPU-gated persistent kernel ----------------------------
// The data is handled in partitions (paper section 4.2: the message is split into partitions of
// at most S x C x N bytes; each partition runs one full round of the ring, then the next one
// starts).  A "slot" is one step of one partition; slots run in order, partition-major.  `acc`
// holds one partition and is reused by the next, so with partitions of a few tens of MiB the
// in-flight partial sums never leave the caches.
//
// What the CPU releases and observes is the gate unit.  By default a unit is a slot.  With
// FTAR_PERSIST_CHUNKS a unit is one ROW of chunks of a slot - chunk c of every portion, i.e. the c-th
// chunk of every rank's work in that step (section 4.2: each step is pipelined over the chunks of a
// portion).  The tiles of a slot are then walked row by row, a worker looks at the gate whenever
// its next tile lies in a later row, and it publishes its progress whenever it moves on to one.
//
// Element i of acc (and of every replica buffer) is only ever touched by the block that owns
// the tile holding i, and the tile -> block assignment is the same in every slot of partitions
// of the same length, so consecutive slots need no synchronisation between blocks: a block-wide
// barrier with workgroup-scope release/acquire between two slots is enough (all waves of a
// block share one CU and its L1).  That also lets the AllGather steps copy 16 bytes per lane
// although the ReduceScatter steps hand each lane 8 bytes of bf16.
// The one exception is a shorter last partition: its portions, and with them its tiles, fall
// elsewhere in acc, so a block may overwrite partial sums that another block has not consumed
// yet.  Before its first slot every worker therefore waits until all workers have finished the
// last ReduceScatter step of the partition before (the last reader of acc): the acc handover.
//
// What the blocks do wait for is the CPU.  The grid is n workers plus one relay block, and the
// relay is the only one that talks to the CPU: it copies the call's gate word from host-pinned
// memory into a mirror in device memory whenever it changes (every worker polling host memory
// over PCIe costs tens of microseconds per step), it watches the two dead-epoch words (a cancel
// by the CPU, a timeout in an earlier call of the same epoch), and it publishes the minimum over
// the workers' progress words back to the CPU.  Before unit u a worker waits on the mirror until
// the unit is released, the call is cancelled, somebody else gave up, or its own wait has lasted
// longer than the timeout (wall clock, 100 MHz, and a spin bound should the clock stand still):
// then it records why and leaves.  A worker that has seen r units released does not look again
// before unit r.  The relay leaves when every worker has left, so the kernel ends no matter what
// the CPU does.  A call whose epoch is already dead when its relay first looks is "skipped": its
// workers leave at their first wait, before anything has been read or written.
__device__ __forceinline__ unsigned long long sys_load(const unsigned long long* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
}
template <typename V>
__device__ __forceinline__ void sys_store(V* p, V v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
}
template <typename V>
__device__ __forceinline__ V dev_load(const V* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <typename V>
__device__ __forceinline__ void dev_store(V* p, V v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Vectors per lane and tile.  8 suits the whole chip; a handful of workgroups is bound by latency,
// not by bandwidth, and gains 40 % from four times as many loads in flight (2 workers on
// 16 x 64 Mi bf16: 106 -> 146 GB/s).
constexpr int kPersistentUnroll = 8;
constexpr int kPersistentUnrollFew = 32;

constexpr unsigned kVerdictTimeout = 1, kVerdictCancel = 2, kVerdictSkipped = 3;

__global__ void k_clear_mirror(DevCtrl* m) {
  unsigned int* w = reinterpret_cast<unsigned int*>(m);
  for (unsigned i = threadIdx.x; i < sizeof(DevCtrl) / 4; i += blockDim.x) w[i] = 0;
}

// The relay block (all its lanes take part in the scan of the workers' progress words).
// leaders: FTAR_PERSIST_PUBLISH - the workers report a unit without writing the L2
// back themselves; the relay keeps one minimum per XCD, the XCD's leader writes its L2 back once for
// everybody (xcd_done), and the progress the CPU sees is the minimum of what has been written back.
__device__ __forceinline__ void relay_loop(Ctrl* ctrl, CallRec* rec, unsigned long long epoch, DevCtrl* mirror,
                                           unsigned n_workers, unsigned long long max_spins, unsigned flags,
                                           bool leaders) {
  __shared__ unsigned s_min;
  __shared__ unsigned s_min_x[kMaxXcds];
  __shared__ int s_last_round;
  __shared__ int s_registered;
  unsigned long long last_gate = 0;
  unsigned last_min = 0, last_pub = 0;
  bool first = true;
  bool registered = !leaders;  // every worker has said which XCD it runs on (it does so before its first wait)
  // max_spins bounds one wait of one worker; every worker leaves after at most n_units such waits
  // plus its work, so the factor below is never reached: it only guarantees termination.
  for (unsigned long long spin = 0; spin < max_spins * 65536ull; ++spin) {
    if (threadIdx.x == 0) {
      // decide first whether this is the last round, then scan: a worker writes its progress word
      // before it counts itself out, so the scan of the last round sees every final value
      s_last_round = __hip_atomic_load(&mirror->exited, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT) >= n_workers;
      s_min = 0xffffffffu;
      if (!registered) {
        unsigned sum = 0;
        for (int x = 0; x < kMaxXcds; ++x) sum += dev_load(&mirror->xcd_workers[x]);
        registered = sum >= n_workers;
      }
      s_registered = registered;
      const unsigned long long d0 = sys_load(&ctrl->dead_epoch), d1 = sys_load(&ctrl->gpu_dead_epoch);
      const bool dead = (d0 > d1 ? d0 : d1) >= epoch;
      if (dead && first) {
        dev_store(&mirror->verdict, kVerdictSkipped);  // before any unit is passed on: nothing will run
      } else if (registered || dead) {  // no unit is passed on before the per-XCD bookkeeping is complete
        unsigned long long g = sys_load(&rec->gate) & 0xffffffffull;
        if (dead) g |= kGateCancel;
        if (g != last_gate) {
          dev_store(&mirror->gate, g);
          last_gate = g;
        }
      }
      first = false;
    }
    if (threadIdx.x < static_cast<unsigned>(kMaxXcds)) s_min_x[threadIdx.x] = 0xffffffffu;
    __syncthreads();
    const bool per_xcd = leaders && s_registered != 0;
    unsigned lo = 0xffffffffu;
    for (unsigned b = threadIdx.x; b < n_workers; b += kThreads) {
      const unsigned v = dev_load(&mirror->worker_unit[b]);
      lo = v < lo ? v : lo;
      if (per_xcd) atomicMin(&s_min_x[dev_load(&mirror->worker_xcd[b]) % kMaxXcds], v);  // written once, before the worker's first wait
    }
    atomicMin(&s_min, lo);
    __syncthreads();
    const int last_round = s_last_round;
    if (threadIdx.x == 0) {
      const unsigned m = s_min;
      unsigned pub = m;  // what the CPU may see
      if (leaders) {
        pub = per_xcd ? 0xffffffffu : 0u;
        if (per_xcd) {
          for (int x = 0; x < kMaxXcds; ++x) {
            if (s_min_x[x] == 0xffffffffu) continue;  // nobody runs there
            dev_store(&mirror->xcd_min[x], s_min_x[x]);
            const unsigned d = dev_load(&mirror->xcd_done[x]);
            pub = d < pub ? d : pub;
          }
          if (pub == 0xffffffffu) pub = 0u;
        }
      }
      if (m != last_min) {
        if (!leaders && (flags & FTAR_PERSIST_PUBLISH)) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
        dev_store(&mirror->min_unit, m);
        last_min = m;
      }
      if (pub != last_pub) {
        sys_store(&rec->progress, static_cast<unsigned long long>(pub));
        last_pub = pub;
      }
      if (last_round) sys_store(&rec->ended, 1ull);  // after the final progress: the call is over
    }
    if (last_round) return;  // the same for every lane
    __builtin_amdgcn_s_sleep(1);
    __syncthreads();  // everybody has read s_last_round before lane 0 writes it again
  }
}

// s_waitcnt vmcnt(0) alone (gfx9 encoding: vmcnt in bits 3:0 and 15:14, expcnt 6:4 and lgkmcnt 11:8 left
// at their maxima): all of the wave's loads have returned and its stores have been taken by the L2.
// A workgroup-scope release does not include it when the workgroup's waves share one compute unit.
constexpr int kWaitVmcnt0 = 0x0F70;

// The XCD this wave runs on (XCC_ID, bits 3:0 of hardware register 20 on gfx942 / gfx950).
__device__ __forceinline__ unsigned xcd_of_this_wave() {
  return __builtin_amdgcn_s_getreg((3 << 11) | (0 << 6) | 20) & 0xfu;
}

// One lane of an XCD's leader: when every worker of the XCD has finished more units than have been
// written back, write the XCD's L2 back (a release at agent scope does) and say so.  A write-back
// serves the whole L2, whoever wrote the lines; 32 workers per XCD each doing their own cost 11 us
// per row against nothing for one (a bare kernel with the same mix of streams).
__device__ __forceinline__ void leader_duty(DevCtrl* mirror, unsigned xcd, unsigned* done) {
  const unsigned v = dev_load(&mirror->xcd_min[xcd]);
  if (v > *done) {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
    dev_store(&mirror->xcd_done[xcd], v);
    *done = v;
  }
}

// A worker counts itself out (one lane).  Its last progress word and verdict must be there before the
// count: waiting for this wave's own stores does that.  A release at agent scope would also write the
// XCD's L2 back, once per worker - 32 write-backs per XCD that the L2 serves one after the other
// (about 11 us in all) for data that the end of the kernel writes back anyway.
__device__ __forceinline__ void count_out(DevCtrl* mirror) {
  __builtin_amdgcn_s_waitcnt(kWaitVmcnt0);
  __hip_atomic_fetch_add(&mirror->exited, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// What a worker needs to wait and to leave.
struct WaitCtx {
  Ctrl* ctrl;
  CallRec* rec;
  DevCtrl* mirror;
  unsigned long long epoch, timeout_ticks, max_spins;
  unsigned long long* s_word;  // LDS: what lane 0 saw
  bool leader;                 // this worker writes its XCD's L2 back for everybody (see leader_duty), also while it waits
  unsigned xcd;
  unsigned* xcd_done;
};

// Records the verdict and counts the worker out (lane 0 only).
__device__ __forceinline__ void leave(const WaitCtx& w, unsigned verdict, unsigned unit) {
  dev_store(&w.mirror->verdict, verdict);
  if (verdict == kVerdictTimeout) sys_store(&w.ctrl->gpu_dead_epoch, w.epoch);  // calls queued behind this one are skipped
  sys_store(&w.rec->blocked_unit, static_cast<unsigned long long>(unit));
  sys_store(&w.rec->status, static_cast<unsigned long long>(verdict));
  count_out(w.mirror);
}

// Block-wide, bounded wait until gate unit `unit` is released.  Returns true to go on (*released is
// then the number of units known to be released); false: the block leaves (already counted out).
__device__ __forceinline__ bool wait_released(const WaitCtx& w, unsigned unit, unsigned* released) {
  if (threadIdx.x == 0) {
    unsigned long long seen = static_cast<unsigned long long>(kVerdictTimeout) << 32;  // unless the loop says otherwise
    const long long t0 = wall_clock64();
    for (unsigned long long spin = 0; spin < w.max_spins; ++spin) {
      const unsigned v = dev_load(&w.mirror->verdict);
      if (v != 0) { seen = static_cast<unsigned long long>(v) << 32; break; }
      const unsigned long long g = dev_load(&w.mirror->gate);
      if ((g & kGateCancel) != 0) { seen = static_cast<unsigned long long>(kVerdictCancel) << 32; break; }
      if ((g & 0xffffffffull) > unit) { seen = g & 0xffffffffull; break; }
      if (static_cast<unsigned long long>(wall_clock64() - t0) > w.timeout_ticks) break;
      if (w.leader) leader_duty(w.mirror, w.xcd, w.xcd_done);  // the CPU may be waiting for exactly this report
      __builtin_amdgcn_s_sleep(4);
    }
    *w.s_word = seen;
  }
  __syncthreads();
  const unsigned long long seen = *w.s_word;
  __syncthreads();  // everybody has read the word before lane 0 can write it again
  const unsigned verdict = static_cast<unsigned>(seen >> 32);
  if (verdict != 0) {  // the same for every lane of the block: all leave together
    if (threadIdx.x == 0) leave(w, verdict, unit);
    return false;
  }
  *released = static_cast<unsigned>(seen);
  return true;
}

// Block-wide, bounded wait until every worker has finished `units` gate units (the acc handover).
__device__ __forceinline__ bool wait_all_done(const WaitCtx& w, unsigned units, unsigned unit_here) {
  if (threadIdx.x == 0) {
    unsigned verdict = kVerdictTimeout;
    const long long t0 = wall_clock64();
    for (unsigned long long spin = 0; spin < w.max_spins; ++spin) {
      if (dev_load(&w.mirror->min_unit) >= units) { verdict = 0; break; }
      if ((dev_load(&w.mirror->gate) & kGateCancel) != 0) { verdict = kVerdictCancel; break; }
      const unsigned v = dev_load(&w.mirror->verdict);
      if (v != 0) { verdict = v; break; }
      if (static_cast<unsigned long long>(wall_clock64() - t0) > w.timeout_ticks) break;
      if (w.leader) leader_duty(w.mirror, w.xcd, w.xcd_done);
      __builtin_amdgcn_s_sleep(4);
    }
    *w.s_word = verdict;
  }
  __syncthreads();
  const unsigned verdict = static_cast<unsigned>(*w.s_word);
  __syncthreads();
  if (verdict != 0) {
    if (threadIdx.x == 0) leave(w, verdict, unit_here);
    return false;
  }
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
  return true;
}

// Soft barrier inside a long step, a performance hint only: the workers of one launch never wait
// for each other, and over a gigabyte of traffic they drift apart, the window of addresses in use
// widens and the DRAM sees less locality (the step kernels avoid that by going out as several
// launches).  Every worker counts itself in at its n-th boundary and waits, bounded, until all
// have; nobody depends on it, and a worker that has left only costs the others the bound.
__device__ __forceinline__ void soft_align(DevCtrl* mirror, unsigned n_workers, unsigned nth) {
  if (threadIdx.x == 0) {
    __hip_atomic_fetch_add(&mirror->align_count, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const unsigned target = nth * n_workers;
    for (int spin = 0; spin < 2000; ++spin) {
      if (static_cast<int>(dev_load(&mirror->align_count) - target) >= 0) break;
      if (dev_load(&mirror->verdict) != 0) break;
      __builtin_amdgcn_s_sleep(2);
    }
  }
  __syncthreads();
}

// ---- rows of chunks ------------------------------------------------------------------
// Tile order of one slot when the gate unit is a row of chunks: row after row, inside a row
// portion after portion, inside a chunk tile after tile (a tile never crosses a chunk's end).
// Portions are whole chunks and differ by at most one chunk, and only the very last chunk of the
// data can be short: all rows but the last two hold N full chunks and are located by division;
// the last (at most two) rows are listed, entry e = (row - uniform_rows) * N + portion.
struct ChunkTab {
  unsigned long long beg[2 * kMaxReplicas], end[2 * kMaxReplicas], tile0[2 * kMaxReplicas + 1];
  unsigned long long uniform_tiles, total_tiles, chunk;
  unsigned rows, uniform_rows, tiles_per_chunk;
};

// One thread fills the table of one partition shape from its portion boundaries.
__device__ void build_chunk_tab(ChunkTab* t, const unsigned long long* seg, int N, unsigned long long chunk,
                                unsigned long long tile_elems) {
  unsigned long long c_min = ~0ull, c_max = 0;
  for (int k = 0; k < N; ++k) {
    const unsigned long long len = seg[k + 1] - seg[k];
    const unsigned long long c = (len + chunk - 1) / chunk;
    c_min = c < c_min ? c : c_min;
    c_max = c > c_max ? c : c_max;
  }
  unsigned long long uni = c_min > 0 ? c_min - 1 : 0;
  if (c_max - uni > 2) uni = c_max - 2;  // cannot happen with portions balanced to one chunk (the host checks)
  t->chunk = chunk;
  t->rows = static_cast<unsigned>(c_max);
  t->uniform_rows = static_cast<unsigned>(uni);
  t->tiles_per_chunk = static_cast<unsigned>((chunk + tile_elems - 1) / tile_elems);
  t->uniform_tiles = uni * static_cast<unsigned long long>(N) * t->tiles_per_chunk;
  unsigned e = 0;
  t->tile0[0] = 0;
  for (unsigned long long c = uni; c < c_max; ++c) {
    for (int k = 0; k < N; ++k, ++e) {
      unsigned long long b = seg[k] + c * chunk;
      if (b > seg[k + 1]) b = seg[k + 1];
      unsigned long long en = b + chunk;
      if (en > seg[k + 1]) en = seg[k + 1];
      t->beg[e] = b;
      t->end[e] = en;
      t->tile0[e + 1] = t->tile0[e] + (en - b + tile_elems - 1) / tile_elems;
    }
  }
  for (unsigned x = e; x < 2 * kMaxReplicas; ++x) {
    t->beg[x] = t->end[x] = 0;
    t->tile0[x + 1] = t->tile0[e];
  }
  t->total_tiles = t->uniform_tiles + t->tile0[e];
}

struct ChunkTile {
  int k;
  unsigned row;
  size_t begin, rem;  // rem: elements from `begin` to the end of the chunk (clipped to the portion)
};

template <size_t kTileElems>
__device__ __forceinline__ ChunkTile chunk_tile_of(const ChunkTab* t, const unsigned long long* seg, int N, size_t g,
                                                   unsigned& e) {
  const size_t uniform_tiles = uniform_u64(t->uniform_tiles);
  const unsigned T = __builtin_amdgcn_readfirstlane(t->tiles_per_chunk);
  const size_t chunk = uniform_u64(t->chunk);
  if (g < uniform_tiles) {
    const size_t per_row = static_cast<size_t>(N) * T;
    const size_t row = g / per_row;
    const unsigned r = static_cast<unsigned>(g - row * per_row);
    const unsigned k = r / T, tt = r - k * T;
    const size_t begin = uniform_u64(seg[k]) + row * chunk + static_cast<size_t>(tt) * kTileElems;
    return ChunkTile{static_cast<int>(k), static_cast<unsigned>(row), begin, chunk - static_cast<size_t>(tt) * kTileElems};
  }
  const size_t gg = g - uniform_tiles;
  while (gg >= uniform_u64(t->tile0[e + 1])) ++e;  // g < total_tiles: ends inside the table
  const size_t begin = uniform_u64(t->beg[e]) + (gg - uniform_u64(t->tile0[e])) * kTileElems;
  const unsigned urows = __builtin_amdgcn_readfirstlane(t->uniform_rows);
  return ChunkTile{static_cast<int>(e % static_cast<unsigned>(N)), urows + e / static_cast<unsigned>(N), begin,
                   uniform_u64(t->end[e]) - begin};
}

// One tile of one ReduceScatter step (MODE) or of an AllGather step (MODE < 0) at portion k.
template <typename T, int VEC, int U, int POL>
__device__ __forceinline__ void ring_one_tile(T* const* s_tab, int N, int step, int k, size_t begin, size_t rem,
                                              float* acc, float scale, size_t buf_off, unsigned long long zpos) {
  float* a = acc + begin;
  const size_t b0 = buf_off + begin;
  if (step < N - 1) {
    if (N == 2) {
      const int p1 = (k + 1) % N;
      T* src[2] = {uniform_ptr(s_tab[k]) + b0, uniform_ptr(s_tab[p1]) + b0};
      const unsigned long long zm = ((zpos >> k) & 1ull) | (((zpos >> p1) & 1ull) << 1);
      sum_block_tile<T, VEC, 2, false, false, U, POL>(src, nullptr, nullptr, src[1], scale, rem, zm);
    } else if (step == 0) {
      const int p1 = (k + 1) % N;
      T* src[2] = {uniform_ptr(s_tab[k]) + b0, uniform_ptr(s_tab[p1]) + b0};
      const unsigned long long zm = ((zpos >> k) & 1ull) | (((zpos >> p1) & 1ull) << 1);
      sum_block_tile<T, VEC, 2, false, true, U, POL>(src, nullptr, a, nullptr, scale, rem, zm);
    } else if (step == N - 2) {
      const int p = (k + N - 1) % N;
      T* src[1] = {uniform_ptr(s_tab[p]) + b0};
      sum_block_tile<T, VEC, 1, true, false, U, POL>(src, a, nullptr, src[0], scale, rem, (zpos >> p) & 1ull);
    } else {
      const int p = (k + step + 1) % N;
      T* src[1] = {uniform_ptr(s_tab[p]) + b0};
      sum_block_tile<T, VEC, 1, true, true, U, POL>(src, a, a, nullptr, scale, rem, (zpos >> p) & 1ull);
    }
  } else {
    // AllGather: the same elements, widest copy (a lane may move other elements than it summed:
    // the barrier before the first AllGather step covers that)
    constexpr int CV = VEC == 1 ? 1 : 16 / static_cast<int>(sizeof(T));
    typedef typename Raw<T, CV>::type R;
    typedef typename Raw<T, 1>::type R1;
    constexpr size_t kTileElems = static_cast<size_t>(kThreads) * U * VEC;
    constexpr int CU = U * VEC / CV;
    const int t = step - (N - 1);
    const T* from = uniform_ptr(s_tab[(k + t + N - 1) % N]) + b0;
    T* to = uniform_ptr(s_tab[(k + t) % N]) + b0;
    const unsigned tid = threadIdx.x;
    if (rem >= kTileElems) {
      R raw[CU];
#pragma unroll
      for (int u = 0; u < CU; ++u) raw[u] = ld<POL>(reinterpret_cast<const R*>(from) + tid + u * kThreads);
#pragma unroll
      for (int u = 0; u < CU; ++u) st<POL>(reinterpret_cast<R*>(to) + tid + u * kThreads, raw[u]);
    } else {
      const size_t n_vec = rem / CV;
      for (size_t v = tid; v < n_vec; v += kThreads)
        st<POL>(reinterpret_cast<R*>(to) + v, ld<POL>(reinterpret_cast<const R*>(from) + v));
      if constexpr (CV > 1) {
        for (size_t e = n_vec * CV + tid; e < rem; e += kThreads)
          st<POL>(reinterpret_cast<R1*>(to) + e, ld<POL>(reinterpret_cast<const R1*>(from) + e));
      }
    }
  }
}

// CH: the gate unit is a row of chunks (FTAR_PERSIST_CHUNKS), else a slot.
template <typename T, int VEC, int POL, int U, bool CH>
__global__ void __launch_bounds__(kThreads)
k_ring_persistent(PtrTable ring, PartGeom geom, SegTable tile_full, SegTable tile_last, int N, float* acc,
                  float scale, Ctrl* ctrl, CallRec* rec, unsigned long long epoch, DevCtrl* mirror,
                  unsigned long long timeout_ticks, unsigned long long max_spins, unsigned flags,
                  unsigned long long zpos, unsigned long long run_tiles) {
  // run_tiles: 0, or the tiles (a multiple of the number of workers, so that a tile keeps its
  // worker) between two soft barriers inside a step
  __shared__ T* s_tab[kMaxReplicas];
  __shared__ unsigned long long s_seg[2][kMaxReplicas + 1], s_tile[2][kMaxReplicas + 1];
  __shared__ unsigned long long s_word;  // what lane 0 saw in a wait
  __shared__ ChunkTab s_chunk[CH ? 2 : 1];
  const unsigned n_workers = gridDim.x - 1;
  if (blockIdx.x == 0) {  // the first block (dispatched first, so always resident) is the relay
    relay_loop(ctrl, rec, epoch, mirror, n_workers, max_spins, flags, (flags & FTAR_PERSIST_PUBLISH) != 0);
    return;
  }
  const unsigned worker = blockIdx.x - 1;
  const unsigned tid = threadIdx.x;
  constexpr size_t kTileElems = static_cast<size_t>(kThreads) * U * VEC;
  if (tid < static_cast<unsigned>(N)) s_tab[tid] = static_cast<T*>(ring.p[tid]);
  if (tid <= static_cast<unsigned>(N)) {
    s_seg[0][tid] = geom.seg_full.begin[tid];
    s_tile[0][tid] = tile_full.begin[tid];
    s_seg[1][tid] = geom.seg_last.begin[tid];
    s_tile[1][tid] = tile_last.begin[tid];
  }
  __syncthreads();
  if constexpr (CH) {
    if (tid == 0) build_chunk_tab(&s_chunk[0], s_seg[0], N, geom.chunk_elems, kTileElems);
    if (tid == 64) build_chunk_tab(&s_chunk[1], s_seg[1], N, geom.chunk_elems, kTileElems);
    __syncthreads();
  }
  // FTAR_PERSIST_PUBLISH: say which XCD this worker runs on; the first
  // one to register on an XCD is its leader (see leader_duty).  Before the first wait, so the relay
  // has every worker's XCD before it passes on a single unit.
  const bool leaders = (flags & FTAR_PERSIST_PUBLISH) != 0;
  unsigned xcd = 0, xcd_done = 0;
  bool leader = false;
  if (leaders) {
    if (tid == 0) {
      const unsigned x = xcd_of_this_wave();
      dev_store(&mirror->worker_xcd[worker], static_cast<unsigned char>(x));
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");  // the relay reads it after it has seen the count
      const unsigned before = __hip_atomic_fetch_add(&mirror->xcd_workers[x], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      s_word = static_cast<unsigned long long>(x) | (before == 0 ? 0x100ull : 0ull);
    }
    __syncthreads();
    xcd = static_cast<unsigned>(s_word & 0xffull);
    leader = (s_word & 0x100ull) != 0;
    __syncthreads();  // everybody has read the word before a wait can write it again
  }
  const WaitCtx wc{ctrl, rec, mirror, epoch, timeout_ticks, max_spins, &s_word, leader, xcd, &xcd_done};
  const unsigned n_steps = static_cast<unsigned>(2 * N - 2);
  // gate units per step of a full partition and of the last one; a slot is one unit unless CH
  const unsigned rows_full = CH ? geom.rows_full : 1u, rows_last = CH ? geom.rows_last : 1u;
  const unsigned units_full = n_steps * rows_full;  // per full partition
  unsigned released = 0;  // units [0, released) are known to be released
  unsigned n_aligned = 0;  // soft barriers inside steps passed so far (the same sequence in every worker)
  // acc handover before a shorter last partition (see above): every worker must have finished
  // the ReduceScatter phase of the partition before
  const bool handover = N >= 3 && geom.n_parts >= 2 && geom.seg_last.begin[N] != geom.part_elems;
  const unsigned hand_units = handover ? (geom.n_parts - 2) * units_full + static_cast<unsigned>(N - 1) * rows_full : 0u;
  for (unsigned part = 0; part < geom.n_parts; ++part) {
    const int sel = part + 1 == geom.n_parts ? 1 : 0;
    const unsigned rows = sel ? rows_last : rows_full;
    const unsigned long long* seg = s_seg[sel];
    const unsigned long long* til = s_tile[sel];
    const size_t off = static_cast<size_t>(part) * geom.part_elems;
    for (unsigned ustep = 0; ustep < n_steps; ++ustep) {
      const int step = static_cast<int>(ustep);
      const unsigned unit0 = part * units_full + ustep * rows;  // first unit of this slot
      if constexpr (!CH) {
        if (unit0 >= released && !wait_released(wc, unit0, &released)) return;
      }
      if (handover && sel == 1 && ustep == 0 && !wait_all_done(wc, hand_units, unit0)) return;
      // first AllGather step: see the block's stores
      if (step == N - 1) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
      if constexpr (CH) {
        const ChunkTab* tab = &s_chunk[sel];
        const size_t total = uniform_u64(tab->total_tiles);
        unsigned e = 0;
        unsigned cur = unit0;  // every unit before `cur` is finished by this worker
        for (size_t g = worker; g < total; g += n_workers) {
          const ChunkTile t = chunk_tile_of<kTileElems>(tab, seg, N, g, e);
          const unsigned unit = unit0 + t.row;
          if (unit != cur) {  // moving on to a later row: the rows before it are done
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
            if (leaders) __builtin_amdgcn_s_waitcnt(kWaitVmcnt0);  // every wave's stores have reached the L2
            __syncthreads();
            if (tid == 0) {
              if ((flags & FTAR_PERSIST_PUBLISH) && !leaders)
                __hip_atomic_store(&mirror->worker_unit[worker], unit, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
              else  // (with leaders: the stores are in the L2, the barrier's release saw to that)
                dev_store(&mirror->worker_unit[worker], unit);
            }
            cur = unit;
          }
          if (leader && tid == 0) leader_duty(mirror, xcd, &xcd_done);
          if (unit >= released && !wait_released(wc, unit, &released)) return;
          ring_one_tile<T, VEC, U, POL>(s_tab, N, step, t.k, t.begin, t.rem, acc, scale, off, zpos);
        }
      } else {
        const size_t slot_tiles = uniform_u64(til[N]);
        const size_t run = static_cast<size_t>(run_tiles);
        for (size_t g0 = 0;;) {
          const size_t g1 = run_tiles == 0 || slot_tiles - g0 < run + run / 2 ? slot_tiles : g0 + run;  // no short last run
          if (step < N - 1) {
            if (N == 2)
              ring_reduce_pass<T, VEC, kRsOnly, U, POL>(s_tab, seg, til, N, step, acc, scale, worker, n_workers, off,
                                                        zpos, g0, g1);
            else if (step == 0)
              ring_reduce_pass<T, VEC, kRsFirst, U, POL>(s_tab, seg, til, N, step, acc, scale, worker, n_workers,
                                                         off, zpos, g0, g1);
            else if (step == N - 2)
              ring_reduce_pass<T, VEC, kRsLast, U, POL>(s_tab, seg, til, N, step, acc, scale, worker, n_workers, off,
                                                        zpos, g0, g1);
            else
              ring_reduce_pass<T, VEC, kRsMid, U, POL>(s_tab, seg, til, N, step, acc, scale, worker, n_workers, off,
                                                       zpos, g0, g1);
          } else {
            // same tiles, widest copy: kThreads*U*VEC == kThreads*(U*VEC/CV)*CV
            constexpr int CV = VEC == 1 ? 1 : 16 / static_cast<int>(sizeof(T));
            ring_allgather_pass<T, CV, U * VEC / CV, POL>(s_tab, seg, til, N, step - (N - 1), worker, n_workers, off,
                                                          g0, g1);
          }
          if (g1 >= slot_tiles) break;
          g0 = g1;
          soft_align(mirror, n_workers, ++n_aligned);
        }
      }
      // A block-wide barrier with workgroup release/acquire is needed (a) before the first
      // AllGather step, whose 16-byte lanes read what other lanes of the block wrote in the last
      // ReduceScatter step, and (b) whenever the slot is reported or the next one needs a wait.
      // Between two ReduceScatter steps, or two AllGather steps, every lane only re-reads its own
      // stores, so slots that are already released run back to back.  Reporting is skipped while
      // the next slot is already released: the progress the CPU sees is then a lower bound, exact
      // whenever the kernel waits.  (With rows of chunks every slot's end is reported.)
      const unsigned done = unit0 + rows;  // units finished once this slot is
      const bool last_slot = part + 1 == geom.n_parts && ustep + 1 == n_steps;
      const bool hand_pub = handover && part + 2 == geom.n_parts && step == N - 2;
      const bool report = CH || done >= released || last_slot || (flags & FTAR_PERSIST_ALIGN) != 0 || hand_pub;
      if (report || step == N - 2) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        if (leaders) __builtin_amdgcn_s_waitcnt(kWaitVmcnt0);
        __syncthreads();
      }
      // With FTAR_PERSIST_PUBLISH the data of the units reported is written back from the XCD's L2
      // before the CPU can see the progress, which is what a NIC reading the buffers on the CPU's
      // signal would need: the workers' stores have reached the L2 (vmcnt(0) above), the XCD's
      // leader writes the L2 back for all of them (leader_duty).
      if (report && tid == 0) {
        if (((flags & FTAR_PERSIST_PUBLISH) && !leaders) || hand_pub)  // the handover orders this block's reads of acc first
          __hip_atomic_store(&mirror->worker_unit[worker], done, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
        else
          dev_store(&mirror->worker_unit[worker], done);
        if (flags & FTAR_PERSIST_ALIGN) {
          // Soft barrier, a performance hint only (bounded, nobody depends on it): blocks that ran
          // ahead wait for the stragglers, so all blocks stay in the same slot and read the same
          // few buffers.  Pays when a step is long (+7 % at 16 x 256 Mi), costs when it is short.
          for (int spin = 0; spin < 4000; ++spin) {
            if (dev_load(&mirror->min_unit) >= done) break;
            __builtin_amdgcn_s_sleep(2);
          }
        }
      }
      if (leader && tid == 0) leader_duty(mirror, xcd, &xcd_done);
      if (flags & FTAR_PERSIST_ALIGN) __syncthreads();
    }
  }
  if (leader && tid == 0) {
    // the leader stays until everything its XCD has written is out of the L2 (bounded like every wait)
    const unsigned total_units = (geom.n_parts - 1) * units_full + n_steps * rows_last;
    const long long t0 = wall_clock64();
    for (unsigned long long spin = 0; spin < max_spins; ++spin) {
      leader_duty(mirror, xcd, &xcd_done);
      if (xcd_done >= total_units) break;
      if (dev_load(&mirror->verdict) != 0 || (dev_load(&mirror->gate) & kGateCancel) != 0) break;
      if (static_cast<unsigned long long>(wall_clock64() - t0) > timeout_ticks) break;
      __builtin_amdgcn_s_sleep(4);
    }
  }
  if (tid == 0) count_out(mirror);
}

template <typename T, int VEC>
struct RingPersistent {
  const PtrTable& ring; int N; const PartGeom& geom; float* acc; float scale; Ctrl* ctrl; CallRec* rec;
  unsigned long long epoch; DevCtrl* mirror; unsigned n_blocks; unsigned long long timeout_ticks; unsigned flags;
  unsigned long long zpos; hipStream_t stream;
  template <int POL> hipError_t operator()(unsigned) const {
    // few workers and enough tiles for all of them even at four times the tile size: big tiles
    const SegTable big = ring_tiles(geom.seg_full, N, VEC, kPersistentUnrollFew);
    // (tuning flag 0x400000 keeps the small tile: several workgroups then fit one compute unit, which is
    // what a stream restricted to a few compute units wants)
    const bool few = n_blocks <= 128 && big.begin[N] >= 2ull * n_blocks && (current_tuning().flags & 0x400000) == 0;
    if (geom.chunk_elems != 0) {
      // rows of chunks: a tile never crosses the end of a chunk, so the big tile only if it fits one
      const size_t big_tile = static_cast<size_t>(kThreads) * kPersistentUnrollFew * VEC;
      if (few && geom.chunk_elems % big_tile == 0) return go<POL, kPersistentUnrollFew, true>();
      return go<POL, kPersistentUnroll, true>();
    }
    if (few) return go<POL, kPersistentUnrollFew, false>();
    return go<POL, kPersistentUnroll, false>();
  }
  template <int POL, int U, bool CH> hipError_t go() const {
    const SegTable tile_full = ring_tiles(geom.seg_full, N, VEC, U);
    const SegTable tile_last = ring_tiles(geom.seg_last, N, VEC, U);
    // Every workgroup must be resident at once: a worker that waits for the CPU keeps its place,
    // and the CPU may be waiting for a worker that has not started.  Clamp to what fits.
    int per_cu = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, k_ring_persistent<T, VEC, POL, U, CH>, kThreads, 0) !=
            hipSuccess || per_cu < 1)
      per_cu = 1;
    const unsigned capacity = static_cast<unsigned>(per_cu) * static_cast<unsigned>(device_cu_count());
    const unsigned workers = n_blocks + 1 > capacity ? capacity - 1 : n_blocks;
    hipLaunchKernelGGL(k_clear_mirror, dim3(1), dim3(256), 0, stream, mirror);
    const dim3 grid(workers + 1), block(kThreads);  // the relay + the workers
    // With FTAR_PERSIST_ALIGN a long step also gets soft barriers inside, one per 256 Mi elements, in
    // whole rounds of the workers (8 x 2e9 bf16: 5.35 -> 5.65 TB/s; shorter runs cost more than they
    // give: every barrier waits for the slowest worker).  Tuning bits 24..27: log2 of the Mi elements.
    unsigned long long run_tiles = 0;
    if (!CH && (flags & FTAR_PERSIST_ALIGN) != 0 && (current_tuning().flags & 0x40) == 0) {
      const int lg = (current_tuning().flags >> 24) & 0xf;
      const size_t run_elems = static_cast<size_t>(1) << (lg ? 20 + lg : 28);
      const size_t tile_elems = static_cast<size_t>(kThreads) * U * VEC;
      run_tiles = (run_elems / tile_elems + workers - 1) / workers * workers;
      if (run_tiles < 4ull * workers) run_tiles = 4ull * workers;
    }
    // one spin of a wait is a sleep plus two loads from device memory: well over 0.1 us
    launch(k_ring_persistent<T, VEC, POL, U, CH>, grid, block, stream, ring, geom, tile_full, tile_last, N, acc,
           scale, ctrl, rec, epoch, mirror, timeout_ticks, timeout_ticks / 10 + 100000, flags, zpos, run_tiles);
    return hipGetLastError();
  }
};

constexpr int kMaxDevices = 64;
std::mutex g_scratch_lock;
void* g_scratch_ptr[kMaxDevices] = {};  // device address of `scratch` on each GPU, once looked up

}  // namespace

hipError_t static_scratch(DevCtrl** mirror, float** acc) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  void* p = nullptr;
  {
    std::lock_guard<std::mutex> hold(g_scratch_lock);
    if (g_scratch_ptr[dev] == nullptr) {
      void* looked_up = nullptr;
      e = hipGetSymbolAddress(&looked_up, HIP_SYMBOL(scratch));
      if (e != hipSuccess) return e;
      if (looked_up == nullptr) return hipErrorInvalidSymbol;
      g_scratch_ptr[dev] = looked_up;
    }
    p = g_scratch_ptr[dev];
  }
  StaticScratch* s = static_cast<StaticScratch*>(p);
  *mirror = &s->mirror;
  *acc = s->acc;
  return hipSuccess;
}

hipError_t launch_ring_persistent(const PtrTable& ring, int n_live, const PartGeom& geom,
                                  ftar_dtype_t dtype, bool vec, float* acc, float scale, Ctrl* ctrl_dev,
                                  CallRec* rec_dev, unsigned long long epoch, DevCtrl* mirror, unsigned n_blocks,
                                  unsigned long long timeout_ticks, unsigned flags, unsigned long long zpos,
                                  hipStream_t stream) {
  // Stores as in the middle ReduceScatter step: what a slot writes, the next one reads.  The
  // partials of one partition are what must fit the Infinity Cache.
  const size_t acc_bytes = (geom.n_parts > 1 ? geom.part_elems : geom.seg_full.begin[n_live]) * 4;
  const LaunchCfg cfg = launch_cfg(1, acc_bytes <= 256 * kMiB ? 1 : 3);
  if (dtype == FTAR_F32) {
    if (vec)
      return with_policy(cfg, RingPersistent<float, 4>{ring, n_live, geom, acc, scale, ctrl_dev, rec_dev, epoch, mirror,
                                                       n_blocks, timeout_ticks, flags, zpos, stream});
    return with_policy(cfg, RingPersistent<float, 1>{ring, n_live, geom, acc, scale, ctrl_dev, rec_dev, epoch, mirror,
                                                     n_blocks, timeout_ticks, flags, zpos, stream});
  }
  if (vec)
    return with_policy(cfg, RingPersistent<bf16, 4>{ring, n_live, geom, acc, scale, ctrl_dev, rec_dev, epoch, mirror,
                                                    n_blocks, timeout_ticks, flags, zpos, stream});
  return with_policy(cfg, RingPersistent<bf16, 1>{ring, n_live, geom, acc, scale, ctrl_dev, rec_dev, epoch, mirror,
                                                  n_blocks, timeout_ticks, flags, zpos, stream});
}

}  // namespace ftar
