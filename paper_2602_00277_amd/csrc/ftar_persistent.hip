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
// relay is the only one that talks to the CPU: it copies the gate word from host-pinned memory
// into a mirror in device memory whenever it changes (every worker polling host memory over
// PCIe costs tens of microseconds per step), and it publishes the minimum over the workers'
// progress words back to the CPU.  Before slot s a worker waits on the mirror until the slot is
// released, the call is cancelled, somebody else gave up, or its own wait has lasted longer than
// the timeout (wall clock, 100 MHz, and a spin bound should the clock stand still): then it
// records why and leaves.  A worker that has seen r slots released does not look again before
// slot r.  The relay leaves when every worker has left, so the kernel ends no matter what the
// CPU does.
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

__global__ void k_clear_mirror(DevCtrl* m) {
  unsigned int* w = reinterpret_cast<unsigned int*>(m);
  for (unsigned i = threadIdx.x; i < sizeof(DevCtrl) / 4; i += blockDim.x) w[i] = 0;
}

// The relay block (all its lanes take part in the scan of the workers' progress words).
__device__ __forceinline__ void relay_loop(Ctrl* ctrl, DevCtrl* mirror, unsigned n_workers,
                                           unsigned long long max_spins, unsigned flags) {
  __shared__ unsigned s_min;
  __shared__ int s_last_round;
  unsigned long long last_gate = 0;
  unsigned last_min = 0;
  // max_spins bounds one wait of one worker; every worker leaves after at most n_slots such waits
  // plus its work, so the factor below is never reached: it only guarantees termination.
  for (unsigned long long spin = 0; spin < max_spins * 65536ull; ++spin) {
    if (threadIdx.x == 0) {
      // decide first whether this is the last round, then scan: a worker writes its progress word
      // before it counts itself out, so the scan of the last round sees every final value
      s_last_round = __hip_atomic_load(&mirror->exited, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT) >= n_workers;
      s_min = 0xffffffffu;
      const unsigned long long g = sys_load(&ctrl->gate);
      if (g != last_gate) {
        dev_store(&mirror->gate, g);
        last_gate = g;
      }
    }
    __syncthreads();
    unsigned lo = 0xffffffffu;
    for (unsigned b = threadIdx.x; b < n_workers; b += kThreads) {
      const unsigned v = dev_load(&mirror->worker_slot[b]);
      lo = v < lo ? v : lo;
    }
    atomicMin(&s_min, lo);
    __syncthreads();
    const int last_round = s_last_round;
    if (threadIdx.x == 0) {
      const unsigned m = s_min;
      if (m != last_min) {
        if (flags & FTAR_PERSIST_PUBLISH) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
        dev_store(&mirror->min_slot, m);
        sys_store(&ctrl->progress, static_cast<unsigned long long>(m));
        last_min = m;
      }
    }
    if (last_round) return;  // the same for every lane
    __builtin_amdgcn_s_sleep(8);
    __syncthreads();  // everybody has read s_last_round before lane 0 writes it again
  }
}

template <typename T, int VEC, int POL, int U>
__global__ void __launch_bounds__(kThreads)
k_ring_persistent(PtrTable ring, PartGeom geom, SegTable tile_full, SegTable tile_last, int N, float* acc,
                  float scale, Ctrl* ctrl, DevCtrl* mirror, unsigned long long timeout_ticks,
                  unsigned long long max_spins, unsigned flags, unsigned long long zpos) {
  __shared__ T* s_tab[kMaxReplicas];
  __shared__ unsigned long long s_seg[2][kMaxReplicas + 1], s_tile[2][kMaxReplicas + 1];
  __shared__ unsigned long long s_gate;  // what lane 0 saw: released slots, or a verdict in bits 32..33
  __shared__ unsigned s_hand;            // verdict of the acc handover wait (0 = go on)
  const unsigned n_workers = gridDim.x - 1;
  if (blockIdx.x == 0) {  // the first block (dispatched first, so always resident) is the relay
    relay_loop(ctrl, mirror, n_workers, max_spins, flags);
    return;
  }
  const unsigned worker = blockIdx.x - 1;
  const unsigned tid = threadIdx.x;
  if (tid < static_cast<unsigned>(N)) s_tab[tid] = static_cast<T*>(ring.p[tid]);
  if (tid <= static_cast<unsigned>(N)) {
    s_seg[0][tid] = geom.seg_full.begin[tid];
    s_tile[0][tid] = tile_full.begin[tid];
    s_seg[1][tid] = geom.seg_last.begin[tid];
    s_tile[1][tid] = tile_last.begin[tid];
  }
  __syncthreads();
  const unsigned n_steps = static_cast<unsigned>(2 * N - 2);
  const unsigned n_slots = geom.n_parts * n_steps;
  unsigned released = 0;  // slots [0, released) are known to be released
  // acc handover before a shorter last partition (see above); hand_pub = the slot whose end every
  // worker publishes, hand_slot = the slot that may only start when all have published it
  const bool handover = N >= 3 && geom.n_parts >= 2 && geom.seg_last.begin[N] != geom.part_elems;
  const unsigned hand_pub = handover ? (geom.n_parts - 2) * n_steps + static_cast<unsigned>(N - 2) : 0xffffffffu;
  const unsigned hand_slot = handover ? (geom.n_parts - 1) * n_steps : 0xffffffffu;
  unsigned part = 0, ustep = 0;
  for (unsigned slot = 0; slot < n_slots; ++slot, ++ustep) {
    if (ustep == n_steps) {
      ustep = 0;
      ++part;
    }
    if (slot >= released) {  // same decision in every lane: `released` comes from shared memory
      if (tid == 0) {
        unsigned long long seen = 1ull << 32;  // verdict 1 (timed out) unless the loop says otherwise
        const long long t0 = wall_clock64();
        for (unsigned long long spin = 0; spin < max_spins; ++spin) {
          const unsigned long long g = dev_load(&mirror->gate);
          if ((g & kGateCancel) != 0) { seen = 2ull << 32; break; }
          if ((g & 0xffffffffull) > slot) { seen = g & 0xffffffffull; break; }
          const unsigned v = dev_load(&mirror->verdict);
          if (v != 0) { seen = static_cast<unsigned long long>(v) << 32; break; }
          if (static_cast<unsigned long long>(wall_clock64() - t0) > timeout_ticks) break;
          __builtin_amdgcn_s_sleep(4);
        }
        s_gate = seen;
      }
      __syncthreads();
      const unsigned long long seen = s_gate;
      const unsigned verdict = static_cast<unsigned>(seen >> 32);
      if (verdict != 0) {  // the same for every lane of the block: all leave together
        if (tid == 0) {
          dev_store(&mirror->verdict, verdict);
          sys_store(&ctrl->blocked_step, static_cast<unsigned long long>(slot));
          sys_store(&ctrl->status, static_cast<unsigned long long>(verdict));
          __hip_atomic_fetch_add(&mirror->exited, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
        }
        return;
      }
      released = static_cast<unsigned>(seen);
    }
    if (slot == hand_slot) {
      if (tid == 0) {
        unsigned verdict = 1;  // timed out unless the loop says otherwise
        const long long t0 = wall_clock64();
        for (unsigned long long spin = 0; spin < max_spins; ++spin) {
          if (dev_load(&mirror->min_slot) > hand_pub) { verdict = 0; break; }
          if ((dev_load(&mirror->gate) & kGateCancel) != 0) { verdict = 2; break; }
          const unsigned v = dev_load(&mirror->verdict);
          if (v != 0) { verdict = v; break; }
          if (static_cast<unsigned long long>(wall_clock64() - t0) > timeout_ticks) break;
          __builtin_amdgcn_s_sleep(4);
        }
        s_hand = verdict;
      }
      __syncthreads();
      const unsigned verdict = s_hand;
      if (verdict != 0) {
        if (tid == 0) {
          dev_store(&mirror->verdict, verdict);
          sys_store(&ctrl->blocked_step, static_cast<unsigned long long>(slot));
          sys_store(&ctrl->status, static_cast<unsigned long long>(verdict));
          __hip_atomic_fetch_add(&mirror->exited, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
        }
        return;
      }
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    }
    const int step = static_cast<int>(ustep);
    // first AllGather step: see the block's stores
    if (step == N - 1) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    const int sel = part + 1 == geom.n_parts ? 1 : 0;
    const unsigned long long* seg = s_seg[sel];
    const unsigned long long* til = s_tile[sel];
    const size_t off = static_cast<size_t>(part) * geom.part_elems;
    if (step < N - 1) {
      if (N == 2)
        ring_reduce_pass<T, VEC, kRsOnly, U, POL>(s_tab, seg, til, N, step, acc, scale, worker, n_workers, off,
                                                  zpos);
      else if (step == 0)
        ring_reduce_pass<T, VEC, kRsFirst, U, POL>(s_tab, seg, til, N, step, acc, scale, worker, n_workers, off,
                                                   zpos);
      else if (step == N - 2)
        ring_reduce_pass<T, VEC, kRsLast, U, POL>(s_tab, seg, til, N, step, acc, scale, worker, n_workers, off,
                                                  zpos);
      else
        ring_reduce_pass<T, VEC, kRsMid, U, POL>(s_tab, seg, til, N, step, acc, scale, worker, n_workers, off,
                                                 zpos);
    } else {
      // same tiles, widest copy: kThreads*U*VEC == kThreads*(U*VEC/CV)*CV
      constexpr int CV = VEC == 1 ? 1 : 16 / static_cast<int>(sizeof(T));
      ring_allgather_pass<T, CV, U * VEC / CV, POL>(s_tab, seg, til, N, step - (N - 1), worker, n_workers, off);
    }
    // A block-wide barrier with workgroup release/acquire is needed (a) before the first
    // AllGather step, whose 16-byte lanes read what other lanes of the block wrote in the last
    // ReduceScatter step, and (b) whenever the slot is reported or the next slot needs a wait
    // (lane 0 then rewrites s_gate).  Between two ReduceScatter steps, or two AllGather steps,
    // every lane only re-reads its own stores, so slots that are already released run back to
    // back.  Reporting is skipped while the next slot is already released: the progress the CPU
    // sees is then a lower bound, exact whenever the kernel waits.
    const bool report = slot + 1 >= released || slot + 1 == n_slots || (flags & FTAR_PERSIST_ALIGN) != 0 ||
                        slot == hand_pub;
    if (report || step == N - 2) {
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
      __syncthreads();
    }
    // With FTAR_PERSIST_PUBLISH the progress store is a release at agent scope: the data of the
    // slots reported is written back from this XCD's L2 before the progress can be seen, which
    // is what a NIC reading the buffers on the CPU's signal would need (one L2 write-back per
    // block and report: 18 % at 64 Mi elements when every slot is reported).
    if (report && tid == 0) {
      if ((flags & FTAR_PERSIST_PUBLISH) || slot == hand_pub)  // the handover orders this block's reads of acc first
        __hip_atomic_store(&mirror->worker_slot[worker], slot + 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
      else
        dev_store(&mirror->worker_slot[worker], slot + 1);
      if (flags & FTAR_PERSIST_ALIGN) {
        // Soft barrier, a performance hint only (bounded, nobody depends on it): blocks that ran
        // ahead wait for the stragglers, so all blocks stay in the same slot and read the same
        // few buffers.  Pays when a step is long (+7 % at 16 x 256 Mi), costs when it is short.
        for (int spin = 0; spin < 4000; ++spin) {
          if (dev_load(&mirror->min_slot) > slot) break;
          __builtin_amdgcn_s_sleep(2);
        }
      }
    }
    if (flags & FTAR_PERSIST_ALIGN) __syncthreads();
  }
  if (tid == 0) __hip_atomic_fetch_add(&mirror->exited, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
}

template <typename T, int VEC>
struct RingPersistent {
  const PtrTable& ring; int N; const PartGeom& geom; float* acc; float scale; Ctrl* ctrl;
  DevCtrl* mirror; unsigned n_blocks; unsigned long long timeout_ticks; unsigned flags;
  unsigned long long zpos; hipStream_t stream;
  template <int POL> hipError_t operator()(unsigned) const {
    // few workers and enough tiles for all of them even at four times the tile size: big tiles
    const SegTable big = ring_tiles(geom.seg_full, N, VEC, kPersistentUnrollFew);
    if (n_blocks <= 128 && big.begin[N] >= 2ull * n_blocks) return go<POL, kPersistentUnrollFew>();
    return go<POL, kPersistentUnroll>();
  }
  template <int POL, int U> hipError_t go() const {
    const SegTable tile_full = ring_tiles(geom.seg_full, N, VEC, U);
    const SegTable tile_last = ring_tiles(geom.seg_last, N, VEC, U);
    // Every workgroup must be resident at once: a worker that waits for the CPU keeps its place,
    // and the CPU may be waiting for a worker that has not started.  Clamp to what fits.
    int per_cu = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, k_ring_persistent<T, VEC, POL, U>, kThreads, 0) !=
            hipSuccess || per_cu < 1)
      per_cu = 1;
    const unsigned capacity = static_cast<unsigned>(per_cu) * static_cast<unsigned>(device_cu_count());
    const unsigned workers = n_blocks + 1 > capacity ? capacity - 1 : n_blocks;
    hipLaunchKernelGGL(k_clear_mirror, dim3(1), dim3(256), 0, stream, mirror);
    const dim3 grid(workers + 1), block(kThreads);  // the relay + the workers
    // one spin of a wait is a sleep plus two loads from device memory: well over 0.1 us
    launch(k_ring_persistent<T, VEC, POL, U>, grid, block, stream, ring, geom, tile_full, tile_last, N, acc,
           scale, ctrl, mirror, timeout_ticks, timeout_ticks / 10 + 100000, flags, zpos);
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
                                  DevCtrl* mirror, unsigned n_blocks, unsigned long long timeout_ticks,
                                  unsigned flags, unsigned long long zpos, hipStream_t stream) {
  // Stores as in the middle ReduceScatter step: what a slot writes, the next one reads.  The
  // partials of one partition are what must fit the Infinity Cache.
  const size_t acc_bytes = (geom.n_parts > 1 ? geom.part_elems : geom.seg_full.begin[n_live]) * 4;
  const LaunchCfg cfg = launch_cfg(1, acc_bytes <= 256 * kMiB ? 1 : 3);
  if (dtype == FTAR_F32) {
    if (vec)
      return with_policy(cfg, RingPersistent<float, 4>{ring, n_live, geom, acc, scale, ctrl_dev, mirror,
                                                       n_blocks, timeout_ticks, flags, zpos, stream});
    return with_policy(cfg, RingPersistent<float, 1>{ring, n_live, geom, acc, scale, ctrl_dev, mirror,
                                                     n_blocks, timeout_ticks, flags, zpos, stream});
  }
  if (vec)
    return with_policy(cfg, RingPersistent<bf16, 4>{ring, n_live, geom, acc, scale, ctrl_dev, mirror,
                                                    n_blocks, timeout_ticks, flags, zpos, stream});
  return with_policy(cfg, RingPersistent<bf16, 1>{ring, n_live, geom, acc, scale, ctrl_dev, mirror,
                                                  n_blocks, timeout_ticks, flags, zpos, stream});
}

}  // namespace ftar
