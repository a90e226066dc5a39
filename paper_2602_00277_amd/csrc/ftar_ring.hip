// Ring all-reduce kernels - one ReduceScatter step, one AllGather step, the whole schedule in one
// pass - and their launchers.

#include "ftar_device.h"

namespace ftar {
namespace {

// One ReduceScatter step over all N portions.
template <typename T, int VEC, int MODE, int U, int POL>
__global__ void __launch_bounds__(kThreads)
k_ring_reduce(PtrTable ring, SegTable seg, SegTable tile0, int N, int step, float* acc, float scale,
              unsigned long long zpos, size_t g_begin, size_t g_end) {
  __shared__ T* s_tab[kMaxReplicas];
  __shared__ unsigned long long s_seg[kMaxReplicas + 1], s_tile[kMaxReplicas + 1];
  stage_ring_tables<T>(ring, seg, tile0, N, s_tab, s_seg, s_tile);
  ring_reduce_pass<T, VEC, MODE, U, POL>(s_tab, s_seg, s_tile, N, step, acc, scale, blockIdx.x, gridDim.x, 0,
                                         zpos, g_begin, g_end);
}

// One AllGather step over all N portions.
template <typename T, int VEC, int U, int POL>
__global__ void __launch_bounds__(kThreads)
k_ring_allgather(PtrTable ring, SegTable seg, SegTable tile0, int N, int step, size_t g_begin, size_t g_end) {
  __shared__ T* s_tab[kMaxReplicas];
  __shared__ unsigned long long s_seg[kMaxReplicas + 1], s_tile[kMaxReplicas + 1];
  stage_ring_tables<T>(ring, seg, tile0, N, s_tab, s_seg, s_tile);
  ring_allgather_pass<T, VEC, U, POL>(s_tab, s_seg, s_tile, N, step, blockIdx.x, gridDim.x, 0, g_begin, g_end);
}

// ---- the ring's result in one pass ------------------------------------------------
// On one device nothing forces the 2N-2 steps to be separate passes over memory: the partial sum
// of an element can stay in a register while its N contributions are added in the ring's order
// (portion k: positions k, k+1, ..., k+N-1 mod N), and the rounded mean can be written straight
// into all N replica buffers.  Same bits as the step schedule, 2*N*E bytes per element instead
// of 4*N*E + 10*N - 20 (N = 16, bf16: 64 instead of 206).
// OWNER: store only into the last buffer of the rotated order, the portion's owner (ring position
// k-1): the state after the ReduceScatter phase instead of the finished all-reduce.
template <typename T, int VEC, int N, int U, int POL, bool ZM, bool OWNER>
__device__ __forceinline__ void onepass_tile(T* const (&buf)[N], float scale, size_t v,
                                             unsigned long long zm) {
  typedef typename Raw<T, VEC>::type R;
  R raw[U][N];
#pragma unroll
  for (int u = 0; u < U; ++u) {
#pragma unroll
    for (int j = 0; j < N; ++j) {
      if (ZM && ((zm >> j) & 1ull)) raw[u][j] = R{};
      else raw[u][j] = ld<POL>(reinterpret_cast<const R*>(buf[j]) + v + u * kThreads);
    }
  }
#pragma unroll
  for (int u = 0; u < U; ++u) {
    float a[VEC], x[VEC];
    widen(raw[u][0], a);
#pragma unroll
    for (int j = 1; j < N; ++j) {
      widen(raw[u][j], x);
#pragma unroll
      for (int e = 0; e < VEC; ++e) a[e] = a[e] + x[e];
    }
#pragma unroll
    for (int e = 0; e < VEC; ++e) a[e] = a[e] * scale;
    const R r = narrow<R, VEC>(a);
    if constexpr (OWNER) {
      st<POL>(reinterpret_cast<R*>(buf[N - 1]) + v + u * kThreads, r);
    } else {
#pragma unroll
      for (int j = 0; j < N; ++j) st<POL>(reinterpret_cast<R*>(buf[j]) + v + u * kThreads, r);
    }
  }
}

// Any N (runtime): loads in groups of G in ring order starting at position k, then N stores.
template <typename T, int VEC, int POL, bool OWNER, int G = 8>
__device__ __forceinline__ void onepass_any_one(T* const* s_tab, int N, int k, size_t base, float scale,
                                                size_t v, unsigned long long zpos) {
  typedef typename Raw<T, VEC>::type R;
  float a[VEC];
  for (int j0 = 0; j0 < N; j0 += G) {
    R raw[G];
#pragma unroll
    for (int jj = 0; jj < G; ++jj)
      if (j0 + jj < N) {
        int p = k + j0 + jj;  // < 2N: one conditional subtraction instead of a division per load
        if (p >= N) p -= N;
        if ((zpos >> p) & 1ull) raw[jj] = R{};
        else raw[jj] = ld<POL>(reinterpret_cast<const R*>(uniform_ptr(s_tab[p]) + base) + v);
      }
#pragma unroll
    for (int jj = 0; jj < G; ++jj) {
      if (j0 + jj < N) {
        float x[VEC];
        widen(raw[jj], x);
        if (j0 + jj == 0) {
#pragma unroll
          for (int e = 0; e < VEC; ++e) a[e] = x[e];
        } else {
#pragma unroll
          for (int e = 0; e < VEC; ++e) a[e] = a[e] + x[e];
        }
      }
    }
  }
#pragma unroll
  for (int e = 0; e < VEC; ++e) a[e] = a[e] * scale;
  const R r = narrow<R, VEC>(a);
  if constexpr (OWNER) {
    st<POL>(reinterpret_cast<R*>(uniform_ptr(s_tab[(k + N - 1) % N]) + base) + v, r);
  } else {
    for (int j = 0; j < N; ++j) st<POL>(reinterpret_cast<R*>(uniform_ptr(s_tab[j]) + base) + v, r);
  }
}

template <typename T, int VEC, int POL, bool OWNER, int G = 8>
__device__ __forceinline__ void onepass_any_range(T* const* s_tab, int N, int k, size_t base, float scale,
                                                  size_t len, unsigned long long zpos) {
  const size_t n_vec = len / VEC;
  for (size_t v = threadIdx.x; v < n_vec; v += kThreads)
    onepass_any_one<T, VEC, POL, OWNER, G>(s_tab, N, k, base, scale, v, zpos);
  if constexpr (VEC > 1) {
    const size_t e = n_vec * VEC + threadIdx.x;
    if (e < len) onepass_any_one<T, 1, POL, OWNER>(s_tab, N, k, base, scale, e, zpos);
  }
}

// NT = compile-time N for the unrolled tile (1..16), or 0: any N through the grouped loop.
template <typename T, int VEC, int NT, int POL, bool OWNER>
__global__ void __launch_bounds__(kThreads)
k_ring_onepass(PtrTable ring, SegTable seg, SegTable tile0, int N, float scale, unsigned long long zpos) {
  __shared__ T* s_tab[kMaxReplicas];
  __shared__ unsigned long long s_seg[kMaxReplicas + 1], s_tile[kMaxReplicas + 1];
  stage_ring_tables<T>(ring, seg, tile0, N, s_tab, s_seg, s_tile);
  constexpr int U = NT == 0 ? 1 : unroll_narrow(NT);
  constexpr size_t kTileElems = static_cast<size_t>(kThreads) * U * VEC;
  const size_t total = uniform_u64(s_tile[N]);
  int k = 0;
  size_t next = uniform_u64(s_tile[1]);
  for (size_t g = blockIdx.x; g < total; g += gridDim.x) {
    const RingTile t = ring_tile_of<kTileElems>(g, k, next, s_seg, s_tile);
    if constexpr (NT > 0) {
      if (t.rem >= kTileElems) {
        T* buf[NT];
        unsigned long long zm = 0;
#pragma unroll
        for (int m = 0; m < NT; ++m) {
          const int p = (t.k + m) % NT;
          buf[m] = uniform_ptr(s_tab[p]) + t.begin;
          zm |= ((zpos >> p) & 1ull) << m;
        }
        if (zm == 0) onepass_tile<T, VEC, NT, U, POL, false, OWNER>(buf, scale, threadIdx.x, 0);
        else onepass_tile<T, VEC, NT, U, POL, true, OWNER>(buf, scale, threadIdx.x, zm);
        continue;
      }
    }
    // whole tiles of a ring of more than 16: all of a vector's loads in flight, up to 32
    if (t.rem >= kTileElems) onepass_any_range<T, VEC, POL, OWNER, (NT == 0 && VEC > 1 ? 32 : 8)>(s_tab, N, t.k, t.begin, scale, kTileElems, zpos);
    else onepass_any_range<T, VEC, POL, OWNER>(s_tab, N, t.k, t.begin, scale, t.rem, zpos);
  }
}

// ---- the whole AllGather phase in one pass ---------------------------------------
// After the ReduceScatter phase portion k is final in the buffer of ring position k-1.  The N-1
// AllGather steps hand it round the ring, one neighbour per step, because a network forces that;
// on one device the owner's copy can be read once and written to the N-1 other buffers directly:
// E + (N-1)E bytes per element instead of 2(N-1)E.  Same bits, of course (bit copies).
template <typename T, int VEC, int U, int POL>
__global__ void __launch_bounds__(kThreads)
k_ring_allgather_all(PtrTable ring, SegTable seg, SegTable tile0, int N) {
  typedef typename Raw<T, VEC>::type R;
  typedef typename Raw<T, 1>::type R1;
  __shared__ T* s_tab[kMaxReplicas];
  __shared__ unsigned long long s_seg[kMaxReplicas + 1], s_tile[kMaxReplicas + 1];
  stage_ring_tables<T>(ring, seg, tile0, N, s_tab, s_seg, s_tile);
  constexpr size_t kTileElems = static_cast<size_t>(kThreads) * U * VEC;
  const unsigned tid = threadIdx.x;
  const size_t total = uniform_u64(s_tile[N]);
  int k = 0;
  size_t next = uniform_u64(s_tile[1]);
  for (size_t g = blockIdx.x; g < total; g += gridDim.x) {
    const RingTile t = ring_tile_of<kTileElems>(g, k, next, s_seg, s_tile);
    const int owner = (t.k + N - 1) % N;
    const T* from = uniform_ptr(s_tab[owner]) + t.begin;
    if (t.rem >= kTileElems) {
      R raw[U];
#pragma unroll
      for (int u = 0; u < U; ++u) raw[u] = ld<POL>(reinterpret_cast<const R*>(from) + tid + u * kThreads);
      for (int m = 1; m < N; ++m) {
        T* to = uniform_ptr(s_tab[(owner + m) % N]) + t.begin;
#pragma unroll
        for (int u = 0; u < U; ++u) st<POL>(reinterpret_cast<R*>(to) + tid + u * kThreads, raw[u]);
      }
    } else {
      const size_t n_vec = t.rem / VEC;
      for (size_t v = tid; v < n_vec; v += kThreads) {
        const R x = ld<POL>(reinterpret_cast<const R*>(from) + v);
        for (int m = 1; m < N; ++m)
          st<POL>(reinterpret_cast<R*>(uniform_ptr(s_tab[(owner + m) % N]) + t.begin) + v, x);
      }
      if constexpr (VEC > 1) {
        const size_t e = n_vec * VEC + tid;
        if (e < t.rem) {
          const R1 x = ld<POL>(reinterpret_cast<const R1*>(from) + e);
          for (int m = 1; m < N; ++m)
            st<POL>(reinterpret_cast<R1*>(uniform_ptr(s_tab[(owner + m) % N]) + t.begin) + e, x);
        }
      }
    }
  }
}

template <typename T, int VEC>
struct RingAllgatherAll {
  const PtrTable& ring; int N; const SegTable& seg; hipStream_t stream;
  template <int POL> hipError_t operator()(unsigned blocks) const {
    constexpr int U = 4;
    const SegTable tiles = ring_tiles(seg, N, VEC, U);
    const dim3 grid(grid_x_for(tiles.begin[N], blocks)), block(kThreads);
    launch(k_ring_allgather_all<T, VEC, U, POL>, grid, block, stream, ring, seg, tiles, N);
    return hipGetLastError();
  }
};

// A long step goes out as several launches, each over a run of the flat tile sequence of 1.25 GiB
// of traffic (512 MiB for the AllGather copy; 8 x 2e9 bf16: middle step 5.7 -> 6.45 TB/s, AllGather
// 5.1 -> 5.95; 0.5 / 0.75 / 1 / 1.25 / 1.5 / 2 GiB per launch give the middle step 6.36 / 6.41 /
// 6.42 / 6.46 / 6.37 / 6.32 TB/s and the copy 5.95 / 5.82 / 5.60 / 5.6 / 5.5 / 5.2): the workgroups
// of a launch never wait for each other and drift apart over gigabytes (as in the one-shot
// reduce); the end of a launch brings them together again.  Tuning flag 0x40 forces one launch;
// bits 24..27 = traffic per launch in units of 256 MiB, for measurement.  A timed call brackets
// the whole series.
constexpr size_t kRingLaunchBytes = static_cast<size_t>(1280) << 20;
constexpr size_t kCopyLaunchBytes = static_cast<size_t>(512) << 20;

template <typename F>
void for_tile_runs(size_t n_tiles, size_t tile_bytes, size_t launch_bytes, F f) {
  const int lg = (current_tuning().flags >> 24) & 0xf;
  size_t per = (lg ? (static_cast<size_t>(lg) << 28) : launch_bytes) / tile_bytes;
  if (per < 1) per = 1;
  if ((current_tuning().flags & 0x40) != 0 || n_tiles <= per + per / 2) per = n_tiles;
  hipEvent_t t_start = nullptr, t_stop = nullptr;
  if (per < n_tiles) take_timing_events(&t_start, &t_stop);
  for (size_t g0 = 0; g0 < n_tiles;) {
    const size_t g1 = n_tiles - g0 < per + per / 2 ? n_tiles : g0 + per;  // no short last launch
    if (per < n_tiles) set_timing_events(g0 == 0 ? t_start : nullptr, g1 == n_tiles ? t_stop : nullptr);
    f(g0, g1);
    g0 = g1;
  }
}

template <typename T, int VEC>
struct RingReduce {
  RingMode mode; const PtrTable& ring; int N; int step; const SegTable& seg; float* acc; float scale;
  unsigned long long zpos; hipStream_t stream;
  template <int MODE, int U, int POL> void go(unsigned blocks) const {
    const SegTable tiles = ring_tiles(seg, N, VEC, U);
    // bytes one tile moves: the replica stream(s) plus the fp32 partial sums, read and written
    const size_t E = sizeof(T), elems = static_cast<size_t>(kThreads) * U * VEC;
    const size_t per_elem = MODE == kRsFirst ? 2 * E + 4 : MODE == kRsMid ? 8 + E : MODE == kRsLast ? 4 + 2 * E : 3 * E;
    for_tile_runs(tiles.begin[N], elems * per_elem, kRingLaunchBytes, [&](size_t g0, size_t g1) {
      const dim3 grid(grid_x_for(g1 - g0, blocks)), block(kThreads);
      launch(k_ring_reduce<T, VEC, MODE, U, POL>, grid, block, stream, ring, seg, tiles, N, step, acc, scale, zpos,
             g0, g1);
    });
  }
  template <int MODE, int POL> void pick_unroll(unsigned blocks) const {
    const int U = ring_unroll(VEC);
    if (U == 2) go<MODE, 2, POL>(blocks);
    else if (U == 8) go<MODE, 8, POL>(blocks);
    else go<MODE, 4, POL>(blocks);
  }
  template <int POL> hipError_t operator()(unsigned blocks) const {
    switch (mode) {
      case kRsFirst: pick_unroll<kRsFirst, POL>(blocks); break;
      case kRsMid: pick_unroll<kRsMid, POL>(blocks); break;
      case kRsLast: pick_unroll<kRsLast, POL>(blocks); break;
      case kRsOnly: pick_unroll<kRsOnly, POL>(blocks); break;
    }
    return hipGetLastError();
  }
};

template <typename T, int VEC>
struct RingAllgather {
  const PtrTable& ring; int N; int step; const SegTable& seg; hipStream_t stream;
  template <int U, int POL> void go(unsigned blocks) const {
    const SegTable tiles = ring_tiles(seg, N, VEC, U);
    const size_t elems = static_cast<size_t>(kThreads) * U * VEC;
    for_tile_runs(tiles.begin[N], elems * 2 * sizeof(T), kCopyLaunchBytes, [&](size_t g0, size_t g1) {
      const dim3 grid(grid_x_for(g1 - g0, blocks)), block(kThreads);
      launch(k_ring_allgather<T, VEC, U, POL>, grid, block, stream, ring, seg, tiles, N, step, g0, g1);
    });
  }
  template <int POL> hipError_t operator()(unsigned blocks) const {
    const int U = ring_unroll(4);
    if (U == 2) go<2, POL>(blocks);
    else if (U == 8) go<8, POL>(blocks);
    else go<4, POL>(blocks);
    return hipGetLastError();
  }
};

template <typename T, int VEC, bool OWNER>
struct RingOnepass {
  const PtrTable& ring; int N; const SegTable& seg; float scale; unsigned long long zpos; hipStream_t stream;
  template <int POL> hipError_t operator()(unsigned blocks) const {
    const int U = (VEC == 1 || N > 16) ? 1 : unroll_narrow(N);  // must match the kernel's tile
    const SegTable tiles = ring_tiles(seg, N, VEC, U);
    const dim3 grid(grid_x_for(tiles.begin[N], blocks)), block(kThreads);
    if (VEC == 1 || N > 16) {
      launch(k_ring_onepass<T, VEC, 0, POL, OWNER>, grid, block, stream, ring, seg, tiles, N, scale, zpos);
      return hipGetLastError();
    }
    switch (N) {
#define FTAR_CASE(n)                                                                                       \
  case n:                                                                                                  \
    launch(k_ring_onepass<T, VEC, (VEC == 1 ? 0 : n), POL, OWNER>, grid, block, stream, ring, seg, tiles, N, \
           scale, zpos);                                                                                   \
    break;
      FTAR_CASE(2) FTAR_CASE(3) FTAR_CASE(4) FTAR_CASE(5) FTAR_CASE(6) FTAR_CASE(7) FTAR_CASE(8)
      FTAR_CASE(9) FTAR_CASE(10) FTAR_CASE(11) FTAR_CASE(12) FTAR_CASE(13) FTAR_CASE(14)
      FTAR_CASE(15) FTAR_CASE(16)
#undef FTAR_CASE
      default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
  }
};

}  // namespace

hipError_t launch_ring_reduce(RingMode mode, const PtrTable& ring, int n_live, int step,
                              const SegTable& seg, ftar_dtype_t dtype, bool vec, float* acc,
                              float scale, unsigned long long zpos, hipStream_t stream) {
  const LaunchCfg cfg = ring_reduce_cfg(mode, seg.begin[n_live]);
  if (dtype == FTAR_F32) {
    if (vec) return with_policy(cfg, RingReduce<float, 4>{mode, ring, n_live, step, seg, acc, scale, zpos, stream});
    return with_policy(cfg, RingReduce<float, 1>{mode, ring, n_live, step, seg, acc, scale, zpos, stream});
  }
  // bf16 lanes take 4 elements: an 8-byte load of the replica stream next to one 16-byte vector of
  // partial sums, so every instruction of a wave covers one contiguous run of memory.  The other
  // shape - 8 elements per lane, a 16-byte bf16 load and TWO partial-sum vectors 32 bytes apart per
  // lane - is kept behind tuning flag 0x200000 for measurement: it is 14 % slower in the middle step
  // (16 x 256 Mi bf16: 5.34 against 6.19 TB/s) and 15 % in the first.
  if (vec && (current_tuning().flags & 0x200000) != 0)
    return with_policy(cfg, RingReduce<bf16, 8>{mode, ring, n_live, step, seg, acc, scale, zpos, stream});
  if (vec) return with_policy(cfg, RingReduce<bf16, 4>{mode, ring, n_live, step, seg, acc, scale, zpos, stream});
  return with_policy(cfg, RingReduce<bf16, 1>{mode, ring, n_live, step, seg, acc, scale, zpos, stream});
}

hipError_t launch_ring_allgather(const PtrTable& ring, int n_live, int step, const SegTable& seg,
                                 ftar_dtype_t dtype, bool vec, hipStream_t stream) {
  const LaunchCfg cfg = ring_allgather_cfg(seg.begin[n_live], dtype == FTAR_F32 ? 4 : 2);
  if (dtype == FTAR_F32) {
    if (vec) return with_policy(cfg, RingAllgather<float, 4>{ring, n_live, step, seg, stream});
    return with_policy(cfg, RingAllgather<float, 1>{ring, n_live, step, seg, stream});
  }
  if (vec) return with_policy(cfg, RingAllgather<bf16, 8>{ring, n_live, step, seg, stream});
  return with_policy(cfg, RingAllgather<bf16, 1>{ring, n_live, step, seg, stream});
}

hipError_t launch_ring_allgather_all(const PtrTable& ring, int n_live, const SegTable& seg, ftar_dtype_t dtype,
                                     bool vec, hipStream_t stream) {
  // one read stream, N-1 written ones: as the one-pass all-reduce
  const LaunchCfg cfg = launch_cfg(1, 3);
  if (dtype == FTAR_F32) {
    if (vec) return with_policy(cfg, RingAllgatherAll<float, 4>{ring, n_live, seg, stream});
    return with_policy(cfg, RingAllgatherAll<float, 1>{ring, n_live, seg, stream});
  }
  if (vec) return with_policy(cfg, RingAllgatherAll<bf16, 8>{ring, n_live, seg, stream});
  return with_policy(cfg, RingAllgatherAll<bf16, 1>{ring, n_live, seg, stream});
}

hipError_t launch_ring_onepass(const PtrTable& ring, int n_live, const SegTable& seg,
                               ftar_dtype_t dtype, bool vec, float scale, unsigned long long zpos,
                               bool owner_only, hipStream_t stream) {
  // N reads and N writes per element, as many write streams as read streams: non-temporal
  // stores and one workgroup per CU are best at every size measured.  Owner only: N reads and one
  // write, the mix of the one-shot reduce, and its choices.
  const LaunchCfg cfg = owner_only ? reduce_cfg(n_live, seg.begin[n_live] * (dtype == FTAR_F32 ? 4 : 2))
                                   : launch_cfg(1, 3);
  if (owner_only) {
    if (dtype == FTAR_F32) {
      if (vec) return with_policy(cfg, RingOnepass<float, 4, true>{ring, n_live, seg, scale, zpos, stream});
      return with_policy(cfg, RingOnepass<float, 1, true>{ring, n_live, seg, scale, zpos, stream});
    }
    if (vec) return with_policy(cfg, RingOnepass<bf16, 8, true>{ring, n_live, seg, scale, zpos, stream});
    return with_policy(cfg, RingOnepass<bf16, 1, true>{ring, n_live, seg, scale, zpos, stream});
  }
  if (dtype == FTAR_F32) {
    if (vec) return with_policy(cfg, RingOnepass<float, 4, false>{ring, n_live, seg, scale, zpos, stream});
    return with_policy(cfg, RingOnepass<float, 1, false>{ring, n_live, seg, scale, zpos, stream});
  }
  if (vec) return with_policy(cfg, RingOnepass<bf16, 8, false>{ring, n_live, seg, scale, zpos, stream});
  return with_policy(cfg, RingOnepass<bf16, 1, false>{ring, n_live, seg, scale, zpos, stream});
}

}  // namespace ftar
