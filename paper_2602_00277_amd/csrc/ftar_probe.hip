// Bare streaming kernels that measure what this GPU's memory system gives for a mix of read and
// written streams - the ceilings the product kernels are compared with.  Measurement only: no
// arithmetic of the method (words are folded with xor so that the loads cannot be dropped).

#include "ftar_device.h"

namespace ftar {
namespace {

// NR read streams, NW written streams, all of n_vec 16-byte vectors.  Every written stream gets
// the xor of the read vectors at the same index (or `fill` when nothing is read).  With NW == 0
// nothing is stored unless the folded word equals `never` in all four lanes of a vector.
template <int NR, int NW, int U, int POL>
__global__ void __launch_bounds__(kThreads)
k_probe_stream(PtrTable tab, size_t n_vec, uint32_t fill, uint32_t never) {
  __shared__ u32x4* s_tab[kMaxReplicas];
  if (threadIdx.x < static_cast<unsigned>(NR + NW)) s_tab[threadIdx.x] = static_cast<u32x4*>(tab.p[threadIdx.x]);
  __syncthreads();
  u32x4* p[NR + NW];
#pragma unroll
  for (int j = 0; j < NR + NW; ++j) p[j] = uniform_ptr(s_tab[j]);
  constexpr size_t kTile = static_cast<size_t>(kThreads) * U;
  const size_t n_tiles = n_vec / kTile;  // the host passes whole tiles only
  for (size_t t = blockIdx.x; t < n_tiles; t += gridDim.x) {
    const size_t v = t * kTile + threadIdx.x;
    u32x4 x[U][NR > 0 ? NR : 1];
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
      for (int j = 0; j < NR; ++j) x[u][j] = ld<POL>(p[j] + v + u * kThreads);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      u32x4 f = {fill, fill, fill, fill};
#pragma unroll
      for (int j = 0; j < NR; ++j) f = j == 0 ? x[u][0] : f ^ x[u][j];
      if constexpr (NW > 0) {
#pragma unroll
        for (int w = 0; w < NW; ++w) st<POL>(p[NR + w] + v + u * kThreads, f);
      } else {
        if (f[0] == never && f[1] == never && f[2] == never && f[3] == never) st<POL>(p[0] + v + u * kThreads, f);
      }
    }
  }
}

// NR read streams and one written stream, the written vectors staged in LDS and written out in
// windows of the wall clock (struct WriteWindow): what the write windows of the many-source
// reductions give on bare streams.  One vector per lane and tile; one workgroup per compute unit.
template <int NR, int POL>
__global__ void __launch_bounds__(kThreads)
k_probe_stream_win(PtrTable tab, size_t n_vec, WriteWindow win) {
  constexpr int kCap = kStageBytes / (kThreads * 16);
  __shared__ u32x4 stage[kCap][kThreads];
  __shared__ u32x4* s_tab[kMaxReplicas];
  if (threadIdx.x < static_cast<unsigned>(NR + 1)) s_tab[threadIdx.x] = static_cast<u32x4*>(tab.p[threadIdx.x]);
  __syncthreads();
  u32x4* p[NR + 1];
#pragma unroll
  for (int j = 0; j < NR + 1; ++j) p[j] = uniform_ptr(s_tab[j]);
  const size_t n_tiles = n_vec / kThreads;  // the host passes whole tiles only
  const size_t gx = gridDim.x;
  unsigned pending = 0;
  size_t first = 0;
  for (size_t t = blockIdx.x; t < n_tiles; t += gx) {
    const unsigned now = static_cast<unsigned>(wall_clock64());
    u32x4 x[NR];
#pragma unroll
    for (int j = 0; j < NR; ++j) x[j] = ld<POL>(p[j] + t * kThreads + threadIdx.x);
    u32x4 f = x[0];
#pragma unroll
    for (int j = 1; j < NR; ++j) f = f ^ x[j];
    if (pending == 0) first = t;
    stage[pending][threadIdx.x] = f;  // a lane only reads back its own slots
    ++pending;
    const bool window = (now & win.period_mask) < win.write_ticks && pending >= win.min_tiles;
    if (pending == static_cast<unsigned>(kCap) || window) {
      for (unsigned k = 0; k < pending; ++k)
        st<POL>(p[NR] + (first + k * gx) * kThreads + threadIdx.x, stage[k][threadIdx.x]);
      pending = 0;
    }
  }
  for (unsigned k = 0; k < pending; ++k) st<POL>(p[NR] + (first + k * gx) * kThreads + threadIdx.x, stage[k][threadIdx.x]);
}

template <int NR>
struct ProbeWin {
  const PtrTable& tab; size_t n_vec; WriteWindow win; hipStream_t stream;
  template <int POL> hipError_t operator()(unsigned) const {
    const size_t tiles = n_vec / kThreads;
    launch(k_probe_stream_win<NR, POL>, dim3(grid_x_for(tiles, static_cast<unsigned>(device_cu_count()))), dim3(kThreads),
           stream, tab, n_vec, win);
    return hipGetLastError();
  }
};

// The same mix on a given number of workgroups of THREADS lanes, U vectors per lane and tile,
// ordinary loads and stores: what a few compute units can move, whatever is in flight.
template <int NR, int NW, int U, int THREADS>
__global__ void __launch_bounds__(THREADS)
k_probe_few(PtrTable tab, size_t n_vec) {
  u32x4* p[NR + NW];
#pragma unroll
  for (int j = 0; j < NR + NW; ++j) p[j] = static_cast<u32x4*>(tab.p[j]);
  constexpr size_t kTile = static_cast<size_t>(THREADS) * U;
  const size_t n_tiles = n_vec / kTile;  // the host passes whole tiles only
  for (size_t t = blockIdx.x; t < n_tiles; t += gridDim.x) {
    const size_t v = t * kTile + threadIdx.x;
    u32x4 x[U][NR];
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
      for (int j = 0; j < NR; ++j) x[u][j] = p[j][v + u * THREADS];
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      u32x4 f = x[u][0];
#pragma unroll
      for (int j = 1; j < NR; ++j) f = f ^ x[u][j];
#pragma unroll
      for (int w = 0; w < NW; ++w) p[NR + w][v + u * THREADS] = f;
    }
  }
}

constexpr int probe_unroll(int streams) { return streams <= 2 ? 8 : streams <= 4 ? 4 : streams <= 8 ? 2 : 1; }

template <int NR, int NW>
struct Probe {
  const PtrTable& tab; size_t n_vec; uint32_t fill; hipStream_t stream;
  template <int POL> hipError_t operator()(unsigned blocks) const {
    constexpr int U = probe_unroll(NR + NW);
    const size_t tiles = n_vec / (static_cast<size_t>(kThreads) * U);
    launch(k_probe_stream<NR, NW, U, POL>, dim3(grid_x_for(tiles, blocks)), dim3(kThreads), stream, tab, n_vec, fill,
           0x9e3779b9u);
    return hipGetLastError();
  }
};

}  // namespace

// Supported mixes only; anything else: hipErrorInvalidValue.
hipError_t launch_probe_stream(const PtrTable& tab, int n_read, int n_written, size_t n_vec, uint32_t fill,
                               hipStream_t stream) {
  // the product kernels' own choices unless the tuning says otherwise: one workgroup per CU from
  // five streams on, non-temporal loads, ordinary stores while what is written fits the cache
  const bool fits = static_cast<size_t>(n_written) * n_vec * 16 <= 256 * kMiB;
  const LaunchCfg cfg = launch_cfg(n_read + n_written <= 2 ? 4 : n_read + n_written <= 4 ? 2 : 1, fits ? 1 : 3);
#define FTAR_PROBE(r, w) \
  if (n_read == r && n_written == w) return with_policy(cfg, Probe<r, w>{tab, n_vec, fill, stream});
  FTAR_PROBE(1, 0) FTAR_PROBE(2, 0) FTAR_PROBE(4, 0) FTAR_PROBE(8, 0) FTAR_PROBE(16, 0)
  FTAR_PROBE(0, 1) FTAR_PROBE(0, 2) FTAR_PROBE(0, 4) FTAR_PROBE(0, 8)
  FTAR_PROBE(1, 1) FTAR_PROBE(2, 1) FTAR_PROBE(3, 1) FTAR_PROBE(4, 1) FTAR_PROBE(7, 1) FTAR_PROBE(8, 1) FTAR_PROBE(16, 1)
  FTAR_PROBE(4, 4) FTAR_PROBE(8, 8)
#undef FTAR_PROBE
  return hipErrorInvalidValue;
}

hipError_t launch_probe_stream_win(const PtrTable& tab, int n_read, size_t n_vec, unsigned period_ticks,
                                   unsigned window_ticks, hipStream_t stream) {
  const LaunchCfg cfg = launch_cfg(1, 3);
  const WriteWindow win{period_ticks - 1u, window_ticks, 4u};
#define FTAR_PROBE(r) \
  if (n_read == r) return with_policy(cfg, ProbeWin<r>{tab, n_vec, win, stream});
  FTAR_PROBE(1) FTAR_PROBE(2) FTAR_PROBE(4) FTAR_PROBE(7) FTAR_PROBE(8) FTAR_PROBE(16)
#undef FTAR_PROBE
  return hipErrorInvalidValue;
}

// n_read 1 or 2, one written stream; (threads, vectors per lane) one of (256, 8), (1024, 8) and, for one
// read stream, (256, 32).
hipError_t launch_probe_few(const PtrTable& tab, int n_read, size_t n_vec, unsigned n_workgroups, unsigned threads,
                            unsigned per_lane, hipStream_t stream) {
#define FTAR_PROBE(r, t, u)                                                                              \
  if (n_read == r && threads == t && per_lane == u) {                                                    \
    launch(k_probe_few<r, 1, u, t>, dim3(n_workgroups), dim3(t), stream, tab, n_vec);                    \
    return hipGetLastError();                                                                            \
  }
  FTAR_PROBE(1, 256, 8) FTAR_PROBE(1, 256, 32) FTAR_PROBE(1, 1024, 8)
  FTAR_PROBE(2, 256, 8) FTAR_PROBE(2, 1024, 8)  // (2, 256, 32) would not fit the registers
#undef FTAR_PROBE
  return hipErrorInvalidValue;
}

}  // namespace ftar
