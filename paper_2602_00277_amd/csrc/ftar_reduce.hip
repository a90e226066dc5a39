// One-shot masked reduction kernels (fixed and runtime number of sources, fp32 result from bf16,
// per-bucket masks) and their launchers.

#include "ftar_device.h"

namespace ftar {
namespace {

// ---- kernels -------------------------------------------------------------

// One-shot masked mean over N live buffers (N fixed at compile time, 1..16).
template <typename T, int VEC, int N, int U, int POL>
__global__ void __launch_bounds__(kThreads)
k_reduce_masked(PtrTable live, T* out, float scale, size_t count, float zterm) {
  __shared__ T* s_tab[kMaxReplicas];
  if (threadIdx.x < static_cast<unsigned>(N)) s_tab[threadIdx.x] = static_cast<T*>(live.p[threadIdx.x]);
  __syncthreads();
  T* src[N];
#pragma unroll
  for (int j = 0; j < N; ++j) src[j] = uniform_ptr(s_tab[j]);
  sum_range_z<T, VEC, N, false, false, U, POL, false, true>(src, nullptr, nullptr, out, scale, count,
                                                            blockIdx.x, gridDim.x, 0, zterm);
}

// One-shot masked mean with write windows: results are staged in LDS (a lane only ever reads back
// what it staged itself, so no barrier is involved) and written out inside the clock windows or
// when the stage is full.  MODE 0: result of the input type; 2: fp32 from bf16; 3: bf16 from fp32.
// One workgroup per compute unit (the stage takes most of its LDS).
template <typename T, int VEC, int N, int U, int POL, int MODE>
__global__ void __launch_bounds__(kThreads)
k_reduce_masked_win(PtrTable live, void* out_, float scale, size_t count, float zterm, WriteWindow win) {
  typedef typename OutVec<T, VEC, MODE>::type O;
  constexpr int kCap = kStageBytes / (kThreads * static_cast<int>(sizeof(O)));  // vectors per lane
  static_assert(kCap >= 2 * U, "room for two tiles at least");
  __shared__ O stage[kCap][kThreads];
  __shared__ T* s_tab[kMaxReplicas];
  const unsigned tid = threadIdx.x;
  if (tid < static_cast<unsigned>(N)) s_tab[tid] = static_cast<T*>(live.p[tid]);
  __syncthreads();
  T* src[N];
#pragma unroll
  for (int j = 0; j < N; ++j) src[j] = uniform_ptr(s_tab[j]);
  O* out = static_cast<O*>(out_);
  const size_t n_vec = count / VEC;
  constexpr size_t kTile = static_cast<size_t>(kThreads) * U;
  const size_t n_tiles = n_vec / kTile;
  const size_t gx = gridDim.x;
  unsigned pending = 0;  // tiles staged, U vectors each
  size_t first = 0;      // tile of stage[0]; the staged tiles are first, first + gx, ...
  for (size_t t = blockIdx.x; t < n_tiles; t += gx) {
    const unsigned now = static_cast<unsigned>(wall_clock64());
    O res[U];
    sum_tile_values<T, VEC, N, MODE, U, POL, true>(src, scale, t * kTile + tid, zterm, res);
    if (pending == 0) first = t;
#pragma unroll
    for (int u = 0; u < U; ++u) stage[pending * U + u][tid] = res[u];
    ++pending;
    const bool window = (now & win.period_mask) < win.write_ticks && pending >= win.min_tiles;
    if ((pending + 1) * U > static_cast<unsigned>(kCap) || window) {
      for (unsigned k = 0; k < pending; ++k) {
#pragma unroll
        for (int u = 0; u < U; ++u)
          st<POL>(out + (first + k * gx) * kTile + tid + u * kThreads, stage[k * U + u][tid]);
      }
      pending = 0;
    }
  }
  for (unsigned k = 0; k < pending; ++k) {
#pragma unroll
    for (int u = 0; u < U; ++u) st<POL>(out + (first + k * gx) * kTile + tid + u * kThreads, stage[k * U + u][tid]);
  }
  // whole vectors past the last full tile and the last count % VEC elements: one workgroup, directly
  if (blockIdx.x == n_tiles % gx) {
    constexpr int kMode = MODE;
    float* fo = static_cast<float*>(out_);
    T* to = static_cast<T*>(out_);
    for (size_t v = n_tiles * kTile + tid; v < n_vec; v += kThreads)
      sum_tile<T, VEC, N, false, kMode, 1, POL, false, true>(src, nullptr, fo, to, scale, v, 0, zterm);
    if constexpr (VEC > 1) {
      const size_t e = n_vec * VEC + tid;
      if (e < count) sum_tile<T, 1, N, false, kMode, 1, POL, false, true>(src, nullptr, fo, to, scale, e, 0, zterm);
    }
  }
}

// The same for any N up to 64: what the specialised kernel above does for up to 16 sources, for the
// 17 to 64 that the paper's 10 to 20 replicas can reach.  One vector per lane and tile, up to 32
// loads per lane in flight (N = 20: 5.1 TB/s with the plain kernel's groups of 8, 5.6 with windows,
// more with all 20 loads in flight).
template <typename T, int VEC, int POL, typename TO>
__global__ void __launch_bounds__(kThreads)
k_reduce_masked_any_win(PtrTable live, int N, TO* out, float scale, size_t count, float zterm, WriteWindow win) {
  typedef typename Raw<TO, VEC>::type RO;
  constexpr int kCap = kStageBytes / (kThreads * static_cast<int>(sizeof(RO)));
  __shared__ RO stage[kCap][kThreads];
  __shared__ T* s_tab[kMaxReplicas];
  const unsigned tid = threadIdx.x;
  if (tid < static_cast<unsigned>(N)) s_tab[tid] = static_cast<T*>(live.p[tid]);
  __syncthreads();
  const size_t n_vec = count / VEC;
  const size_t n_tiles = n_vec / kThreads;
  const size_t gx = gridDim.x;
  RO* o = reinterpret_cast<RO*>(out);
  unsigned pending = 0;
  size_t first = 0;
  for (size_t t = blockIdx.x; t < n_tiles; t += gx) {
    const unsigned now = static_cast<unsigned>(wall_clock64());
    const RO r = sum_any_value<T, VEC, POL, TO, 32>(s_tab, 0, N, scale, t * kThreads + tid, zterm);
    if (pending == 0) first = t;
    stage[pending][tid] = r;
    ++pending;
    const bool window = (now & win.period_mask) < win.write_ticks && pending >= win.min_tiles;
    if (pending == static_cast<unsigned>(kCap) || window) {
      for (unsigned k = 0; k < pending; ++k) st<POL>(o + (first + k * gx) * kThreads + tid, stage[k][tid]);
      pending = 0;
    }
  }
  for (unsigned k = 0; k < pending; ++k) st<POL>(o + (first + k * gx) * kThreads + tid, stage[k][tid]);
  // whole vectors past the last full tile and the last count % VEC elements: one workgroup, directly
  if (blockIdx.x == n_tiles % gx) {
    const size_t v = n_tiles * kThreads + tid;
    if (v < n_vec) sum_any_one<T, VEC, POL, TO>(s_tab, 0, N, out, scale, v, zterm);
    if constexpr (VEC > 1) {
      const size_t e = n_vec * VEC + tid;
      if (e < count) sum_any_one<T, 1, POL, TO>(s_tab, 0, N, out, scale, e, zterm);
    }
  }
}

// The same with a result of the other element type, 4 elements per lane and vector: an fp32 result
// from bf16 inputs (8-byte loads, 16-byte stores) or a bf16 result from fp32 inputs (16-byte loads,
// 8-byte stores).  TI = input type; out is float* for bf16 inputs and bf16* for fp32 inputs.
template <typename TI, int VEC, int N, int U, int POL>
__global__ void __launch_bounds__(kThreads)
k_reduce_masked_cvt(PtrTable live, void* out, float scale, size_t count, float zterm) {
  __shared__ TI* s_tab[kMaxReplicas];
  if (threadIdx.x < static_cast<unsigned>(N)) s_tab[threadIdx.x] = static_cast<TI*>(live.p[threadIdx.x]);
  __syncthreads();
  TI* src[N];
#pragma unroll
  for (int j = 0; j < N; ++j) src[j] = uniform_ptr(s_tab[j]);
  constexpr int kMode = __is_same(TI, float) ? 3 : 2;
  sum_range_z<TI, VEC, N, false, kMode, U, POL, false, true>(src, nullptr, static_cast<float*>(out), nullptr,
                                                             scale, count, blockIdx.x, gridDim.x, 0, zterm);
}

// One-shot masked mean, any N up to 64 (also the element-wise path for unaligned buffers).
template <typename T, int VEC, int POL, typename TO = T>
__global__ void __launch_bounds__(kThreads)
k_reduce_masked_any(PtrTable live, int N, TO* out, float scale, size_t count, float zterm) {
  __shared__ T* s_tab[kMaxReplicas];
  if (threadIdx.x < static_cast<unsigned>(N)) s_tab[threadIdx.x] = static_cast<T*>(live.p[threadIdx.x]);
  __syncthreads();
  sum_any_range<T, VEC, POL, TO>(s_tab, 0, N, out, scale, count, blockIdx.x, gridDim.x, zterm);
}

// Every participant is a zero-gradient one: the mean is +0.0 (all-zero bits in both element types).
__global__ void __launch_bounds__(kThreads)
k_fill_zero(uint16_t* head16, uint32_t* out32, size_t n32, uint16_t* tail16) {
  for (size_t i = static_cast<size_t>(blockIdx.x) * kThreads + threadIdx.x; i < n32;
       i += static_cast<size_t>(gridDim.x) * kThreads)
    out32[i] = 0u;
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    if (head16 != nullptr) *head16 = 0;
    if (tail16 != nullptr) *tail16 = 0;
  }
}

constexpr int kBucketUnroll = 4;  // vectors per lane in one tile of the bucketed kernel

WriteWindow reduce_window(int n_src, size_t out_bytes);

template <typename T, int VEC, int N, int POL>
__device__ __forceinline__ void bucket_tile_n(T* const* s_tab, T* out, float scale, size_t begin,
                                              size_t rem) {
  constexpr int UN = unroll_narrow(N) < kBucketUnroll ? unroll_narrow(N) : kBucketUnroll;
  T* src[N];
#pragma unroll
  for (int j = 0; j < N; ++j) src[j] = uniform_ptr(s_tab[j]) + begin;
  if (rem >= static_cast<size_t>(kThreads) * kBucketUnroll * VEC) {
#pragma unroll
    for (int it = 0; it < kBucketUnroll / UN; ++it)
      sum_tile<T, VEC, N, false, false, UN, POL>(src, nullptr, nullptr, out + begin, scale,
                                                 static_cast<size_t>(it) * kThreads * UN + threadIdx.x);
  } else {
    sum_range<T, VEC, N, false, false, 1, POL>(src, nullptr, nullptr, out + begin, scale, rem, 0u, 1u);
  }
}

// Masked mean with one live mask per bucket.  When a block's next tile lies in another bucket it
// re-compacts that bucket's mask into the LDS pointer table (lane r places replica r at the rank
// of its bit) and switches to the loop specialised for that bucket's N.
template <typename T, int VEC, int POL>
__global__ void __launch_bounds__(kThreads)
k_reduce_bucketed(PtrTable all, int n_replicas, BucketTable masks, ScaleTable scales,
                  size_t first_elem, size_t bucket_elems, size_t last_len, int n_buckets,
                  size_t tiles_per_bucket, size_t total_tiles, T* out) {
  // last_len = length of this launch's last bucket; tiles_per_bucket = ceil(bucket_elems / tile);
  // total_tiles = (n_buckets-1)*tiles_per_bucket + ceil(last_len / tile): all computed on the host.
  __shared__ T* s_tab[kMaxReplicas];
  constexpr size_t kTileElems = static_cast<size_t>(kThreads) * kBucketUnroll * VEC;
  int cur = -1, N = 0;
  float scale = 0.0f;
  for (size_t g = blockIdx.x; g < total_tiles; g += gridDim.x) {
    const int b = static_cast<int>(g / tiles_per_bucket);
    const size_t in_bucket = (g - b * tiles_per_bucket) * kTileElems;  // offset of the tile in its bucket
    const size_t begin = first_elem + b * bucket_elems + in_bucket;
    const size_t rem = (b == n_buckets - 1 ? last_len : bucket_elems) - in_bucket;
    if (b != cur) {  // same for every lane of the block
      __syncthreads();                 // nobody still reads the previous bucket's table
      const unsigned long long mask = masks.mask[b];
      const unsigned r = threadIdx.x;
      if (r < static_cast<unsigned>(n_replicas) && ((mask >> r) & 1ull))
        s_tab[__popcll(mask & ((1ull << r) - 1ull))] = static_cast<T*>(all.p[r]);
      __syncthreads();
      cur = b;
      N = __popcll(mask);
      scale = scales.s[N];
    }
    bool done = false;
    if constexpr (VEC > 1) {
      done = true;
      switch (N) {
#define FTAR_CASE(n) case n: bucket_tile_n<T, VEC, n, POL>(s_tab, out, scale, begin, rem); break;
        FTAR_CASE(1) FTAR_CASE(2) FTAR_CASE(3) FTAR_CASE(4) FTAR_CASE(5) FTAR_CASE(6) FTAR_CASE(7)
        FTAR_CASE(8) FTAR_CASE(9) FTAR_CASE(10) FTAR_CASE(11) FTAR_CASE(12) FTAR_CASE(13)
        FTAR_CASE(14) FTAR_CASE(15) FTAR_CASE(16)
#undef FTAR_CASE
        default: done = false; break;
      }
    }
    if (!done) {
      if (rem >= kTileElems) sum_any_range<T, VEC, POL>(s_tab, begin, N, out + begin, scale, kTileElems, 0u, 1u, -0.0f);
      else sum_any_range<T, VEC, POL>(s_tab, begin, N, out + begin, scale, rem, 0u, 1u, -0.0f);
    }
  }
}

// The same tile with its results left in the LDS stage instead of memory: lane_stage points at this
// lane's slot of the first of the tile's kBucketUnroll result vectors; slots are kThreads apart.
template <typename T, int VEC, int N, int POL>
__device__ __forceinline__ void bucket_tile_n_staged(T* const* s_tab, float scale, size_t begin,
                                                     typename Raw<T, VEC>::type* lane_stage) {
  constexpr int UN = unroll_narrow(N) < kBucketUnroll ? unroll_narrow(N) : kBucketUnroll;
  typedef typename Raw<T, VEC>::type R;
  T* src[N];
#pragma unroll
  for (int j = 0; j < N; ++j) src[j] = uniform_ptr(s_tab[j]) + begin;
#pragma unroll
  for (int it = 0; it < kBucketUnroll / UN; ++it) {
    R res[UN];
    sum_tile_values<T, VEC, N, 0, UN, POL, false>(src, scale, static_cast<size_t>(it) * kThreads * UN + threadIdx.x,
                                                  0.0f, res);
#pragma unroll
    for (int u = 0; u < UN; ++u) lane_stage[(it * UN + u) * kThreads] = res[u];
  }
}

// k_reduce_bucketed with write windows (see WriteWindow): whole tiles leave their results in the LDS
// stage; they are written out inside the clock windows or when the stage is full.  Short tiles (the
// end of a bucket) are written directly, as in the plain kernel.  One workgroup per compute unit.
template <typename T, int VEC, int POL>
__global__ void __launch_bounds__(kThreads)
k_reduce_bucketed_win(PtrTable all, int n_replicas, BucketTable masks, ScaleTable scales,
                      size_t first_elem, size_t bucket_elems, size_t last_len, int n_buckets,
                      size_t tiles_per_bucket, size_t total_tiles, T* out, WriteWindow win) {
  typedef typename Raw<T, VEC>::type R;
  constexpr int kCapTiles = kStageBytes / (kThreads * static_cast<int>(sizeof(R)) * kBucketUnroll);
  __shared__ R stage[kCapTiles * kBucketUnroll][kThreads];
  __shared__ T* s_tab[kMaxReplicas];
  constexpr size_t kTileElems = static_cast<size_t>(kThreads) * kBucketUnroll * VEC;
  const unsigned tid = threadIdx.x;
  const size_t gx = gridDim.x;
  int cur = -1, N = 0;
  float scale = 0.0f;
  unsigned pending = 0;  // tiles staged
  size_t first = 0;      // flat index of the first staged tile; the others follow at distance gx,
                         // except that directly written tiles are skipped: `skipped` marks them
  unsigned skipped = 0;  // bit k: the k-th tile since `first` was written directly
  unsigned span = 0;     // tiles since `first`, staged or skipped
  for (size_t g = blockIdx.x; g < total_tiles; g += gx) {
    const unsigned now = static_cast<unsigned>(wall_clock64());
    const int b = static_cast<int>(g / tiles_per_bucket);
    const size_t in_bucket = (g - b * tiles_per_bucket) * kTileElems;
    const size_t begin = first_elem + b * bucket_elems + in_bucket;
    const size_t rem = (b == n_buckets - 1 ? last_len : bucket_elems) - in_bucket;
    if (b != cur) {
      __syncthreads();
      const unsigned long long mask = masks.mask[b];
      if (tid < static_cast<unsigned>(n_replicas) && ((mask >> tid) & 1ull))
        s_tab[__popcll(mask & ((1ull << tid) - 1ull))] = static_cast<T*>(all.p[tid]);
      __syncthreads();
      cur = b;
      N = __popcll(mask);
      scale = scales.s[N];
    }
    if (pending == 0) {
      first = g;
      skipped = 0;
      span = 0;
    }
    bool staged = false;
    if (rem >= kTileElems) {
      R* lane_stage = &stage[pending * kBucketUnroll][tid];
      staged = true;
      switch (N) {
#define FTAR_CASE(n) case n: bucket_tile_n_staged<T, VEC, n, POL>(s_tab, scale, begin, lane_stage); break;
        FTAR_CASE(1) FTAR_CASE(2) FTAR_CASE(3) FTAR_CASE(4) FTAR_CASE(5) FTAR_CASE(6) FTAR_CASE(7)
        FTAR_CASE(8) FTAR_CASE(9) FTAR_CASE(10) FTAR_CASE(11) FTAR_CASE(12) FTAR_CASE(13)
        FTAR_CASE(14) FTAR_CASE(15) FTAR_CASE(16)
#undef FTAR_CASE
        default:  // 17 to 64 live replicas: the generic sum, all of a vector's loads in flight (up to 32)
#pragma unroll
          for (int u = 0; u < kBucketUnroll; ++u)
            lane_stage[u * kThreads] =
                sum_any_value<T, VEC, POL, T, 32>(s_tab, begin, N, scale, tid + static_cast<size_t>(u) * kThreads, -0.0f);
          break;
      }
    }
    if (staged) {
      ++pending;
    } else {
      skipped |= 1u << span;
      if (rem >= kTileElems) sum_any_range<T, VEC, POL>(s_tab, begin, N, out + begin, scale, kTileElems, 0u, 1u, -0.0f);
      else sum_any_range<T, VEC, POL>(s_tab, begin, N, out + begin, scale, rem, 0u, 1u, -0.0f);
    }
    ++span;
    const bool window = (now & win.period_mask) < win.write_ticks && pending >= win.min_tiles;
    const bool last_iter = g + gx >= total_tiles;
    if (pending == static_cast<unsigned>(kCapTiles) || span == 32u || window || last_iter) {
      unsigned k = 0;
      for (unsigned i = 0; i < span; ++i) {
        if ((skipped >> i) & 1u) continue;
        const size_t gi = first + i * gx;
        const size_t bi = gi / tiles_per_bucket;
        R* o = reinterpret_cast<R*>(out + first_elem + bi * bucket_elems + (gi - bi * tiles_per_bucket) * kTileElems);
#pragma unroll
        for (int u = 0; u < kBucketUnroll; ++u) st<POL>(o + tid + u * kThreads, stage[k * kBucketUnroll + u][tid]);
        ++k;
      }
      pending = 0;
    }
  }
}

// Tuning flag bit 5 selects the wide tiles for the one-shot reduce (default: narrow).
bool wide_tiles() { return (current_tuning().flags & 0x20) != 0; }

template <typename T, int VEC>
struct ReduceFixed {
  const PtrTable& live; int N; size_t count; T* out; float scale; float zterm; hipStream_t stream;
  template <int POL> hipError_t operator()(unsigned blocks) const {
    const bool wide = wide_tiles();
    const int U = wide ? unroll_wide(N) : unroll_narrow(N);
    const size_t tiles = count / VEC / (static_cast<size_t>(kThreads) * U);
    const dim3 grid(grid_x_for(tiles, blocks)), block(kThreads);
    switch (N) {
#define FTAR_CASE(n)                                                                              \
  case n:                                                                                         \
    if (wide)                                                                                     \
      launch(k_reduce_masked<T, VEC, n, unroll_wide(n), POL>, grid, block, stream, live, out, scale, \
             count, zterm);                                                                       \
    else                                                                                          \
      launch(k_reduce_masked<T, VEC, n, unroll_narrow(n), POL>, grid, block, stream, live, out,    \
             scale, count, zterm);                                                                \
    break;
      FTAR_CASE(1) FTAR_CASE(2) FTAR_CASE(3) FTAR_CASE(4) FTAR_CASE(5) FTAR_CASE(6) FTAR_CASE(7)
      FTAR_CASE(8) FTAR_CASE(9) FTAR_CASE(10) FTAR_CASE(11) FTAR_CASE(12) FTAR_CASE(13)
      FTAR_CASE(14) FTAR_CASE(15) FTAR_CASE(16)
#undef FTAR_CASE
      default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
  }
};

template <typename T, int VEC, typename TO = T>
struct ReduceAny {
  const PtrTable& live; int N; size_t count; TO* out; float scale; float zterm; hipStream_t stream;
  template <int POL> hipError_t operator()(unsigned blocks) const {
    const size_t tiles = (count / VEC + kThreads - 1) / kThreads;
    const dim3 grid(grid_x_for(tiles, blocks)), block(kThreads);
    launch(k_reduce_masked_any<T, VEC, POL, TO>, grid, block, stream, live, N, out, scale, count, zterm);
    return hipGetLastError();
  }
};

// Result of the other element type: 4 elements per lane and vector.  bf16 inputs (8-byte loads)
// take the wide tiles, fp32 inputs (16-byte loads) the narrow ones: the same bytes in flight as the
// same-type kernel has.
template <typename TI>
struct ReduceFixedCvt {
  const PtrTable& live; int N; size_t count; void* out; float scale; float zterm; hipStream_t stream;
  template <int POL> hipError_t operator()(unsigned blocks) const {
    constexpr bool kWide = !__is_same(TI, float);
    const int U = kWide ? unroll_wide(N) : unroll_narrow(N);
    const size_t tiles = count / 4 / (static_cast<size_t>(kThreads) * U);
    const dim3 grid(grid_x_for(tiles, blocks)), block(kThreads);
    switch (N) {
#define FTAR_CASE(n)                                                                               \
  case n:                                                                                          \
    launch(k_reduce_masked_cvt<TI, 4, n, (kWide ? unroll_wide(n) : unroll_narrow(n)), POL>, grid, block, \
           stream, live, out, scale, count, zterm);                                                \
    break;
      FTAR_CASE(1) FTAR_CASE(2) FTAR_CASE(3) FTAR_CASE(4) FTAR_CASE(5) FTAR_CASE(6) FTAR_CASE(7)
      FTAR_CASE(8) FTAR_CASE(9) FTAR_CASE(10) FTAR_CASE(11) FTAR_CASE(12) FTAR_CASE(13)
      FTAR_CASE(14) FTAR_CASE(15) FTAR_CASE(16)
#undef FTAR_CASE
      default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
  }
};

// When the write windows are used and with which period (tuning flags for measurement: 0x80 never,
// 0x100000 whenever the kernel can; bits 12..15 = log2 of the period in ticks, bits 16..19 = log2 of
// period / window).  From six sources on they pay at every size beyond a few tiles per workgroup,
// together with non-temporal stores (8 x 64 Mi bf16, replica 3 dead: 6.16 -> 6.75 TB/s; 8 x 16 Mi:
// 5.46 -> 5.84; with ordinary stores, which a small output would otherwise get, nothing is gained;
// per-bucket masks, 8 x 64 Mi bf16: 5.8 -> 6.5).
// With four or five sources only when the whole output is too large for the Infinity Cache (4 + 1
// streams of 128 MiB: 6.3 TB/s plain, 5.7 staged; of 1 GiB: 5.5 and 5.7).  The period grows with
// the number of sources: the stage must hold what one period produces.
WriteWindow reduce_window(int n_src, size_t out_bytes) {
  const int flags = current_tuning().flags;
  WriteWindow w{0u, 0u, 0u};
  if (n_src < 4 || n_src > kMaxReplicas || (flags & 0x80) != 0) return w;
  if ((flags & 0x100000) == 0) {
    if (n_src < 6 && out_bytes <= 256 * kMiB) return w;
    if (out_bytes < 16 * kMiB) return w;
  }
  int lg = n_src > 16 ? 13 : n_src >= 6 ? 12 : 11;  // 82 us, 41 us, 20 us
  int div = n_src >= 6 ? 3 : 2;                     // window = period / 8, period / 4
  if ((flags >> 12) & 0xf) lg = (flags >> 12) & 0xf;
  if ((flags >> 16) & 0xf) div = (flags >> 16) & 0xf;
  w.period_mask = (1u << lg) - 1u;
  w.write_ticks = (1u << lg) >> div;
  w.min_tiles = 4;
  return w;
}

// MODE as in k_reduce_masked_win.  One workgroup per compute unit.
template <typename T, int VEC, int MODE>
struct ReduceWin {
  const PtrTable& live; int N; size_t count; void* out; float scale; float zterm; WriteWindow win; hipStream_t stream;
  template <int POL> hipError_t operator()(unsigned) const {
    // 8-byte loads (fp32 from bf16): twice the vectors for the same bytes in flight; tuning flag 0x20 too
    const bool wide = MODE == 2 || wide_tiles();
    const int U = wide ? unroll_wide(N) : unroll_narrow(N);
    const size_t tiles = count / VEC / (static_cast<size_t>(kThreads) * U);
    const dim3 grid(grid_x_for(tiles, static_cast<unsigned>(device_cu_count()))), block(kThreads);
    switch (N) {
#define FTAR_CASE(n)                                                                                        \
  case n:                                                                                                   \
    if (wide)                                                                                               \
      launch(k_reduce_masked_win<T, VEC, n, unroll_wide(n), POL, MODE>, grid, block, stream, live, out, scale, \
             count, zterm, win);                                                                            \
    else                                                                                                    \
      launch(k_reduce_masked_win<T, VEC, n, unroll_narrow(n), POL, MODE>, grid, block, stream, live, out,    \
             scale, count, zterm, win);                                                                     \
    break;
      FTAR_CASE(4) FTAR_CASE(5) FTAR_CASE(6) FTAR_CASE(7) FTAR_CASE(8) FTAR_CASE(9) FTAR_CASE(10)
      FTAR_CASE(11) FTAR_CASE(12) FTAR_CASE(13) FTAR_CASE(14) FTAR_CASE(15) FTAR_CASE(16)
#undef FTAR_CASE
      default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
  }
};

template <typename T, int VEC, typename TO>
struct ReduceAnyWin {
  const PtrTable& live; int N; size_t count; TO* out; float scale; float zterm; WriteWindow win; hipStream_t stream;
  template <int POL> hipError_t operator()(unsigned) const {
    const size_t tiles = count / VEC / kThreads;
    const dim3 grid(grid_x_for(tiles, static_cast<unsigned>(device_cu_count()))), block(kThreads);
    launch(k_reduce_masked_any_win<T, VEC, POL, TO>, grid, block, stream, live, N, out, scale, count, zterm, win);
    return hipGetLastError();
  }
};

// whole_out_bytes: output size of the whole call (a long call goes out as several launches)
template <typename TI, typename TO>
hipError_t reduce_masked_cvt(const PtrTable& live, int N, size_t count, bool vec, void* out, float scale,
                             float zterm, size_t whole_out_bytes, const WriteWindow& win, hipStream_t stream) {
  // staged results go out with non-temporal stores whatever the size (see reduce_window)
  const LaunchCfg cfg = vec && win.period_mask != 0 ? launch_cfg(1, 3) : reduce_cfg(N, whole_out_bytes);
  TO* o = static_cast<TO*>(out);
  if (vec && win.period_mask != 0 && N > 16)
    return with_policy(cfg, ReduceAnyWin<TI, 4, TO>{live, N, count, o, scale, zterm, win, stream});
  if (vec && win.period_mask != 0)
    return with_policy(cfg, ReduceWin<TI, 4, (__is_same(TI, float) ? 3 : 2)>{live, N, count, out, scale, zterm, win, stream});
  if (vec && N <= 16) return with_policy(cfg, ReduceFixedCvt<TI>{live, N, count, out, scale, zterm, stream});
  if (vec) return with_policy(cfg, ReduceAny<TI, 4, TO>{live, N, count, o, scale, zterm, stream});
  return with_policy(cfg, ReduceAny<TI, 1, TO>{live, N, count, o, scale, zterm, stream});
}

template <typename T, int VECW>
hipError_t reduce_masked_typed(const PtrTable& live, int N, size_t count, bool vec, void* out,
                               float scale, float zterm, size_t whole_out_bytes, const WriteWindow& win,
                               hipStream_t stream) {
  T* o = static_cast<T*>(out);
  const LaunchCfg cfg = vec && win.period_mask != 0 ? launch_cfg(1, 3) : reduce_cfg(N, whole_out_bytes);
  if (vec && win.period_mask != 0 && N > 16)
    return with_policy(cfg, ReduceAnyWin<T, VECW, T>{live, N, count, o, scale, zterm, win, stream});
  if (vec && win.period_mask != 0)
    return with_policy(cfg, ReduceWin<T, VECW, 0>{live, N, count, out, scale, zterm, win, stream});
  if (vec && N <= 16) return with_policy(cfg, ReduceFixed<T, VECW>{live, N, count, o, scale, zterm, stream});
  if (vec) return with_policy(cfg, ReduceAny<T, VECW>{live, N, count, o, scale, zterm, stream});
  return with_policy(cfg, ReduceAny<T, 1>{live, N, count, o, scale, zterm, stream});
}

template <typename T, int VEC>
struct Bucketed {
  const PtrTable& all; int n_replicas; const BucketTable& masks; int n_buckets; size_t first_elem;
  size_t bucket_elems; size_t count; const ScaleTable& scales; T* out; WriteWindow win; hipStream_t stream;
  template <int POL> hipError_t operator()(unsigned blocks) const {
    const size_t tile_elems = static_cast<size_t>(kThreads) * kBucketUnroll * VEC;
    const size_t tiles_per_bucket = (bucket_elems + tile_elems - 1) / tile_elems;
    const size_t last_begin = first_elem + static_cast<size_t>(n_buckets - 1) * bucket_elems;
    const size_t last_len = count - last_begin < bucket_elems ? count - last_begin : bucket_elems;
    const size_t tiles = static_cast<size_t>(n_buckets - 1) * tiles_per_bucket +
                         (last_len + tile_elems - 1) / tile_elems;
    if constexpr (VEC > 1) {
      if (win.period_mask != 0) {  // staged results, one workgroup per compute unit
        const dim3 grid(grid_x_for(tiles, static_cast<unsigned>(device_cu_count()))), block(kThreads);
        launch(k_reduce_bucketed_win<T, VEC, POL>, grid, block, stream, all, n_replicas, masks, scales, first_elem,
               bucket_elems, last_len, n_buckets, tiles_per_bucket, tiles, out, win);
        return hipGetLastError();
      }
    }
    const dim3 grid(grid_x_for(tiles, blocks)), block(kThreads);
    launch(k_reduce_bucketed<T, VEC, POL>, grid, block, stream, all, n_replicas, masks, scales,
                                                               first_elem, bucket_elems, last_len,
                                                               n_buckets, tiles_per_bucket, tiles, out);
    return hipGetLastError();
  }
};

template <typename T, int VECW>
hipError_t bucketed_typed(const PtrTable& all, int n_replicas, const BucketTable& masks,
                          int n_buckets, size_t first_elem, size_t bucket_elems, size_t count,
                          const ScaleTable& scales, bool vec, void* out, hipStream_t stream) {
  T* o = static_cast<T*>(out);
  const WriteWindow win = reduce_window(n_replicas, count * sizeof(T));
  // staged results: non-temporal stores whatever the size (8 x 64 Mi bf16, buckets of 25 Mi: 5.8 -> 6.5 TB/s)
  const LaunchCfg cfg = vec && win.period_mask != 0 ? launch_cfg(1, 3) : bucketed_cfg(n_replicas, count * sizeof(T));
  if (vec)
    return with_policy(cfg, Bucketed<T, VECW>{all, n_replicas, masks, n_buckets, first_elem, bucket_elems, count,
                                              scales, o, win, stream});
  return with_policy(cfg, Bucketed<T, 1>{all, n_replicas, masks, n_buckets, first_elem, bucket_elems, count,
                                         scales, o, WriteWindow{0u, 0u, 0u}, stream});
}

}  // namespace

hipError_t launch_reduce_masked(const PtrTable& live, int n_src, size_t count, ftar_dtype_t dtype,
                                ftar_dtype_t out_dtype, bool vec, void* out, float scale,
                                bool zero_participants, size_t whole_count, hipStream_t stream) {
  if (whole_count < count) whole_count = count;
  if (n_src == 0) {  // nothing to read; bf16 buffers are only 2-byte aligned: head/tail by halves
    if (!zero_participants) return hipErrorInvalidValue;
    const size_t bytes = count * (out_dtype == FTAR_F32 ? 4 : 2);
    char* o = static_cast<char*>(out);
    uint16_t *head = nullptr, *odd = nullptr;
    size_t left = bytes;
    if (reinterpret_cast<uintptr_t>(o) % 4 != 0) {  // 2-byte aligned bf16: first half alone
      head = reinterpret_cast<uint16_t*>(o);
      o += 2;
      left -= 2;
    }
    const size_t n32 = left / 4;
    if (left % 4) odd = reinterpret_cast<uint16_t*>(o + n32 * 4);
    const unsigned blocks = static_cast<unsigned>(std::min<size_t>((n32 + kThreads - 1) / kThreads + 1,
                                                                  static_cast<size_t>(device_cu_count()) * 8));
    launch(k_fill_zero, dim3(blocks), dim3(kThreads), stream, head, reinterpret_cast<uint32_t*>(o), n32, odd);
    return hipGetLastError();
  }
  const float zterm = zero_participants ? 0.0f : -0.0f;
  // A long reduction goes out as several launches of about 1 GiB of traffic each.  The blocks of
  // a launch stride over their tiles without ever waiting for each other; over some 100 MiB per
  // stream they drift apart, the window of addresses in use widens and the DRAM sees less
  // locality (8 x 2e9 bf16: 5.14 TB/s as one launch, 5.65 TB/s in launches of 128 MiB per stream).
  // Tuning flag 0x40 forces one launch.
  const size_t es_in = dtype == FTAR_F32 ? 4 : 2, es_out = out_dtype == FTAR_F32 ? 4 : 2;
  const WriteWindow win = reduce_window(n_src, whole_count * es_out);
  size_t chunk = (static_cast<size_t>(1) << 30) / (static_cast<size_t>(n_src) * es_in + es_out);
  chunk &= ~static_cast<size_t>(0xffff);  // whole tiles of every shape, 16-byte aligned in both types
  // (with write windows the workgroups meet at every window: one launch is then best, 6.4 -> 6.6 TB/s)
  if ((current_tuning().flags & 0x40) != 0 || count <= chunk + chunk / 2 || win.period_mask != 0) chunk = count;
  hipEvent_t t_start = nullptr, t_stop = nullptr;
  if (chunk < count) take_timing_events(&t_start, &t_stop);
  for (size_t first = 0; first < count; first += chunk) {
    const size_t len = count - first < chunk + chunk / 2 ? count - first : chunk;  // no short last launch
    PtrTable part = live;
    for (int j = 0; j < n_src; ++j) part.p[j] = static_cast<char*>(live.p[j]) + first * es_in;
    void* o = static_cast<char*>(out) + first * es_out;
    if (chunk < count)  // the events of a timed call bracket the whole series
      set_timing_events(first == 0 ? t_start : nullptr, first + len >= count ? t_stop : nullptr);
    hipError_t e;
    if (out_dtype != dtype && dtype == FTAR_BF16)
      e = reduce_masked_cvt<bf16, float>(part, n_src, len, vec, o, scale, zterm, whole_count * es_out, win, stream);
    else if (out_dtype != dtype)
      e = reduce_masked_cvt<float, bf16>(part, n_src, len, vec, o, scale, zterm, whole_count * es_out, win, stream);
    else if (dtype == FTAR_F32)
      e = reduce_masked_typed<float, 4>(part, n_src, len, vec, o, scale, zterm, whole_count * es_out, win, stream);
    else
      e = reduce_masked_typed<bf16, 8>(part, n_src, len, vec, o, scale, zterm, whole_count * es_out, win, stream);
    if (e != hipSuccess) return e;
    if (len != chunk) break;
  }
  return hipSuccess;
}

hipError_t launch_reduce_bucketed(const PtrTable& all, int n_replicas, const BucketTable& masks,
                                  int n_buckets, size_t first_elem, size_t bucket_elems,
                                  size_t count, const ScaleTable& scales, ftar_dtype_t dtype,
                                  bool vec, void* out, hipStream_t stream) {
  if (dtype == FTAR_F32)
    return bucketed_typed<float, 4>(all, n_replicas, masks, n_buckets, first_elem, bucket_elems,
                                    count, scales, vec, out, stream);
  return bucketed_typed<bf16, 8>(all, n_replicas, masks, n_buckets, first_elem, bucket_elems, count,
                                 scales, vec, out, stream);
}

}  // namespace ftar
