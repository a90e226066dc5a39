// HIP kernels (gfx950 / CDNA4) of the FTAR data path and their launchers.
//
// Everything here is a streaming, HBM-bandwidth-bound elementwise pass: a few
// fp32 additions per 16-byte load, no data reuse, no contraction - so no MFMA
// and no LDS tiling of data.  What matters is (1) every wave instruction
// touching a contiguous run of full cache lines (lane t reads 16 bytes at
// 16*t: 1 KiB per wave instruction), (2) many independent loads in flight per
// lane before the first use (the paper's instruction-level-parallelism remark,
// section 4.2 "Optimizations", applied at full rather than minimal occupancy),
// (3) a persistent grid that strides over tiles so consecutive tiles are in
// flight on different XCDs at the same time, and (4) non-temporal accesses,
// since no byte is touched twice.  LDS holds only the compact pointer table the
// CPU resolved from the live mask; pointers are pulled from it into scalar
// registers, so address arithmetic stays on the scalar unit.
//
// Arithmetic contract (identical in every kernel): exact widening to fp32,
// fp32 additions in the stated order starting from the first operand, one
// multiplication by `scale`, one rounding (nearest-even) to the output type.
// Compiled with -ffp-contract=off; fp32 denormals are not flushed.

#include <hip/hip_ext.h>

#include "ftar_internal.h"

namespace ftar {
namespace {

constexpr int kThreads = 256;          // 4 waves of 64 lanes: one per SIMD of a CU

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

struct bf16 {  // storage tag: the upper 16 bits of an IEEE-754 binary32
  uint16_t bits;
};

// Raw<T, VEC>: the register image of VEC consecutive elements of T.
template <typename T, int VEC> struct Raw;
template <> struct Raw<float, 4> { typedef f32x4 type; };
template <> struct Raw<float, 1> { typedef float type; };
template <> struct Raw<bf16, 8> { typedef u32x4 type; };
template <> struct Raw<bf16, 4> { typedef u32x2 type; };
template <> struct Raw<bf16, 1> { typedef uint16_t type; };

template <int POL, typename R>
__device__ __forceinline__ R ld(const R* p) {
  if constexpr ((POL & 1) != 0) return __builtin_nontemporal_load(p);
  else return *p;
}

template <int POL, typename R>
__device__ __forceinline__ void st(R* p, R v) {
  if constexpr ((POL & 2) != 0) __builtin_nontemporal_store(v, p);
  else *p = v;
}

// ---- widening: exact -------------------------------------------------------
__device__ __forceinline__ void widen(f32x4 r, float (&x)[4]) {
  x[0] = r[0]; x[1] = r[1]; x[2] = r[2]; x[3] = r[3];
}
__device__ __forceinline__ void widen(float r, float (&x)[1]) { x[0] = r; }
__device__ __forceinline__ void widen(u32x4 r, float (&x)[8]) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    x[2 * i] = __uint_as_float(r[i] << 16);
    x[2 * i + 1] = __uint_as_float(r[i] & 0xffff0000u);
  }
}
__device__ __forceinline__ void widen(u32x2 r, float (&x)[4]) {
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    x[2 * i] = __uint_as_float(r[i] << 16);
    x[2 * i + 1] = __uint_as_float(r[i] & 0xffff0000u);
  }
}
__device__ __forceinline__ void widen(uint16_t r, float (&x)[1]) {
  x[0] = __uint_as_float(static_cast<uint32_t>(r) << 16);
}

// ---- narrowing: round to nearest, ties to even; NaN stays a (quiet) NaN ------
__device__ __forceinline__ uint32_t bf16_rne(float f) {
  const uint32_t u = __float_as_uint(f);
  const uint32_t rounded = (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
  const uint32_t quiet = ((u >> 16) | 0x40u) & 0xffffu;
  return ((u & 0x7fffffffu) > 0x7f800000u) ? quiet : rounded;
}

template <typename R, int VEC>
__device__ __forceinline__ R narrow(const float (&x)[VEC]) {
  if constexpr (__is_same(R, f32x4)) {
    f32x4 r = {x[0], x[1], x[2], x[3]};
    return r;
  } else if constexpr (__is_same(R, float)) {
    return x[0];
  } else if constexpr (__is_same(R, u32x4)) {
    u32x4 r;
#pragma unroll
    for (int i = 0; i < 4; ++i) r[i] = bf16_rne(x[2 * i]) | (bf16_rne(x[2 * i + 1]) << 16);
    return r;
  } else if constexpr (__is_same(R, u32x2)) {
    u32x2 r;
#pragma unroll
    for (int i = 0; i < 2; ++i) r[i] = bf16_rne(x[2 * i]) | (bf16_rne(x[2 * i + 1]) << 16);
    return r;
  } else {
    return static_cast<uint16_t>(bf16_rne(x[0]));
  }
}

// A pointer read from LDS is the same in every lane: move it to scalar registers.
template <typename P>
__device__ __forceinline__ P* uniform_ptr(P* p) {
  const uint64_t u = reinterpret_cast<uint64_t>(p);
  const uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(u));
  const uint32_t hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(u >> 32));
  return reinterpret_cast<P*>((static_cast<uint64_t>(hi) << 32) | lo);
}

// ---- one tile of the sum --------------------------------------------------
// For U vectors per lane (vector v + u*kThreads):
//   a = ACC_IN ? acc_in : x_0 ;  a = a + x_j for the remaining sources in order;
//   ACC_OUT == 1: acc_out = a (fp32, unscaled);  ACC_OUT == 0: out = cvt(scale * a);
//   ACC_OUT == 2: acc_out = scale * a (fp32 result from any input type)
// Every load of the tile is issued before the first use.  `out` may alias
// src[NSRC-1] (the in-place last ReduceScatter step): a lane only ever writes
// the elements it has itself already loaded.
// zm: bit j set = source j is a zero-gradient participant: it contributes +0.0 and its buffer is
// not read (the pointer may be anything).  The bits are the same for the whole wave.
// ZM = false compiles the loads without the tests (zm is then ignored): callers pick it when zm == 0.
// ZT = true adds `zterm` to the finished sum before it is scaled: +0.0 when zero-gradient
// participants were left out of src altogether, -0.0 (the identity of IEEE addition) otherwise.
// x_1 + ... + x_n with +0.0 terms anywhere in between equals (x_1 + ... + x_n) + 0.0 bit for bit:
// a +0.0 term only ever changes a running sum of -0.0, and that happens iff every x_i is -0.0.
template <typename T, int VEC, int NSRC, bool ACC_IN, int ACC_OUT, int U, int POL, bool ZM = false,
          bool ZT = false>
__device__ __forceinline__ void sum_tile(T* const (&src)[NSRC], const float* acc_in, float* acc_out,
                                         T* out, float scale, size_t v, unsigned long long zm = 0,
                                         float zterm = 0.0f) {
  static_assert(!(ACC_IN || ACC_OUT) || VEC <= 4, "fp32 partials are moved 4 at a time");
  typedef typename Raw<T, VEC>::type R;
  typedef typename Raw<float, (VEC == 1 ? 1 : 4)>::type A;
  R raw[U][NSRC];
  A ain[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
#pragma unroll
    for (int j = 0; j < NSRC; ++j) {
      if (ZM && ((zm >> j) & 1ull)) raw[u][j] = R{};  // all-zero bits are +0.0 in both element types
      else raw[u][j] = ld<POL>(reinterpret_cast<const R*>(src[j]) + v + u * kThreads);
    }
  }
  if constexpr (ACC_IN) {
#pragma unroll
    for (int u = 0; u < U; ++u) ain[u] = ld<POL>(reinterpret_cast<const A*>(acc_in) + v + u * kThreads);
  }
#pragma unroll
  for (int u = 0; u < U; ++u) {
    float a[VEC], x[VEC];
    if constexpr (ACC_IN) widen(ain[u], a);
    else widen(raw[u][0], a);
#pragma unroll
    for (int j = (ACC_IN ? 0 : 1); j < NSRC; ++j) {
      widen(raw[u][j], x);
#pragma unroll
      for (int e = 0; e < VEC; ++e) a[e] = a[e] + x[e];
    }
    if constexpr (ACC_OUT == 1) {
      st<POL>(reinterpret_cast<A*>(acc_out) + v + u * kThreads, narrow<A, VEC>(a));
    } else {
      if constexpr (ZT) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) a[e] = a[e] + zterm;
      }
#pragma unroll
      for (int e = 0; e < VEC; ++e) a[e] = a[e] * scale;
      if constexpr (ACC_OUT == 2) st<POL>(reinterpret_cast<A*>(acc_out) + v + u * kThreads, narrow<A, VEC>(a));
      else st<POL>(reinterpret_cast<R*>(out) + v + u * kThreads, narrow<R, VEC>(a));
    }
  }
}

// Persistent loop of block bx of gx over the `len` elements that start at the
// given pointers: full tiles grid-strided, then one block finishes the whole
// vectors past the last full tile and the last len % VEC single elements.
template <typename T, int VEC, int NSRC, bool ACC_IN, int ACC_OUT, int U, int POL, bool ZM,
          bool ZT = false>
__device__ __forceinline__ void sum_range_z(T* const (&src)[NSRC], const float* acc_in, float* acc_out,
                                            T* out, float scale, size_t len, unsigned bx,
                                            unsigned gx, unsigned long long zm, float zterm = 0.0f) {
  const unsigned tid = threadIdx.x;
  const size_t n_vec = len / VEC;
  constexpr size_t kTile = static_cast<size_t>(kThreads) * U;
  const size_t n_tiles = n_vec / kTile;
  for (size_t t = bx; t < n_tiles; t += gx)
    sum_tile<T, VEC, NSRC, ACC_IN, ACC_OUT, U, POL, ZM, ZT>(src, acc_in, acc_out, out, scale, t * kTile + tid, zm, zterm);
  if (bx == n_tiles % gx) {
    for (size_t v = n_tiles * kTile + tid; v < n_vec; v += kThreads)
      sum_tile<T, VEC, NSRC, ACC_IN, ACC_OUT, 1, POL, ZM, ZT>(src, acc_in, acc_out, out, scale, v, zm, zterm);
    if constexpr (VEC > 1) {
      const size_t e = n_vec * VEC + tid;
      if (e < len) sum_tile<T, 1, NSRC, ACC_IN, ACC_OUT, 1, POL, ZM, ZT>(src, acc_in, acc_out, out, scale, e, zm, zterm);
    }
  }
}

template <typename T, int VEC, int NSRC, bool ACC_IN, bool ACC_OUT, int U, int POL>
__device__ __forceinline__ void sum_range(T* const (&src)[NSRC], const float* acc_in, float* acc_out,
                                          T* out, float scale, size_t len, unsigned bx,
                                          unsigned gx, unsigned long long zm = 0) {
  if (zm == 0) sum_range_z<T, VEC, NSRC, ACC_IN, ACC_OUT, U, POL, false>(src, acc_in, acc_out, out, scale, len, bx, gx, 0);
  else sum_range_z<T, VEC, NSRC, ACC_IN, ACC_OUT, U, POL, true>(src, acc_in, acc_out, out, scale, len, bx, gx, zm);
}

// Vectors per lane per tile for an N-source sum.  Two choices per N are compiled: "wide"
// (about 16 x 16-byte loads in flight per lane) and "narrow" (half of that).
__host__ __device__ constexpr int unroll_wide(int n_src) {
  return n_src <= 2 ? 8 : n_src <= 4 ? 4 : n_src <= 8 ? 2 : 1;
}
__host__ __device__ constexpr int unroll_narrow(int n_src) {
  return unroll_wide(n_src) > 1 ? unroll_wide(n_src) / 2 : 1;
}

// ---- any number of sources (runtime N): loads in groups of 8 ---------------
template <typename T, int VEC, int POL, typename TO = T>
__device__ __forceinline__ void sum_any_one(T* const* s_tab, size_t base, int N, TO* out, float scale,
                                            size_t v, float zterm) {
  typedef typename Raw<T, VEC>::type R;
  typedef typename Raw<TO, VEC>::type RO;
  float a[VEC];
  for (int j0 = 0; j0 < N; j0 += 8) {
    R raw[8];
#pragma unroll
    for (int jj = 0; jj < 8; ++jj)
      if (j0 + jj < N) raw[jj] = ld<POL>(reinterpret_cast<const R*>(uniform_ptr(s_tab[j0 + jj]) + base) + v);
#pragma unroll
    for (int jj = 0; jj < 8; ++jj) {
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
  for (int e = 0; e < VEC; ++e) a[e] = (a[e] + zterm) * scale;
  st<POL>(reinterpret_cast<RO*>(out) + v, narrow<RO, VEC>(a));
}

template <typename T, int VEC, int POL, typename TO = T>
__device__ __forceinline__ void sum_any_range(T* const* s_tab, size_t base, int N, TO* out, float scale,
                                              size_t len, unsigned bx, unsigned gx, float zterm) {
  const size_t n_vec = len / VEC;
  for (size_t v = static_cast<size_t>(bx) * kThreads + threadIdx.x; v < n_vec;
       v += static_cast<size_t>(gx) * kThreads)
    sum_any_one<T, VEC, POL, TO>(s_tab, base, N, out, scale, v, zterm);
  if constexpr (VEC > 1) {
    if (bx == 0) {
      const size_t e = n_vec * VEC + threadIdx.x;
      if (e < len) sum_any_one<T, 1, POL, TO>(s_tab, base, N, out, scale, e, zterm);
    }
  }
}

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

// The same with an fp32 result from bf16 inputs: 8-byte loads, 16-byte stores.
template <int VEC, int N, int U, int POL>
__global__ void __launch_bounds__(kThreads)
k_reduce_masked_f32out(PtrTable live, float* out, float scale, size_t count, float zterm) {
  __shared__ bf16* s_tab[kMaxReplicas];
  if (threadIdx.x < static_cast<unsigned>(N)) s_tab[threadIdx.x] = static_cast<bf16*>(live.p[threadIdx.x]);
  __syncthreads();
  bf16* src[N];
#pragma unroll
  for (int j = 0; j < N; ++j) src[j] = uniform_ptr(s_tab[j]);
  sum_range_z<bf16, VEC, N, false, 2, U, POL, false, true>(src, nullptr, out, nullptr, scale, count,
                                                           blockIdx.x, gridDim.x, 0, zterm);
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

__device__ __forceinline__ unsigned long long uniform_u64(unsigned long long x) {
  const uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(x));
  const uint32_t hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(x >> 32));
  return (static_cast<unsigned long long>(hi) << 32) | lo;
}

// One block-wide tile starting at the given pointers, `rem` = elements left in the portion
// from there: the unrolled body when a whole tile is left, the checked loop over `rem` otherwise.
// (Written as a branch on `rem`, not as min(rem, tile): hipcc 7.2 miscompiles a select on a
// wave-uniform 64-bit unsigned compare here, reading a stale SCC.)
template <typename T, int VEC, int NSRC, bool ACC_IN, bool ACC_OUT, int U, int POL>
__device__ __forceinline__ void sum_block_tile(T* const (&src)[NSRC], const float* acc_in,
                                               float* acc_out, T* out, float scale, size_t rem,
                                               unsigned long long zm = 0) {
  if (rem >= static_cast<size_t>(kThreads) * U * VEC) {
    if (zm == 0) sum_tile<T, VEC, NSRC, ACC_IN, ACC_OUT, U, POL, false>(src, acc_in, acc_out, out, scale, threadIdx.x, 0);
    else sum_tile<T, VEC, NSRC, ACC_IN, ACC_OUT, U, POL, true>(src, acc_in, acc_out, out, scale, threadIdx.x, zm);
  } else {
    sum_range<T, VEC, NSRC, ACC_IN, ACC_OUT, 1, POL>(src, acc_in, acc_out, out, scale, rem, 0u, 1u, zm);
  }
}

// The kernels below walk the whole element range as ONE sequence of tiles, grid-strided, and
// look up which portion (or bucket) a tile belongs to.  All blocks then work inside one narrow
// moving window of `acc` and of one or two replica buffers, which keeps few DRAM rows open;
// giving every portion its own share of the grid instead opens N windows in 2N buffers at once
// and costs about 10 % of the bandwidth at 16 portions.

constexpr int kBucketUnroll = 4;  // vectors per lane in one tile of the bucketed kernel

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

// Portion lookup shared by the ring kernels: tile g of the flat sequence -> portion k and the
// tile's first element.  s_tile[k] = number of tiles before portion k.
struct RingTile {
  int k;
  size_t begin, rem;  // rem = elements from `begin` to the end of portion k (may exceed one tile)
};

template <size_t kTileElems>
__device__ __forceinline__ RingTile ring_tile_of(size_t g, int& k, size_t& next,
                                                 const unsigned long long* s_seg,
                                                 const unsigned long long* s_tile) {
  while (g >= next) {  // also steps over empty portions
    ++k;
    next = uniform_u64(s_tile[k + 1]);
  }
  const size_t begin = uniform_u64(s_seg[k]) + (g - uniform_u64(s_tile[k])) * kTileElems;
  return RingTile{k, begin, uniform_u64(s_seg[k + 1]) - begin};
}

// Stages the ring's pointer table, portion boundaries and tile prefix in LDS (block-wide).
template <typename T>
__device__ __forceinline__ void stage_ring_tables(const PtrTable& ring, const SegTable& seg,
                                                  const SegTable& tile0, int N, T** s_tab,
                                                  unsigned long long* s_seg,
                                                  unsigned long long* s_tile) {
  const unsigned tid = threadIdx.x;
  if (tid < static_cast<unsigned>(N)) s_tab[tid] = static_cast<T*>(ring.p[tid]);
  if (tid <= static_cast<unsigned>(N)) {
    s_seg[tid] = seg.begin[tid];
    s_tile[tid] = tile0.begin[tid];
  }
  __syncthreads();
}

// Block bx of gx's share of one ReduceScatter step: tiles bx, bx + gx, ...
template <typename T, int VEC, int MODE, int U, int POL>
__device__ __forceinline__ void ring_reduce_pass(T* const* s_tab, const unsigned long long* s_seg,
                                                 const unsigned long long* s_tile, int N, int step,
                                                 float* acc, float scale, unsigned bx, unsigned gx,
                                                 size_t buf_off = 0, unsigned long long zpos = 0) {
  // zpos: bit p set = the replica at ring position p is a zero-gradient participant
  // buf_off: first element of the partition in the replica buffers (acc is partition-relative)
  constexpr size_t kTileElems = static_cast<size_t>(kThreads) * U * VEC;
  const size_t total = uniform_u64(s_tile[N]);
  int k = 0;
  size_t next = uniform_u64(s_tile[1]);
  for (size_t g = bx; g < total; g += gx) {
    const RingTile t = ring_tile_of<kTileElems>(g, k, next, s_seg, s_tile);
    float* a = acc + t.begin;  // never dereferenced in the N == 2 mode
    const size_t b0 = buf_off + t.begin;
    if constexpr (MODE == kRsFirst) {
      const int p1 = (t.k + 1) % N;
      T* src[2] = {uniform_ptr(s_tab[t.k]) + b0, uniform_ptr(s_tab[p1]) + b0};
      const unsigned long long zm = ((zpos >> t.k) & 1ull) | (((zpos >> p1) & 1ull) << 1);
      sum_block_tile<T, VEC, 2, false, true, U, POL>(src, nullptr, a, nullptr, scale, t.rem, zm);
    } else if constexpr (MODE == kRsMid) {
      const int p = (t.k + step + 1) % N;
      T* src[1] = {uniform_ptr(s_tab[p]) + b0};
      sum_block_tile<T, VEC, 1, true, true, U, POL>(src, a, a, nullptr, scale, t.rem, (zpos >> p) & 1ull);
    } else if constexpr (MODE == kRsLast) {
      const int p = (t.k + N - 1) % N;
      T* src[1] = {uniform_ptr(s_tab[p]) + b0};
      sum_block_tile<T, VEC, 1, true, false, U, POL>(src, a, nullptr, src[0], scale, t.rem, (zpos >> p) & 1ull);
    } else {  // kRsOnly, N == 2
      const int p1 = (t.k + 1) % N;
      T* src[2] = {uniform_ptr(s_tab[t.k]) + b0, uniform_ptr(s_tab[p1]) + b0};
      const unsigned long long zm = ((zpos >> t.k) & 1ull) | (((zpos >> p1) & 1ull) << 1);
      sum_block_tile<T, VEC, 2, false, false, U, POL>(src, nullptr, nullptr, src[1], scale, t.rem, zm);
    }
  }
}

// Block bx of gx's share of one AllGather step: bit copy from ring position k+t-1 to k+t.
template <typename T, int VEC, int U, int POL>
__device__ __forceinline__ void ring_allgather_pass(T* const* s_tab, const unsigned long long* s_seg,
                                                    const unsigned long long* s_tile, int N, int step,
                                                    unsigned bx, unsigned gx, size_t buf_off = 0) {
  typedef typename Raw<T, VEC>::type R;
  typedef typename Raw<T, 1>::type R1;
  constexpr size_t kTileElems = static_cast<size_t>(kThreads) * U * VEC;
  const unsigned tid = threadIdx.x;
  const size_t total = uniform_u64(s_tile[N]);
  int k = 0;
  size_t next = uniform_u64(s_tile[1]);
  for (size_t g = bx; g < total; g += gx) {
    const RingTile t = ring_tile_of<kTileElems>(g, k, next, s_seg, s_tile);
    const T* from = uniform_ptr(s_tab[(t.k + step + N - 1) % N]) + buf_off + t.begin;
    T* to = uniform_ptr(s_tab[(t.k + step) % N]) + buf_off + t.begin;
    if (t.rem >= kTileElems) {
      R raw[U];
#pragma unroll
      for (int u = 0; u < U; ++u) raw[u] = ld<POL>(reinterpret_cast<const R*>(from) + tid + u * kThreads);
#pragma unroll
      for (int u = 0; u < U; ++u) st<POL>(reinterpret_cast<R*>(to) + tid + u * kThreads, raw[u]);
    } else {
      const size_t n_vec = t.rem / VEC;
      for (size_t v = tid; v < n_vec; v += kThreads)
        st<POL>(reinterpret_cast<R*>(to) + v, ld<POL>(reinterpret_cast<const R*>(from) + v));
      if constexpr (VEC > 1) {
        const size_t e = n_vec * VEC + tid;
        if (e < t.rem) reinterpret_cast<R1*>(to)[e] = reinterpret_cast<const R1*>(from)[e];
      }
    }
  }
}

// One ReduceScatter step over all N portions.
template <typename T, int VEC, int MODE, int U, int POL>
__global__ void __launch_bounds__(kThreads)
k_ring_reduce(PtrTable ring, SegTable seg, SegTable tile0, int N, int step, float* acc, float scale,
              unsigned long long zpos) {
  __shared__ T* s_tab[kMaxReplicas];
  __shared__ unsigned long long s_seg[kMaxReplicas + 1], s_tile[kMaxReplicas + 1];
  stage_ring_tables<T>(ring, seg, tile0, N, s_tab, s_seg, s_tile);
  ring_reduce_pass<T, VEC, MODE, U, POL>(s_tab, s_seg, s_tile, N, step, acc, scale, blockIdx.x, gridDim.x, 0,
                                         zpos);
}

// One AllGather step over all N portions.
template <typename T, int VEC, int U, int POL>
__global__ void __launch_bounds__(kThreads)
k_ring_allgather(PtrTable ring, SegTable seg, SegTable tile0, int N, int step) {
  __shared__ T* s_tab[kMaxReplicas];
  __shared__ unsigned long long s_seg[kMaxReplicas + 1], s_tile[kMaxReplicas + 1];
  stage_ring_tables<T>(ring, seg, tile0, N, s_tab, s_seg, s_tile);
  ring_allgather_pass<T, VEC, U, POL>(s_tab, s_seg, s_tile, N, step, blockIdx.x, gridDim.x);
}

// ---- the ring's result in one pass ------------------------------------------------
// On one device nothing forces the 2N-2 steps to be separate passes over memory: the partial sum
// of an element can stay in a register while its N contributions are added in the ring's order
// (portion k: positions k, k+1, ..., k+N-1 mod N), and the rounded mean can be written straight
// into all N replica buffers.  Same bits as the step schedule, 2*N*E bytes per element instead
// of 4*N*E + 10*N - 20 (N = 16, bf16: 64 instead of 206).
template <typename T, int VEC, int N, int U, int POL, bool ZM>
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
#pragma unroll
    for (int j = 0; j < N; ++j) st<POL>(reinterpret_cast<R*>(buf[j]) + v + u * kThreads, r);
  }
}

// Any N (runtime): loads in groups of 8 in ring order starting at position k, then N stores.
template <typename T, int VEC, int POL>
__device__ __forceinline__ void onepass_any_one(T* const* s_tab, int N, int k, size_t base, float scale,
                                                size_t v, unsigned long long zpos) {
  typedef typename Raw<T, VEC>::type R;
  float a[VEC];
  for (int j0 = 0; j0 < N; j0 += 8) {
    R raw[8];
#pragma unroll
    for (int jj = 0; jj < 8; ++jj)
      if (j0 + jj < N) {
        const int p = (k + j0 + jj) % N;
        if ((zpos >> p) & 1ull) raw[jj] = R{};
        else raw[jj] = ld<POL>(reinterpret_cast<const R*>(uniform_ptr(s_tab[p]) + base) + v);
      }
#pragma unroll
    for (int jj = 0; jj < 8; ++jj) {
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
  for (int j = 0; j < N; ++j) st<POL>(reinterpret_cast<R*>(uniform_ptr(s_tab[j]) + base) + v, r);
}

template <typename T, int VEC, int POL>
__device__ __forceinline__ void onepass_any_range(T* const* s_tab, int N, int k, size_t base, float scale,
                                                  size_t len, unsigned long long zpos) {
  const size_t n_vec = len / VEC;
  for (size_t v = threadIdx.x; v < n_vec; v += kThreads)
    onepass_any_one<T, VEC, POL>(s_tab, N, k, base, scale, v, zpos);
  if constexpr (VEC > 1) {
    const size_t e = n_vec * VEC + threadIdx.x;
    if (e < len) onepass_any_one<T, 1, POL>(s_tab, N, k, base, scale, e, zpos);
  }
}

// NT = compile-time N for the unrolled tile (1..16), or 0: any N through the grouped loop.
template <typename T, int VEC, int NT, int POL>
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
        if (zm == 0) onepass_tile<T, VEC, NT, U, POL, false>(buf, scale, threadIdx.x, 0);
        else onepass_tile<T, VEC, NT, U, POL, true>(buf, scale, threadIdx.x, zm);
        continue;
      }
    }
    if (t.rem >= kTileElems) onepass_any_range<T, VEC, POL>(s_tab, N, t.k, t.begin, scale, kTileElems, zpos);
    else onepass_any_range<T, VEC, POL>(s_tab, N, t.k, t.begin, scale, t.rem, zpos);
  }
}

// ---- the whole ring as one CPU-gated persistent kernel ----------------------------
// The data is handled in partitions (paper section 4.2: the message is split into partitions of
// at most S x C x N bytes; each partition runs one full round of the ring, then the next one
// starts).  A "slot" is one step of one partition; slots run in order, partition-major.  `acc`
// holds one partition and is reused by the next, so with partitions of a few tens of MiB the
// in-flight partial sums never leave the caches.
//
// Element i of acc (and of every replica buffer) is only ever touched by the block that owns
// the tile holding i, and the tile -> block assignment is the same in every slot, so consecutive
// slots need no synchronisation between blocks: a block-wide barrier with workgroup-scope
// release/acquire between two slots is enough (all waves of a block share one CU and its L1).
// That also lets the AllGather steps copy 16 bytes per lane although the ReduceScatter steps
// hand each lane 8 bytes of bf16.
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

constexpr int kPersistentUnroll = 8;

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

template <typename T, int VEC, int POL>
__global__ void __launch_bounds__(kThreads)
k_ring_persistent(PtrTable ring, PartGeom geom, SegTable tile_full, SegTable tile_last, int N, float* acc,
                  float scale, Ctrl* ctrl, DevCtrl* mirror, unsigned long long timeout_ticks,
                  unsigned long long max_spins, unsigned flags, unsigned long long zpos) {
  __shared__ T* s_tab[kMaxReplicas];
  __shared__ unsigned long long s_seg[2][kMaxReplicas + 1], s_tile[2][kMaxReplicas + 1];
  __shared__ unsigned long long s_gate;  // what lane 0 saw: released slots, or a verdict in bits 32..33
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
  constexpr int U = kPersistentUnroll;
  const unsigned n_steps = static_cast<unsigned>(2 * N - 2);
  const unsigned n_slots = geom.n_parts * n_steps;
  unsigned released = 0;  // slots [0, released) are known to be released
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
    const int step = static_cast<int>(ustep);
    if (step == N - 1) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");  // first AllGather step: see the block's stores
    const int sel = part + 1 == geom.n_parts ? 1 : 0;
    const unsigned long long* seg = s_seg[sel];
    const unsigned long long* til = s_tile[sel];
    const size_t off = static_cast<size_t>(part) * geom.part_elems;
    if (step < N - 1) {
      if (N == 2) ring_reduce_pass<T, VEC, kRsOnly, U, POL>(s_tab, seg, til, N, step, acc, scale, worker, n_workers, off, zpos);
      else if (step == 0) ring_reduce_pass<T, VEC, kRsFirst, U, POL>(s_tab, seg, til, N, step, acc, scale, worker, n_workers, off, zpos);
      else if (step == N - 2) ring_reduce_pass<T, VEC, kRsLast, U, POL>(s_tab, seg, til, N, step, acc, scale, worker, n_workers, off, zpos);
      else ring_reduce_pass<T, VEC, kRsMid, U, POL>(s_tab, seg, til, N, step, acc, scale, worker, n_workers, off, zpos);
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
    const bool report = slot + 1 >= released || slot + 1 == n_slots || (flags & FTAR_PERSIST_ALIGN) != 0;
    if (report || step == N - 2) {
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
      __syncthreads();
    }
    // With FTAR_PERSIST_PUBLISH the progress store is a release at agent scope: the data of the
    // slots reported is written back from this XCD's L2 before the progress can be seen, which
    // is what a NIC reading the buffers on the CPU's signal would need (one L2 write-back per
    // block and report: 18 % at 64 Mi elements when every slot is reported).
    if (report && tid == 0) {
      if (flags & FTAR_PERSIST_PUBLISH)
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

// ---- launch geometry and access policy -----------------------------------------
// Defaults come from sweeps on MI355X.  Bare probe kernels there reach about 6.9 TB/s for pure
// reads, 5.8 TB/s for pure writes and 6.0-6.4 TB/s for 7 reads + 1 write.  Two things matter:
//  * Few waves.  One workgroup per CU (one wave per SIMD) with just enough loads in flight
//    beats high occupancy by 5-10 %: all blocks then advance through one narrow window of
//    every stream and few DRAM rows are open at a time.  Kernels with little in flight per
//    wave (one or two streams) need 2-4 workgroups per CU instead.
//  * The 256 MB Infinity Cache.  Non-temporal loads always help.  Stores: what one ring step
//    writes is what the next step reads; when that fits the cache, ordinary stores keep it
//    there (up to 6.8 TB/s of algorithmic bytes); when it does not, non-temporal stores are
//    10-20 % faster than ordinary ones.
struct LaunchCfg {
  unsigned blocks;  // grid budget
  int pol;          // bit 0: non-temporal loads, bit 1: non-temporal stores
};

constexpr size_t kMiB = static_cast<size_t>(1) << 20;

// Tuning overrides: blocks_per_cu > 0 replaces the default; flags with bit 4 set carry an
// explicit policy in their low two bits.
LaunchCfg launch_cfg(int default_blocks_per_cu, int default_pol) {
  const Tuning t = current_tuning();
  const int per_cu = t.blocks_per_cu > 0 ? t.blocks_per_cu : default_blocks_per_cu;
  LaunchCfg c;
  c.blocks = static_cast<unsigned>(device_cu_count()) * static_cast<unsigned>(per_cu);
  c.pol = (t.flags & 0x10) ? (t.flags & 3) : default_pol;
  return c;
}

// N-reads-one-write reduction: fewer workgroups the more streams there are; ordinary stores
// while the output fits the Infinity Cache, non-temporal ones beyond (matters for N <= 4).
LaunchCfg reduce_cfg(int n_live, size_t out_bytes) {
  const bool big = out_bytes > 256 * kMiB;
  const int per_cu = n_live <= 2 ? 4 : (n_live <= 4 && !big) ? 2 : 1;
  return launch_cfg(per_cu, big ? 3 : 1);
}

LaunchCfg ring_reduce_cfg(RingMode mode, size_t count) {
  if (mode == kRsMid) return launch_cfg(1, count * 4 <= 256 * kMiB ? 1 : 3);
  return launch_cfg(2, 3);
}

LaunchCfg ring_allgather_cfg(size_t count, size_t elem_bytes) {
  return launch_cfg(2, count * elem_bytes <= 192 * kMiB ? 1 : 3);
}

// Every kernel goes through here.  Normally a plain launch; when the caller armed a pair of
// timing events for this thread's next launch, the dispatch itself records them (begin and end
// of the kernel on the GPU, without the command processor's gap between two dispatches).
template <typename... KArgs, typename... Args>
void launch(void (*kernel)(KArgs...), dim3 grid, dim3 block, hipStream_t stream, const Args&... args) {
  hipEvent_t start = nullptr, stop = nullptr;
  take_timing_events(&start, &stop);
  if (start || stop)
    hipExtLaunchKernelGGL(kernel, grid, block, 0, stream, start, stop, 0, static_cast<KArgs>(args)...);
  else
    hipLaunchKernelGGL(kernel, grid, block, 0, stream, static_cast<KArgs>(args)...);
}

unsigned grid_x_for(size_t n_tiles, unsigned budget) {
  if (budget < 1) budget = 1;
  if (n_tiles < 1) return 1;
  return n_tiles < budget ? static_cast<unsigned>(n_tiles) : budget;
}

// Calls f.template operator()<POL>(blocks) for the runtime policy.
template <typename F>
hipError_t with_policy(const LaunchCfg& cfg, F f) {
  switch (cfg.pol) {
    case 0: return f.template operator()<0>(cfg.blocks);
    case 1: return f.template operator()<1>(cfg.blocks);
    case 2: return f.template operator()<2>(cfg.blocks);
    default: return f.template operator()<3>(cfg.blocks);
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
                                                                                  count, zterm);  \
    else                                                                                          \
      launch(k_reduce_masked<T, VEC, n, unroll_narrow(n), POL>, grid, block, stream, live, out,    \
                                                                                    scale, count, zterm); \
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

// bf16 in, fp32 out: 4 elements per lane and vector (8-byte loads), as many vectors in flight
// as the wide tiles of the same-type kernel have bytes.
struct ReduceFixedF32Out {
  const PtrTable& live; int N; size_t count; float* out; float scale; float zterm; hipStream_t stream;
  template <int POL> hipError_t operator()(unsigned blocks) const {
    const int U = unroll_wide(N);
    const size_t tiles = count / 4 / (static_cast<size_t>(kThreads) * U);
    const dim3 grid(grid_x_for(tiles, blocks)), block(kThreads);
    switch (N) {
#define FTAR_CASE(n)                                                                               \
  case n:                                                                                          \
    launch(k_reduce_masked_f32out<4, n, unroll_wide(n), POL>, grid, block, stream, live, out, scale, \
           count, zterm);                                                                          \
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

hipError_t reduce_masked_f32out(const PtrTable& live, int N, size_t count, bool vec, float* out,
                                float scale, float zterm, hipStream_t stream) {
  const LaunchCfg cfg = reduce_cfg(N, count * sizeof(float));
  if (vec && N <= 16) return with_policy(cfg, ReduceFixedF32Out{live, N, count, out, scale, zterm, stream});
  if (vec) return with_policy(cfg, ReduceAny<bf16, 4, float>{live, N, count, out, scale, zterm, stream});
  return with_policy(cfg, ReduceAny<bf16, 1, float>{live, N, count, out, scale, zterm, stream});
}

template <typename T, int VECW>
hipError_t reduce_masked_typed(const PtrTable& live, int N, size_t count, bool vec, void* out,
                               float scale, float zterm, hipStream_t stream) {
  T* o = static_cast<T*>(out);
  const LaunchCfg cfg = reduce_cfg(N, count * sizeof(T));
  if (vec && N <= 16) return with_policy(cfg, ReduceFixed<T, VECW>{live, N, count, o, scale, zterm, stream});
  if (vec) return with_policy(cfg, ReduceAny<T, VECW>{live, N, count, o, scale, zterm, stream});
  return with_policy(cfg, ReduceAny<T, 1>{live, N, count, o, scale, zterm, stream});
}

template <typename T, int VEC>
struct Bucketed {
  const PtrTable& all; int n_replicas; const BucketTable& masks; int n_buckets; size_t first_elem;
  size_t bucket_elems; size_t count; const ScaleTable& scales; T* out; hipStream_t stream;
  template <int POL> hipError_t operator()(unsigned blocks) const {
    const size_t tile_elems = static_cast<size_t>(kThreads) * kBucketUnroll * VEC;
    const size_t tiles_per_bucket = (bucket_elems + tile_elems - 1) / tile_elems;
    const size_t last_begin = first_elem + static_cast<size_t>(n_buckets - 1) * bucket_elems;
    const size_t last_len = count - last_begin < bucket_elems ? count - last_begin : bucket_elems;
    const size_t tiles = static_cast<size_t>(n_buckets - 1) * tiles_per_bucket +
                         (last_len + tile_elems - 1) / tile_elems;
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
  if (vec)
    return with_policy(reduce_cfg(n_replicas, (count - first_elem) * sizeof(T)), Bucketed<T, VECW>{all, n_replicas, masks, n_buckets, first_elem, bucket_elems,
                                         count, scales, o, stream});
  return with_policy(reduce_cfg(n_replicas, (count - first_elem) * sizeof(T)), Bucketed<T, 1>{all, n_replicas, masks, n_buckets, first_elem, bucket_elems,
                                    count, scales, o, stream});
}

// Vectors per lane per tile in the ring kernels: tuning flag bits 8..11 (2, 4 or 8), default 4.
int ring_unroll() {
  const int u = (current_tuning().flags >> 8) & 0xf;
  return (u == 2 || u == 8) ? u : 4;
}

// Tiles before each portion (tile = kThreads*U*vec elements; the last tile of a portion may be short).
SegTable ring_tiles(const SegTable& seg, int N, int vec, int U) {
  SegTable t;
  const size_t tile_elems = static_cast<size_t>(kThreads) * U * vec;
  t.begin[0] = 0;
  for (int k = 0; k < N; ++k)
    t.begin[k + 1] = t.begin[k] + (seg.begin[k + 1] - seg.begin[k] + tile_elems - 1) / tile_elems;
  for (int k = N + 1; k <= kMaxReplicas; ++k) t.begin[k] = t.begin[N];
  return t;
}

template <typename T, int VEC>
struct RingReduce {
  RingMode mode; const PtrTable& ring; int N; int step; const SegTable& seg; float* acc; float scale;
  unsigned long long zpos; hipStream_t stream;
  template <int MODE, int U, int POL> void go(unsigned blocks) const {
    const SegTable tiles = ring_tiles(seg, N, VEC, U);
    const dim3 grid(grid_x_for(tiles.begin[N], blocks)), block(kThreads);
    launch(k_ring_reduce<T, VEC, MODE, U, POL>, grid, block, stream, ring, seg, tiles, N, step, acc, scale, zpos);
  }
  template <int MODE, int POL> void pick_unroll(unsigned blocks) const {
    const int U = ring_unroll();
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
    const dim3 grid(grid_x_for(tiles.begin[N], blocks)), block(kThreads);
    launch(k_ring_allgather<T, VEC, U, POL>, grid, block, stream, ring, seg, tiles, N, step);
  }
  template <int POL> hipError_t operator()(unsigned blocks) const {
    const int U = ring_unroll();
    if (U == 2) go<2, POL>(blocks);
    else if (U == 8) go<8, POL>(blocks);
    else go<4, POL>(blocks);
    return hipGetLastError();
  }
};

template <typename T, int VEC>
struct RingOnepass {
  const PtrTable& ring; int N; const SegTable& seg; float scale; unsigned long long zpos; hipStream_t stream;
  template <int POL> hipError_t operator()(unsigned blocks) const {
    const int U = (VEC == 1 || N > 16) ? 1 : unroll_narrow(N);  // must match the kernel's tile
    const SegTable tiles = ring_tiles(seg, N, VEC, U);
    const dim3 grid(grid_x_for(tiles.begin[N], blocks)), block(kThreads);
    if (VEC == 1 || N > 16) {
      launch(k_ring_onepass<T, VEC, 0, POL>, grid, block, stream, ring, seg, tiles, N, scale, zpos);
      return hipGetLastError();
    }
    switch (N) {
#define FTAR_CASE(n) \
  case n: launch(k_ring_onepass<T, VEC, (VEC == 1 ? 0 : n), POL>, grid, block, stream, ring, seg, tiles, N, scale, zpos); break;
      FTAR_CASE(2) FTAR_CASE(3) FTAR_CASE(4) FTAR_CASE(5) FTAR_CASE(6) FTAR_CASE(7) FTAR_CASE(8)
      FTAR_CASE(9) FTAR_CASE(10) FTAR_CASE(11) FTAR_CASE(12) FTAR_CASE(13) FTAR_CASE(14)
      FTAR_CASE(15) FTAR_CASE(16)
#undef FTAR_CASE
      default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
  }
};

template <typename T, int VEC>
struct RingPersistent {
  const PtrTable& ring; int N; const PartGeom& geom; float* acc; float scale; Ctrl* ctrl;
  DevCtrl* mirror; unsigned n_blocks; unsigned long long timeout_ticks; unsigned flags;
  unsigned long long zpos; hipStream_t stream;
  template <int POL> hipError_t operator()(unsigned) const {
    const SegTable tile_full = ring_tiles(geom.seg_full, N, VEC, kPersistentUnroll);
    const SegTable tile_last = ring_tiles(geom.seg_last, N, VEC, kPersistentUnroll);
    // Every workgroup must be resident at once: a worker that waits for the CPU keeps its place,
    // and the CPU may be waiting for a worker that has not started.  Clamp to what fits.
    int per_cu = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, k_ring_persistent<T, VEC, POL>, kThreads, 0) !=
            hipSuccess || per_cu < 1)
      per_cu = 1;
    const unsigned capacity = static_cast<unsigned>(per_cu) * static_cast<unsigned>(device_cu_count());
    const unsigned workers = n_blocks + 1 > capacity ? capacity - 1 : n_blocks;
    hipLaunchKernelGGL(k_clear_mirror, dim3(1), dim3(256), 0, stream, mirror);
    const dim3 grid(workers + 1), block(kThreads);  // the relay + the workers
    // one spin of a wait is a sleep plus two loads from device memory: well over 0.1 us
    launch(k_ring_persistent<T, VEC, POL>, grid, block, stream, ring, geom, tile_full, tile_last, N, acc,
           scale, ctrl, mirror, timeout_ticks, timeout_ticks / 10 + 100000, flags, zpos);
    return hipGetLastError();
  }
};

}  // namespace

// ---- exported launchers ----------------------------------------------------

hipError_t launch_reduce_masked(const PtrTable& live, int n_src, size_t count, ftar_dtype_t dtype,
                                ftar_dtype_t out_dtype, bool vec, void* out, float scale,
                                bool zero_participants, hipStream_t stream) {
  if (out_dtype != dtype && !(dtype == FTAR_BF16 && out_dtype == FTAR_F32)) return hipErrorInvalidValue;
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
  if (out_dtype != dtype)
    return reduce_masked_f32out(live, n_src, count, vec, static_cast<float*>(out), scale, zterm, stream);
  if (dtype == FTAR_F32)
    return reduce_masked_typed<float, 4>(live, n_src, count, vec, out, scale, zterm, stream);
  return reduce_masked_typed<bf16, 8>(live, n_src, count, vec, out, scale, zterm, stream);
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

hipError_t launch_ring_reduce(RingMode mode, const PtrTable& ring, int n_live, int step,
                              const SegTable& seg, ftar_dtype_t dtype, bool vec, float* acc,
                              float scale, unsigned long long zpos, hipStream_t stream) {
  if (dtype == FTAR_F32) {
    if (vec) return with_policy(ring_reduce_cfg(mode, seg.begin[n_live]), RingReduce<float, 4>{mode, ring, n_live, step, seg, acc, scale, zpos, stream});
    return with_policy(ring_reduce_cfg(mode, seg.begin[n_live]), RingReduce<float, 1>{mode, ring, n_live, step, seg, acc, scale, zpos, stream});
  }
  if (vec) return with_policy(ring_reduce_cfg(mode, seg.begin[n_live]), RingReduce<bf16, 4>{mode, ring, n_live, step, seg, acc, scale, zpos, stream});
  return with_policy(ring_reduce_cfg(mode, seg.begin[n_live]), RingReduce<bf16, 1>{mode, ring, n_live, step, seg, acc, scale, zpos, stream});
}

hipError_t launch_ring_allgather(const PtrTable& ring, int n_live, int step, const SegTable& seg,
                                 ftar_dtype_t dtype, bool vec, hipStream_t stream) {
  if (dtype == FTAR_F32) {
    if (vec) return with_policy(ring_allgather_cfg(seg.begin[n_live], 4), RingAllgather<float, 4>{ring, n_live, step, seg, stream});
    return with_policy(ring_allgather_cfg(seg.begin[n_live], 4), RingAllgather<float, 1>{ring, n_live, step, seg, stream});
  }
  if (vec) return with_policy(ring_allgather_cfg(seg.begin[n_live], 2), RingAllgather<bf16, 8>{ring, n_live, step, seg, stream});
  return with_policy(ring_allgather_cfg(seg.begin[n_live], 2), RingAllgather<bf16, 1>{ring, n_live, step, seg, stream});
}

hipError_t launch_ring_onepass(const PtrTable& ring, int n_live, const SegTable& seg,
                               ftar_dtype_t dtype, bool vec, float scale, unsigned long long zpos,
                               hipStream_t stream) {
  // N reads and N writes per element, as many write streams as read streams: non-temporal
  // stores and one workgroup per CU are best at every size measured
  const LaunchCfg cfg = launch_cfg(1, 3);
  if (dtype == FTAR_F32) {
    if (vec) return with_policy(cfg, RingOnepass<float, 4>{ring, n_live, seg, scale, zpos, stream});
    return with_policy(cfg, RingOnepass<float, 1>{ring, n_live, seg, scale, zpos, stream});
  }
  if (vec) return with_policy(cfg, RingOnepass<bf16, 8>{ring, n_live, seg, scale, zpos, stream});
  return with_policy(cfg, RingOnepass<bf16, 1>{ring, n_live, seg, scale, zpos, stream});
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
