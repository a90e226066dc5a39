// Device helpers and launch plumbing shared by the kernel files (ftar_reduce.hip, ftar_ring.hip,
// ftar_persistent.hip, ftar_probe.hip).  Everything here is a template or inline and lives in an
// unnamed namespace: each file gets its own copy.
//
// Every kernel built from these is a streaming, HBM-bandwidth-bound elementwise pass: a few
// fp32 additions per 16-byte load, no data reuse, no contraction - so no MFMA
// and no LDS tiling of data.  What matters is (1) every wave instruction
// touching a contiguous run of full cache lines (lane t reads 16 bytes at
// 16*t: 1 KiB per wave instruction), (2) many independent loads in flight per
// lane before the first use (the paper's instruction-level-parallelism remark,
// section 4.2 "Optimizations"), (3) a persistent grid of few workgroups that
// strides over tiles, so the whole chip works inside one narrow window of every
// stream, and (4) non-temporal loads, since no byte is read twice (stores are
// non-temporal only where nobody reads the data soon).  LDS holds only the compact pointer table the
// CPU resolved from the live mask; pointers are pulled from it into scalar
// registers, so address arithmetic stays on the scalar unit.
//
// Arithmetic contract (identical in every kernel): exact widening to fp32,
// fp32 additions in the stated order starting from the first operand, one
// multiplication by `scale`, one rounding (nearest-even) to the output type.
// Compiled with -ffp-contract=off; fp32 denormals are not flushed.

#ifndef FTAR_DEVICE_H_
#define FTAR_DEVICE_H_

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

// Every pointer the kernels dereference is device (global) memory, but most of them reach the
// kernels through a table, as generic pointers.  Saying "global" at the access gives global_load /
// global_store instead of flat ones: those return in order, so the compiler may wait for just the
// loads a computation needs (s_waitcnt vmcnt(k)) and sum the first vectors of a tile while the
// last ones are still in flight; a flat load forces a wait for everything outstanding.
#define FTAR_GLOBAL __attribute__((address_space(1)))

template <int POL, typename R>
__device__ __forceinline__ R ld(const R* p) {
  const FTAR_GLOBAL R* g = (const FTAR_GLOBAL R*)p;
  if constexpr ((POL & 1) != 0) return __builtin_nontemporal_load(g);
  else return *g;
}

template <int POL, typename R>
__device__ __forceinline__ void st(R* p, R v) {
  FTAR_GLOBAL R* g = (FTAR_GLOBAL R*)p;
  if constexpr ((POL & 2) != 0) __builtin_nontemporal_store(v, g);
  else *g = v;
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
// gfx950 converts in hardware (v_cvt_pk_bf16_f32, two values per instruction).  On all 2^32
// patterns it gives what the integer rule gives - add 0x7fff plus the lowest kept bit, shift by
// 16; NaN: sign and upper payload kept, quiet bit set; fp32 denormals are not flushed.
__device__ __forceinline__ uint32_t bf16_rne2(float lo, float hi) {  // lo in bits 0..15
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  typedef float f32x2 __attribute__((ext_vector_type(2)));
  const f32x2 v = {lo, hi};
  const bf16x2 r = __builtin_convertvector(v, bf16x2);
  uint32_t u;
  __builtin_memcpy(&u, &r, 4);
  return u;
}
__device__ __forceinline__ uint32_t bf16_rne(float f) { return bf16_rne2(f, 0.0f) & 0xffffu; }

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
    for (int i = 0; i < 4; ++i) r[i] = bf16_rne2(x[2 * i], x[2 * i + 1]);
    return r;
  } else if constexpr (__is_same(R, u32x2)) {
    u32x2 r;
#pragma unroll
    for (int i = 0; i < 2; ++i) r[i] = bf16_rne2(x[2 * i], x[2 * i + 1]);
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
//   ACC_OUT == 2: acc_out = scale * a (fp32 result from any input type);
//   ACC_OUT == 3: acc_out = bf16(scale * a) (bf16 result from fp32 inputs)
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
  static_assert(ACC_OUT != 3 || __is_same(T, float), "mode 3 narrows fp32 inputs");
  static_assert((ACC_OUT != 2 && ACC_OUT != 3) || VEC <= 4, "results of the other type are moved 4 at a time");
  typedef typename Raw<T, VEC>::type R;
  typedef typename Raw<float, (VEC == 1 ? 1 : 4)>::type A;
  // fp32 partial sums move as 16-byte vectors: a lane that takes 8 elements (one 16-byte bf16
  // vector) takes two of them, at vector indices 2v and 2v + 1, so acc keeps its natural order
  constexpr int AV = VEC == 8 ? 2 : 1;
  R raw[U][NSRC];
  A ain[U][AV];
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
    for (int u = 0; u < U; ++u) {
#pragma unroll
      for (int q = 0; q < AV; ++q)
        ain[u][q] = ld<POL>(reinterpret_cast<const A*>(acc_in) + (v + u * kThreads) * AV + q);
    }
  }
#pragma unroll
  for (int u = 0; u < U; ++u) {
    float a[VEC], x[VEC];
    if constexpr (ACC_IN && VEC == 8) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        a[e] = ain[u][0][e];
        a[4 + e] = ain[u][1][e];
      }
    } else if constexpr (ACC_IN) {
      widen(ain[u][0], a);
    } else {
      widen(raw[u][0], a);
    }
#pragma unroll
    for (int j = (ACC_IN ? 0 : 1); j < NSRC; ++j) {
      widen(raw[u][j], x);
#pragma unroll
      for (int e = 0; e < VEC; ++e) a[e] = a[e] + x[e];
    }
    if constexpr (ACC_OUT == 1 && VEC == 8) {
      const f32x4 lo = {a[0], a[1], a[2], a[3]}, hi = {a[4], a[5], a[6], a[7]};
      st<POL>(reinterpret_cast<f32x4*>(acc_out) + (v + u * kThreads) * 2, lo);
      st<POL>(reinterpret_cast<f32x4*>(acc_out) + (v + u * kThreads) * 2 + 1, hi);
    } else if constexpr (ACC_OUT == 1) {
      st<POL>(reinterpret_cast<A*>(acc_out) + v + u * kThreads, narrow<A, VEC>(a));
    } else {
      if constexpr (ZT) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) a[e] = a[e] + zterm;
      }
#pragma unroll
      for (int e = 0; e < VEC; ++e) a[e] = a[e] * scale;
      if constexpr (ACC_OUT == 2) {
        st<POL>(reinterpret_cast<A*>(acc_out) + v + u * kThreads, narrow<A, VEC>(a));
      } else if constexpr (ACC_OUT == 3) {
        typedef typename Raw<bf16, VEC>::type B;
        st<POL>(reinterpret_cast<B*>(acc_out) + v + u * kThreads, narrow<B, VEC>(a));
      } else {
        st<POL>(reinterpret_cast<R*>(out) + v + u * kThreads, narrow<R, VEC>(a));
      }
    }
  }
}

// The result vector type of a tile for each store mode of sum_tile.
template <typename T, int VEC, int ACC_OUT> struct OutVec { typedef typename Raw<T, VEC>::type type; };
template <typename T, int VEC> struct OutVec<T, VEC, 2> { typedef typename Raw<float, (VEC == 1 ? 1 : 4)>::type type; };
template <typename T, int VEC> struct OutVec<T, VEC, 3> { typedef typename Raw<bf16, VEC>::type type; };

// sum_tile without the stores: the U finished result vectors of the tile (modes 0, 2 and 3), for
// kernels that stage their results and write them out later.  Same loads, same arithmetic.
template <typename T, int VEC, int NSRC, int ACC_OUT, int U, int POL, bool ZT>
__device__ __forceinline__ void sum_tile_values(T* const (&src)[NSRC], float scale, size_t v, float zterm,
                                                typename OutVec<T, VEC, ACC_OUT>::type (&res)[U]) {
  static_assert(ACC_OUT == 0 || ACC_OUT == 2 || ACC_OUT == 3, "finished results only");
  static_assert(ACC_OUT == 0 || VEC <= 4, "results of the other type are moved 4 at a time");
  typedef typename Raw<T, VEC>::type R;
  typedef typename OutVec<T, VEC, ACC_OUT>::type O;
  R raw[U][NSRC];
#pragma unroll
  for (int u = 0; u < U; ++u) {
#pragma unroll
    for (int j = 0; j < NSRC; ++j) raw[u][j] = ld<POL>(reinterpret_cast<const R*>(src[j]) + v + u * kThreads);
  }
#pragma unroll
  for (int u = 0; u < U; ++u) {
    float a[VEC], x[VEC];
    widen(raw[u][0], a);
#pragma unroll
    for (int j = 1; j < NSRC; ++j) {
      widen(raw[u][j], x);
#pragma unroll
      for (int e = 0; e < VEC; ++e) a[e] = a[e] + x[e];
    }
    if constexpr (ZT) {
#pragma unroll
      for (int e = 0; e < VEC; ++e) a[e] = a[e] + zterm;
    }
#pragma unroll
    for (int e = 0; e < VEC; ++e) a[e] = a[e] * scale;
    res[u] = narrow<O, VEC>(a);
  }
}

// ---- write windows ------------------------------------------------------------------------
// A sum over many streams writes little (1/(N+1) of its bytes), but every write that lands among
// the reads costs the memory more than its share: 8 streams read alone run at 6.9 TB/s, one
// stream written alone at 6.4 TB/s, yet the plain 8 + 1 mix only reaches 5.6-5.7 TB/s.  Counters
// show no stall in the L2 <-> fabric path and the loss does not respond to more loads in flight,
// cache-policy bits, store bursts of a single workgroup or stream alignment; it does respond to
// WHEN the chip writes.  So a workgroup stages its finished vectors in LDS and writes them out
// only inside windows of the 100 MHz wall clock, which is the same for all compute units: the
// whole chip then reads for tens of microseconds and writes in one short burst, with no
// communication between workgroups (8 + 1 streams of 1 GiB: 5.7 -> 6.5 TB/s; of 3 GiB: 5.6 ->
// 6.4), always with non-temporal stores.  It pays from four sources on (from six on at any size,
// see reduce_window); with a third or more of the bytes written the LDS cannot hold a long enough
// period and nothing is gained.  Nor when the result goes back into one of the
// buffers just read: the one-pass ReduceScatter loses with windows (8 x 1 Gi bf16: 5.6 TB/s plain,
// 4.9 staged) and keeps its plain stores.  A full stage is written out at once, whatever the clock
// says, so progress never depends on the clock.
struct WriteWindow {
  unsigned period_mask;  // period - 1, period a power of two in 10 ns ticks; 0 = no staging at all
  unsigned write_ticks;  // the window is [0, write_ticks) of every period
  unsigned min_tiles;    // flush in a window only with at least this many tiles staged
};

constexpr int kStageBytes = 144 * 1024;  // of the 160 KiB of LDS a compute unit has

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
// G: loads a lane has in flight; the N sources are taken G at a time, always in ascending order.
template <typename T, int VEC, int POL, typename TO = T, int G = 8>
__device__ __forceinline__ typename Raw<TO, VEC>::type sum_any_value(T* const* s_tab, size_t base, int N, float scale,
                                                                     size_t v, float zterm) {
  typedef typename Raw<T, VEC>::type R;
  typedef typename Raw<TO, VEC>::type RO;
  float a[VEC];
  for (int j0 = 0; j0 < N; j0 += G) {
    R raw[G];
#pragma unroll
    for (int jj = 0; jj < G; ++jj)
      if (j0 + jj < N) raw[jj] = ld<POL>(reinterpret_cast<const R*>(uniform_ptr(s_tab[j0 + jj]) + base) + v);
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
  for (int e = 0; e < VEC; ++e) a[e] = (a[e] + zterm) * scale;
  return narrow<RO, VEC>(a);
}

template <typename T, int VEC, int POL, typename TO = T>
__device__ __forceinline__ void sum_any_one(T* const* s_tab, size_t base, int N, TO* out, float scale,
                                            size_t v, float zterm) {
  typedef typename Raw<TO, VEC>::type RO;
  st<POL>(reinterpret_cast<RO*>(out) + v, sum_any_value<T, VEC, POL, TO>(s_tab, base, N, scale, v, zterm));
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
                                                 size_t buf_off = 0, unsigned long long zpos = 0,
                                                 size_t g_begin = 0, size_t g_end = ~static_cast<size_t>(0)) {
  // zpos: bit p set = the replica at ring position p is a zero-gradient participant
  // buf_off: first element of the partition in the replica buffers (acc is partition-relative)
  // [g_begin, g_end): the part of the flat tile sequence this launch covers (clipped to the whole)
  constexpr size_t kTileElems = static_cast<size_t>(kThreads) * U * VEC;
  const size_t all = uniform_u64(s_tile[N]);
  const size_t total = g_end < all ? g_end : all;
  int k = 0;
  size_t next = uniform_u64(s_tile[1]);
  for (size_t g = g_begin + bx; g < total; g += gx) {
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
                                                    unsigned bx, unsigned gx, size_t buf_off = 0,
                                                    size_t g_begin = 0, size_t g_end = ~static_cast<size_t>(0)) {
  typedef typename Raw<T, VEC>::type R;
  typedef typename Raw<T, 1>::type R1;
  constexpr size_t kTileElems = static_cast<size_t>(kThreads) * U * VEC;
  const unsigned tid = threadIdx.x;
  const size_t all = uniform_u64(s_tile[N]);
  const size_t total = g_end < all ? g_end : all;
  int k = 0;
  size_t next = uniform_u64(s_tile[1]);
  for (size_t g = g_begin + bx; g < total; g += gx) {
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
        if (e < t.rem) st<POL>(reinterpret_cast<R1*>(to) + e, ld<POL>(reinterpret_cast<const R1*>(from) + e));
      }
    }
  }
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
inline LaunchCfg launch_cfg(int default_blocks_per_cu, int default_pol) {
  const Tuning t = current_tuning();
  const int per_cu = t.blocks_per_cu > 0 ? t.blocks_per_cu : default_blocks_per_cu;
  LaunchCfg c;
  c.blocks = static_cast<unsigned>(device_cu_count()) * static_cast<unsigned>(per_cu);
  c.pol = (t.flags & 0x10) ? (t.flags & 3) : default_pol;
  return c;
}

// N-reads-one-write reduction: fewer workgroups the more streams there are; ordinary stores
// while the output fits the Infinity Cache, non-temporal ones beyond (matters for N <= 4).
inline LaunchCfg reduce_cfg(int n_live, size_t out_bytes) {
  const bool big = out_bytes > 256 * kMiB;
  const int per_cu = n_live <= 2 ? 4 : (n_live <= 4 && !big) ? 2 : 1;
  return launch_cfg(per_cu, big ? 3 : 1);
}

// The first step's partial sums are what the second step reads, the last step's results are what
// the first AllGather step reads: ordinary stores leave them in the Infinity Cache (8 x 64 Mi bf16
// inside the whole schedule: first step 87 -> 79 us, last step 87 -> 80 us against non-temporal
// stores; no difference once nothing fits any more).
// Per-bucket masks: the tile body re-specialises per bucket and runs four short sub-tiles, so two
// workgroups per CU keep more loads in flight (8 x 64 Mi bf16: 167 -> 158 us); over long streams
// (8 x 512 Mi fp32) the extra blocks drift apart and one per CU is 3 % faster.
inline LaunchCfg bucketed_cfg(int n_replicas, size_t out_bytes) {
  LaunchCfg c = reduce_cfg(n_replicas, out_bytes);
  if (out_bytes <= 512 * kMiB && current_tuning().blocks_per_cu <= 0) {
    const LaunchCfg two = launch_cfg(2, c.pol);
    if (two.blocks > c.blocks) c.blocks = two.blocks;
  }
  return c;
}

inline LaunchCfg ring_reduce_cfg(RingMode mode, size_t count) {
  if (mode == kRsMid) return launch_cfg(1, count * 4 <= 256 * kMiB ? 1 : 3);
  // First and last step: ordinary stores while the next step can find them in the cache.  Beyond
  // that non-temporal stores, and the last step (three quarters of its bytes are reads) with one
  // workgroup per CU (16 x 256 Mi bf16: last step 4.97 -> 6.43 TB/s, first step 5.69 -> 6.04).
  if (count * 4 <= 512 * kMiB) return launch_cfg(2, 1);
  return launch_cfg(mode == kRsLast ? 1 : 2, 3);
}

inline LaunchCfg ring_allgather_cfg(size_t count, size_t elem_bytes) {
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

inline unsigned grid_x_for(size_t n_tiles, unsigned budget) {
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

// Vectors per lane per tile in the ring kernels: tuning flag bits 8..11 (2, 4 or 8); default 4, or 2
// when a lane's vector is 8 elements wide (the same bytes in flight).
inline int ring_unroll(int vec) {
  const int u = (current_tuning().flags >> 8) & 0xf;
  return (u == 2 || u == 4 || u == 8) ? u : vec == 8 ? 2 : 4;
}

// Tiles before each portion (tile = kThreads*U*vec elements; the last tile of a portion may be short).
inline SegTable ring_tiles(const SegTable& seg, int N, int vec, int U) {
  SegTable t;
  const size_t tile_elems = static_cast<size_t>(kThreads) * U * vec;
  t.begin[0] = 0;
  for (int k = 0; k < N; ++k)
    t.begin[k + 1] = t.begin[k] + (seg.begin[k + 1] - seg.begin[k] + tile_elems - 1) / tile_elems;
  for (int k = N + 1; k <= kMaxReplicas; ++k) t.begin[k] = t.begin[N];
  return t;
}

}  // namespace
}  // namespace ftar

#endif  // FTAR_DEVICE_H_
