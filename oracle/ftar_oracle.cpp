// CPU oracle for the GPU data path of the Fault Tolerant All Reduce (FTAR).
//
// THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE.  It is a slow, plain,
// single-threaded statement of what the data path must compute, used only by
// the tests, the smoke check and the CPU-baseline leg of the benchmark.  It
// shares no code, header, table or helper with the HIP library and never
// calls it.  Build: g++ -O2 -ffp-contract=off (no fast-math, no intrinsics,
// default MXCSR so fp32 denormals are kept).
//
// What the paper fixes (section 4.1 "Overview" and section 4.2 "Efficient
// Fault Tolerant All Reduce"):
//   * same-rank GPUs of the participating replicas exchange gradients to
//     obtain the elementwise SUM over the participants (4.1);
//   * who participates is decided on the CPU by the reconfig function (4.2,
//     "CPU-GPU interaction"); here that decision is the live_mask;
//   * the exchange is a ring all-reduce, a ReduceScatter phase and an
//     AllGather phase of N-1 steps each; replica i starts by sending its i-th
//     portion to its right neighbour, every receiver reduces on arrival and
//     forwards (4.2, "Ring algorithm");
//   * intermediate ReduceScatter results live only in the send buffer, the
//     last ReduceScatter step also stores into the local data buffer, every
//     AllGather step stores into the local data buffer (4.2, "Optimizations").
// What the paper leaves open and this oracle fixes (each is a stated reading):
//   * result is the MEAN: the fp32 sum is multiplied once by
//     scale = 1.0f/(float)N computed by one fp32 division; sum_only=1 gives
//     the paper's literal sum (scale 1);
//   * inputs are fp32 or bf16, partial sums are carried in fp32 and rounded
//     once at the end (round-to-nearest-even for bf16);
//   * one-shot order: ascending replica index, the accumulator STARTS from
//     the first live value (not from +0), so one live replica is the bitwise
//     identity;
//   * ring order: ring position p = rank of the replica among the live ones,
//     right neighbour = (p+1) mod N, so portion k absorbs positions
//     k, k+1, ..., k+N-1 (mod N) in that order and ends at position k-1;
//   * portions ("segments") are whole chunks balanced to +-1 chunk:
//     seg_begin[k] = min(count, floor(k*n_chunks/N)*chunk_elems);
//   * the paper's step numbering for the store rule names N operations in a
//     phase of N-1 steps; it is read as off by one: steps are 0..N-2.
//
// Pins (tests/test_oracle_*.py): single-live identity, identical inputs give
// mean == input, dropping replica k == sum over the rest, power-of-two
// linearity, brute force on 16-element inputs against a separately written
// numpy.float32 loop, fp64 summation bound, bf16 conversion against torch's
// converter, per-rank message-passing ring == closed-form ring, all-reduce
// postcondition, the store rule, hand-derived ring schedule fixtures.
// No function here is "parity unpinned".

#include <cstddef>
#include <cstdint>
#include <cmath>
#include <cstring>
#include <vector>

namespace {

enum { DT_F32 = 0, DT_BF16 = 1 };

// ---- bf16 <-> fp32 -------------------------------------------------------
// bf16 is the upper half of an IEEE-754 binary32.  Widening is exact.
float bf16_bits_to_f32(uint16_t h) {
    uint32_t u = static_cast<uint32_t>(h) << 16;
    float f;
    std::memcpy(&f, &u, 4);
    return f;
}

// Narrowing: round to nearest, ties to even, on the 16 discarded bits.
// NaN stays NaN (sign kept, quiet bit forced); overflow rounds to infinity.
uint16_t f32_to_bf16_bits(float f) {
    uint32_t u;
    std::memcpy(&u, &f, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) {
        return static_cast<uint16_t>((u >> 16) | 0x0040u);
    }
    uint32_t keep_lsb = (u >> 16) & 1u;
    u += 0x7fffu + keep_lsb;
    return static_cast<uint16_t>(u >> 16);
}

// ---- element access by dtype ---------------------------------------------
float load_f32(const void* buf, size_t i, int dtype) {
    if (dtype == DT_F32) return static_cast<const float*>(buf)[i];
    return bf16_bits_to_f32(static_cast<const uint16_t*>(buf)[i]);
}

void store_cvt(void* buf, size_t i, int dtype, float v) {
    if (dtype == DT_F32) static_cast<float*>(buf)[i] = v;
    else static_cast<uint16_t*>(buf)[i] = f32_to_bf16_bits(v);
}

size_t elem_bytes(int dtype) { return dtype == DT_F32 ? 4 : 2; }

// ---- membership and geometry ---------------------------------------------
// ring[] = live replica indices in ascending order; returns N, or a negative
// code for an unusable mask (-1: arguments, -2: no live, -3: bit beyond n).
int live_ring(int n, uint64_t mask, int* ring) {
    if (n < 1 || n > 64) return -1;
    if (n < 64 && (mask >> n) != 0) return -3;
    int N = 0;
    for (int r = 0; r < n; ++r)
        if ((mask >> r) & 1u) ring[N++] = r;
    if (N == 0) return -2;
    return N;
}

float mean_scale(int N) { return 1.0f / static_cast<float>(N); }

void segment_bounds(int N, size_t count, size_t chunk, size_t* seg_begin) {
    size_t n_chunks = (count + chunk - 1) / chunk;
    for (int k = 0; k < N; ++k) {
        // floor(k*n_chunks/N) without overflow concerns at our sizes
        unsigned __int128 q = static_cast<unsigned __int128>(k) * n_chunks / static_cast<unsigned>(N);
        unsigned __int128 b = q * chunk;
        seg_begin[k] = b > count ? count : static_cast<size_t>(b);
    }
    seg_begin[N] = count;
}

int segment_of(const size_t* seg_begin, int N, size_t i) {
    int k = 0;
    while (k + 1 < N && i >= seg_begin[k + 1]) ++k;  // also steps over empty portions
    return k;
}

}  // namespace

extern "C" {

uint32_t oracle_bf16_to_f32_bits(uint16_t h) {
    float f = bf16_bits_to_f32(h);
    uint32_t u;
    std::memcpy(&u, &f, 4);
    return u;
}

uint16_t oracle_f32_bits_to_bf16(uint32_t bits) {
    float f;
    std::memcpy(&f, &bits, 4);
    return f32_to_bf16_bits(f);
}

void oracle_f32_to_bf16_array(const float* in, uint16_t* out, size_t count) {
    for (size_t i = 0; i < count; ++i) out[i] = f32_to_bf16_bits(in[i]);
}

void oracle_bf16_to_f32_array(const uint16_t* in, float* out, size_t count) {
    for (size_t i = 0; i < count; ++i) out[i] = bf16_bits_to_f32(in[i]);
}

// Live ring: ascending live replica indices (section 4.2: the group is
// whoever reconfig admits).  Returns N or a negative code.
int oracle_live_ring(int n, uint64_t mask, int* ring) { return live_ring(n, mask, ring); }

// fp32 bits of the averaging factor for N participants.
uint32_t oracle_scale_bits(int N) {
    float s = mean_scale(N);
    uint32_t u;
    std::memcpy(&u, &s, 4);
    return u;
}

// Portion boundaries (section 4.2 splits the data into N portions made of
// fixed-size chunks; the balancing rule is this build's reading).
// seg_begin has N+1 entries.  Returns N or a negative code.
int oracle_geometry(int n, uint64_t mask, size_t count, size_t chunk_elems, size_t* seg_begin) {
    int ring[64];
    int N = live_ring(n, mask, ring);
    if (N < 0) return N;
    if (count == 0 || chunk_elems == 0) return -1;
    segment_bounds(N, count, chunk_elems, seg_begin);
    return N;
}

// One-shot masked reduction (section 4.1: sum over the participants; mean
// by this build's reading).  bufs: n host pointers, dead entries unused.
//   out[i] = cvt(scale * (((x_ring0[i] + x_ring1[i]) + ...) + x_ringN-1[i]))
int oracle_reduce_masked(const void* const* bufs, int n, uint64_t mask, size_t count,
                         int dtype, int sum_only, void* out) {
    int ring[64];
    int N = live_ring(n, mask, ring);
    if (N < 0) return N;
    const float scale = sum_only ? 1.0f : mean_scale(N);
    for (size_t i = 0; i < count; ++i) {
        float a = load_f32(bufs[ring[0]], i, dtype);
        for (int j = 1; j < N; ++j) a = a + load_f32(bufs[ring[j]], i, dtype);
        a = a * scale;
        store_cvt(out, i, dtype, a);
    }
    return N;
}

// Zero-gradient participants (section 4.3, "Non-blocking Catch Up": a replica that is catching
// up takes part in the exchange and sends a zero gradient).  Replicas in zero_mask (a subset of
// live_mask) take part - they count among the N participants and, in a ring, receive the result -
// but contribute +0.0 and their buffers are never read.  The divisor is the number of
// participants, or with contributors_only the number of replicas that really contribute.
// By definition this is oracle_reduce_masked over buffers in which the zero participants hold
// +0.0 everywhere (tests pin exactly that), with the other divisor if asked.
int oracle_reduce_masked_zero(const void* const* bufs, int n, uint64_t live_mask, uint64_t zero_mask,
                              int contributors_only, size_t count, int dtype, void* out) {
  int ring[64];
  int N = live_ring(n, live_mask, ring);
  if (N < 0) return N;
  if ((zero_mask & ~live_mask) != 0) return -3;
  int Z = 0;
  for (int j = 0; j < N; ++j) Z += (zero_mask >> ring[j]) & 1u;
  const int divisor = contributors_only ? N - Z : N;
  if (divisor <= 0) return -2;
  const float scale = 1.0f / static_cast<float>(divisor);
  for (size_t i = 0; i < count; ++i) {
    float a = ((zero_mask >> ring[0]) & 1u) ? 0.0f : load_f32(bufs[ring[0]], i, dtype);
    for (int j = 1; j < N; ++j)
      a = a + (((zero_mask >> ring[j]) & 1u) ? 0.0f : load_f32(bufs[ring[j]], i, dtype));
    a = a * scale;
    store_cvt(out, i, dtype, a);
  }
  return N;
}

// Delivery variants of the one-shot reduction: the result type may be fp32 although the inputs
// are bf16 (the one rounding to the output type is then the identity), and the operation may be
// the plain sum of section 4.1 instead of this build's mean.  Otherwise as
// oracle_reduce_masked_zero.
int oracle_reduce_masked_ex(const void* const* bufs, int n, uint64_t live_mask, uint64_t zero_mask,
                            int contributors_only, size_t count, int in_dtype, int out_dtype,
                            int sum_only, void* out) {
  int ring[64];
  int N = live_ring(n, live_mask, ring);
  if (N < 0) return N;
  if ((zero_mask & ~live_mask) != 0) return -3;
  int Z = 0;
  for (int j = 0; j < N; ++j) Z += (zero_mask >> ring[j]) & 1u;
  const int divisor = contributors_only ? N - Z : N;
  if (divisor <= 0) return -2;
  const float scale = sum_only ? 1.0f : 1.0f / static_cast<float>(divisor);
  for (size_t i = 0; i < count; ++i) {
    float a = ((zero_mask >> ring[0]) & 1u) ? 0.0f : load_f32(bufs[ring[0]], i, in_dtype);
    for (int j = 1; j < N; ++j)
      a = a + (((zero_mask >> ring[j]) & 1u) ? 0.0f : load_f32(bufs[ring[j]], i, in_dtype));
    a = a * scale;
    store_cvt(out, i, out_dtype, a);
  }
  return N;
}

// Learning-rate intervention factors of section 6.2: "linear" = healthy replicas / all replicas,
// "sqrt" = the square root of that ratio.  Healthy = taking part and contributing a gradient
// (a zero-gradient participant trains on no data in this step).  linear is the fp32 quotient of
// the two counts; root is the binary64 square root of the binary64 quotient, rounded to fp32.
int oracle_lr_factors(int n, uint64_t live_mask, uint64_t zero_mask, float* linear, float* root) {
  int ring[64];
  int N = live_ring(n, live_mask, ring);
  if (N < 0) return N;
  if ((zero_mask & ~live_mask) != 0) return -3;
  int healthy = 0;
  for (int j = 0; j < N; ++j) healthy += ((zero_mask >> ring[j]) & 1u) ? 0 : 1;
  *linear = static_cast<float>(healthy) / static_cast<float>(n);
  *root = static_cast<float>(std::sqrt(static_cast<double>(healthy) / static_cast<double>(n)));
  return N;
}

// Ring all-reduce with zero-gradient participants, closed form for the element range
// [begin, begin+len): as oracle_ring_closed_form with +0.0 in place of the zero participants'
// values.  Every participant, the zero ones included, ends with this value.
int oracle_ring_closed_form_zero(const void* const* bufs, int n, uint64_t live_mask, uint64_t zero_mask,
                                 int contributors_only, size_t count, size_t chunk_elems, int dtype,
                                 size_t begin, size_t len, void* out) {
  int ring[64];
  int N = live_ring(n, live_mask, ring);
  if (N < 0) return N;
  if ((zero_mask & ~live_mask) != 0) return -3;
  if (count == 0 || chunk_elems == 0 || begin > count || len > count - begin) return -1;
  int Z = 0;
  for (int j = 0; j < N; ++j) Z += (zero_mask >> ring[j]) & 1u;
  const int divisor = contributors_only ? N - Z : N;
  if (divisor <= 0) return -2;
  const float scale = 1.0f / static_cast<float>(divisor);
  std::vector<size_t> sb(N + 1);
  segment_bounds(N, count, chunk_elems, sb.data());
  for (size_t j = 0; j < len; ++j) {
    int k = segment_of(sb.data(), N, begin + j);
    int r0 = ring[k];
    float a = ((zero_mask >> r0) & 1u) ? 0.0f : load_f32(bufs[r0], j, dtype);
    for (int m = 1; m < N; ++m) {
      int r = ring[(k + m) % N];
      a = a + (((zero_mask >> r) & 1u) ? 0.0f : load_f32(bufs[r], j, dtype));
    }
    if (N > 1) a = a * scale;
    store_cvt(out, j, dtype, a);
  }
  return N;
}

// The same sum carried in binary64 with a binary64 1/N: the "exact" value
// the error bounds are stated against.  out: count doubles.
int oracle_reduce_f64(const void* const* bufs, int n, uint64_t mask, size_t count,
                      int dtype, int sum_only, double* out, double* abs_sum) {
    int ring[64];
    int N = live_ring(n, mask, ring);
    if (N < 0) return N;
    const double scale = sum_only ? 1.0 : 1.0 / static_cast<double>(N);
    for (size_t i = 0; i < count; ++i) {
        double a = 0.0, m = 0.0;
        for (int j = 0; j < N; ++j) {
            double x = static_cast<double>(load_f32(bufs[ring[j]], i, dtype));
            a += x;
            m += x < 0 ? -x : x;
        }
        out[i] = a * scale;
        if (abs_sum) abs_sum[i] = m * scale;
    }
    return N;
}

// Ring all-reduce as message passing between ranks (section 4.2, "Ring
// algorithm" and the store rule under "Optimizations").  Every ring position
// has its local data buffer (bufs[ring[p]], updated in place), a send buffer
// and a receive buffer.  The "network" moves each position's send buffer into
// its right neighbour's receive buffer at the start of every step.
// Runs the first rs_steps ReduceScatter steps and then the first ag_steps
// AllGather steps (ag_steps must be 0 unless rs_steps == N-1).
// acc_image (optional, count floats): after the call, for every portion whose
// partial sum is still in flight, the fp32 contents of the send buffer that
// holds it, laid out at the portion's element range.
int oracle_ring_per_rank(void* const* bufs, int n, uint64_t mask, size_t count,
                         size_t chunk_elems, int dtype, int sum_only, int rs_steps,
                         int ag_steps, float* acc_image) {
    int ring[64];
    int N = live_ring(n, mask, ring);
    if (N < 0) return N;
    if (count == 0 || chunk_elems == 0) return -1;
    if (rs_steps < 0 || rs_steps > N - 1 || ag_steps < 0 || ag_steps > N - 1) return -4;
    if (ag_steps > 0 && rs_steps != N - 1) return -4;
    std::vector<size_t> sb(N + 1);
    segment_bounds(N, count, chunk_elems, sb.data());
    const float scale = sum_only ? 1.0f : mean_scale(N);
    if (N == 1) return N;  // a ring of one exchanges nothing

    size_t max_len = 0;
    for (int k = 0; k < N; ++k)
        if (sb[k + 1] - sb[k] > max_len) max_len = sb[k + 1] - sb[k];

    // In-flight payloads: fp32 partial sums during ReduceScatter, final values
    // in the data's own dtype (kept as raw 32-bit words here) during AllGather.
    std::vector<std::vector<float>> send(N, std::vector<float>(max_len));
    std::vector<std::vector<float>> recv(N, std::vector<float>(max_len));
    std::vector<int> send_seg(N), recv_seg(N);

    // Before the first step: position p stages its own portion p for sending.
    for (int p = 0; p < N; ++p) {
        send_seg[p] = p;
        for (size_t j = 0, len = sb[p + 1] - sb[p]; j < len; ++j)
            send[p][j] = load_f32(bufs[ring[p]], sb[p] + j, dtype);
    }

    for (int s = 0; s < rs_steps; ++s) {
        for (int p = 0; p < N; ++p) {  // transfer: left neighbour -> me
            int left = (p + N - 1) % N;
            recv[p] = send[left];
            recv_seg[p] = send_seg[left];
        }
        const bool last = (s == N - 2);
        for (int p = 0; p < N; ++p) {  // reduce on arrival
            int k = recv_seg[p];
            void* local = bufs[ring[p]];
            for (size_t j = 0, len = sb[k + 1] - sb[k]; j < len; ++j) {
                float r = recv[p][j] + load_f32(local, sb[k] + j, dtype);
                if (!last) {
                    send[p][j] = r;  // result kept only in the send buffer
                } else {
                    r = r * scale;
                    store_cvt(local, sb[k] + j, dtype, r);       // final result to the user
                    send[p][j] = load_f32(local, sb[k] + j, dtype);  // and staged for AllGather
                }
            }
            send_seg[p] = k;
        }
    }

    if (acc_image) {
        for (size_t i = 0; i < count; ++i) acc_image[i] = 0.0f;
        if (rs_steps < N - 1) {
            for (int p = 0; p < N; ++p) {
                int k = send_seg[p];
                for (size_t j = 0, len = sb[k + 1] - sb[k]; j < len; ++j)
                    acc_image[sb[k] + j] = send[p][j];
            }
        }
    }

    for (int t = 0; t < ag_steps; ++t) {
        for (int p = 0; p < N; ++p) {
            int left = (p + N - 1) % N;
            recv[p] = send[left];
            recv_seg[p] = send_seg[left];
        }
        for (int p = 0; p < N; ++p) {  // store what arrived, forward it next step
            int k = recv_seg[p];
            void* local = bufs[ring[p]];
            for (size_t j = 0, len = sb[k + 1] - sb[k]; j < len; ++j) {
                // payload is already a value of the data's dtype: the store is a bit copy
                store_cvt(local, sb[k] + j, dtype, recv[p][j]);
                send[p][j] = recv[p][j];
            }
            send_seg[p] = k;
        }
    }
    return N;
}

// Which portion position p receives at ReduceScatter step s and at AllGather
// step t, taken from the message-passing simulation itself (used by the
// schedule fixture test).  Outputs are N*(N-1) ints, [step][position].
int oracle_ring_schedule(int n, uint64_t mask, int* rs_recv_seg, int* ag_recv_seg) {
    int ring[64];
    int N = live_ring(n, mask, ring);
    if (N < 0) return N;
    std::vector<int> send_seg(N), recv_seg(N);
    for (int p = 0; p < N; ++p) send_seg[p] = p;
    for (int phase = 0; phase < 2; ++phase) {
        int* out = phase == 0 ? rs_recv_seg : ag_recv_seg;
        for (int s = 0; s < N - 1; ++s) {
            for (int p = 0; p < N; ++p) recv_seg[p] = send_seg[(p + N - 1) % N];
            for (int p = 0; p < N; ++p) {
                out[s * N + p] = recv_seg[p];
                send_seg[p] = recv_seg[p];
            }
        }
    }
    return N;
}

// Closed form of the finished ring all-reduce for the element range
// [begin, begin+len): element i of portion k is
//   cvt(scale * (x_ring[k] + x_ring[k+1] + ... + x_ring[k+N-1 mod N])) summed in
// that order, and every live replica ends with that value.
// bufs[r] points at element `begin` of replica r's ORIGINAL data; out gets len
// elements of the data's dtype.
int oracle_ring_closed_form(const void* const* bufs, int n, uint64_t mask, size_t count,
                            size_t chunk_elems, int dtype, int sum_only, size_t begin,
                            size_t len, void* out) {
    int ring[64];
    int N = live_ring(n, mask, ring);
    if (N < 0) return N;
    if (count == 0 || chunk_elems == 0 || begin > count || len > count - begin) return -1;
    std::vector<size_t> sb(N + 1);
    segment_bounds(N, count, chunk_elems, sb.data());
    const float scale = sum_only ? 1.0f : mean_scale(N);
    for (size_t j = 0; j < len; ++j) {
        int k = segment_of(sb.data(), N, begin + j);
        float a = load_f32(bufs[ring[k]], j, dtype);
        for (int m = 1; m < N; ++m) a = a + load_f32(bufs[ring[(k + m) % N]], j, dtype);
        if (N > 1) a = a * scale;
        store_cvt(out, j, dtype, a);
    }
    return N;
}

// fp32 partial sums in flight after `rs_steps` non-final ReduceScatter steps,
// closed form, for the element range [begin, begin+len):
//   acc[i] = x_ring[k] + x_ring[k+1] + ... + x_ring[k+rs_steps]   (1 <= rs_steps <= N-2)
int oracle_ring_partial(const void* const* bufs, int n, uint64_t mask, size_t count,
                        size_t chunk_elems, int dtype, int rs_steps, size_t begin,
                        size_t len, float* acc) {
    int ring[64];
    int N = live_ring(n, mask, ring);
    if (N < 0) return N;
    if (count == 0 || chunk_elems == 0 || begin > count || len > count - begin) return -1;
    if (rs_steps < 1 || rs_steps > N - 2) return -4;
    std::vector<size_t> sb(N + 1);
    segment_bounds(N, count, chunk_elems, sb.data());
    for (size_t j = 0; j < len; ++j) {
        int k = segment_of(sb.data(), N, begin + j);
        float a = load_f32(bufs[ring[k]], j, dtype);
        for (int m = 1; m <= rs_steps; ++m) a = a + load_f32(bufs[ring[(k + m) % N]], j, dtype);
        acc[j] = a;
    }
    return N;
}

size_t oracle_elem_bytes(int dtype) { return elem_bytes(dtype); }

}  // extern "C"
