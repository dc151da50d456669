// Channel-salience statistics and top-k selection (Section 4.2, Eq. 6-8).
//
// Everything that decides an index is exact: |q| sums and key ranges are integers
// in units of 2^-24 (every finite fp16 is a multiple of it), so the reductions may
// run in any order; the score is one binary64 product.
#include "mixkvq_internal.h"

namespace mixkvq {

// ---------------------------------------------------------------------------
// accumulator clear
// ---------------------------------------------------------------------------
__global__ void zero_u64_kernel(unsigned long long* sums, size_t n_sums, unsigned long long* counts, size_t n_counts) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n_sums) sums[i] = 0ull;
  else if (i < n_sums + n_counts) counts[i - n_sums] = 0ull;
}

// the sums and the counts of the view's pairs (two ranges: a view of some sequences of the batch is not contiguous)
hipError_t launch_zero_qacc(const CacheView& v, hipStream_t s) {
  const size_t n_sums = (size_t)v.P * kD, n = n_sums + (size_t)v.P;
  zero_u64_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s>>>(v.qacc, n_sums, v.qcnt, (size_t)v.P);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Eq. 6: sum of |q| per KV head and channel, over tokens and the g query heads
// of the group.  Streaming form: a workgroup takes `rows` rows of one query head;
// 16 threads cover a row of 256 bytes with one 16-byte load each, 16 rows per pass,
// eight passes in flight.  Per-thread 64-bit sums, one LDS reduction over the 16 row
// lanes, one 64-bit atomic per channel and workgroup (integers: any order is exact).
// ---------------------------------------------------------------------------
constexpr int kStreamThreads = 256;
constexpr int kMinRowsPerWG = 512, kMaxRowsPerWG = 2048;
constexpr int kInFlight = 8;      // 16-byte loads a thread has in flight

// Rows one workgroup takes: 512, or up to 2048 when that still leaves every compute unit tens of workgroups (fewer
// reductions and atomics per byte streamed: +2 % on a 5 GB tensor).
static int rows_per_workgroup(int64_t pairs_times_heads, int L) {
  int rows = kMinRowsPerWG;
  while (rows < kMaxRowsPerWG && pairs_times_heads * ((L + 2 * rows - 1) / (2 * rows)) >= 4096) rows *= 2;
  return rows;
}

// The per-thread sums run in binary64, which is exact here: every |fp16| is a multiple of 2^-24 below 2^16, so up to
// 2^13 of them add without rounding in a 53-bit significand (a thread adds at most kMaxRowsPerWG / 16 = 128 per channel);
// the sum times 2^24 is the exact integer.
typedef _Float16 sh2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void add8(double (&acc)[8], uint4 v) {
  const unsigned w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const sh2 h = __builtin_bit_cast(sh2, w[i]);
    acc[2 * i] += __builtin_fabs((double)(float)h[0]);
    acc[2 * i + 1] += __builtin_fabs((double)(float)h[1]);
  }
}

template <bool BF>      // BF: the tensor holds bfloat16 (converted to binary16 on entry)
__global__ void __launch_bounds__(kStreamThreads)
qabs_accumulate_kernel(const __half* __restrict__ q, int Lq, Strides3 qs, int Hkv, int g, int rows,
                       unsigned long long* __restrict__ qacc, unsigned long long* __restrict__ qcnt) {
  __shared__ unsigned long long sAcc[16][kD];
  const int p = blockIdx.x, b = p / Hkv, j = p % Hkv, tid = threadIdx.x;
  const int hh = blockIdx.y % g, chunk = blockIdx.y / g;
  const int c = tid & 15, r = tid >> 4;
  const int t0 = chunk * rows, t1 = min(Lq, t0 + rows);
  const __half* base = q + (int64_t)b * qs.b + (int64_t)(j * g + hh) * qs.h + 8 * c;
  static_assert(kMaxRowsPerWG / 16 <= 8192, "per-thread binary64 sums must stay exact");
  double acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = 0.0;
  int t = t0 + r;
  constexpr int NF = kInFlight;
  for (; t + 16 * (NF - 1) < t1; t += 16 * NF) {
    uint4 v[NF];
#pragma unroll
    for (int u = 0; u < NF; ++u) v[u] = *reinterpret_cast<const uint4*>(base + (int64_t)(t + 16 * u) * qs.t);
#pragma unroll
    for (int u = 0; u < NF; ++u) add8(acc, as_f16x8(v[u], BF));
  }
  for (; t < t1; t += 16) add8(acc, as_f16x8(*reinterpret_cast<const uint4*>(base + (int64_t)t * qs.t), BF));
#pragma unroll
  for (int i = 0; i < 8; ++i) sAcc[r][8 * c + i] = (unsigned long long)(acc[i] * 16777216.0);
  __syncthreads();
  if (tid < kD) {
    unsigned long long sum = 0;
#pragma unroll
    for (int rr = 0; rr < 16; ++rr) sum += sAcc[rr][tid];
    atomicAdd(&qacc[(size_t)p * kD + tid], sum);
  }
  if (tid == 0) atomicAdd(&qcnt[p], (unsigned long long)(t1 - t0));
}

// Fallback for tensors whose rows are not 16-byte aligned: one thread per channel.
__global__ void __launch_bounds__(kD) qabs_accumulate_unaligned_kernel(const __half* __restrict__ q, int Lq, Strides3 qs,
                                                                      int Hkv, int g, int rows, int bf16,
                                                                      unsigned long long* __restrict__ qacc,
                                                                      unsigned long long* __restrict__ qcnt) {
  const int p = blockIdx.x, b = p / Hkv, j = p % Hkv, d = threadIdx.x;
  const int hh = blockIdx.y % g, chunk = blockIdx.y / g;
  const int t0 = chunk * rows, t1 = min(Lq, t0 + rows);
  const __half* base = q + (int64_t)b * qs.b + (int64_t)(j * g + hh) * qs.h + d;
  unsigned long long acc = 0;
  for (int t = t0; t < t1; ++t) acc += fix24_abs(in_bits(base + (int64_t)t * qs.t, bf16));
  atomicAdd(&qacc[(size_t)p * kD + d], acc);
  if (d == 0) atomicAdd(&qcnt[p], (unsigned long long)(t1 - t0));
}

static bool rows_aligned16(const void* ptr, Strides3 st) {
  return (reinterpret_cast<uintptr_t>(ptr) & 15u) == 0 && st.b % 8 == 0 && st.h % 8 == 0 && st.t % 8 == 0;
}

hipError_t launch_qabs_accumulate(const CacheView& v, const __half* q, int Lq, Strides3 qs, hipStream_t s) {
  const int rows = rows_per_workgroup((int64_t)v.P * v.g, Lq);
  dim3 grid(v.P, v.g * ((Lq + rows - 1) / rows));
  if (!rows_aligned16(q, qs))
    qabs_accumulate_unaligned_kernel<<<grid, dim3(kD), 0, s>>>(q, Lq, qs, v.cfg.Hkv, v.g, rows, v.cfg.in_dtype, v.qacc, v.qcnt);
  else if (v.cfg.in_dtype)
    qabs_accumulate_kernel<true><<<grid, dim3(kStreamThreads), 0, s>>>(q, Lq, qs, v.cfg.Hkv, v.g, rows, v.qacc, v.qcnt);
  else
    qabs_accumulate_kernel<false><<<grid, dim3(kStreamThreads), 0, s>>>(q, Lq, qs, v.cfg.Hkv, v.g, rows, v.qacc, v.qcnt);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Eq. 7: per-channel min and max of the keys over L tokens.  Same streaming form; the
// running min/max are kept on packed 16-bit keys that order like the fp16 values
// (sign-magnitude -> two's complement), two channels per instruction, and only the
// workgroup's result is converted to the exact integers the atomics work on.
// ---------------------------------------------------------------------------
typedef short s16x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ s16x2 order_key(unsigned w) {     // involution: also maps keys back to fp16 bits
  const s16x2 v = __builtin_bit_cast(s16x2, w);
  return v ^ ((v >> 15) & (short)0x7fff);
}

__global__ void range_init_kernel(long long* mn, long long* mx, int n) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) {
    mn[i] = 0x7fffffffffffffffll;
    mx[i] = -0x7fffffffffffffffll - 1;
  }
}

template <bool BF>
__global__ void __launch_bounds__(kStreamThreads)
key_range_kernel(const __half* __restrict__ k, int L, Strides3 ks, int Hkv, int rows, long long* __restrict__ mn,
                 long long* __restrict__ mx) {
  __shared__ unsigned sLo[16][kD / 2], sHi[16][kD / 2];
  const int p = blockIdx.x, b = p / Hkv, j = p % Hkv, tid = threadIdx.x;
  const int c = tid & 15, r = tid >> 4;
  const int t0 = blockIdx.y * rows, t1 = min(L, t0 + rows);
  const __half* base = k + (int64_t)b * ks.b + (int64_t)j * ks.h + 8 * c;
  s16x2 lo[4], hi[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    lo[i] = s16x2{(short)0x7fff, (short)0x7fff};
    hi[i] = s16x2{(short)-0x8000, (short)-0x8000};
  }
  auto upd = [&](uint4 v) {
    const unsigned w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const s16x2 key = order_key(w[i]);
      lo[i] = __builtin_elementwise_min(lo[i], key);
      hi[i] = __builtin_elementwise_max(hi[i], key);
    }
  };
  int t = t0 + r;
  constexpr int NF = kInFlight;
  for (; t + 16 * (NF - 1) < t1; t += 16 * NF) {
    uint4 v[NF];
#pragma unroll
    for (int u = 0; u < NF; ++u) v[u] = *reinterpret_cast<const uint4*>(base + (int64_t)(t + 16 * u) * ks.t);
#pragma unroll
    for (int u = 0; u < NF; ++u) upd(as_f16x8(v[u], BF));
  }
  for (; t < t1; t += 16) upd(as_f16x8(*reinterpret_cast<const uint4*>(base + (int64_t)t * ks.t), BF));
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    sLo[r][4 * c + i] = __builtin_bit_cast(unsigned, lo[i]);
    sHi[r][4 * c + i] = __builtin_bit_cast(unsigned, hi[i]);
  }
  __syncthreads();
  if (tid < kD / 2) {
    s16x2 l = __builtin_bit_cast(s16x2, sLo[0][tid]), h = __builtin_bit_cast(s16x2, sHi[0][tid]);
#pragma unroll
    for (int rr = 1; rr < 16; ++rr) {
      l = __builtin_elementwise_min(l, __builtin_bit_cast(s16x2, sLo[rr][tid]));
      h = __builtin_elementwise_max(h, __builtin_bit_cast(s16x2, sHi[rr][tid]));
    }
    const unsigned lb = __builtin_bit_cast(unsigned, order_key(__builtin_bit_cast(unsigned, l)));
    const unsigned hb = __builtin_bit_cast(unsigned, order_key(__builtin_bit_cast(unsigned, h)));
    const size_t o = (size_t)p * kD + 2 * tid;
    if (t1 > t0) {
      atomicMin(&mn[o], fix24((unsigned short)(lb & 0xffffu)));
      atomicMin(&mn[o + 1], fix24((unsigned short)(lb >> 16)));
      atomicMax(&mx[o], fix24((unsigned short)(hb & 0xffffu)));
      atomicMax(&mx[o + 1], fix24((unsigned short)(hb >> 16)));
    }
  }
}

__global__ void __launch_bounds__(kD) key_range_unaligned_kernel(const __half* __restrict__ k, int L, Strides3 ks,
                                                                int Hkv, int rows, int bf16, long long* __restrict__ mn,
                                                                long long* __restrict__ mx) {
  const int p = blockIdx.x, b = p / Hkv, j = p % Hkv, d = threadIdx.x;
  const int t0 = blockIdx.y * rows;
  const int t1 = min(L, t0 + rows);
  const __half* base = k + (int64_t)b * ks.b + (int64_t)j * ks.h + d;
  long long lo = 0x7fffffffffffffffll, hi = -0x7fffffffffffffffll - 1;
  for (int t = t0; t < t1; ++t) {
    long long x = fix24(in_bits(base + (int64_t)t * ks.t, bf16));
    lo = x < lo ? x : lo;
    hi = x > hi ? x : hi;
  }
  atomicMin(&mn[(size_t)p * kD + d], lo);
  atomicMax(&mx[(size_t)p * kD + d], hi);
}

// ---------------------------------------------------------------------------
// Eq. 8 + top-k.  One workgroup per (batch, KV head) pair, one thread per channel.
// rank_d = number of channels that beat d (higher score, or equal score and lower index).
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(kD) select_topk_kernel(CacheView cv, const long long* __restrict__ mn,
                                                        const long long* __restrict__ mx, uint8_t* __restrict__ sel) {
  __shared__ double sA[kD];
  __shared__ unsigned char sTier[kD];
  const mixkvq_config& cfg = cv.cfg;
  const int p = blockIdx.x, d = threadIdx.x, k16 = cfg.k16, ks = cfg.k16 + cfg.k4;
  const long long rng = mx[(size_t)p * kD + d] - mn[(size_t)p * kD + d];
  const double A = cfg.score_mode ? (double)rng : (double)cv.qacc[(size_t)p * kD + d] * (double)rng;
  uint8_t* out = sel + (size_t)p * ks;
  if (d < ks) out[d] = MIXKVQ_NO_CHANNEL;     // entries no channel claims (threshold policy)
  sA[d] = A;
  __syncthreads();
  const double thr16 = cfg.policy == 1 ? score_threshold(cfg.tau16, cv.qcnt[p], cfg.score_mode) : 0.0;
  const double thr4 = cfg.policy == 1 ? score_threshold(cfg.tau4, cv.qcnt[p], cfg.score_mode) : 0.0;
  int rank = 0, c16 = 0, c_any = 0;
  for (int e = 0; e < kD; ++e) {
    const double o = sA[e];
    rank += (o > A) || (o == A && e < d);
    c16 += o > thr16;
    c_any += (o > thr16) || (o > thr4);
  }
  int n16, n4;
  tier_sizes(cfg, c16, c_any, &n16, &n4);
  const unsigned char tier = rank < n16 ? 2 : (rank < n16 + n4 ? 1 : 0);
  sTier[d] = tier;
  __syncthreads();
  if (tier) {
    int pos = 0;
    for (int e = 0; e < d; ++e) pos += sTier[e] == tier;
    out[(tier == 2 ? 0 : k16) + pos] = (uint8_t)d;
  }
}

size_t select_workspace_bytes(const mixkvq_config& c) {
  // minima and maxima per (pair, channel), then one selection per pair
  return (size_t)c.B * c.Hkv * kD * 2 * sizeof(long long) + (size_t)c.B * c.Hkv * kD;
}

uint8_t* select_scratch(const CacheView& v) { return v.ws + (size_t)v.P * kD * 2 * sizeof(long long); }

// One run of tokens into the range arrays.
static void launch_key_range(const CacheView& v, const __half* k, int L, Strides3 ks, bool bf16, long long* mn, long long* mx,
                             hipStream_t s) {
  const int rows = rows_per_workgroup(v.P, L);
  dim3 grid(v.P, (L + rows - 1) / rows);
  if (!rows_aligned16(k, ks))
    key_range_unaligned_kernel<<<grid, dim3(kD), 0, s>>>(k, L, ks, v.cfg.Hkv, rows, bf16 ? 1 : 0, mn, mx);
  else if (bf16)
    key_range_kernel<true><<<grid, dim3(kStreamThreads), 0, s>>>(k, L, ks, v.cfg.Hkv, rows, mn, mx);
  else
    key_range_kernel<false><<<grid, dim3(kStreamThreads), 0, s>>>(k, L, ks, v.cfg.Hkv, rows, mn, mx);
}

hipError_t launch_select2(const CacheView& v, const __half* kA, int LA, Strides3 sA, const __half* kB, int LB, Strides3 sB,
                          uint8_t* sel, hipStream_t s) {
  long long* mn = (long long*)v.ws;
  long long* mx = mn + (size_t)v.P * kD;
  const int n = v.P * kD;
  range_init_kernel<<<dim3((n + 255) / 256), dim3(256), 0, s>>>(mn, mx, n);
  if (LA > 0) launch_key_range(v, kA, LA, sA, false, mn, mx, s);       // window rows are binary16 already
  if (LB > 0) launch_key_range(v, kB, LB, sB, v.cfg.in_dtype != 0, mn, mx, s);
  select_topk_kernel<<<dim3(v.P), dim3(kD), 0, s>>>(v, mn, mx, sel);
  return hipGetLastError();
}

hipError_t launch_select(const CacheView& v, const __half* k, int L, Strides3 ks, uint8_t* sel, hipStream_t s) {
  return launch_select2(v, nullptr, 0, Strides3{0, 0, 0}, k, L, ks, sel, s);
}

}  // namespace mixkvq
