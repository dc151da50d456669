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
__global__ void zero_u64_kernel(unsigned long long* p, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0ull;
}

hipError_t launch_zero_qacc(const CacheView& v, hipStream_t s) {
  size_t n = (size_t)v.P * (kD + 1);
  zero_u64_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s>>>(v.qacc, n);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Eq. 6: sum of |q| per KV head and channel, over tokens and the g query heads
// of the group.  One thread per channel; 128-bit loads are not needed for the
// decode case (one token), and the prefill case streams rows of 256 bytes.
// ---------------------------------------------------------------------------
constexpr int kQTokensPerBlock = 64;

__global__ void __launch_bounds__(kD) qabs_accumulate_kernel(const __half* __restrict__ q, int Lq, Strides3 qs, int Hkv,
                                                            int g, unsigned long long* __restrict__ qacc,
                                                            unsigned long long* __restrict__ qcnt) {
  const int p = blockIdx.x, b = p / Hkv, j = p % Hkv, d = threadIdx.x;
  const int t0 = blockIdx.y * kQTokensPerBlock;
  const int t1 = min(Lq, t0 + kQTokensPerBlock);
  unsigned long long acc = 0;
  for (int hh = 0; hh < g; ++hh) {
    const __half* base = q + (int64_t)b * qs.b + (int64_t)(j * g + hh) * qs.h + d;
    for (int t = t0; t < t1; ++t) acc += fix24_abs(h2bits(base[(int64_t)t * qs.t]));
  }
  atomicAdd(&qacc[(size_t)p * kD + d], acc);
  if (d == 0) atomicAdd(&qcnt[p], (unsigned long long)g * (unsigned long long)(t1 - t0));
}

hipError_t launch_qabs_accumulate(const CacheView& v, const __half* q, int Lq, Strides3 qs, hipStream_t s) {
  dim3 grid(v.P, (Lq + kQTokensPerBlock - 1) / kQTokensPerBlock);
  qabs_accumulate_kernel<<<grid, dim3(kD), 0, s>>>(q, Lq, qs, v.cfg.Hkv, v.g, v.qacc, v.qcnt);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Eq. 7: per-channel min and max of the keys over L tokens (exact integers).
// ---------------------------------------------------------------------------
constexpr int kKTokensPerBlock = 256;

__global__ void range_init_kernel(long long* mn, long long* mx, int n) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) {
    mn[i] = 0x7fffffffffffffffll;
    mx[i] = -0x7fffffffffffffffll - 1;
  }
}

__global__ void __launch_bounds__(kD) key_range_kernel(const __half* __restrict__ k, int L, Strides3 ks, int Hkv,
                                                      long long* __restrict__ mn, long long* __restrict__ mx) {
  const int p = blockIdx.x, b = p / Hkv, j = p % Hkv, d = threadIdx.x;
  const int t0 = blockIdx.y * kKTokensPerBlock;
  const int t1 = min(L, t0 + kKTokensPerBlock);
  const __half* base = k + (int64_t)b * ks.b + (int64_t)j * ks.h + d;
  long long lo = 0x7fffffffffffffffll, hi = -0x7fffffffffffffffll - 1;
  for (int t = t0; t < t1; ++t) {
    long long x = fix24(h2bits(base[(int64_t)t * ks.t]));
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
__device__ __forceinline__ void rank_and_emit(double A, int d, int k16, int k4, double* sA, unsigned char* sTier,
                                              uint8_t* out) {
  sA[d] = A;
  __syncthreads();
  int rank = 0;
  for (int e = 0; e < kD; ++e) {
    double o = sA[e];
    rank += (o > A) || (o == A && e < d);
  }
  unsigned char tier = rank < k16 ? 2 : (rank < k16 + k4 ? 1 : 0);
  sTier[d] = tier;
  __syncthreads();
  if (tier) {
    int pos = 0;
    for (int e = 0; e < d; ++e) pos += sTier[e] == tier;
    out[(tier == 2 ? 0 : k16) + pos] = (uint8_t)d;
  }
}

__global__ void __launch_bounds__(kD) select_topk_kernel(const unsigned long long* __restrict__ qacc,
                                                        const long long* __restrict__ mn,
                                                        const long long* __restrict__ mx, int k16, int k4,
                                                        int score_mode, uint8_t* __restrict__ sel) {
  __shared__ double sA[kD];
  __shared__ unsigned char sTier[kD];
  const int p = blockIdx.x, d = threadIdx.x;
  const long long rng = mx[(size_t)p * kD + d] - mn[(size_t)p * kD + d];
  const double A = score_mode ? (double)rng : (double)qacc[(size_t)p * kD + d] * (double)rng;
  rank_and_emit(A, d, k16, k4, sA, sTier, sel + (size_t)p * (k16 + k4));
}

size_t select_workspace_bytes(const mixkvq_config& c) { return (size_t)c.B * c.Hkv * kD * 2 * sizeof(long long); }

hipError_t launch_select(const CacheView& v, const __half* k, int L, Strides3 ks, uint8_t* sel, hipStream_t s) {
  long long* mn = (long long*)v.ws;
  long long* mx = mn + (size_t)v.P * kD;
  const int n = v.P * kD;
  range_init_kernel<<<dim3((n + 255) / 256), dim3(256), 0, s>>>(mn, mx, n);
  dim3 grid(v.P, (L + kKTokensPerBlock - 1) / kKTokensPerBlock);
  key_range_kernel<<<grid, dim3(kD), 0, s>>>(k, L, ks, v.cfg.Hkv, mn, mx);
  select_topk_kernel<<<dim3(v.P), dim3(kD), 0, s>>>(v.qacc, mn, mx, v.cfg.k16, v.cfg.k4, v.cfg.score_mode, sel);
  return hipGetLastError();
}

}  // namespace mixkvq
