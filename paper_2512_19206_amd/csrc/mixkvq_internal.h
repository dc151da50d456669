// Internal declarations shared by the host API and the kernel launchers of libmixkvq.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>
#include "mixkvq.h"

namespace mixkvq {

__device__ __forceinline__ unsigned short h2bits(__half h) { return __half_as_ushort(h); }

constexpr int kD = 128;             // head dimension of the hot path
constexpr int kMaxR = 128;          // most tokens in one block record
constexpr int kMaxWindow = 256;     // the one residual length above kMaxR: its blocks are stored as two records
constexpr int kMaxSplits = 64;      // split-K ceiling per (batch, KV head) pair
constexpr int kSplitTargetWGs = 1024;   // sizes the workspace: split ceiling = kSplitTargetWGs / pairs
constexpr int kDecodeTargetWGs = 512;   // workgroups the decode launch aims for
constexpr int kMaxRec = 24576;      // largest supported block record in bytes (it is staged whole in LDS)

struct Layout : mixkvq_block_layout_t {};

struct Strides3 { int64_t b, h, t; };

// One new token per sequence that the decode launch itself moves into fp16 row `row` of every pair
// (k == nullptr: none).
struct NewToken { const __half* k; const __half* v; Strides3 st; int row; };

// Token counts per sequence for batches whose sequences differ in length, passed by value to the decode kernels
// (enabled == 0: every sequence has the counts given as scalar arguments).
constexpr int kMaxRaggedB = 256;
struct SeqCounts {
  int32_t enabled;
  int32_t n_blocks[kMaxRaggedB];      // quantized blocks of sequence b
  uint16_t n_fp16[kMaxRaggedB];       // its fp16 rows in use (sink + residual window)
};

// Device-visible view of a cache: plain data passed by value to kernels.
struct CacheView {
  mixkvq_config cfg;
  Layout lay;
  int32_t P;             // B * Hkv
  int32_t g;             // Hq / Hkv
  int32_t NB;            // block capacity per pair = T_max / R
  int32_t S;             // sink rows per pair (cfg.sink)
  int32_t RW;            // fp16 rows per pair = S + R: the sink rows, then the residual window
  uint8_t* blocks;       // [P][NB][rec_bytes], or with a block table a pool [slots][Hkv][rec_bytes]
  const int32_t* table;  // nullptr, or [B][NB]: pool slot of block i of sequence b
  __half* res_k;         // [P][RW][D]
  __half* res_v;
  unsigned long long* qacc;  // [P][D]
  unsigned long long* qcnt;  // [P]
  uint8_t* ws;
};

// Index (in records) of block `blk` of pair p inside cv.blocks.
__device__ __forceinline__ size_t record_index(const CacheView& cv, int p, int blk) {
  if (cv.table) {
    const int Hkv = cv.cfg.Hkv, b = p / Hkv, j = p % Hkv;
    return (size_t)cv.table[(size_t)b * cv.NB + blk] * Hkv + j;
  }
  return (size_t)p * cv.NB + blk;
}

int compute_layout(const mixkvq_config& c, Layout* out);   // MIXKVQ_OK or MIXKVQ_EINVAL
int rec_tokens(const mixkvq_config& c);                    // tokens per block record: min(R, kMaxR)
int max_splits_for(int P);                                 // split-K ceiling used to size the workspace

// ---- kernel launchers (each returns a hipError_t from the launch) ----
hipError_t launch_zero_qacc(const CacheView& v, hipStream_t s);
hipError_t launch_qabs_accumulate(const CacheView& v, const __half* q, int Lq, Strides3 qs, hipStream_t s);
hipError_t launch_select(const CacheView& v, const __half* k, int L, Strides3 ks, uint8_t* sel, hipStream_t s);
// The same over two runs of tokens: LA rows of the residual windows (binary16, kA = first row of the view's first pair,
// strides of the fp16-row buffers) followed by LB rows of the caller's tensor (kB, its strides and dtype).
hipError_t launch_select2(const CacheView& v, const __half* kA, int LA, Strides3 sA, const __half* kB, int LB, Strides3 sB,
                          uint8_t* sel, hipStream_t s);
uint8_t* select_scratch(const CacheView& v);   // room for one selection [P][k16 + k4] behind the range arrays in the workspace
hipError_t launch_flush(const CacheView& v, const __half* k_new, const __half* v_new, Strides3 kvs,
                        int r0, int first_block, int n_flush, const uint8_t* sel, hipStream_t s);
// n tokens starting at new-token index src_first go to fp16 rows dst_row.. of every pair (row 0 = first sink row,
// row S = first row of the residual window)
hipError_t launch_residual_copy(const CacheView& v, const __half* k_new, const __half* v_new, Strides3 kvs,
                                int src_first, int dst_row, int n, hipStream_t s);
// n_fp16: fp16 tokens of every pair = rows [0, n_fp16) of its fp16 rows (the sink, then the window; the window only
// holds tokens once the sink is full, so the rows in use are contiguous)
// With sc != nullptr (sequences of different lengths) n_blocks and n_fp16 are the largest counts of the batch, a
// sequence without tokens is skipped (output 0, lse -inf), and a new token (nt) goes to the last fp16 row in use.
hipError_t launch_decode(const CacheView& v, const __half* q, __half* out, float* lse, float scale,
                         int n_blocks, int n_fp16, int accumulate_q, NewToken nt, const SeqCounts* sc, hipStream_t s,
                         hipEvent_t ev_start, hipEvent_t ev_stop, int* path,   // *path: MIXKVQ_PATH_* of the launch
                         float* part = nullptr);   // split-K partials; nullptr: the cache's workspace
// bytes of split-K partials that launch would write
size_t decode_launch_partials_bytes(const CacheView& v, int n_blocks, int n_fp16);
// The library's own partials buffer for callers that cannot allocate: a file-scope device array of
// kNoAllocScratchBytes on every GPU; *out is its address on the current device (looked up once per device).
constexpr size_t kNoAllocScratchBytes = 8u << 20;
hipError_t noalloc_scratch(void** out);

size_t decode_workspace_bytes(const mixkvq_config& c);
size_t decode_partials_bytes(const mixkvq_config& c);
size_t select_workspace_bytes(const mixkvq_config& c);

// ---- small device helpers used by several kernels ----

// |x| * 2^24 of an fp16 as an exact integer (< 2^40).
__device__ __forceinline__ unsigned long long fix24_abs(unsigned short h) {
  unsigned e = (h >> 10) & 31u, m = h & 1023u;
  return e ? ((unsigned long long)(1024u + m) << (e - 1)) : (unsigned long long)m;
}
__device__ __forceinline__ long long fix24(unsigned short h) {
  long long v = (long long)fix24_abs(h);
  return (h & 0x8000u) ? -v : v;
}

// ---- input precision: bfloat16 tensors enter as the nearest binary16 (ties to even), saturated at +-65504 ----
__device__ __forceinline__ unsigned bf16x2_to_f16x2(unsigned w) {
  const float lo = __builtin_amdgcn_fmed3f(__uint_as_float(w << 16), -65504.f, 65504.f);
  const float hi = __builtin_amdgcn_fmed3f(__uint_as_float(w & 0xffff0000u), -65504.f, 65504.f);
  const __half2 r = __float22half2_rn(make_float2(lo, hi));
  return __builtin_bit_cast(unsigned, r);
}
__device__ __forceinline__ unsigned short bf16_to_f16_bits(unsigned short b) {
  return (unsigned short)(bf16x2_to_f16x2((unsigned)b) & 0xffffu);
}
// eight input elements (16 bytes) as eight binary16
__device__ __forceinline__ uint4 as_f16x8(uint4 v, bool bf16) {
  if (bf16) {
    v.x = bf16x2_to_f16x2(v.x);
    v.y = bf16x2_to_f16x2(v.y);
    v.z = bf16x2_to_f16x2(v.z);
    v.w = bf16x2_to_f16x2(v.w);
  }
  return v;
}
// one input element's binary16 bit pattern
__device__ __forceinline__ unsigned short in_bits(const __half* p, bool bf16) {
  const unsigned short b = h2bits(*p);
  return bf16 ? bf16_to_f16_bits(b) : b;
}
// fp32 -> bfloat16 bits, round to nearest even (finite values)
__device__ __forceinline__ unsigned short f32_to_bf16_bits(float x) {
  const unsigned u = __float_as_uint(x);
  return (unsigned short)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}

// Token (inside the block) of code i of value word tg; see the record layout in mixkvq.h.
__device__ __forceinline__ int value_word_token(int tg, int i, int interleave) {
  return interleave ? 64 * (tg >> 2) + 8 * (tg & 3) + (i & 7) + 32 * (i >> 3) : 16 * tg + i;
}

// Threshold of Section 4.2 in the units of the integer score sum|q|_d * range_d (units 2^-48):
// A_d = (sum|q|_d 2^-24 / count) * (range_d 2^-24 / 3) > tau  <=>  score_d > tau * 3 * 2^48 * count, the right-hand
// side formed in binary64 from left to right; with the error-only score, range_d > tau * 3 * 2^24.
__device__ __forceinline__ double score_threshold(double tau, unsigned long long count, int score_mode) {
  if (score_mode) return (tau * 3.0) * 16777216.0;
  return ((tau * 3.0) * 281474976710656.0) * (double)count;
}

// Sizes of the fp16 and the 4-bit tier of one block: the budgets themselves, or under the threshold policy the
// number of channels that pass (c16 above tau16, c_any above the lower of the two thresholds) cut to the capacities.
__device__ __forceinline__ void tier_sizes(const mixkvq_config& cfg, int c16, int c_any, int* n16, int* n4) {
  if (cfg.policy == 1) {
    *n16 = c16 < cfg.k16 ? c16 : cfg.k16;
    const int rest = c_any - *n16;
    *n4 = rest < cfg.k4 ? rest : cfg.k4;
  } else {
    *n16 = cfg.k16;
    *n4 = cfg.k4;
  }
}

}  // namespace mixkvq
