// Internal declarations shared by the host API and the kernel launchers of libmixkvq.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>
#include "mixkvq.h"

namespace mixkvq {

constexpr int kD = 128;             // head dimension of the hot path
constexpr int kMaxR = 128;          // largest residual window / flush unit
constexpr int kMaxSplits = 64;      // split-K ceiling per (batch, KV head) pair
constexpr int kSplitTargetWGs = 1024;   // sizes the workspace: split ceiling = kSplitTargetWGs / pairs
constexpr int kDecodeTargetWGs = 512;   // workgroups the decode launch aims for
constexpr int kMaxRec = 24576;      // largest supported block record in bytes (it is staged whole in LDS)

struct Layout : mixkvq_block_layout_t {};

struct Strides3 { int64_t b, h, t; };

// One new token per sequence that the decode launch itself moves into residual-window row `row`
// (k == nullptr: none).
struct NewToken { const __half* k; const __half* v; Strides3 st; int row; };

// Device-visible view of a cache: plain data passed by value to kernels.
struct CacheView {
  mixkvq_config cfg;
  Layout lay;
  int32_t P;             // B * Hkv
  int32_t g;             // Hq / Hkv
  int32_t NB;            // block capacity per pair = T_max / R
  uint8_t* blocks;       // [P][NB][rec_bytes]
  __half* res_k;         // [P][R][D]
  __half* res_v;
  unsigned long long* qacc;  // [P][D]
  unsigned long long* qcnt;  // [P]
  uint8_t* ws;
};

int compute_layout(const mixkvq_config& c, Layout* out);   // MIXKVQ_OK or MIXKVQ_EINVAL
int max_splits_for(int P);                                 // split-K ceiling used to size the workspace

// ---- kernel launchers (each returns a hipError_t from the launch) ----
hipError_t launch_zero_qacc(const CacheView& v, hipStream_t s);
hipError_t launch_qabs_accumulate(const CacheView& v, const __half* q, int Lq, Strides3 qs, hipStream_t s);
hipError_t launch_select(const CacheView& v, const __half* k, int L, Strides3 ks, uint8_t* sel, hipStream_t s);
hipError_t launch_flush(const CacheView& v, const __half* k_new, const __half* v_new, Strides3 kvs,
                        int r0, int first_block, int n_flush, const uint8_t* sel, hipStream_t s);
hipError_t launch_residual_copy(const CacheView& v, const __half* k_new, const __half* v_new, Strides3 kvs,
                                int src_first, int dst_first, int n, hipStream_t s);
hipError_t launch_decode(const CacheView& v, const __half* q, __half* out, float* lse, float scale,
                         int n_blocks, int n_res, int accumulate_q, NewToken nt, hipStream_t s, hipEvent_t ev_start,
                         hipEvent_t ev_stop);

size_t decode_workspace_bytes(const mixkvq_config& c);
size_t decode_partials_bytes(const mixkvq_config& c);
size_t select_workspace_bytes(const mixkvq_config& c);

// ---- small device helpers used by several kernels ----
__device__ __forceinline__ unsigned short h2bits(__half h) { return __half_as_ushort(h); }

// |x| * 2^24 of an fp16 as an exact integer (< 2^40).
__device__ __forceinline__ unsigned long long fix24_abs(unsigned short h) {
  unsigned e = (h >> 10) & 31u, m = h & 1023u;
  return e ? ((unsigned long long)(1024u + m) << (e - 1)) : (unsigned long long)m;
}
__device__ __forceinline__ long long fix24(unsigned short h) {
  long long v = (long long)fix24_abs(h);
  return (h & 0x8000u) ? -v : v;
}

}  // namespace mixkvq
