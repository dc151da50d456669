// Split-K decode attention over the mixed-precision cache (Section 3.1, Eq. 1, with
// keys and values dequantized on the fly by Eq. 3) and the log-sum-exp merge of the
// splits.
#include <stdlib.h>
#include <string.h>
#include <mutex>
#include "mixkvq_internal.h"

namespace mixkvq {

constexpr int kDecThreads = 256;
constexpr int kMaxG = 8;
constexpr int kPartStride = kD + 2;   // floats per (split, head): O[D], m, l

size_t decode_partials_bytes(const mixkvq_config& c) {
  const int P = c.B * c.Hkv;
  const size_t n = (size_t)P * (max_splits_for(P) + 1) * (c.Hq / c.Hkv) * kPartStride * sizeof(float);
  return (n + 255) / 256 * 256;
}
size_t decode_workspace_bytes(const mixkvq_config& c) { return decode_partials_bytes(c); }

// ---------------------------------------------------------------------------
// Reference-grade split kernel: plain vector ALU, one workgroup per (pair, split).
// Threads play two roles per block of R tokens: (token, head-half) for q.K and the
// softmax update, (channel, head-half) for P.V.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(kDecThreads)
decode_split_kernel(CacheView cv, const __half* __restrict__ q, float scale, int n_blocks, int n_fp16, int n_splits,
                    float* __restrict__ part, SeqCounts sc) {
  __shared__ __align__(16) unsigned char sRec[kMaxRec];
  __shared__ float sQ[kMaxG][kD];
  __shared__ float sP[kMaxG][kMaxR];
  __shared__ float sM[kMaxG], sL[kMaxG], sAlpha[kMaxG];
  __shared__ unsigned char sLoList[kD];
  __shared__ unsigned char sIsHi[kD];
  __shared__ int sNLo;                     // 2-bit channels of the staged block

  const mixkvq_config& cfg = cv.cfg;
  const Layout& lay = cv.lay;
  const int R = cfg.R, Gk = cfg.Gk, Gv = cfg.Gv, k4 = cfg.k4, k16 = cfg.k16, ks = k4 + k16, g = cv.g;
  const int p = blockIdx.x, split = blockIdx.y, tid = threadIdx.x;
  const int b = p / cfg.Hkv, j = p % cfg.Hkv;
  if (sc.enabled) {      // sequences of different lengths: this pair's own counts
    n_blocks = sc.n_blocks[b];
    n_fp16 = sc.n_fp16[b];
  }
  const int lane_lo = tid & (kD - 1), half = tid >> 7;   // role index and head half
  const int h0 = half * 4;                               // heads h0 .. h0+3 (< g)

  for (int i = tid; i < g * kD; i += kDecThreads)
    sQ[i / kD][i % kD] = __half2float(__ushort_as_half(in_bits(q + ((size_t)b * cfg.Hq + (size_t)j * g) * kD + i,
                                                               cfg.in_dtype != 0)));
  if (tid < kMaxG) { sM[tid] = -INFINITY; sL[tid] = 0.f; }

  float acc[4] = {0.f, 0.f, 0.f, 0.f};   // O[h0+i][channel lane_lo]

  const int blk0 = (int)((long long)n_blocks * split / n_splits);
  const int blk1 = (int)((long long)n_blocks * (split + 1) / n_splits);
  // the last split also takes the fp16 rows (sink, then residual window) in chunks of up to kMaxR tokens
  const int n_chunks = (split == n_splits - 1) ? (n_fp16 + kMaxR - 1) / kMaxR : 0;
  const int n_iter = (blk1 - blk0) + n_chunks;
  const __half* fk = cv.res_k + (size_t)p * cv.RW * kD;
  const __half* fv = cv.res_v + (size_t)p * cv.RW * kD;

  for (int it = 0; it < n_iter; ++it) {
    const bool is_res = it >= blk1 - blk0;
    const int row0 = is_res ? (it - (blk1 - blk0)) * kMaxR : 0;       // first fp16 row of this chunk
    const int nt = is_res ? (n_fp16 - row0 < kMaxR ? n_fp16 - row0 : kMaxR) : R;
    __syncthreads();
    const uint8_t* rec = cv.blocks + (is_res ? 0 : record_index(cv, p, blk0 + it)) * lay.rec_bytes;
    if (!is_res) {
      for (int i = tid; i < lay.rec_bytes / 16; i += kDecThreads)
        reinterpret_cast<uint4*>(sRec)[i] = reinterpret_cast<const uint4*>(rec)[i];
      if (tid < kD) sIsHi[tid] = 0;
      __syncthreads();
      if (tid < ks && sRec[lay.off_idx + tid] < kD) sIsHi[sRec[lay.off_idx + tid]] = 1;   // skips unused entries
      __syncthreads();
      if (tid < kD && !sIsHi[tid]) {
        int pos = 0;
        for (int e = 0; e < tid; ++e) pos += !sIsHi[e];
        sLoList[pos] = (unsigned char)tid;
      }
      if (tid == 0) {
        int c = 0;
        for (int e = 0; e < kD; ++e) c += !sIsHi[e];
        sNLo = c;
      }
      __syncthreads();
    }

    // ---- logits: thread (token t = lane_lo, heads h0..h0+3) ----
    if (lane_lo < nt && h0 < g) {
      const int t = lane_lo;
      float s[4] = {0.f, 0.f, 0.f, 0.f};
      if (is_res) {
        const __half* row = fk + (size_t)(row0 + t) * kD;
        for (int d = 0; d < kD; ++d) {
          const float kv = __half2float(row[d]);
#pragma unroll
          for (int i = 0; i < 4; ++i) s[i] += sQ[(h0 + i) & 7][d] * kv;
        }
      } else {
        const int grp = t / Gk;
        const unsigned* klo = reinterpret_cast<const unsigned*>(sRec + lay.off_klo) + t * lay.Wlo;
        const __half* ls = reinterpret_cast<const __half*>(sRec + lay.off_klo_s) + grp * lay.NLp;
        const __half* lz = reinterpret_cast<const __half*>(sRec + lay.off_klo_z) + grp * lay.NLp;
        for (int jj = 0; jj < sNLo; ++jj) {
          const unsigned c = (klo[jj >> 4] >> (16 * (jj & 1) + 2 * ((jj & 15) >> 1))) & 3u;
          const float kv = (float)c * __half2float(ls[jj]) + __half2float(lz[jj]);
          const int d = sLoList[jj];
#pragma unroll
          for (int i = 0; i < 4; ++i) s[i] += sQ[(h0 + i) & 7][d] * kv;
        }
        const unsigned* k4w = reinterpret_cast<const unsigned*>(sRec + lay.off_k4) + t * lay.W4;
        const __half* hs = reinterpret_cast<const __half*>(sRec + lay.off_k4_s) + grp * k4;
        const __half* hz = reinterpret_cast<const __half*>(sRec + lay.off_k4_z) + grp * k4;
        for (int jj = 0; jj < k4; ++jj) {
          const unsigned c = (k4w[jj >> 3] >> (16 * (jj & 1) + 4 * ((jj & 7) >> 1))) & 15u;
          const float kv = (float)c * __half2float(hs[jj]) + __half2float(hz[jj]);
          const int d = sRec[lay.off_idx + k16 + jj];
          if (d >= kD) break;      // the tier ends at the first unused entry
#pragma unroll
          for (int i = 0; i < 4; ++i) s[i] += sQ[(h0 + i) & 7][d] * kv;
        }
        const __half* k16p = reinterpret_cast<const __half*>(sRec + lay.off_k16) + t * k16;
        for (int jj = 0; jj < k16; ++jj) {
          const float kv = __half2float(k16p[jj]);
          const int d = sRec[lay.off_idx + jj];
          if (d >= kD) break;
#pragma unroll
          for (int i = 0; i < 4; ++i) s[i] += sQ[(h0 + i) & 7][d] * kv;
        }
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (h0 + i < g) sP[h0 + i][t] = s[i] * scale;
    }
    __syncthreads();

    // ---- online softmax: wave w owns heads w and w+4 ----
    {
      const int wave = tid >> 6, lane = tid & 63;
      for (int h = wave; h < g; h += 4) {
        float x0 = lane < nt ? sP[h][lane] : -INFINITY;
        float x1 = lane + 64 < nt ? sP[h][lane + 64] : -INFINITY;
        float mx = fmaxf(x0, x1);
        for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
        const float m_old = sM[h];
        const float m_new = fmaxf(m_old, mx);
        const float e0 = lane < nt ? __expf(x0 - m_new) : 0.f;
        const float e1 = lane + 64 < nt ? __expf(x1 - m_new) : 0.f;
        float sum = e0 + e1;
        for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
        if (lane < nt) sP[h][lane] = e0;
        if (lane + 64 < nt) sP[h][lane + 64] = e1;
        if (lane == 0) {
          const float alpha = __expf(m_old - m_new);   // exp(-inf) = 0 on the first block
          sAlpha[h] = alpha;
          sM[h] = m_new;
          sL[h] = sL[h] * alpha + sum;
        }
      }
    }
    __syncthreads();

    // ---- P.V: thread (channel d = lane_lo, heads h0..h0+3) ----
    if (h0 < g) {
      const int d = lane_lo;
#pragma unroll
      for (int i = 0; i < 4; ++i) acc[i] *= sAlpha[(h0 + i) & 7];
      if (is_res) {
        for (int t = 0; t < nt; ++t) {
          const float vv = __half2float(fv[(size_t)(row0 + t) * kD + d]);
#pragma unroll
          for (int i = 0; i < 4; ++i) acc[i] += sP[(h0 + i) & 7][t] * vv;
        }
      } else {
        const int vg = d / Gv;
        const unsigned* vw = reinterpret_cast<const unsigned*>(sRec + lay.off_v);
        const __half* vs = reinterpret_cast<const __half*>(sRec + lay.off_v_s);
        const __half* vz = reinterpret_cast<const __half*>(sRec + lay.off_v_z);
        for (int tg = 0; tg < R / 16; ++tg) {
          const unsigned w = vw[tg * kD + d];
#pragma unroll
          for (int i16 = 0; i16 < 16; ++i16) {
            const int t = value_word_token(tg, i16, lay.v_interleave);
            const float vv = (float)((w >> (16 * (i16 & 1) + 2 * (i16 >> 1))) & 3u) * __half2float(vs[t * lay.NVG + vg]) +
                             __half2float(vz[t * lay.NVG + vg]);
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[i] += sP[(h0 + i) & 7][t] * vv;
          }
        }
      }
    }
  }
  __syncthreads();
  // ---- partial result of this split ----
  float* out = part + ((size_t)p * n_splits + split) * g * kPartStride;
#pragma unroll
  for (int i = 0; i < 4; ++i)
    if (h0 + i < g) out[(h0 + i) * kPartStride + lane_lo] = acc[i];
  if (tid < g) {
    out[tid * kPartStride + kD] = sM[tid];
    out[tid * kPartStride + kD + 1] = sL[tid];
  }
}

// ---------------------------------------------------------------------------
// Merge of the splits: m* = max m_i, l* = sum l_i e^(m_i - m*), O = sum O_i e^(m_i - m*) / l*.
// One workgroup per (batch, query head), one thread per channel.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(kD) decode_merge_kernel(const float* __restrict__ part, int n_splits, int g, int Hq,
                                                         int out_bf16, __half* __restrict__ out, float* __restrict__ lse) {
  const int bh = blockIdx.x, b = bh / Hq, h = bh % Hq, d = threadIdx.x;
  const int Hkv = Hq / g, j = h / g, hh = h % g;
  const int p = b * Hkv + j;
  const float* base = part + ((size_t)p * n_splits * g + hh) * kPartStride;
  const size_t stride = (size_t)g * kPartStride;
  float m = -INFINITY;
#pragma unroll 8
  for (int s = 0; s < n_splits; ++s) m = fmaxf(m, base[s * stride + kD]);
  float l = 0.f, o = 0.f;
#pragma unroll 8
  for (int s = 0; s < n_splits; ++s) {
    const float ms = base[s * stride + kD];
    const float w = ms == -INFINITY ? 0.f : __expf(ms - m);
    l += base[s * stride + kD + 1] * w;
    o += base[s * stride + d] * w;
  }
  const float r = l > 0.f ? o / l : 0.f;       // l == 0: a sequence without tokens
  reinterpret_cast<unsigned short*>(out)[(size_t)bh * kD + d] =
      out_bf16 ? f32_to_bf16_bits(r) : __half_as_ushort(__float2half_rn(r));
  if (lse && d == 0) lse[bh] = l > 0.f ? m + __logf(l) : -INFINITY;
}

bool try_launch_decode_mfma(const CacheView& v, const __half* q, float scale, int n_blocks, int n_res, int n_splits,
                            float* part, __half* out, float* lse, int accumulate_q, NewToken nt, const SeqCounts& sc,
                            hipStream_t s, hipEvent_t ev_start, hipEvent_t ev_stop, hipError_t* err);

// Split count of a decode launch (one rule for every caller): enough workgroups to fill the chip (tunable through
// MIXKVQ_DECODE_WGS for experiments), never above the ceiling the workspace was sized for.  *n_splits_mc is the count
// the matrix-core kernel takes: its fp16 rows are cut into sub-units of 32 tokens and a wavefront takes at most one of
// them, so a pair needs at least as many wavefronts (4 per workgroup) as it has sub-units.
static void choose_splits(const CacheView& v, int n_blocks, int n_fp16, int* n_splits_out, int* n_splits_mc_out) {
  static const int target_wgs = [] {
    const char* e = getenv("MIXKVQ_DECODE_WGS");
    int t = e ? atoi(e) : 0;
    return t > 0 ? t : kDecodeTargetWGs;
  }();
  int n_splits = target_wgs / v.P;
  if (n_splits > max_splits_for(v.P)) n_splits = max_splits_for(v.P);
  if (n_splits > n_blocks) n_splits = n_blocks;
  if (n_splits < 1) n_splits = 1;
  int n_splits_mc = n_splits;
  const int min_splits = ((n_fp16 + 31) / 32 + 3) / 4;
  if (n_splits_mc < min_splits) n_splits_mc = min_splits;
  *n_splits_out = n_splits;
  *n_splits_mc_out = n_splits_mc;
}

size_t decode_launch_partials_bytes(const CacheView& v, int n_blocks, int n_fp16) {
  int n_splits, n_splits_mc;
  choose_splits(v, n_blocks, n_fp16, &n_splits, &n_splits_mc);
  const int n = n_splits_mc > n_splits ? n_splits_mc : n_splits;
  return (size_t)v.P * n * v.g * kPartStride * sizeof(float);
}

// ---------------------------------------------------------------------------
// Split-K partials for callers that cannot allocate (and pass no workspace): one array per GPU, resident from the
// moment the library is loaded until the process ends.  Every launch writes all the partials it later reads, so
// nothing has to be cleared; launches that share it must not overlap on one GPU.
// In host code the array's name is only a handle: the device address comes from hipGetSymbolAddress, once per
// device with that device current, and is what the kernels get.
// ---------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[kNoAllocScratchBytes];

hipError_t noalloc_scratch(void** out) {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static void* ptrs[kMaxDevices] = {};
  int device = 0;
  if (hipError_t e = hipGetDevice(&device); e != hipSuccess) return e;
  if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(mu);
  if (!ptrs[device]) {
    void* p = nullptr;
    if (hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)); e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    ptrs[device] = p;
  }
  *out = ptrs[device];
  return hipSuccess;
}

hipError_t launch_decode(const CacheView& v, const __half* q, __half* out, float* lse, float scale, int n_blocks,
                         int n_fp16, int accumulate_q, NewToken nt, const SeqCounts* sc_in, hipStream_t s,
                         hipEvent_t ev_start, hipEvent_t ev_stop, int* path, float* part) {
  static const SeqCounts kLockStep = [] { SeqCounts z; memset(&z, 0, sizeof(z)); return z; }();
  const SeqCounts& sc = sc_in ? *sc_in : kLockStep;
  int n_splits, n_splits_mc;
  choose_splits(v, n_blocks, n_fp16, &n_splits, &n_splits_mc);
  if (!part) part = reinterpret_cast<float*>(v.ws);
  hipError_t e = hipSuccess;
  if (n_splits_mc <= max_splits_for(v.P) &&
      try_launch_decode_mfma(v, q, scale, n_blocks, n_fp16, n_splits_mc, part, out, lse, accumulate_q, nt, sc, s,
                             ev_start, ev_stop, &e)) {
    *path = MIXKVQ_PATH_MATRIX;
    return e;
  }
  *path = MIXKVQ_PATH_VECTOR;
  if (nt.k) {   // this path does not move the new token itself
    e = launch_residual_copy(v, nt.k, nt.v, nt.st, 0, nt.row, 1, s);
    if (e != hipSuccess) return e;
  }
  if (accumulate_q) {
    Strides3 qs{(int64_t)v.cfg.Hq * kD, (int64_t)kD, (int64_t)kD};
    if (!sc.enabled) {
      e = launch_qabs_accumulate(v, q, 1, qs, s);
      if (e != hipSuccess) return e;
    } else {      // sequences without tokens are skipped
      for (int b = 0; b < v.cfg.B; ++b) {
        if (sc.n_blocks[b] == 0 && sc.n_fp16[b] == 0) continue;
        CacheView vb = v;
        vb.cfg.B = 1;
        vb.P = v.cfg.Hkv;
        vb.qacc += (size_t)b * v.cfg.Hkv * kD;
        vb.qcnt += (size_t)b * v.cfg.Hkv;
        e = launch_qabs_accumulate(vb, q + (size_t)b * v.cfg.Hq * kD, 1, qs, s);
        if (e != hipSuccess) return e;
      }
    }
  }
  if (ev_start) (void)hipEventRecord(ev_start, s);
  decode_split_kernel<<<dim3(v.P, n_splits), dim3(kDecThreads), 0, s>>>(v, q, scale, n_blocks, n_fp16, n_splits, part, sc);
  if (ev_stop) (void)hipEventRecord(ev_stop, s);
  decode_merge_kernel<<<dim3(v.cfg.B * v.cfg.Hq), dim3(kD), 0, s>>>(part, n_splits, v.g, v.cfg.Hq, v.cfg.in_dtype, out, lse);
  return hipGetLastError();
}

}  // namespace mixkvq
