// Quantize-and-pack of whole R-token blocks (the KeyQuant step of Appendix D.1)
// and the residual-window copy.
//
// One workgroup turns one block of one (batch, KV head) pair into its record:
// channel selection for the block (unless the caller fixed it), per-channel key
// groups at 2 bit / 4 bit / raw fp16, per-token 2-bit values.  The arithmetic of
// Eq. 2 is done in IEEE binary32 steps (subtract, correctly rounded divide, round
// half to even), so codes, scales and zero-points are reproducible bit for bit.
#include "mixkvq_internal.h"

// Eq. 2 must round exactly as written: no fused multiply-add contraction in this file.
#pragma clang fp contract(off)

namespace mixkvq {

constexpr int kFlushThreads = 256;
constexpr int kRowPad = 8;                 // halfs of padding per LDS row (keeps 16-byte alignment)
constexpr int kRowStride = kD + kRowPad;   // 136 halfs = 272 bytes

struct GroupParams { float s, z; unsigned short s16, z16; };

// Scale and zero-point of one group from its fp16 minimum and maximum (Eq. 2-3).
__device__ __forceinline__ GroupParams group_params(float mn, float mx, float levels) {
  mn = mn + 0.0f;   // -0 -> +0
  mx = mx + 0.0f;
  GroupParams r;
  __half z16 = __float2half_rn(mn);          // exact: mn is an fp16 value
  float s32 = (mx - mn) / levels;            // IEEE divide
  __half s16 = __float2half_rn(s32);
  r.s16 = h2bits(s16);
  r.z16 = h2bits(z16);
  r.s = __half2float(s16);
  r.z = __half2float(z16);
  return r;
}

__device__ __forceinline__ unsigned encode(float x, float z, float s, float top) {
  if (!(s > 0.f)) return 0u;
  float c = rintf((x - z) / s);
  c = fminf(fmaxf(c, 0.f), top);
  return (unsigned)c;
}

// Token `i` of the block being flushed: stream position pos = f*R + i of
// (old residual ++ new tokens); positions < r0 live in the residual window.
__device__ __forceinline__ const __half* token_row(const __half* res, const __half* fresh, Strides3 st, int p, int Hkv,
                                                  int R, int r0, int pos) {
  if (pos < r0) return res + ((size_t)p * R + pos) * kD;
  const int b = p / Hkv, j = p % Hkv;
  return fresh + (int64_t)b * st.b + (int64_t)j * st.h + (int64_t)(pos - r0) * st.t;
}

__device__ __forceinline__ void load_tile(__half* sT, const __half* res, const __half* fresh, Strides3 st, int p, int Hkv,
                                          int R, int r0, int pos0) {
  // R rows of 256 bytes; 16 threads per row, 16 bytes each
  for (int idx = threadIdx.x; idx < R * 16; idx += kFlushThreads) {
    const int t = idx >> 4, c = idx & 15;
    const __half* row = token_row(res, fresh, st, p, Hkv, R, r0, pos0 + t);
    uint4 v = *reinterpret_cast<const uint4*>(row + c * 8);
    *reinterpret_cast<uint4*>(sT + t * kRowStride + c * 8) = v;
  }
}

__global__ void __launch_bounds__(kFlushThreads)
flush_block_kernel(CacheView cv, const __half* __restrict__ k_new, const __half* __restrict__ v_new, Strides3 st, int r0,
                   int first_block, const uint8_t* __restrict__ sel_in) {
  __shared__ __align__(16) __half sT[kMaxR * kRowStride];   // K tile, then V tile
  __shared__ double sA[kD];
  __shared__ unsigned char sTier[kD];      // 0: 2 bit, 1: 4 bit, 2: fp16
  __shared__ unsigned char sPos[kD];       // position of the channel inside its tier
  __shared__ unsigned char sLoList[kD];    // 2-bit channels, ascending
  __shared__ unsigned char sHiList[kD];    // fp16 tier then 4-bit tier
  __shared__ float sS[8 * kD], sZ[8 * kD]; // [group][channel] scale / zero-point of the channel's tier
  __shared__ unsigned sKmax[8];            // per group: largest stored scale (fp16 bits; scales are >= 0)

  const mixkvq_config& cfg = cv.cfg;
  const Layout& lay = cv.lay;
  const int R = cfg.R, Gk = cfg.Gk, Gv = cfg.Gv, k4 = cfg.k4, k16 = cfg.k16, ks = k4 + k16;
  const int p = blockIdx.x, f = blockIdx.y, tid = threadIdx.x;
  uint8_t* rec = cv.blocks + ((size_t)p * cv.NB + first_block + f) * lay.rec_bytes;

  // zero the record's padding by clearing the small planes that may have holes
  // (index bytes and the tails of the scale/zero planes); full planes are overwritten below.
  for (int i = tid; i < lay.off_klo / 4; i += kFlushThreads) reinterpret_cast<unsigned*>(rec)[i] = 0u;

  load_tile(sT, cv.res_k, k_new, st, p, cfg.Hkv, R, r0, f * R);
  if (tid < 8) sKmax[tid] = 0u;
  __syncthreads();

  // ---- channel tiers --------------------------------------------------
  if (sel_in == nullptr && ks > 0) {
    double A = 0.0;
    if (tid < kD) {
      long long lo = 0x7fffffffffffffffll, hi = -0x7fffffffffffffffll - 1;
      for (int t = 0; t < R; ++t) {
        long long x = fix24(h2bits(sT[t * kRowStride + tid]));
        lo = x < lo ? x : lo;
        hi = x > hi ? x : hi;
      }
      const long long rng = hi - lo;
      A = cfg.score_mode ? (double)rng : (double)cv.qacc[(size_t)p * kD + tid] * (double)rng;
      sA[tid] = A;
    }
    __syncthreads();
    if (tid < kD) {
      int rank = 0;
      for (int e = 0; e < kD; ++e) {
        double o = sA[e];
        rank += (o > A) || (o == A && e < tid);
      }
      sTier[tid] = rank < k16 ? 2 : (rank < ks ? 1 : 0);
    }
  } else {
    if (tid < kD) sTier[tid] = 0;
    __syncthreads();
    if (tid < ks) sTier[sel_in[(size_t)p * ks + tid]] = tid < k16 ? 2 : 1;
  }
  __syncthreads();
  if (tid < kD) {
    const unsigned char tier = sTier[tid];
    int pos = 0;
    for (int e = 0; e < tid; ++e) pos += sTier[e] == tier;
    sPos[tid] = (unsigned char)pos;
    if (tier == 0) sLoList[pos] = (unsigned char)tid;
    else {
      const int slot = (tier == 2 ? 0 : k16) + pos;
      sHiList[slot] = (unsigned char)tid;
      rec[lay.off_idx + slot] = (uint8_t)tid;
    }
  }
  __syncthreads();

  // ---- key group parameters: one (group, channel) item per thread ----
  const int NG = lay.NG;
  for (int it = tid; it < NG * kD; it += kFlushThreads) {
    const int grp = it / kD, d = it % kD;
    const unsigned char tier = sTier[d];
    if (tier == 2) continue;
    float mn = __half2float(sT[(grp * Gk) * kRowStride + d]), mx = mn;
    for (int t = 1; t < Gk; ++t) {
      float x = __half2float(sT[(grp * Gk + t) * kRowStride + d]);
      mn = fminf(mn, x);
      mx = fmaxf(mx, x);
    }
    GroupParams gp = group_params(mn, mx, tier ? 15.f : 3.f);
    sS[grp * kD + d] = gp.s;
    sZ[grp * kD + d] = gp.z;
    const int pos = sPos[d];
    atomicMax(&sKmax[grp], (unsigned)gp.s16);
    if (tier == 0) {
      reinterpret_cast<unsigned short*>(rec + lay.off_klo_s)[grp * lay.NLp + pos] = gp.s16;
      reinterpret_cast<unsigned short*>(rec + lay.off_klo_z)[grp * lay.NLp + pos] = gp.z16;
    } else {
      reinterpret_cast<unsigned short*>(rec + lay.off_k4_s)[grp * k4 + pos] = gp.s16;
      reinterpret_cast<unsigned short*>(rec + lay.off_k4_z)[grp * k4 + pos] = gp.z16;
    }
  }
  __syncthreads();
  if (tid < NG) reinterpret_cast<unsigned short*>(rec + lay.off_kmax)[tid] = (unsigned short)sKmax[tid];

  // ---- 2-bit key words: [token][Wlo] ------------------------------------
  for (int it = tid; it < R * lay.Wlo; it += kFlushThreads) {
    const int t = it / lay.Wlo, wd = it % lay.Wlo, grp = t / Gk;
    unsigned w = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int jj = wd * 16 + i;
      if (jj < lay.NL) {
        const int d = sLoList[jj];
        w |= encode(__half2float(sT[t * kRowStride + d]), sZ[grp * kD + d], sS[grp * kD + d], 3.f) << (16 * (i & 1) + 2 * (i >> 1));
      }
    }
    reinterpret_cast<unsigned*>(rec + lay.off_klo)[it] = w;
  }
  // ---- 4-bit key words: [token][k4/8] -------------------------------------
  for (int it = tid; it < R * lay.W4; it += kFlushThreads) {
    const int t = it / lay.W4, wd = it % lay.W4, grp = t / Gk;
    unsigned w = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int d = sHiList[k16 + wd * 8 + i];
      w |= encode(__half2float(sT[t * kRowStride + d]), sZ[grp * kD + d], sS[grp * kD + d], 15.f) << (16 * (i & 1) + 4 * (i >> 1));
    }
    reinterpret_cast<unsigned*>(rec + lay.off_k4)[it] = w;
  }
  // ---- fp16 tier: [token][k16] ------------------------------------------
  for (int it = tid; it < R * k16; it += kFlushThreads) {
    const int t = it / k16, i = it % k16;
    reinterpret_cast<__half*>(rec + lay.off_k16)[it] = sT[t * kRowStride + sHiList[i]];
  }
  __syncthreads();

  // ---- values -----------------------------------------------------------------
  load_tile(sT, cv.res_v, v_new, st, p, cfg.Hkv, R, r0, f * R);
  __syncthreads();
  const int NVG = lay.NVG;
  float* sVS = sS;   // [token][NVG] (R * NVG <= 128 * 8)
  float* sVZ = sZ;
  for (int it = tid; it < R * NVG; it += kFlushThreads) {
    const int t = it / NVG, vg = it % NVG;
    const __half* row = sT + t * kRowStride + vg * Gv;
    float mn = __half2float(row[0]), mx = mn;
    for (int d = 1; d < Gv; ++d) {
      float x = __half2float(row[d]);
      mn = fminf(mn, x);
      mx = fmaxf(mx, x);
    }
    GroupParams gp = group_params(mn, mx, 3.f);
    sVS[it] = gp.s;
    sVZ[it] = gp.z;
    reinterpret_cast<unsigned short*>(rec + lay.off_v_s)[it] = gp.s16;
    reinterpret_cast<unsigned short*>(rec + lay.off_v_z)[it] = gp.z16;
  }
  __syncthreads();
  // value words: [token group][channel], 16 codes along tokens
  for (int it = tid; it < (R / 16) * kD; it += kFlushThreads) {
    const int tg = it / kD, d = it % kD, vg = d / Gv;
    unsigned w = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int t = tg * 16 + i;
      w |= encode(__half2float(sT[t * kRowStride + d]), sVZ[t * NVG + vg], sVS[t * NVG + vg], 3.f) << (16 * (i & 1) + 2 * (i >> 1));
    }
    reinterpret_cast<unsigned*>(rec + lay.off_v)[it] = w;
  }
}

hipError_t launch_flush(const CacheView& v, const __half* k_new, const __half* v_new, Strides3 kvs, int r0,
                        int first_block, int n_flush, const uint8_t* sel, hipStream_t s) {
  // grid.y is limited to 65535 blocks per launch
  for (int f0 = 0; f0 < n_flush; f0 += 32768) {
    const int nf = n_flush - f0 < 32768 ? n_flush - f0 : 32768;
    // shift the stream origin so that block index 0 of this launch is block f0 of the call
    flush_block_kernel<<<dim3(v.P, nf), dim3(kFlushThreads), 0, s>>>(v, k_new, v_new, kvs, r0 - f0 * v.cfg.R,
                                                                    first_block + f0, sel);
  }
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// residual-window copy: n tokens starting at new-token index src_first go to
// window rows dst_first.. of every pair.
// ---------------------------------------------------------------------------
__global__ void residual_copy_kernel(CacheView cv, const __half* __restrict__ k_new, const __half* __restrict__ v_new,
                                     Strides3 st, int src_first, int dst_first, int n) {
  const int p = blockIdx.x, b = p / cv.cfg.Hkv, j = p % cv.cfg.Hkv;
  for (int idx = blockIdx.y * blockDim.x + threadIdx.x; idx < n * 16; idx += gridDim.y * blockDim.x) {
    const int t = idx >> 4, c = idx & 15;
    const int64_t src = (int64_t)b * st.b + (int64_t)j * st.h + (int64_t)(src_first + t) * st.t + c * 8;
    const size_t dst = ((size_t)p * cv.cfg.R + dst_first + t) * kD + c * 8;
    *reinterpret_cast<uint4*>(cv.res_k + dst) = *reinterpret_cast<const uint4*>(k_new + src);
    *reinterpret_cast<uint4*>(cv.res_v + dst) = *reinterpret_cast<const uint4*>(v_new + src);
  }
}

hipError_t launch_residual_copy(const CacheView& v, const __half* k_new, const __half* v_new, Strides3 kvs,
                                int src_first, int dst_first, int n, hipStream_t s) {
  const int threads = n * 16 < 256 ? 64 : 256;
  int gy = (n * 16 + threads - 1) / threads;
  if (gy > 8) gy = 8;
  residual_copy_kernel<<<dim3(v.P, gy), dim3(threads), 0, s>>>(v, k_new, v_new, kvs, src_first, dst_first, n);
  return hipGetLastError();
}

}  // namespace mixkvq
