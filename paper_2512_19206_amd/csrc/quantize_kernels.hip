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
  mn = mn == 0.f ? 0.f : mn;   // -0 -> +0
  mx = mx == 0.f ? 0.f : mx;
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

// First row of pair p's residual window inside the pair's fp16 rows (the sink rows come first).
__device__ __forceinline__ const __half* window_rows(const CacheView& cv, const __half* res, int p) {
  return res + ((size_t)p * cv.RW + cv.S) * kD;
}

// Token `i` of the block being flushed: stream position pos = f*R + i of
// (old residual ++ new tokens); positions < r0 live in the residual window `win` of the pair.
__device__ __forceinline__ const __half* token_row(const __half* win, const __half* fresh, Strides3 st, int p, int Hkv,
                                                  int r0, int pos) {
  if (pos < r0) return win + (size_t)pos * kD;
  const int b = p / Hkv, j = p % Hkv;
  return fresh + (int64_t)b * st.b + (int64_t)j * st.h + (int64_t)(pos - r0) * st.t;
}

__device__ __forceinline__ void load_tile(__half* sT, const __half* win, const __half* fresh, Strides3 st, int p, int Hkv,
                                          int R, int r0, int pos0, bool bf16) {
  // R rows of 256 bytes; 16 threads per row, 16 bytes each.  Window rows are binary16 already; rows of the
  // caller's tensor may be bfloat16.
  for (int idx = threadIdx.x; idx < R * 16; idx += kFlushThreads) {
    const int t = idx >> 4, c = idx & 15;
    const __half* row = token_row(win, fresh, st, p, Hkv, r0, pos0 + t);
    uint4 v = as_f16x8(*reinterpret_cast<const uint4*>(row + c * 8), bf16 && pos0 + t >= r0);
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
  __shared__ unsigned sKmax[9];            // per key group: largest stored scale (fp16 bits; scales are >= 0); [8]: values
  __shared__ int sN[3];                    // channels per tier

  const mixkvq_config& cfg = cv.cfg;
  const Layout& lay = cv.lay;
  const int R = cfg.R, Gk = cfg.Gk, Gv = cfg.Gv, k4 = cfg.k4, k16 = cfg.k16, ks = k4 + k16;
  const int p = blockIdx.x, f = blockIdx.y, tid = threadIdx.x;
  uint8_t* rec = cv.blocks + record_index(cv, p, first_block + f) * lay.rec_bytes;

  // zero the record's padding by clearing the small planes that may have holes
  // (index bytes and the tails of the scale/zero planes); full planes are overwritten below.
  // (under the threshold policy the channel lists start out as "no channel")
  for (int i = tid; i < lay.off_klo / 4; i += kFlushThreads)
    reinterpret_cast<unsigned*>(rec)[i] = (cfg.policy == 1 && i < ks / 4) ? 0xffffffffu : 0u;

  load_tile(sT, window_rows(cv, cv.res_k, p), k_new, st, p, cfg.Hkv, R, r0, f * R, cfg.in_dtype != 0);
  if (tid < 9) sKmax[tid] = 0u;
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
      const double thr16 = cfg.policy == 1 ? score_threshold(cfg.tau16, cv.qcnt[p], cfg.score_mode) : 0.0;
      const double thr4 = cfg.policy == 1 ? score_threshold(cfg.tau4, cv.qcnt[p], cfg.score_mode) : 0.0;
      int rank = 0, c16 = 0, c_any = 0;
      for (int e = 0; e < kD; ++e) {
        double o = sA[e];
        rank += (o > A) || (o == A && e < tid);
        c16 += o > thr16;
        c_any += (o > thr16) || (o > thr4);
      }
      int n16, n4;
      tier_sizes(cfg, c16, c_any, &n16, &n4);
      sTier[tid] = rank < n16 ? 2 : (rank < n16 + n4 ? 1 : 0);
    }
  } else {
    if (tid < kD) sTier[tid] = 0;
    __syncthreads();
    if (tid < ks) {
      const unsigned ch = sel_in[(size_t)p * ks + tid];
      if (ch < (unsigned)kD) sTier[ch] = tid < k16 ? 2 : 1;     // MIXKVQ_NO_CHANNEL: an unused entry
    }
  }
  __syncthreads();
  if (tid < 3) {
    int c = 0;
    for (int e = 0; e < kD; ++e) c += sTier[e] == tid;
    sN[tid] = c;
  }
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
      if (jj < sN[0]) {
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
      if (wd * 8 + i < sN[1]) {
        const int d = sHiList[k16 + wd * 8 + i];
        w |= encode(__half2float(sT[t * kRowStride + d]), sZ[grp * kD + d], sS[grp * kD + d], 15.f) << (16 * (i & 1) + 4 * (i >> 1));
      }
    }
    reinterpret_cast<unsigned*>(rec + lay.off_k4)[it] = w;
  }
  // ---- fp16 tier: [token][k16] ------------------------------------------
  for (int it = tid; it < R * k16; it += kFlushThreads) {
    const int t = it / k16, i = it % k16;
    reinterpret_cast<__half*>(rec + lay.off_k16)[it] = i < sN[2] ? sT[t * kRowStride + sHiList[i]] : __ushort_as_half(0);
  }
  __syncthreads();

  // ---- values -----------------------------------------------------------------
  load_tile(sT, window_rows(cv, cv.res_v, p), v_new, st, p, cfg.Hkv, R, r0, f * R, cfg.in_dtype != 0);
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
    atomicMax(&sKmax[8], (unsigned)gp.s16);
    reinterpret_cast<unsigned short*>(rec + lay.off_v_s)[it] = gp.s16;
    reinterpret_cast<unsigned short*>(rec + lay.off_v_z)[it] = gp.z16;
  }
  __syncthreads();
  if (tid == 0) reinterpret_cast<unsigned short*>(rec + lay.off_kmax)[NG] = (unsigned short)sKmax[8];
  // value words: [token group][channel], 16 codes along tokens
  for (int it = tid; it < (R / 16) * kD; it += kFlushThreads) {
    const int tg = it / kD, d = it % kD, vg = d / Gv;
    unsigned w = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int t = value_word_token(tg, i, lay.v_interleave);
      w |= encode(__half2float(sT[t * kRowStride + d]), sVZ[t * NVG + vg], sVS[t * NVG + vg], 3.f) << (16 * (i & 1) + 2 * (i >> 1));
    }
    reinterpret_cast<unsigned*>(rec + lay.off_v)[it] = w;
  }
}

// ---------------------------------------------------------------------------
// The same record, built for throughput (Gk a multiple of 16, Gv >= 16, 16-byte aligned rows):
//   - both tiles are fetched with all loads in flight at once (the value tile waits in registers while the
//     keys are encoded);
//   - minima and maxima are taken with packed fp16 instructions, two channels at a time, first per chunk of
//     16 tokens (all threads), then per group / per block;
//   - positions inside the tiers come from wavefront ballots;
//   - in the encode loops a thread keeps the parameters of its channels (keys) or tokens (values) in registers
//     and only the element itself comes from LDS; a code costs one fused multiply-add, a rounding and its share
//     of the check that the shortcut is safe (see code_fast); the few codes that fail the check are redone with
//     Eq. 2's division.
// The codes, scales and zero-points are bit-identical to those of flush_block_kernel.
// ---------------------------------------------------------------------------
typedef _Float16 fh2 __attribute__((ext_vector_type(2)));
// Row stride of the staged tile in this kernel: 65 words, an odd number, so that the rows a wavefront reads in one
// instruction (8 consecutive tokens x 8 word columns 8 words apart in the key loop, 64 tokens in the 4-bit loop) fall
// into different LDS banks; rows are then only 4-byte aligned, and a 16-byte piece is staged with four 4-byte writes.
constexpr int kFastStride = kD + 2;

#ifdef MIXKVQ_PHASE_CLOCKS
// Profiling aid, not part of the default build: 100 MHz timestamps of the phases of the first 1024 workgroups.
__device__ unsigned long long g_flush_clock[1024 * 16];
#define MIXKVQ_FPHASE(K_)                                                      \
  if (threadIdx.x == 0 && blockIdx.x + gridDim.x * blockIdx.y < 1024)          \
    g_flush_clock[(blockIdx.x + gridDim.x * blockIdx.y) * 16 + (K_)] = wall_clock64();
#else
#define MIXKVQ_FPHASE(K_)
#endif

// Minima and maxima are taken with the packed fp16 instructions, two values at a time.  Which zero they return for
// {-0, +0} does not matter: group_params() and the integer range both take -0 as +0.
__device__ __forceinline__ fh2 as_h2(unsigned w) { return __builtin_bit_cast(fh2, w); }
__device__ __forceinline__ unsigned short h_bits(_Float16 h) { return __builtin_bit_cast(unsigned short, h); }

// Fast form of Eq. 2's code: q0 = x*r + nz in one fused multiply-add, with r the reciprocal of the scale and
// nz = -z*r, both per group.  Against the quotient q that Eq. 2 defines (fp32 subtract, correctly rounded divide):
//   |q0 - q| <= |q| (2^-23 [rcp] + 2^-24 [fma] + 2^-23 [the two roundings of q]) + |z r| 2^-24,
// i.e. below 2.9e-6 for two-bit codes (q <= 3.002) and below 6.5e-6 for four-bit codes (q <= 15.008) as long as
// |z r| <= 32 and the scale is a normal binary16 (its rounding is then fine enough that no quotient passes the top
// code by more than 0.008).  So whenever q0 is further than EPS (2^-18, 2^-16) from every half-integer, rint(q0) IS
// the code Eq. 2 defines, with no clamp needed; `dev` collects the largest distance from the nearest integer over a
// word, and the caller redoes a word with dev > 1/2 - EPS with the IEEE division.  Groups outside those conditions
// get (r, nz) = (0, 1/2): every q0 is 1/2, so all their words are redone.  Scale 0 gets (0, 0): code 0.
// The code is returned as a float: the callers build each half-word of a packed word as an exact fp32 sum
// c_0 + c_1 2^w + c_2 2^2w + ... (< 2^16) with one fused multiply-add per code and convert once per half-word.
constexpr float kEps2 = 3.814697265625e-6f, kEps4 = 1.52587890625e-5f;
__device__ __forceinline__ void fast_params(float s, float z, float* r, float* nz) {
  float rr = s > 0.f ? __builtin_amdgcn_rcpf(s) : 0.f;
  float nn = -z * rr;
  if (s > 0.f && (s < 6.103515625e-05f || !(fabsf(nn) <= 32.f))) {
    rr = 0.f;
    nn = 0.5f;
  }
  *r = rr;
  *nz = nn;
}
__device__ __forceinline__ float code_fast(__half x, float r, float nz, float& dev) {
  const float q0 = __builtin_fmaf(__half2float(x), r, nz);
  const float c = rintf(q0);
  dev = fmaxf(dev, fabsf(q0 - c));
  return c;
}
// Eq. 2's code itself (IEEE division) as a float, from the group's packed parameters (scale | zero-point << 16, binary16 bits).
__device__ __forceinline__ float code_exact(__half x, unsigned sz, float top) {
  const float s = __half2float(__ushort_as_half((unsigned short)(sz & 0xffffu)));
  const float z = __half2float(__ushort_as_half((unsigned short)(sz >> 16)));
  if (!(s > 0.f)) return 0.f;
  return fminf(fmaxf(rintf((__half2float(x) - z) / s), 0.f), top);
}
// code i of a word sits at bit 16 (i & 1) + W (i >> 1): even codes in the low half-word, odd codes in the high one
template <int W>
__device__ __forceinline__ void add_code(float (&half)[2], int i, float c) {
  half[i & 1] = __builtin_fmaf(c, (float)(1u << (W * (i >> 1))), half[i & 1]);
}
__device__ __forceinline__ unsigned join_halves(const float (&half)[2]) {
  return (unsigned)half[0] | ((unsigned)half[1] << 16);
}

// largest value over the wavefront (every lane must take part)
__device__ __forceinline__ unsigned wave_max_u32(unsigned v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const unsigned other = (unsigned)__shfl_xor((int)v, o);
    v = other > v ? other : v;
  }
  return v;
}

// 16-byte piece `idx` of the tile that starts at stream position pos0; `res_p` and `fresh_p` are the pair's
// residual window and its slice of the caller's tensor (token 0 of this call).
__device__ __forceinline__ uint4 load_chunk(const __half* res_p, const __half* fresh_p, int64_t stride_t, int r0, int pos0,
                                            int idx, bool bf16) {
  const int pos = pos0 + (idx >> 4), c = idx & 15;
  const __half* row = pos < r0 ? res_p + (size_t)pos * kD : fresh_p + (int64_t)(pos - r0) * stride_t;
  return as_f16x8(*reinterpret_cast<const uint4*>(row + c * 8), bf16 && pos >= r0);   // window rows are binary16 already
}

__global__ void __launch_bounds__(kFlushThreads, 3)   // three workgroups per CU (LDS) = three wavefronts per SIMD
flush_block_fast_kernel(CacheView cv, const __half* __restrict__ k_new, const __half* __restrict__ v_new, Strides3 st,
                        int r0, int first_block, const uint8_t* __restrict__ sel_in) {
  __shared__ __align__(16) __half sT[kMaxR * kFastStride];   // K tile, then V tile
  __shared__ double sA[kD];
  __shared__ unsigned char sTier[kD];      // 0: 2 bit, 1: 4 bit, 2: fp16
  __shared__ unsigned char sPos[kD];       // position of the channel inside its tier
  __shared__ unsigned char sLoList[kD];    // 2-bit channels, ascending
  __shared__ unsigned char sHiList[kD];    // fp16 tier then 4-bit tier
  // parameters of the groups, keys: [group][channel], values: [token][value group]: the pair (r, nz) of the fast
  // codes, and scale | zero-point << 16 (binary16 bits) for the codes that are redone with the division
  __shared__ __align__(16) float sRN[2 * 8 * kD];
  float* const sR = sRN;               // r
  float* const sNZ = sRN + 8 * kD;     // nz
  __shared__ unsigned sSZ[8 * kD];
  __shared__ unsigned sKmax[9];            // [8]: largest value scale
  __shared__ unsigned sChunk[2][kMaxR / 16][kD / 2];   // (min, max) keys per 16-token chunk and channel pair
  unsigned (*sCLo)[kD / 2] = sChunk[0];
  unsigned (*sCHi)[kD / 2] = sChunk[1];
  __shared__ int sCnt[6];                  // channels per tier in wavefront 0, then in wavefront 1

  const int R = cv.cfg.R, Gk = cv.cfg.Gk, Gv = cv.cfg.Gv, k4 = cv.cfg.k4, k16 = cv.cfg.k16, ks = k4 + k16;
  const int Hkv = cv.cfg.Hkv, score_mode = cv.cfg.score_mode, policy = cv.cfg.policy;
  const bool bf16 = cv.cfg.in_dtype != 0;
  const int rec_bytes = cv.lay.rec_bytes, off_idx = cv.lay.off_idx, off_kmax = cv.lay.off_kmax,
            off_klo_s = cv.lay.off_klo_s, off_klo_z = cv.lay.off_klo_z, off_k4_s = cv.lay.off_k4_s,
            off_k4_z = cv.lay.off_k4_z, off_klo = cv.lay.off_klo, off_k4 = cv.lay.off_k4, off_k16 = cv.lay.off_k16,
            off_v = cv.lay.off_v, off_v_s = cv.lay.off_v_s, off_v_z = cv.lay.off_v_z, NLp = cv.lay.NLp,
            Wlo = cv.lay.Wlo, W4 = cv.lay.W4, NG = cv.lay.NG, NVG = cv.lay.NVG;
  const int p = blockIdx.x, f = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  uint8_t* rec = cv.blocks + record_index(cv, p, first_block + f) * rec_bytes;
  const int n_chunks16 = R * 16;           // 16-byte pieces of a tile
  const int n_ch = R / 16;                 // chunks of 16 tokens

  MIXKVQ_FPHASE(0)
  // ---- the key tile first; the value tile is requested once the keys are staged in LDS, so that the wait for the
  //      keys is a wait for 32 KiB and the values arrive while the keys are encoded ------------------------------
  uint4 kreg[8], vreg[8];
  const int64_t pair_off = (int64_t)(p / Hkv) * st.b + (int64_t)(p % Hkv) * st.h;
  const __half* res_kp = window_rows(cv, cv.res_k, p);
  const __half* res_vp = window_rows(cv, cv.res_v, p);
  const int pos0 = f * R;
  // the usual case: the whole tile comes from one place, rows a constant stride apart; else it straddles the end of
  // the residual window (first block of an append onto a partly filled window)
  const bool one_place = pos0 >= r0 || pos0 + R <= r0;
  const bool from_res = pos0 + R <= r0;
  const int64_t row_stride = from_res ? (int64_t)kD : st.t;
  const int64_t first = (int64_t)(from_res ? pos0 : pos0 - r0) + (tid >> 4);
  const bool v_pending = one_place && bf16 && !from_res;     // the value tile in registers still holds bfloat16
  if (one_place) {
    const __half* kp = (from_res ? res_kp : k_new + pair_off) + first * row_stride + (tid & 15) * 8;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      kreg[i] = make_uint4(0u, 0u, 0u, 0u);
      if (tid + kFlushThreads * i < n_chunks16) kreg[i] = *reinterpret_cast<const uint4*>(kp + 16 * i * row_stride);
    }
    if (bf16 && !from_res) {     // rows of the caller's bfloat16 tensors enter as binary16 (the values when they are staged)
#pragma unroll
      for (int i = 0; i < 8; ++i) kreg[i] = as_f16x8(kreg[i], true);
    }
  } else {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int idx = tid + kFlushThreads * i;
      kreg[i] = make_uint4(0u, 0u, 0u, 0u);
      if (idx < n_chunks16) kreg[i] = load_chunk(res_kp, k_new + pair_off, st.t, r0, pos0, idx, bf16);
    }
  }
  // zero the small planes of the record (index bytes, tails of the scale/zero planes)
  // (under the threshold policy the channel lists start out as "no channel")
  for (int i = tid; i < off_klo / 4; i += kFlushThreads)
    reinterpret_cast<unsigned*>(rec)[i] = (policy == 1 && i < ks / 4) ? 0xffffffffu : 0u;
  if (tid < 9) sKmax[tid] = 0u;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int idx = tid + kFlushThreads * i;
    if (idx < n_chunks16) {
      unsigned* dst = reinterpret_cast<unsigned*>(sT + (idx >> 4) * kFastStride + (idx & 15) * 8);
      dst[0] = kreg[i].x; dst[1] = kreg[i].y; dst[2] = kreg[i].z; dst[3] = kreg[i].w;
    }
  }
  if (one_place) {
    const __half* vp = (from_res ? res_vp : v_new + pair_off) + first * row_stride + (tid & 15) * 8;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      vreg[i] = make_uint4(0u, 0u, 0u, 0u);
      if (tid + kFlushThreads * i < n_chunks16) vreg[i] = *reinterpret_cast<const uint4*>(vp + 16 * i * row_stride);
    }
  } else {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int idx = tid + kFlushThreads * i;
      vreg[i] = make_uint4(0u, 0u, 0u, 0u);
      if (idx < n_chunks16) vreg[i] = load_chunk(res_vp, v_new + pair_off, st.t, r0, pos0, idx, bf16);
    }
  }
  __syncthreads();

  MIXKVQ_FPHASE(1)
  // ---- minimum / maximum per chunk of 16 tokens and channel pair -----------------------------
  {
    const int d2 = tid & 63;
    const unsigned* sT32 = reinterpret_cast<const unsigned*>(sT);
    for (int ch = tid >> 6; ch < n_ch; ch += 4) {
      fh2 lo = as_h2(sT32[(16 * ch) * (kFastStride / 2) + d2]), hi = lo;
#pragma unroll
      for (int t = 1; t < 16; ++t) {
        const fh2 key = as_h2(sT32[(16 * ch + t) * (kFastStride / 2) + d2]);
        lo = __builtin_elementwise_min(lo, key);
        hi = __builtin_elementwise_max(hi, key);
      }
      sCLo[ch][d2] = __builtin_bit_cast(unsigned, lo);
      sCHi[ch][d2] = __builtin_bit_cast(unsigned, hi);
    }
  }
  __syncthreads();

  MIXKVQ_FPHASE(2)
  // ---- channel tiers ------------------------------------------------------------------------
  if (sel_in == nullptr && ks > 0) {
    double A = 0.0;
    if (tid < kD) {
      const _Float16* cl = reinterpret_cast<const _Float16*>(&sCLo[0][0]);
      const _Float16* chh = reinterpret_cast<const _Float16*>(&sCHi[0][0]);
      _Float16 lo = cl[tid], hi = chh[tid];
      for (int ch = 1; ch < n_ch; ++ch) {
        const _Float16 a = cl[ch * kD + tid], b2 = chh[ch * kD + tid];
        lo = a < lo ? a : lo;
        hi = b2 > hi ? b2 : hi;
      }
      const long long rng = fix24(h_bits(hi)) - fix24(h_bits(lo));
      A = score_mode ? (double)rng : (double)cv.qacc[(size_t)p * kD + tid] * (double)rng;
      sA[tid] = A;
    }
    __syncthreads();
    // rank of every channel (number of channels that beat it) and, under the threshold policy, how many channels
    // pass each threshold: the two halves of the workgroup each compare against 64 of the channels
    {
      const int d = tid & (kD - 1), e0 = (tid >> 7) * (kD / 2);
      const double Ad = sA[d];
      int rank = 0, c16 = 0, c_any = 0;
      if (policy == 1) {
        const double thr16 = score_threshold(cv.cfg.tau16, cv.qcnt[p], score_mode);
        const double thr4 = score_threshold(cv.cfg.tau4, cv.qcnt[p], score_mode);
        for (int e = e0; e < e0 + kD / 2; ++e) {
          const double o = sA[e];
          rank += (o > Ad) || (o == Ad && e < d);
          c16 += o > thr16;
          c_any += (o > thr16) || (o > thr4);
        }
      } else {
        for (int e = e0; e < e0 + kD / 2; ++e) {
          const double o = sA[e];
          rank += (o > Ad) || (o == Ad && e < d);
        }
      }
      unsigned* sPart = reinterpret_cast<unsigned*>(sR);      // not yet in use: [2][kD] packed partial counts
      sPart[tid] = (unsigned)rank | ((unsigned)c16 << 8) | ((unsigned)c_any << 16);     // each count <= 64
      __syncthreads();
      if (tid < kD) {
        const unsigned both = sPart[tid] + sPart[tid + kD];                              // each count <= 128: no carry
        rank = (int)(both & 0xffu);
        c16 = (int)((both >> 8) & 0xffu);
        c_any = (int)((both >> 16) & 0xffu);
        int n16, n4;
        tier_sizes(cv.cfg, c16, c_any, &n16, &n4);
        sTier[tid] = rank < n16 ? 2 : (rank < n16 + n4 ? 1 : 0);
      }
    }
  } else {
    if (tid < kD) sTier[tid] = 0;
    __syncthreads();
    if (tid < ks) {
      const unsigned ch = sel_in[(size_t)p * ks + tid];
      if (ch < (unsigned)kD) sTier[ch] = tid < k16 ? 2 : 1;     // MIXKVQ_NO_CHANNEL: an unused entry
    }
  }
  __syncthreads();
  // position of every channel inside its tier: ballots over the two wavefronts that hold the channels
  {
    const int tier = tid < kD ? sTier[tid] : 3;
    const unsigned long long m0 = __ballot(tier == 0), m1 = __ballot(tier == 1), m2 = __ballot(tier == 2);
    if (lane == 0 && wave < 2) {
      sCnt[3 * wave] = __popcll(m0);
      sCnt[3 * wave + 1] = __popcll(m1);
      sCnt[3 * wave + 2] = __popcll(m2);
    }
    __syncthreads();
    if (tid < kD) {
      const unsigned long long mine = tier == 0 ? m0 : (tier == 1 ? m1 : m2);
      const int pos = __popcll(mine & ((1ull << lane) - 1ull)) + (wave == 1 ? sCnt[tier] : 0);
      sPos[tid] = (unsigned char)pos;
      if (tier == 0) sLoList[pos] = (unsigned char)tid;
      else {
        const int slot = (tier == 2 ? 0 : k16) + pos;
        sHiList[slot] = (unsigned char)tid;
        rec[off_idx + slot] = (uint8_t)tid;
      }
    }
  }
  __syncthreads();

  // sizes of the tiers of this block (the budgets, or what passed the thresholds)
  // (the same for every thread: kept in scalar registers)
  const int n_lo = __builtin_amdgcn_readfirstlane(sCnt[0] + sCnt[3]), n_4 = __builtin_amdgcn_readfirstlane(sCnt[1] + sCnt[4]),
            n_16 = __builtin_amdgcn_readfirstlane(sCnt[2] + sCnt[5]);

  MIXKVQ_FPHASE(3)
  // ---- key group parameters from the chunk extrema ------------------------------------------
  {
    const _Float16* cl = reinterpret_cast<const _Float16*>(&sCLo[0][0]);
    const _Float16* chh = reinterpret_cast<const _Float16*>(&sCHi[0][0]);
    const int cpg = Gk / 16;     // chunks per group
    // (a wavefront's 64 items of one pass belong to one group: its largest scale is reduced over the wavefront first,
    //  one LDS atomic per wavefront and pass)
    for (int it = tid; it < NG * kD; it += kFlushThreads) {
      const int grp = it / kD, d = it % kD;
      const unsigned char tier = sTier[d];
      unsigned s16v = 0u;
      if (tier != 2) {
        _Float16 lo = cl[(grp * cpg) * kD + d], hi = chh[(grp * cpg) * kD + d];
        for (int c = 1; c < cpg; ++c) {
          const _Float16 a = cl[(grp * cpg + c) * kD + d], b2 = chh[(grp * cpg + c) * kD + d];
          lo = a < lo ? a : lo;
          hi = b2 > hi ? b2 : hi;
        }
        const GroupParams gp = group_params((float)lo, (float)hi, tier ? 15.f : 3.f);
        sSZ[grp * kD + d] = (unsigned)gp.s16 | ((unsigned)gp.z16 << 16);
        fast_params(gp.s, gp.z, &sR[grp * kD + d], &sNZ[grp * kD + d]);
        const int pos = sPos[d];
        s16v = gp.s16;
        if (tier == 0) {
          reinterpret_cast<unsigned short*>(rec + off_klo_s)[grp * NLp + pos] = gp.s16;
          reinterpret_cast<unsigned short*>(rec + off_klo_z)[grp * NLp + pos] = gp.z16;
        } else {
          reinterpret_cast<unsigned short*>(rec + off_k4_s)[grp * k4 + pos] = gp.s16;
          reinterpret_cast<unsigned short*>(rec + off_k4_z)[grp * k4 + pos] = gp.z16;
        }
      }
      const unsigned wmax = wave_max_u32(s16v);
      if (lane == 0) atomicMax(&sKmax[grp], wmax);
    }
  }
  __syncthreads();
  if (tid < NG) reinterpret_cast<unsigned short*>(rec + off_kmax)[tid] = (unsigned short)sKmax[tid];

  MIXKVQ_FPHASE(4)
  // ---- 2-bit key words [token][Wlo]: thread = (word column, token lane); the 16 channels of the column
  //      and their parameters stay in registers ---------------------------------------------------------
  {
    const int wd = tid & 7, tl = tid >> 3;
    if (wd < Wlo) {
      int doff[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int jj = 16 * wd + i;
        doff[i] = jj < n_lo ? (int)sLoList[jj] : -1;
      }
      for (int grp = 0; grp < NG; ++grp) {
        float rc[16], nz[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int d = doff[i] < 0 ? 0 : doff[i];
          rc[i] = doff[i] < 0 ? 0.f : sR[grp * kD + d];   // (0, 0) gives code 0: the padding of the last word
          nz[i] = doff[i] < 0 ? 0.f : sNZ[grp * kD + d];
        }
        // LDS address of each of the 16 elements in this thread's first token of the group; its other tokens are 32
        // rows further each, a compile-time distance once the loop is unrolled (no address arithmetic per element)
        const __half* col[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) col[i] = sT + (grp * Gk + tl) * kFastStride + (doff[i] < 0 ? 0 : doff[i]);
        const int n_it = (Gk - tl + 31) / 32;      // tokens tl, tl + 32, ... below Gk: at most 4 (Gk <= 128)
#pragma unroll
        for (int k = 0; k < kMaxR / 32; ++k) {
          if (k >= n_it) break;
          const int t = grp * Gk + tl + 32 * k;
          float hw[2] = {0.f, 0.f};
          float dev[4] = {0.f, 0.f, 0.f, 0.f};     // per run of four codes: the search below stays short
#pragma unroll
          for (int i = 0; i < 16; ++i)
            add_code<2>(hw, i, code_fast(col[i][k * 32 * kFastStride], rc[i], nz[i], dev[i >> 2]));
          // some quotient sits next to a rounding boundary (exact ties are common: about every other pass has one)
          if (__any(fmaxf(fmaxf(dev[0], dev[1]), fmaxf(dev[2], dev[3])) > 0.5f - kEps2)) {
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
              if (!__any(dev[i4] > 0.5f - kEps2)) continue;
#pragma unroll
              for (int i = 4 * i4; i < 4 * i4 + 4; ++i) {     // find the codes concerned and correct them
                const int d = doff[i] < 0 ? 0 : doff[i];
                const __half x = col[i][k * 32 * kFastStride];
                float dv = 0.f;
                const float c = code_fast(x, rc[i], nz[i], dv);
                if (__any(dv > 0.5f - kEps2))
                  add_code<2>(hw, i, code_exact(x, doff[i] < 0 ? 0u : sSZ[grp * kD + d], 3.f) - c);
              }
            }
          }
          const unsigned w = join_halves(hw);
          reinterpret_cast<unsigned*>(rec + off_klo)[t * Wlo + wd] = w;
        }
      }
    }
  }
  MIXKVQ_FPHASE(5)
  // ---- 4-bit key words: [token][k4/8] -------------------------------------
  // (a thread keeps its token; the two halves of the workgroup alternate over the words: no divisions by run-time values)
  for (int wd = tid >> 7; wd < W4; wd += 2) {
    const int t = tid & 127;
    if (t >= R) break;
    const int grp = t / Gk, it = t * W4 + wd;
    float hw[2] = {0.f, 0.f};
    float dev[2] = {0.f, 0.f};
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const bool used = wd * 8 + i < n_4;                    // an unused entry gets (0, 0), i.e. code 0
      const int d = used ? sHiList[k16 + wd * 8 + i] : 0;
      add_code<4>(hw, i, code_fast(sT[t * kFastStride + d], used ? sR[grp * kD + d] : 0.f,
                                   used ? sNZ[grp * kD + d] : 0.f, dev[i >> 2]));
    }
    if (__any(fmaxf(dev[0], dev[1]) > 0.5f - kEps4)) {     // some quotient sits next to a rounding boundary
#pragma unroll
      for (int i4 = 0; i4 < 2; ++i4) {
        if (!__any(dev[i4] > 0.5f - kEps4)) continue;
#pragma unroll
        for (int i = 4 * i4; i < 4 * i4 + 4; ++i) {
          const bool used = wd * 8 + i < n_4;
          const int d = used ? sHiList[k16 + wd * 8 + i] : 0;
          float dv = 0.f;
          const float c = code_fast(sT[t * kFastStride + d], used ? sR[grp * kD + d] : 0.f, used ? sNZ[grp * kD + d] : 0.f, dv);
          if (__any(dv > 0.5f - kEps4))
            add_code<4>(hw, i, code_exact(sT[t * kFastStride + d], used ? sSZ[grp * kD + d] : 0u, 15.f) - c);
        }
      }
    }
    const unsigned w = join_halves(hw);
    reinterpret_cast<unsigned*>(rec + off_k4)[it] = w;
  }
  // ---- fp16 tier: [token][k16] ------------------------------------------
  for (int i = tid >> 7; i < k16; i += 2) {
    const int t = tid & 127;
    if (t < R) reinterpret_cast<__half*>(rec + off_k16)[t * k16 + i] = i < n_16 ? sT[t * kFastStride + sHiList[i]] : __ushort_as_half(0);
  }
  __syncthreads();

  MIXKVQ_FPHASE(6)
  // ---- values ---------------------------------------------------------------------------------
  // The tile goes to LDS; on the way every thread reduces its 16-byte pieces (still in registers) to the minimum
  // and maximum per token and value group: 16 threads cover a row, a group is Gv/8 neighbouring threads, and the
  // pair (min, -max) is reduced with packed fp16 minima over DPP lane exchanges inside the row of 16.
  {
    const int c = tid & 15, lpg = Gv / 8;                 // lpg = 2, 4, 8 or 16 (Gv divides 128)
    const int lpg_shift = 31 - __builtin_clz(lpg);
    unsigned* sRow = &sChunk[0][0][0];     // [token][value group] packed (min, -max); <= 128 * 8 entries
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int row = (tid >> 4) + 16 * i;
      if (row < R) {
        const uint4 v = as_f16x8(vreg[i], v_pending);
        unsigned* dst = reinterpret_cast<unsigned*>(sT + row * kFastStride + c * 8);
        dst[0] = v.x; dst[1] = v.y; dst[2] = v.z; dst[3] = v.w;
        const fh2 k0 = as_h2(v.x), k1 = as_h2(v.y), k2 = as_h2(v.z), k3 = as_h2(v.w);
        const fh2 lo2 = __builtin_elementwise_min(__builtin_elementwise_min(k0, k1), __builtin_elementwise_min(k2, k3));
        const fh2 hi2 = __builtin_elementwise_max(__builtin_elementwise_max(k0, k1), __builtin_elementwise_max(k2, k3));
        fh2 m;
        m[0] = lo2[0] < lo2[1] ? lo2[0] : lo2[1];
        m[1] = -(hi2[0] > hi2[1] ? hi2[0] : hi2[1]);
        int mi = __builtin_bit_cast(int, m);
#define MIXKVQ_DPP_MIN(CTRL)                                                                                   \
  mi = __builtin_bit_cast(int, __builtin_elementwise_min(                                                      \
      __builtin_bit_cast(fh2, mi), __builtin_bit_cast(fh2, __builtin_amdgcn_update_dpp(mi, mi, CTRL, 0xf, 0xf, false))));
        if (lpg >= 2) MIXKVQ_DPP_MIN(0xB1)     // quad_perm [1,0,3,2]
        if (lpg >= 4) MIXKVQ_DPP_MIN(0x4E)     // quad_perm [2,3,0,1]
        if (lpg >= 8) MIXKVQ_DPP_MIN(0x141)    // row_half_mirror
        if (lpg >= 16) MIXKVQ_DPP_MIN(0x140)   // row_mirror
#undef MIXKVQ_DPP_MIN
        if ((c & (lpg - 1)) == 0) sRow[row * NVG + (c >> lpg_shift)] = (unsigned)mi;
      }
    }
    MIXKVQ_FPHASE(7)
    __syncthreads();
    unsigned vmax_t = 0u;
    for (int it = tid; it < R * NVG; it += kFlushThreads) {
      const fh2 mm = as_h2(sRow[it]);
      const GroupParams gp = group_params((float)mm[0], -(float)mm[1], 3.f);
      sSZ[it] = (unsigned)gp.s16 | ((unsigned)gp.z16 << 16);
      fast_params(gp.s, gp.z, &sR[it], &sNZ[it]);
      vmax_t = gp.s16 > vmax_t ? gp.s16 : vmax_t;
      reinterpret_cast<unsigned short*>(rec + off_v_s)[it] = gp.s16;
      reinterpret_cast<unsigned short*>(rec + off_v_z)[it] = gp.z16;
    }
    const unsigned wmax = wave_max_u32(vmax_t);       // every lane is here: the loop above has ended for all
    if (lane == 0) atomicMax(&sKmax[8], wmax);
  }
  __syncthreads();
  if (tid == 0) reinterpret_cast<unsigned short*>(rec + off_kmax)[NG] = (unsigned short)sKmax[8];
  MIXKVQ_FPHASE(8)
  // value words [token group][channel], 16 codes along tokens: the 16 tokens' parameters in registers
  {
    const int d = tid & (kD - 1), vg = d / Gv;
    const int ilv = cv.lay.v_interleave;
    for (int tg = tid >> 7; tg < n_ch; tg += 2) {
      // tokens of the word: two runs of 8 (tok0 .. tok0+7 and tok1 .. tok1+7), consecutive unless interleaved; each run
      // gets one base address, so that the elements sit at compile-time offsets from it
      const int tok0 = value_word_token(tg, 0, ilv), tok1 = tok0 + (ilv ? 32 : 8);
      const __half* const col0 = sT + tok0 * kFastStride + d;
      const __half* const col1 = sT + tok1 * kFastStride + d;
      float rc[16], nz[16];
      if (NVG == 1) {
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
          const int t4 = (i4 >> 1 ? tok1 : tok0) + 4 * (i4 & 1);
          const float4 a = *reinterpret_cast<const float4*>(sR + t4);
          const float4 b2 = *reinterpret_cast<const float4*>(sNZ + t4);
          rc[4 * i4] = a.x; rc[4 * i4 + 1] = a.y; rc[4 * i4 + 2] = a.z; rc[4 * i4 + 3] = a.w;
          nz[4 * i4] = b2.x; nz[4 * i4 + 1] = b2.y; nz[4 * i4 + 2] = b2.z; nz[4 * i4 + 3] = b2.w;
        }
      } else {
        const float* const r0 = sR + tok0 * NVG + vg, * const r1 = sR + tok1 * NVG + vg;
        const float* const z0 = sNZ + tok0 * NVG + vg, * const z1 = sNZ + tok1 * NVG + vg;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          rc[i] = (i < 8 ? r0 : r1)[(i & 7) * NVG];
          nz[i] = (i < 8 ? z0 : z1)[(i & 7) * NVG];
        }
      }
      float hw[2] = {0.f, 0.f};
      float dev[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int i = 0; i < 16; ++i)
        add_code<2>(hw, i, code_fast((i < 8 ? col0 : col1)[(i & 7) * kFastStride], rc[i], nz[i], dev[i >> 2]));
      // some quotient sits next to a rounding boundary
      if (__any(fmaxf(fmaxf(dev[0], dev[1]), fmaxf(dev[2], dev[3])) > 0.5f - kEps2)) {
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
          if (!__any(dev[i4] > 0.5f - kEps2)) continue;
#pragma unroll
          for (int i = 4 * i4; i < 4 * i4 + 4; ++i) {
            const int t = (i < 8 ? tok0 : tok1) + (i & 7);
            float dv = 0.f;
            const float c = code_fast(sT[t * kFastStride + d], rc[i], nz[i], dv);
            if (__any(dv > 0.5f - kEps2)) add_code<2>(hw, i, code_exact(sT[t * kFastStride + d], sSZ[t * NVG + vg], 3.f) - c);
          }
        }
      }
      const unsigned w = join_halves(hw);
      reinterpret_cast<unsigned*>(rec + off_v)[tg * kD + d] = w;
    }
  }
  MIXKVQ_FPHASE(9)
}

hipError_t launch_flush(const CacheView& v, const __half* k_new, const __half* v_new, Strides3 kvs, int r0,
                        int first_block, int n_flush, const uint8_t* sel, hipStream_t s) {
  // the throughput kernel needs 16-token chunks inside key groups, whole 16-byte pieces inside value groups and
  // 16-byte aligned rows; anything else takes the general kernel
  const bool aligned = ((reinterpret_cast<uintptr_t>(k_new) | reinterpret_cast<uintptr_t>(v_new)) & 15u) == 0 &&
                       kvs.b % 8 == 0 && kvs.h % 8 == 0 && kvs.t % 8 == 0;
  static const bool force_general = getenv("MIXKVQ_FLUSH_GENERAL") != nullptr;
  const bool fast = aligned && v.cfg.Gk % 16 == 0 && v.cfg.Gv % 16 == 0 && !force_general;
  // grid.y is limited to 65535 blocks per launch
  for (int f0 = 0; f0 < n_flush; f0 += 32768) {
    const int nf = n_flush - f0 < 32768 ? n_flush - f0 : 32768;
    // shift the stream origin so that block index 0 of this launch is block f0 of the call
    if (fast)
      flush_block_fast_kernel<<<dim3(v.P, nf), dim3(kFlushThreads), 0, s>>>(v, k_new, v_new, kvs, r0 - f0 * v.cfg.R,
                                                                           first_block + f0, sel);
    else
      flush_block_kernel<<<dim3(v.P, nf), dim3(kFlushThreads), 0, s>>>(v, k_new, v_new, kvs, r0 - f0 * v.cfg.R,
                                                                      first_block + f0, sel);
  }
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// copy into the fp16 rows: n tokens starting at new-token index src_first go to rows dst_row.. of every pair
// (row 0 = first sink row, row S = first row of the residual window).
// ---------------------------------------------------------------------------
__global__ void residual_copy_kernel(CacheView cv, const __half* __restrict__ k_new, const __half* __restrict__ v_new,
                                     Strides3 st, int src_first, int dst_row, int n) {
  const int p = blockIdx.x, b = p / cv.cfg.Hkv, j = p % cv.cfg.Hkv;
  for (int idx = blockIdx.y * blockDim.x + threadIdx.x; idx < n * 16; idx += gridDim.y * blockDim.x) {
    const int t = idx >> 4, c = idx & 15;
    const int64_t src = (int64_t)b * st.b + (int64_t)j * st.h + (int64_t)(src_first + t) * st.t + c * 8;
    const size_t dst = ((size_t)p * cv.RW + dst_row + t) * kD + c * 8;
    const bool bf16 = cv.cfg.in_dtype != 0;
    *reinterpret_cast<uint4*>(cv.res_k + dst) = as_f16x8(*reinterpret_cast<const uint4*>(k_new + src), bf16);
    *reinterpret_cast<uint4*>(cv.res_v + dst) = as_f16x8(*reinterpret_cast<const uint4*>(v_new + src), bf16);
  }
}

hipError_t launch_residual_copy(const CacheView& v, const __half* k_new, const __half* v_new, Strides3 kvs,
                                int src_first, int dst_row, int n, hipStream_t s) {
  const int threads = n * 16 < 256 ? 64 : 256;
  int gy = (n * 16 + threads - 1) / threads;
  if (gy > 8) gy = 8;
  residual_copy_kernel<<<dim3(v.P, gy), dim3(threads), 0, s>>>(v, k_new, v_new, kvs, src_first, dst_row, n);
  return hipGetLastError();
}

}  // namespace mixkvq

#ifdef MIXKVQ_PHASE_CLOCKS
extern "C" int mixkvq_debug_flush_clocks(void* host_dst, size_t bytes) {
  (void)hipDeviceSynchronize();
  return (int)hipMemcpyFromSymbol(host_dst, HIP_SYMBOL(mixkvq::g_flush_clock), bytes);
}
#endif
