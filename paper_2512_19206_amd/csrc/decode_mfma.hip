// Split-K decode attention on the matrix cores (Section 3.1, Eq. 1; keys and values
// dequantized by Eq. 3 without ever materialising them).
//
// One wavefront owns one block record of R tokens at a time and keeps running
// softmax statistics for the g query heads of the KV head.  Both contractions use
// v_mfma_f32_16x16x32_f16 in the transposed form
//     S^T[token][col] = K_codes[token][slot] . Qs^T[slot][col]
//     O^T[chan][col]  = V_codes^T[chan][token] . Ps^T[token][col]
// so that the accumulator layout of the first product (token along the register
// index, column along lane%16) is exactly the B-operand layout of the second one.
//
// Dequantization is folded into the small operands (Eq. 3, x~ = c*s + z):
//   keys    q.(c*s+z) = sum_d (q_d s_d) c_d + sum_d q_d z_d     -> Qs = q*s per block, plus a bias per head
//   values  sum_t p_t (c_t s_t + z_t) = sum_t (p_t s_t) c_t + sum_t p_t z_t
// The big operands are the raw packed codes: `word & 0x00030003 << 2p` leaves two
// codes in the mantissa bits of an fp16 pair, i.e. the fp16 SUBNORMALS c * 4^p * 2^-24,
// which the gfx950 matrix cores multiply exactly; 4^-p goes into the small operand
// and 2^24 into the final scale.  One shift and eight ANDs unpack 16 codes.
//
// Columns 0..7 of the small key operand hold the fp16 head of q*s for heads 0..7 and
// columns 8..15 its exact fp16 tail (q*s - head, one fused multiply-add), so the
// product keeps ~22 bits of q*s at no extra matrix instruction; the two halves are
// added after the product with one DPP add.
#include "mixkvq_internal.h"

namespace mixkvq {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

constexpr int kMfmaThreads = 256;
constexpr int kWaves = kMfmaThreads / 64;
constexpr int kKPartMax = 8192;                 // bytes of a record before the value plane (staged in LDS)
constexpr int kVMetaMax = 1024;                 // value scales + zero-points of one block
constexpr int kWaveLds = kKPartMax + kVMetaMax + 256;   // + channel lists
constexpr int kPartStrideM = kD + 2;

__device__ __forceinline__ f32x4 mfma(u32x4 a, u32x4 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}
typedef _Float16 h2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ unsigned pk_mul(unsigned a, unsigned b) {
  return __builtin_bit_cast(unsigned, __builtin_bit_cast(h2, a) * __builtin_bit_cast(h2, b));
}
// a*b - c in one rounding per half
__device__ __forceinline__ unsigned pk_fma_neg(unsigned a, unsigned b, unsigned c) {
  return __builtin_bit_cast(unsigned, __builtin_elementwise_fma(__builtin_bit_cast(h2, a), __builtin_bit_cast(h2, b),
                                                                -__builtin_bit_cast(h2, c)));
}
__device__ __forceinline__ unsigned pk_max(unsigned a, unsigned b) {
  return __builtin_bit_cast(unsigned, __builtin_elementwise_max(__builtin_bit_cast(h2, a), __builtin_bit_cast(h2, b)));
}
__device__ __forceinline__ float dot2(unsigned a, unsigned b, float c) {
  return __builtin_amdgcn_fdot2(__builtin_bit_cast(h2, a), __builtin_bit_cast(h2, b), c, false);
}
__device__ __forceinline__ unsigned cvt_pk(float lo, float hi) {
  __half2 r = __float22half2_rn(make_float2(lo, hi));
  return __builtin_bit_cast(unsigned, r);
}
__device__ __forceinline__ float half_lo(unsigned v) { return __half2float(__ushort_as_half((unsigned short)(v & 0xffffu))); }
__device__ __forceinline__ float half_hi(unsigned v) { return __half2float(__ushort_as_half((unsigned short)(v >> 16))); }
// max / sum over the four lanes l, l^16, l^32, l^48
__device__ __forceinline__ float xkg_max(float v) {
  auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  v = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
  auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}
__device__ __forceinline__ float xkg_sum(float v) {
  auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  v = __uint_as_float(a[0]) + __uint_as_float(a[1]);
  auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}
// value of lane+8 inside each row of 16 lanes (0 for lanes 8..15)
__device__ __forceinline__ float row_shl8(float v) {
  return __uint_as_float(__builtin_amdgcn_update_dpp(0u, __float_as_uint(v), 0x108, 0xF, 0xF, true));
}

// position exponent of code r%8 of a 16-code word after unpacking: value = c * 4^sc * 2^-24
__device__ __host__ constexpr int sc2(int r) { return r < 5 ? r : r - 3; }
// the same for nibble r%4 of an 8-nibble word: value = c * 4^sc * 2^-24
__device__ __host__ constexpr int sc4(int e) { return (e & 1) ? 2 : 0; }

// two-bit word -> the two A operands (4 VGPRs each) of the MFMA steps x = 0, 1
__device__ __forceinline__ void unpack2(unsigned w, u32x4& a0, u32x4& a1) {
  const unsigned w6 = w >> 6;
  a0[0] = w & 0x00030003u; a0[1] = w & 0x000C000Cu; a0[2] = w & 0x00300030u; a0[3] = w & 0x00C000C0u;
  a1[0] = w & 0x03000300u; a1[1] = w6 & 0x00300030u; a1[2] = w6 & 0x00C000C0u; a1[3] = w6 & 0x03000300u;
}
// four-bit word -> one A operand: pairs (0,4) (1,5) (2,6) (3,7)
__device__ __forceinline__ u32x4 unpack4(unsigned w) {
  const unsigned w8 = w >> 8;
  u32x4 a;
  a[0] = w & 0x000F000Fu; a[1] = w & 0x00F000F0u; a[2] = w8 & 0x000F000Fu; a[3] = w8 & 0x00F000F0u;
  return a;
}

template <int K4, int K16>
struct Tiers {
  static constexpr int NL = kD - K4 - K16;
  static constexpr int Wlo = (NL + 15) / 16;
  static constexpr int NLp = Wlo * 16;
  static constexpr int NLU = (NL + 7) / 8;     // 8-slot units of the 2-bit plane
  static constexpr int W4 = K4 / 8;            // 8-slot units (= words) of the 4-bit plane
  static_assert(NLU + W4 <= 16, "the 2-bit and 4-bit tiers must fit four MFMA steps");
  static_assert(K16 <= 32, "the fp16 tier must fit one MFMA step");
};

// unit (8 slots) handled by lane group kg in MFMA step s = 2u + x: linear index ui = 8u + 2kg + x;
// ui < NLU: half x of 2-bit word 4u+kg; NLU <= ui < NLU+W4: 4-bit word ui-NLU; else empty.

template <int K4, int K16, int NVG, int NKL>
__global__ void __launch_bounds__(kMfmaThreads, 2)
decode_mfma_kernel(CacheView cv, const __half* __restrict__ q, float scale_log2e, int n_blocks, int n_res, int n_splits,
                   float* __restrict__ part, int accumulate_q) {
  using T = Tiers<K4, K16>;
  extern __shared__ __align__(16) unsigned char smem[];
  // scalars of the by-value view (kept in SGPRs; no references into the kernel argument)
  const int R = cv.cfg.R, g = cv.g, Hq = cv.cfg.Hq, Hkv = cv.cfg.Hkv, Gk = cv.cfg.Gk, NB = cv.NB;
  const int rec_bytes = cv.lay.rec_bytes, off_idx = cv.lay.off_idx, off_klo_s = cv.lay.off_klo_s,
            off_klo_z = cv.lay.off_klo_z, off_k4_s = cv.lay.off_k4_s, off_k4_z = cv.lay.off_k4_z,
            off_klo = cv.lay.off_klo, off_k4 = cv.lay.off_k4, off_k16 = cv.lay.off_k16, off_v = cv.lay.off_v,
            off_v_s = cv.lay.off_v_s;
  const unsigned char* const blocks = cv.blocks;
  const int p = blockIdx.x, split = blockIdx.y, tid = threadIdx.x;
  const int b = p / Hkv, jkv = p % Hkv;
  const int wave = tid >> 6, lane = tid & 63, n = lane & 15, kg = lane >> 4;
  const int head = n & 7, role = n >> 3;     // role 0: head of q*s, role 1: tail
  const bool live = head < g;

  __half* sQn = reinterpret_cast<__half*>(smem);                   // [8][128] normalised q
  int* sEq = reinterpret_cast<int*>(smem + 2048);                   // [8] exponents
  unsigned char* wbase = smem + 2048 + 64 + wave * kWaveLds;        // this wave's private region
  unsigned char* sK = wbase;                                        // record bytes [0, off_v)
  unsigned char* sVm = wbase + kKPartMax;                           // v_s, v_z planes
  unsigned char* sLo = wbase + kKPartMax + kVMetaMax;               // 2-bit channel list [128], then salient idx [<=64]

  // ---- normalise q per head: qn = q * 2^-Eq with max|qn| in [1/2, 1) ----
  if (tid < 8 * 32) {
    const int h = tid >> 5, l32 = tid & 31;
    float v[4];
    float mx = 0.f;
    for (int i = 0; i < 4; ++i) {
      v[i] = h < g ? __half2float(q[((size_t)b * Hq + jkv * g + h) * kD + l32 * 4 + i]) : 0.f;
      mx = fmaxf(mx, fabsf(v[i]));
    }
    for (int o = 16; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 32));
    int ef = (int)((__float_as_uint(mx) >> 23) & 0xff) - 127 + 15;   // fp16 exponent field of the maximum
    if (ef < 1) ef = 1;
    const int eq = ef - 14;
    for (int i = 0; i < 4; ++i) sQn[h * kD + l32 * 4 + i] = __float2half_rn(ldexpf(v[i], -eq));
    if (l32 == 0) sEq[h] = eq;
  }
  __syncthreads();
  const int Eq = sEq[head];

  const int blk_lo = (int)((long long)n_blocks * split / n_splits);
  const int blk_hi = (int)((long long)n_blocks * (split + 1) / n_splits);

  // ---- per-lane constants -------------------------------------------------
  const int m_ = n;                                   // A-operand row
  const int tokbase = 16 * (m_ >> 2) + (m_ & 3);      // token of row m in tile (h, x): 64h + tokbase + {0,8,4,12}[x]
  const int nck = off_v >> 4;                     // 16-byte chunks of the key part
  const int nvm = (rec_bytes - off_v_s) >> 4; // chunks of the value scale/zero planes

  // running state (log2 domain)
  float m_run = -INFINITY, l_run = 0.f;
  float zacc[NVG][5];
  f32x4 O[2][4];   // [x'][q]: channels 64x' + 16kg + 4i + q
#pragma unroll
  for (int a = 0; a < NVG; ++a)
#pragma unroll
    for (int c = 0; c < 5; ++c) zacc[a][c] = 0.f;
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int c = 0; c < 4; ++c) O[a][c] = f32x4{0.f, 0.f, 0.f, 0.f};

  // q in slot order (rebuilt when the block's channel selection changes)
  unsigned qn[4][4];                  // [step][vgpr]: normalised q pairs
  unsigned q16[4];                    // fp16-tier q pairs of this lane's chunk (role 0 only)
  unsigned sel_prev[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) sel_prev[i] = 0xffffffffu;
#pragma unroll
  for (int s = 0; s < 4; ++s)
#pragma unroll
    for (int e = 0; e < 4; ++e) qn[s][e] = 0u;
#pragma unroll
  for (int e = 0; e < 4; ++e) q16[e] = 0u;

  // prefetch registers
  u32x4 kreg[NKL];
  u32x4 vmreg;
  u32x4 vreg[2][2];   // [h][x]

  // Loads of one block into the prefetch registers.  Indices beyond the end of a plane are
  // clamped (the data is loaded twice and stored once) so that every load is unconditional.
#define MIXKVQ_ISSUE_K_LOADS(BLK)                                                                             \
  {                                                                                                          \
    const unsigned char* rec_ = blocks + ((size_t)p * NB + (BLK)) * rec_bytes;                              \
    _Pragma("unroll") for (int c = 0; c < NKL; ++c) {                                                       \
      const int idx_ = c * 64 + lane;                                                                        \
      kreg[c] = reinterpret_cast<const u32x4*>(rec_)[idx_ < nck ? idx_ : nck - 1];                          \
    }                                                                                                        \
    vmreg = reinterpret_cast<const u32x4*>(rec_ + off_v_s)[lane < nvm ? lane : nvm - 1];                    \
  }
#define MIXKVQ_ISSUE_V_LOADS(BLK)                                                                           \
  {                                                                                                          \
    const unsigned char* rec_ = blocks + ((size_t)p * NB + (BLK)) * rec_bytes;                              \
    const unsigned* vw_ = reinterpret_cast<const unsigned*>(rec_ + off_v);                                  \
    _Pragma("unroll") for (int h = 0; h < 2; ++h) _Pragma("unroll") for (int x = 0; x < 2; ++x)             \
        vreg[h][x] = *reinterpret_cast<const u32x4*>(vw_ + (4 * (h * 64 < R ? h : 0) + kg) * kD + 64 * x + 4 * n); \
  }

  int blk = blk_lo + wave;
  if (blk < blk_hi) {
    MIXKVQ_ISSUE_K_LOADS(blk)
    MIXKVQ_ISSUE_V_LOADS(blk)
  }

  for (; blk < blk_hi; blk += kWaves) {
    // ---- stage the key part and value metadata in LDS (wave-private: no barrier needed) ----
#pragma unroll
    for (int c = 0; c < NKL; ++c) {
      const int idx = c * 64 + lane;
      if (idx < nck) reinterpret_cast<u32x4*>(sK)[idx] = kreg[c];
    }
    if (lane < nvm) reinterpret_cast<u32x4*>(sVm)[lane] = vmreg;
    if (blk + kWaves < blk_hi) MIXKVQ_ISSUE_K_LOADS(blk + kWaves)

    // ---- channel selection of this block: rebuild q in slot order if it changed ----
    if (K4 + K16 > 0) {
      bool changed = false;
#pragma unroll
      for (int i = 0; i < (K4 + K16 + 3) / 4; ++i) {
        const unsigned wv = reinterpret_cast<const unsigned*>(sK + off_idx)[i];
        changed |= wv != sel_prev[i];
        sel_prev[i] = wv;
      }
      if (__builtin_amdgcn_readfirstlane((int)changed)) {
        // list of 2-bit channels: lanes cover channels lane and lane+64
        unsigned char* sIdx = sLo + kD;
        if (lane < K4 + K16) sIdx[lane] = sK[off_idx + lane];
        unsigned long long m0 = 0, m1 = 0;   // bitmap of salient channels
#pragma unroll
        for (int i = 0; i < K4 + K16; ++i) {
          const int ch = sK[off_idx + i];
          if (ch < 64) m0 |= 1ull << ch; else m1 |= 1ull << (ch - 64);
        }
        {
          const int ch0 = lane, ch1 = lane + 64;
          if (!((m0 >> ch0) & 1)) sLo[ch0 - __popcll(m0 & ((1ull << ch0) - 1))] = (unsigned char)ch0;
          if (!((m1 >> lane) & 1))
            sLo[ch1 - __popcll(m0) - __popcll(m1 & ((1ull << lane) - 1))] = (unsigned char)ch1;
        }
        // gather
        const __half* qrow = sQn + head * kD;
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
          for (int x = 0; x < 2; ++x) {
            const int ui = 8 * u + 2 * kg + x;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              float lo = 0.f, hi = 0.f;
              if (ui < T::NLU) {
                const int j0 = 16 * (4 * u + kg) + 4 * x + e, j1 = j0 + 8;
                if (j0 < T::NL) lo = __half2float(qrow[sLo[j0]]);
                if (j1 < T::NL) hi = __half2float(qrow[sLo[j1]]);
              } else if (ui - T::NLU < T::W4) {
                const int a0 = 8 * (ui - T::NLU) + e;
                lo = __half2float(qrow[sIdx[K16 + a0]]);
                hi = __half2float(qrow[sIdx[K16 + a0 + 4]]);
              }
              if (!live) { lo = 0.f; hi = 0.f; }
              qn[2 * u + x][e] = cvt_pk(lo, hi);
            }
          }
        if (K16 > 0) {
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int a0 = 8 * kg + 2 * e;
            float lo = 0.f, hi = 0.f;
            if (live && role == 0) {
              if (a0 < K16) lo = __half2float(qrow[sIdx[a0]]);
              if (a0 + 1 < K16) hi = __half2float(qrow[sIdx[a0 + 1]]);
            }
            q16[e] = cvt_pk(lo, hi);
          }
        }
      }
    } else if (sel_prev[0] == 0xffffffffu) {
      sel_prev[0] = 0;
      const __half* qrow = sQn + head * kD;
#pragma unroll
      for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int x = 0; x < 2; ++x)
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int j0 = 16 * (4 * u + kg) + 4 * x + e;
            float lo = live ? __half2float(qrow[j0]) : 0.f, hi = live ? __half2float(qrow[j0 + 8]) : 0.f;
            qn[2 * u + x][e] = cvt_pk(lo, hi);
          }
    }

    // operands that live across the super-groups of one key group
    u32x4 Bq[4];
    float zdot = 0.f, C = 0.f, Cz = 0.f, zc = 0.f;
#pragma unroll
    for (int hsg = 0; hsg < 2; ++hsg) {       // super-groups of 64 tokens
      if (64 * hsg < R) {
      if ((64 * hsg) % Gk == 0) {
        const int grp = (64 * hsg) / Gk;
      // ---- small key operand of this group: Qs = qg * s, bias = sum q z ----------------
      unsigned sp[4][4];     // scales of this lane's slots, paired like the codes
      zdot = 0.f;
      unsigned smax2 = 0u;
#pragma unroll
      for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int x = 0; x < 2; ++x) {
          const int ui = 8 * u + 2 * kg + x;
          // byte offsets of the two 4-entry runs (A: low halves, B: high halves) inside the record
          int oa_s, ob_s, oa_z, ob_z;
          if (ui < T::NLU) {
            const int j0 = 16 * (4 * u + kg) + 4 * x;
            oa_s = off_klo_s + 2 * (grp * T::NLp + j0);
            ob_s = oa_s + 16;
            oa_z = off_klo_z + 2 * (grp * T::NLp + j0);
            ob_z = oa_z + 16;
          } else if (ui - T::NLU < T::W4) {
            const int a0 = 8 * (ui - T::NLU);
            oa_s = off_k4_s + 2 * (grp * K4 + a0);
            ob_s = oa_s + 8;
            oa_z = off_k4_z + 2 * (grp * K4 + a0);
            ob_z = oa_z + 8;
          } else {   // empty unit: q is 0 there; read any finite scale
            oa_s = ob_s = off_klo_s;
            oa_z = ob_z = off_klo_z;
          }
          const uint2 sa = *reinterpret_cast<const uint2*>(sK + oa_s), sb = *reinterpret_cast<const uint2*>(sK + ob_s);
          const uint2 za = *reinterpret_cast<const uint2*>(sK + oa_z), zb = *reinterpret_cast<const uint2*>(sK + ob_z);
          const int s = 2 * u + x;
          sp[s][0] = __builtin_amdgcn_perm(sb.x, sa.x, 0x05040100u);
          sp[s][1] = __builtin_amdgcn_perm(sb.x, sa.x, 0x07060302u);
          sp[s][2] = __builtin_amdgcn_perm(sb.y, sa.y, 0x05040100u);
          sp[s][3] = __builtin_amdgcn_perm(sb.y, sa.y, 0x07060302u);
          zdot = dot2(qn[s][0], __builtin_amdgcn_perm(zb.x, za.x, 0x05040100u), zdot);
          zdot = dot2(qn[s][1], __builtin_amdgcn_perm(zb.x, za.x, 0x07060302u), zdot);
          zdot = dot2(qn[s][2], __builtin_amdgcn_perm(zb.y, za.y, 0x05040100u), zdot);
          zdot = dot2(qn[s][3], __builtin_amdgcn_perm(zb.y, za.y, 0x07060302u), zdot);
#pragma unroll
          for (int e = 0; e < 4; ++e) smax2 = pk_max(smax2, sp[s][e]);
        }
      zdot = xkg_sum(zdot);
      if (role) zdot = 0.f;
      // block exponent: scales are multiplied by 2^e0 so that the largest lands in [2^14, 2^15) (e0 <= 15),
      // and by 4^-sc, the position factor of the code they meet in the product
      float smax = fmaxf(half_lo(smax2), half_hi(smax2));
      smax = xkg_max(smax);
      int efs = (int)((__float_as_uint(smax) >> 23) & 0xff) - 127 + 15;
      if (efs < 1) efs = 1;
      efs = __builtin_amdgcn_readfirstlane(efs);
      const int e0 = 29 - efs < 15 ? 29 - efs : 15;
#pragma unroll
      for (int s = 0; s < 4; ++s)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int ui = 8 * (s >> 1) + 2 * kg + (s & 1);
          const int sc = ui < T::NLU ? sc2(4 * (s & 1) + e) : sc4(e);
          const unsigned mult = ((unsigned)(15 + e0 - 2 * sc) << 10) * 0x00010001u;   // fp16 pair 2^(e0 - 2 sc)
          const unsigned sn = pk_mul(sp[s][e], mult);
          const unsigned hi = pk_mul(qn[s][e], sn);
          const unsigned lo = pk_fma_neg(qn[s][e], sn, hi);
          Bq[s][e] = role ? lo : hi;
        }
      // logits in the log2 domain: x2 = S * C + Z * Cz
      Cz = ldexpf(scale_log2e, Eq);
      C = ldexpf(scale_log2e, 24 - e0 + Eq);
      zc = zdot * Cz;

      }
      {
        // ---- S^T tiles: tile x holds tokens 64*hsg + 16*(row/4) + row%4 + {0,8,4,12}[x] ----
        f32x4 S[4];
#pragma unroll
        for (int x = 0; x < 4; ++x) {
          const int off_x = (x == 0 ? 0 : x == 1 ? 8 : x == 2 ? 4 : 12);
          const int tok = 64 * hsg + tokbase + off_x;
          f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int u = 0; u < 2; ++u) {
            u32x4 a0 = {0u, 0u, 0u, 0u}, a1 = {0u, 0u, 0u, 0u};
            const int ui0 = 8 * u + 2 * kg;
            if (8 * u + 7 < T::NLU) {          // every lane group has a full 2-bit word here
              const unsigned w = *reinterpret_cast<const unsigned*>(sK + off_klo + 4 * (tok * T::Wlo + 4 * u + kg));
              unpack2(w, a0, a1);
            } else {
              if (ui0 < T::NLU) {
                const unsigned w = *reinterpret_cast<const unsigned*>(sK + off_klo + 4 * (tok * T::Wlo + 4 * u + kg));
                u32x4 t0, t1;
                unpack2(w, t0, t1);
                a0 = t0;
                if (ui0 + 1 < T::NLU) a1 = t1;
              }
              if (T::W4 > 0) {
                if (ui0 >= T::NLU && ui0 - T::NLU < T::W4)
                  a0 = unpack4(*reinterpret_cast<const unsigned*>(sK + off_k4 + 4 * (tok * T::W4 + ui0 - T::NLU)));
                if (ui0 + 1 >= T::NLU && ui0 + 1 - T::NLU < T::W4)
                  a1 = unpack4(*reinterpret_cast<const unsigned*>(sK + off_k4 + 4 * (tok * T::W4 + ui0 + 1 - T::NLU)));
              }
            }
            acc = mfma(a0, Bq[2 * u], acc);
            acc = mfma(a1, Bq[2 * u + 1], acc);
          }
          S[x] = acc;
        }
        f32x4 S16[4];
        if (K16 > 0) {
#pragma unroll
          for (int x = 0; x < 4; ++x) {
            const int off_x = (x == 0 ? 0 : x == 1 ? 8 : x == 2 ? 4 : 12);
            const int tok = 64 * hsg + tokbase + off_x;
            u32x4 a = {0u, 0u, 0u, 0u};
            if (8 * kg < K16) {
              const unsigned char* src = sK + off_k16 + 2 * (tok * K16 + 8 * kg);
              const uint2 v0 = *reinterpret_cast<const uint2*>(src);
              a[0] = v0.x; a[1] = v0.y;
              if (8 * kg + 4 < K16) {
                const uint2 v1 = *reinterpret_cast<const uint2*>(src + 8);
                a[2] = v1.x; a[3] = v1.y;
              }
            }
            u32x4 bq = {q16[0], q16[1], q16[2], q16[3]};
            S16[x] = mfma(a, bq, f32x4{zdot, zdot, zdot, zdot});
          }
        }

        // ---- logits, running maximum ----
        float x2[4][4];
        float mx = -INFINITY;
#pragma unroll
        for (int x = 0; x < 4; ++x)
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const float s = S[x][i] + row_shl8(S[x][i]);
            x2[x][i] = K16 > 0 ? fmaf(s, C, S16[x][i] * Cz) : fmaf(s, C, zc);
            mx = fmaxf(mx, x2[x][i]);
          }
        mx = xkg_max(mx);
        const float m_new = fmaxf(m_run, mx);
        if (__builtin_amdgcn_readfirstlane((int)__any(m_new > m_run))) {
          const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);   // exp2(-inf) = 0 on the first block
          l_run *= alpha;
#pragma unroll
          for (int a = 0; a < NVG; ++a)
#pragma unroll
            for (int c = 0; c < 5; ++c) zacc[a][c] *= alpha;
#pragma unroll
          for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int c = 0; c < 4; ++c) O[a][c] *= alpha;
          m_run = m_new;
        }

        // ---- p, value-side small operand Ps = p * s_v * 4^-sc ----
        // this lane's tokens: 64*hsg + 16*kg + r, r = i + {0,8,4,12}[x]; their scale/zero-point entries
        unsigned vs[NVG][8], vz[NVG][8];   // fp16 pairs: entry r -> [r/2] half r%2
        {
          const int t0 = 64 * hsg + 16 * kg;
          if (NVG == 1) {
            const uint4* ps = reinterpret_cast<const uint4*>(sVm + 2 * t0);
            const uint4* pz = reinterpret_cast<const uint4*>(sVm + 2 * R + 2 * t0);
            const uint4 s0 = ps[0], s1 = ps[1], z0 = pz[0], z1 = pz[1];
            vs[0][0] = s0.x; vs[0][1] = s0.y; vs[0][2] = s0.z; vs[0][3] = s0.w;
            vs[0][4] = s1.x; vs[0][5] = s1.y; vs[0][6] = s1.z; vs[0][7] = s1.w;
            vz[0][0] = z0.x; vz[0][1] = z0.y; vz[0][2] = z0.z; vz[0][3] = z0.w;
            vz[0][4] = z1.x; vz[0][5] = z1.y; vz[0][6] = z1.z; vz[0][7] = z1.w;
          } else {
            // [token][2] layout: token r at dword r, value group a in half a
            const uint4* ps = reinterpret_cast<const uint4*>(sVm + 4 * t0);
            const uint4* pz = reinterpret_cast<const uint4*>(sVm + 4 * R + 4 * t0);
#pragma unroll
            for (int c = 0; c < 4; ++c) {
              const uint4 sv = ps[c], zv = pz[c];
              const unsigned sw[4] = {sv.x, sv.y, sv.z, sv.w}, zw[4] = {zv.x, zv.y, zv.z, zv.w};
#pragma unroll
              for (int k2 = 0; k2 < 2; ++k2) {
                // tokens 4c+2k2, 4c+2k2+1 -> pair index (4c+2k2)/2
                vs[0][2 * c + k2] = __builtin_amdgcn_perm(sw[2 * k2 + 1], sw[2 * k2], 0x05040100u);
                vs[NVG - 1][2 * c + k2] = __builtin_amdgcn_perm(sw[2 * k2 + 1], sw[2 * k2], 0x07060302u);
                vz[0][2 * c + k2] = __builtin_amdgcn_perm(zw[2 * k2 + 1], zw[2 * k2], 0x05040100u);
                vz[NVG - 1][2 * c + k2] = __builtin_amdgcn_perm(zw[2 * k2 + 1], zw[2 * k2], 0x07060302u);
              }
            }
          }
        }
        u32x4 Bp[NVG][2];   // [value group][PV step]: step 0 pairs tiles (0,1), step 1 pairs tiles (2,3)
        float lsum = 0.f;
#pragma unroll
        for (int st = 0; st < 2; ++st)
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int sc = st == 0 ? i : sc2(4 + i);
            const float pa = __builtin_amdgcn_exp2f(x2[2 * st][i] - m_run - 2.f * sc);       // tile 2st:   token r = i + (st ? 4 : 0)
            const float pb = __builtin_amdgcn_exp2f(x2[2 * st + 1][i] - m_run - 2.f * sc);   // tile 2st+1: token r + 8
            lsum = fmaf(pa + pb, (float)(1 << (2 * sc)), lsum);
            const int ra = i + (st ? 4 : 0), rb = ra + 8;
#pragma unroll
            for (int a = 0; a < NVG; ++a) {
              const float sa = (ra & 1) ? half_hi(vs[a][ra >> 1]) : half_lo(vs[a][ra >> 1]);
              const float sb = (rb & 1) ? half_hi(vs[a][rb >> 1]) : half_lo(vs[a][rb >> 1]);
              const float za = (ra & 1) ? half_hi(vz[a][ra >> 1]) : half_lo(vz[a][ra >> 1]);
              const float zb = (rb & 1) ? half_hi(vz[a][rb >> 1]) : half_lo(vz[a][rb >> 1]);
              Bp[a][st][i] = cvt_pk(pa * sa, pb * sb);
              zacc[a][sc] = fmaf(pa, za, fmaf(pb, zb, zacc[a][sc]));
            }
          }
        l_run += lsum;

        // ---- O^T += V_codes^T . Ps^T ----
#pragma unroll
        for (int xp = 0; xp < 2; ++xp) {
          const u32x4 vw = vreg[hsg][xp];
          const unsigned w4[4] = {vw.x, vw.y, vw.z, vw.w};
#pragma unroll
          for (int qq = 0; qq < 4; ++qq) {
            u32x4 a0, a1;
            unpack2(w4[qq], a0, a1);
            const int a = NVG == 1 ? 0 : xp;
            O[xp][qq] = mfma(a0, Bp[a][0], O[xp][qq]);
            O[xp][qq] = mfma(a1, Bp[a][1], O[xp][qq]);
          }
        }
      }
      }
    }
    if (blk + kWaves < blk_hi) MIXKVQ_ISSUE_V_LOADS(blk + kWaves)
  }

  // ---- wave results -> workgroup partial ------------------------------------------
  // sums over the four lane groups of a column
  l_run = xkg_sum(l_run);
  float zsum[NVG];
#pragma unroll
  for (int a = 0; a < NVG; ++a) {
    float z = 0.f;
#pragma unroll
    for (int c = 0; c < 5; ++c) z = fmaf(zacc[a][c], (float)(1 << (2 * c)), z);
    zsum[a] = xkg_sum(z);
  }
  __syncthreads();   // every wave is done with its private LDS region
  float* sM = reinterpret_cast<float*>(smem + 2048 + 64);          // [waves][8]
  float* sO = sM + kWaves * 8;                                     // [8][128] + [8] l
  if (kg == 0 && role == 0) sM[wave * 8 + head] = m_run;
  for (int i = tid; i < 8 * kD + 8; i += kMfmaThreads) sO[i] = 0.f;
  __syncthreads();
  float m_wg = -INFINITY;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) m_wg = fmaxf(m_wg, sM[w * 8 + head]);
  const float wscale = m_run == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m_run - m_wg);
  for (int w = 0; w < kWaves; ++w) {   // one wave at a time: the sum order is fixed
    if (wave == w && role == 0 && live) {
#pragma unroll
      for (int xp = 0; xp < 2; ++xp)
#pragma unroll
        for (int qq = 0; qq < 4; ++qq)
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int ch = 64 * xp + 16 * kg + 4 * i + qq;
            const int a = NVG == 1 ? 0 : xp;
            sO[head * kD + ch] += fmaf(O[xp][qq][i], 16777216.f, zsum[a]) * wscale;
          }
      if (kg == 0) sO[8 * kD + head] += l_run * wscale;
    }
    __syncthreads();
  }
  // natural-log domain for the merge kernel: m_e = m2 * ln2
  float* out = part + ((size_t)p * (n_splits + 1) + split) * g * kPartStrideM;
  for (int i = tid; i < g * kD; i += kMfmaThreads) out[(i / kD) * kPartStrideM + (i % kD)] = sO[i];
  if (tid < g) {
    float mw = -INFINITY;
    for (int w = 0; w < kWaves; ++w) mw = fmaxf(mw, sM[w * 8 + tid]);
    out[tid * kPartStrideM + kD] = mw * 0.6931471805599453f;
    out[tid * kPartStrideM + kD + 1] = sO[8 * kD + tid];
  }
}

// ---------------------------------------------------------------------------
// Residual window (fp16 keys and values) and the |q| accumulator: one workgroup
// per pair, plain vector ALU; it writes partial number n_splits.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
decode_residual_kernel(CacheView cv, const __half* __restrict__ q, float scale, int n_res, int n_splits,
                       float* __restrict__ part, int accumulate_q) {
  __shared__ float sQ[8][kD];
  __shared__ float sP[8][kMaxR];
  __shared__ float sM[8], sL[8];
  const mixkvq_config& cfg = cv.cfg;
  const int R = cfg.R, g = cv.g;
  const int p = blockIdx.x, tid = threadIdx.x;
  const int b = p / cfg.Hkv, j = p % cfg.Hkv;
  const __half* qp = q + ((size_t)b * cfg.Hq + (size_t)j * g) * kD;
  for (int i = tid; i < g * kD; i += 256) sQ[i / kD][i % kD] = __half2float(qp[i]);
  if (accumulate_q && tid < kD) {
    unsigned long long acc = 0;
    for (int h = 0; h < g; ++h) acc += fix24_abs(h2bits(qp[h * kD + tid]));
    cv.qacc[(size_t)p * kD + tid] += acc;     // one writer per element
    if (tid == 0) cv.qcnt[p] += (unsigned long long)g;
  }
  __syncthreads();
  // logits: thread (token, head half)
  const int t = tid & 127, h0 = (tid >> 7) * 4;
  if (t < n_res && h0 < g) {
    float s[4] = {0.f, 0.f, 0.f, 0.f};
    const __half* row = cv.res_k + ((size_t)p * R + t) * kD;
    for (int d8 = 0; d8 < kD; d8 += 8) {
      const uint4 raw = *reinterpret_cast<const uint4*>(row + d8);
      const unsigned ww[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const float k0 = half_lo(ww[c]), k1 = half_hi(ww[c]);
#pragma unroll
        for (int i = 0; i < 4; ++i) s[i] = fmaf(sQ[(h0 + i) & 7][d8 + 2 * c + 1], k1, fmaf(sQ[(h0 + i) & 7][d8 + 2 * c], k0, s[i]));
      }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (h0 + i < g) sP[h0 + i][t] = s[i] * scale;
  }
  __syncthreads();
  {
    const int wave = tid >> 6, lane = tid & 63;
    for (int h = wave; h < g; h += 4) {
      const float x0 = lane < n_res ? sP[h][lane] : -INFINITY;
      const float x1 = lane + 64 < n_res ? sP[h][lane + 64] : -INFINITY;
      float mx = fmaxf(x0, x1);
      for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
      const float e0 = lane < n_res ? __expf(x0 - mx) : 0.f;
      const float e1 = lane + 64 < n_res ? __expf(x1 - mx) : 0.f;
      float sum = e0 + e1;
      for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
      if (lane < n_res) sP[h][lane] = e0;
      if (lane + 64 < n_res) sP[h][lane + 64] = e1;
      if (lane == 0) { sM[h] = mx; sL[h] = sum; }
    }
  }
  __syncthreads();
  const int d = tid & 127;
  float* out = part + ((size_t)p * (n_splits + 1) + n_splits) * g * kPartStrideM;
  if (h0 < g) {
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    for (int tt = 0; tt < n_res; ++tt) {
      const float vv = __half2float(cv.res_v[((size_t)p * R + tt) * kD + d]);
#pragma unroll
      for (int i = 0; i < 4; ++i) acc[i] = fmaf(sP[(h0 + i) & 7][tt], vv, acc[i]);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (h0 + i < g) out[(h0 + i) * kPartStrideM + d] = acc[i];
  }
  if (tid < g) {
    out[tid * kPartStrideM + kD] = n_res > 0 ? sM[tid] : -INFINITY;
    out[tid * kPartStrideM + kD + 1] = n_res > 0 ? sL[tid] : 0.f;
  }
}

template <int K4, int K16, int NVG, int NKL>
static hipError_t launch_one(const CacheView& v, const __half* q, float scale, int n_blocks, int n_res, int n_splits,
                             float* part, hipStream_t s, hipEvent_t ev_start, hipEvent_t ev_stop) {
  auto kern = decode_mfma_kernel<K4, K16, NVG, NKL>;
  const size_t lds = 2048 + 64 + (size_t)kWaves * kWaveLds;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  if (ev_start) (void)hipEventRecord(ev_start, s);
  kern<<<dim3(v.P, n_splits), dim3(kMfmaThreads), lds, s>>>(v, q, scale * 1.4426950408889634f, n_blocks, n_res, n_splits,
                                                            part, 0);
  if (ev_stop) (void)hipEventRecord(ev_stop, s);
  return hipGetLastError();
}

// Returns true and launches when the configuration is one the matrix-core kernel covers.
bool try_launch_decode_mfma(const CacheView& v, const __half* q, float scale, int n_blocks, int n_res, int n_splits,
                            float* part, int accumulate_q, hipStream_t s, hipEvent_t ev_start, hipEvent_t ev_stop,
                            hipError_t* err) {
  const mixkvq_config& c = v.cfg;
  if (c.R % 64 != 0 || c.Gk % 64 != 0 || c.Gv % 64 != 0 || n_blocks < 1) return false;
  if (v.lay.off_v > kKPartMax || v.lay.rec_bytes - v.lay.off_v_s > kVMetaMax) return false;
  const int nvg = v.lay.NVG;
  const int nkl = (v.lay.off_v / 16 + 63) / 64;
  hipError_t e = hipErrorInvalidValue;
  bool ok = true;
#define MIXKVQ_CASE(K4_, K16_, NVG_, NKL_)                                                                          \
  if (c.k4 == K4_ && c.k16 == K16_ && nvg == NVG_ && nkl <= NKL_)                                                   \
    e = launch_one<K4_, K16_, NVG_, NKL_>(v, q, scale, n_blocks, n_res, n_splits, part, s, ev_start, ev_stop);     \
  else
  MIXKVQ_CASE(16, 0, 1, 6)
  MIXKVQ_CASE(0, 12, 1, 8)
  MIXKVQ_CASE(0, 0, 1, 6)
  MIXKVQ_CASE(8, 0, 1, 6)
  MIXKVQ_CASE(24, 0, 1, 6)
  MIXKVQ_CASE(32, 0, 1, 6)
  MIXKVQ_CASE(16, 0, 2, 6)
  MIXKVQ_CASE(0, 12, 2, 8)
  MIXKVQ_CASE(8, 4, 1, 8)
  MIXKVQ_CASE(0, 32, 1, 8)
  ok = false;
#undef MIXKVQ_CASE
  if (!ok) return false;
  if (e == hipSuccess) {
    decode_residual_kernel<<<dim3(v.P), dim3(256), 0, s>>>(v, q, scale, n_res, n_splits, part, accumulate_q);
    e = hipGetLastError();
  }
  *err = e;
  return true;
}

}  // namespace mixkvq
