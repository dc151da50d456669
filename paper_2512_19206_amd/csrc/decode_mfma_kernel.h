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
// This header holds the kernel template and its launcher; the .hip files that include it hold the tables of
// instantiated variants (one translation unit per table, so that they compile in parallel).
#pragma once
#include <hip/hip_ext.h>
#include <atomic>
#include "mixkvq_internal.h"

namespace mixkvq {


typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

constexpr int kMfmaThreads = 256;
constexpr int kComputeUnits = 256;              // MI355X
constexpr int kWaves = kMfmaThreads / 64;
constexpr int kKPartMax = 12288;                // bytes of a record before the value plane (staged in LDS)
constexpr int kVMetaMax = 2048;                 // value scales + zero-points of one block
constexpr int kQsStride = 168;                  // halfs per head row of the slot-ordered q table (160 slots + padding)
constexpr int kQsBytes = 8 * kQsStride * 2;
constexpr int kWaveLds = kKPartMax + kVMetaMax + 256 + kQsBytes;   // + a spare 256 bytes + slot-ordered q
constexpr int kHdrLds = 2048 + 256 + 2048 + 2048;   // normalised q [8][128], exponents and wave maxima, q transposed [128][8], raw q [8][128]
constexpr int kPartStrideM = kD + 2;
constexpr int kPBoost = 8;                      // softmax weights go to the matrix cores as p * 2^kPBoost (see mfma_part)
constexpr unsigned kBigScale = 0x5BF8u;         // fp16 255: the largest value scale for which p' * s cannot overflow

#if defined(MIXKVQ_PHASE_CLOCKS) && defined(MIXKVQ_MFMA_MAIN_TU)
// Profiling aid, not part of the default build: 100 MHz timestamps of each wavefront's phases.
__device__ unsigned long long g_phase_clock[4096 * 16];
#define MIXKVQ_PHASE(K_)                                                                              \
  if (lane == 0)                                                                                      \
    g_phase_clock[((blockIdx.y * gridDim.x + blockIdx.x) * kWaves + wave) % 4096 * 16 + (K_)] = wall_clock64();
// slots 12 and 13: the shader clock at the first and the last phase
#define MIXKVQ_PHASE_CYCLES(K_)                                                                       \
  if (lane == 0)                                                                                      \
    g_phase_clock[((blockIdx.y * gridDim.x + blockIdx.x) * kWaves + wave) % 4096 * 16 + (K_)] = clock64();
#else
#define MIXKVQ_PHASE(K_)
#define MIXKVQ_PHASE_CYCLES(K_)
#endif

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
__device__ __forceinline__ unsigned row_shl8u(unsigned v) { return __builtin_amdgcn_update_dpp(0u, v, 0x108, 0xF, 0xF, true); }
// value of lane (i+8)%16 inside each row of 16 lanes
__device__ __forceinline__ float row_ror8(float v) {
  return __uint_as_float(__builtin_amdgcn_update_dpp(0u, __float_as_uint(v), 0x128, 0xF, 0xF, true));
}

// Small operands of the two value steps of one register of softmax weights: P*s as an fp16 head plus its exact fp16
// remainder (one fused multiply-add), so that the value products carry ~22 bits of p*s like the key products do of
// q*s.  In lanes 0..7 of a row `p` holds the token pair of step 0, in lanes 8..15 the pair of step 1.  Step 0 gets
// the head in columns 0..7 and the tail of the same pairs in columns 8..15; step 1 gets the head of lanes 8..15
// moved to columns 0..7 while columns 8..15 keep their own tail.  Columns 8..15 of the output accumulate the
// tail products; the halves are added once, after the last record.
__device__ __forceinline__ void ps_operands(unsigned p, unsigned sv, u32x4& b0, u32x4& b1, int i) {
  const unsigned pm = pk_mul(p, sv);
  const unsigned pt = pk_fma_neg(p, sv, pm);
  b0[i] = __builtin_amdgcn_update_dpp(pm, pt, 0x118, 0xF, 0xC, false);   // row_shr:8 into lanes 8..15 only
  b1[i] = __builtin_amdgcn_update_dpp(pt, pm, 0x108, 0xF, 0x3, false);   // row_shl:8 into lanes 0..7 only
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
// four-bit word -> one A operand: code pairs (0,1) (2,3) (4,5) (6,7)
__device__ __forceinline__ u32x4 unpack4(unsigned w) {
  const unsigned w8 = w >> 8;
  u32x4 a;
  a[0] = w & 0x000F000Fu; a[1] = w & 0x00F000F0u; a[2] = w8 & 0x000F000Fu; a[3] = w8 & 0x00F000F0u;
  return a;
}

// Lanes of a wavefront hand data to each other through the wavefront's own LDS region.  The hardware keeps a
// wavefront's LDS operations in order, so no instruction is needed, but the compiler must be told that what a
// lane reads may have been written by another lane (else it may reuse a value the lane loaded earlier).
__device__ __forceinline__ void wave_lds_handoff() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Channel of A-row `row` of the value product (xp, qq), i.e. which value code word a lane holds in element qq of
// vreg[.][xp].  All 16 rows of one product must share a value group (the small operand carries the group's
// scales): with groups of 64 or 128 channels row r of (xp, qq) is channel 64 xp + 4 r + qq; with groups of 32
// channels (NVG = 4) it is channel 32 (2 xp + qq/2) + 2 r + qq%2, and (xp, qq) belongs to value group 2 xp + qq/2.
template <int NVG>
__device__ __forceinline__ constexpr int value_channel(int xp, int qq, int row) {
  return NVG == 4 ? 32 * (2 * xp + (qq >> 1)) + 2 * row + (qq & 1) : 64 * xp + 4 * row + qq;
}
template <int NVG>
__device__ __forceinline__ constexpr int value_group(int xp, int qq) {
  return NVG == 4 ? 2 * xp + (qq >> 1) : (NVG == 2 ? xp : 0);
}

// THR = 1: threshold policy.  K4 and K16 are capacities, a block's channel lists may hold unused entries
// (MIXKVQ_NO_CHANNEL) and the 2-bit planes have room for every channel.
template <int K4, int K16, int THR>
struct Tiers {
  static constexpr int NL = THR ? kD : kD - K4 - K16;
  static constexpr int Wlo = (NL + 15) / 16;   // 2-bit words per token
  static constexpr int NLp = Wlo * 16;
  static constexpr int NU = (Wlo + 3) / 4;     // word rounds: lane group kg takes 2-bit word 4u + kg in round u
  static constexpr int W4 = K4 / 8;            // 4-bit words per token
  static_assert(W4 <= 4, "the 4-bit tier must fit one MFMA step");
  static_assert(K16 <= 32, "the fp16 tier must fit one MFMA step");
};

// Which 1-KiB pieces of the key part the FIRST 64 tokens of a record of 128 tokens with one key group need
// (the small planes, the first half of each code plane): a wavefront stages those, works on the first half while
// the other pieces may still be on their way, and stages the rest before the second half.  The plane offsets
// are those of mixkvq_block_layout for R = Gk = 128; the launcher checks them against the cache's layout.
template <int K4, int K16, int THR>
struct HalfSplit {
  static constexpr int al(int n) { return (n + 15) / 16 * 16; }
  static constexpr int ks = K4 + K16, NL = THR ? kD : kD - ks, Wlo = (NL + 15) / 16, NLp = 16 * Wlo, W4 = K4 / 8;
  static constexpr int off_klo = al(ks) + al(4) + 2 * al(NLp * 2) + 2 * al(K4 * 2);
  static constexpr int off_k4 = off_klo + al(128 * Wlo * 4);
  static constexpr int off_k16 = off_k4 + al(128 * W4 * 4);
  static constexpr int off_v = off_k16 + al(128 * K16 * 2);
  static constexpr bool overlaps(int c, int lo, int hi) { return lo < hi && 1024 * c < hi && lo < 1024 * (c + 1); }
  static constexpr bool early(int c) {
    return overlaps(c, 0, off_klo + 64 * Wlo * 4) || overlaps(c, off_k4, off_k4 + 64 * W4 * 4) ||
           overlaps(c, off_k16, off_k16 + 64 * K16 * 2);
  }
};

// Contraction slots.  Every lane group runs the same code; a lane group whose word does not
// exist reads a clamped address and meets a zero in the small operand.
//   2-bit tier, step 2u+x (u < NU, x = 0,1): lane group kg unpacks half x of word c = 4u+kg;
//       VGPR e pairs channels j and j+1 of the 2-bit list, j = 16c + 8x + 2e, position factor 4^sc2(4x+e)
//   4-bit tier, one step: lane group kg unpacks word kg; VGPR e pairs tier entries 8kg+2e, 8kg+2e+1
//   fp16 tier, one step: lane group kg takes tier entries 8kg .. 8kg+7 as they are

// merge of the split partials (one kernel for every variant; defined beside the main table)
constexpr int kMergeLds = 64 + ((kMaxSplits + 1) * 8 * 2 + 16) * 4;
hipError_t launch_merge_pair(const CacheView& v, const float* part, int n_splits, __half* out, float* lse, hipStream_t s);


template <int K4, int K16, int NVG, int NKL, int RG, int THR, int G32, int PG, int RH>
__device__ __forceinline__ void mfma_part(const CacheView& cv, const __half* __restrict__ q, float scale_log2e,
                                          int n_blocks, int n_res, int n_splits, float* __restrict__ part,
                                          int accumulate_q, const NewToken& nt, const SeqCounts& sc, unsigned char* smem,
                                          __half* __restrict__ fin_out, float* __restrict__ fin_lse) {
  using T = Tiers<K4, K16, THR>;
  constexpr int NU = T::NU;
  // scalars of the by-value view (kept in SGPRs; no references into the kernel argument)
  // RG = 1: R = Gk = 128 known at compile time (one straight-line body per block record)
  // G32 = 1: key groups of 32 tokens.  A tile of 16 tokens must lie in ONE key group (its small operand carries
  // that group's scales), so tiles 0, 1 take the first 32 tokens of a 64-token span and tiles 2, 3 the second 32,
  // each lane group owning 8 tokens of either half; the value words of such a cache are interleaved to match
  // (codes 0..7 from the first half, 8..15 from the second: see the record layout).
  // RH = 1: records of 32 tokens (R = Gk = 32): a record is HALF a 64-token span.  The lanes of token groups 2 and 3
  // (kg >= 2) then have no tokens: their logits are -inf, and they load the value words and value scales of token
  // group 0 instead (finite numbers that meet weights of exactly zero).
  static_assert(!(G32 && RG), "RG fixes Gk = 128");
  static_assert(!(RH && (G32 || RG)), "RH is the plain tile order on a record of 32 tokens");
  const int R = RG ? 128 : cv.cfg.R, Gk = RG ? 128 : (G32 ? 32 : cv.cfg.Gk);
  const int g = cv.g, Hq = cv.cfg.Hq, Hkv = cv.cfg.Hkv, NB = cv.NB;
  const int rec_bytes = cv.lay.rec_bytes, off_idx = cv.lay.off_idx, off_klo_s = cv.lay.off_klo_s,
            off_klo_z = cv.lay.off_klo_z, off_k4_s = cv.lay.off_k4_s, off_k4_z = cv.lay.off_k4_z,
            off_kmax = cv.lay.off_kmax, off_klo = cv.lay.off_klo, off_k4 = cv.lay.off_k4, off_k16 = cv.lay.off_k16, off_v = cv.lay.off_v,
            off_v_s = cv.lay.off_v_s;
  const unsigned char* const blocks = cv.blocks;
  const int p = blockIdx.x, split = blockIdx.y, tid = threadIdx.x;
  const int b = p / Hkv, jkv = p % Hkv;
  bool skip_pair = false;
  if (sc.enabled) {      // sequences of different lengths: this pair's own counts; a sequence without tokens is skipped
    n_blocks = sc.n_blocks[b];
    n_res = sc.n_fp16[b];
    skip_pair = n_blocks == 0 && n_res == 0;
  }
  // (the wavefront index is the same in all lanes: as a scalar it keeps record indices and addresses off the vector ALU)
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, n = lane & 15, kg = lane >> 4;
  // Two workgroups share a compute unit, and among wavefronts of equal priority a SIMD issues from the OLDER one
  // first.  With one round of workgroups (at most two per compute unit, all resident from the start) the workgroups
  // of the second half of the grid are the younger ones everywhere: measured, their wavefronts finished 30 % later
  // than their neighbours, which then left the SIMDs to a single wavefront each for the last quarter of the kernel.
  // The younger wavefronts therefore raise their priority during five of every eight half-records (s_setprio only
  // reorders instruction issue): each of the two then wins about half of the time and both finish nearly together.
  const int n_wgs = gridDim.x * gridDim.y;
  const bool younger = n_wgs > kComputeUnits && n_wgs <= 2 * kComputeUnits &&
                       (int)(blockIdx.y * gridDim.x + blockIdx.x) >= kComputeUnits;
  const int head = n & 7, role = n >> 3;     // role 0: head of q*s, role 1: tail
  const bool live = head < g;

  __half* sQn = reinterpret_cast<__half*>(smem);                   // [8][128] normalised q
  int* sEq = reinterpret_cast<int*>(smem + 2048);                   // [8] exponents
  __half* sQt = reinterpret_cast<__half*>(smem + 2048 + 256);       // [128][8]: the 8 heads of a channel in 16 bytes
  unsigned short* sQraw = reinterpret_cast<unsigned short*>(smem + 2048 + 256 + 2048);   // [8][128] q as given
  unsigned char* wbase = smem + kHdrLds + wave * kWaveLds;           // this wave's private region
  unsigned char* sK = wbase;                                        // record bytes [0, NKL KiB)
  unsigned char* sVm = wbase + kKPartMax;                           // v_s, v_z planes
  unsigned short* sQs = reinterpret_cast<unsigned short*>(wbase + kKPartMax + kVMetaMax + 256);   // [8][kQsStride]

  // Work units of the pair: its block records, then the residual window in sub-units of 32 tokens, dealt
  // round-robin over all wavefronts of the pair's workgroups.
  const int gw = split * kWaves + wave, n_gw = n_splits * kWaves;
  // The wavefronts of a workgroup take neighbouring records at the same time (wavefront w of workgroup s
  // takes units s*4 + w, then + 4*n_splits, ...): the chip streams a few long contiguous ranges.
  const int blk_lo = gw;
  const int blk_hi = n_blocks;
  const int blk_step = n_gw;
  // fp16 rows (sink tokens, then the residual window; n_res counts both): sub-units of 32 tokens follow the
  // records in the same round-robin deal
  const int n_sub = (n_res + 31) >> 5;     // <= 12 (sink + window <= 384 rows) and <= n_gw (the launcher sees to it)
  // unit n_blocks + j belongs to wavefront (n_blocks + j) % n_gw; n_sub <= n_gw, so one division serves them all
  const int first_sub_gw = n_blocks % n_gw;
  int my_sub = gw - first_sub_gw;
  if (my_sub < 0) my_sub += n_gw;
  if (my_sub >= n_sub) my_sub = -1;
  // one wavefront per pair (the next in the deal, never one with a sub-unit unless the pair has a single
  // workgroup) stores this step's new token and adds |q| to the accumulator
  const bool bookkeeper =
      (first_sub_gw + n_sub >= n_gw ? first_sub_gw + n_sub - n_gw : first_sub_gw + n_sub) == gw && !skip_pair;

  // ---- per-lane constants -------------------------------------------------
  // token of A-row n in tile (h, x): 64h + tokbase + {0,1,8,9}[x]  (G32: 8 (n/4) + 2 (n%4) + {0,1,32,33}[x])
  const int tokbase = (G32 ? 8 : 16) * (n >> 2) + 2 * (n & 3);
  const bool no_tokens = RH && kg >= 2;     // this lane's token group lies past the end of a 32-token record
  const int kgv = no_tokens ? 0 : kg;       // the token group whose value words and scales it reads
  const int rec_chunks = rec_bytes >> 4;
  const int nvm = (rec_bytes - off_v_s) >> 4;     // 16-byte chunks of the value scale/zero planes
  // LDS byte offsets of this lane's words in token `tokbase` (clamped to existing words)
  // With 8 two-bit words per token a token's row is 32 bytes, and the 16 tokens a lane group reads in one
  // instruction (even or odd tokens, 2 apart, in four runs 16 apart) would share 4 of the 64 LDS banks.  Such a
  // plane (SWZ) is staged with its 16-byte pieces permuted inside every aligned run of four: piece J goes to
  // J ^ ((J >> 5) & 3), i.e. bits 4..5 of the token index are XORed into the two address bits that are the same for
  // all lanes of an instruction; the 64 lanes then cover all banks.
  constexpr bool SWZ = T::Wlo == 8 && NKL <= 8;     // (variants that stage more pieces have no registers to spare for the permuted piece indices)
  constexpr int kOffx[4] = {0, 1, G32 ? 32 : 8, G32 ? 33 : 9};      // token offsets of the four tiles of a 64-token span
  int lo_word_off[NU][SWZ ? 4 : 1];     // [round][tile] (one entry per round without the permutation)
#pragma unroll
  for (int u = 0; u < NU; ++u) {
    const int c = 4 * u + kg < T::Wlo ? 4 * u + kg : T::Wlo - 1;
    if (SWZ) {
#pragma unroll
      for (int x = 0; x < 4; ++x) {
        const int tk = tokbase + kOffx[x], piece = 2 * tk + (c >> 2);
        lo_word_off[u][x] = off_klo + 16 * (piece ^ ((piece >> 5) & 3)) + 4 * (c & 3) - 4 * kOffx[x] * T::Wlo;
      }
    } else {
      lo_word_off[u][0] = off_klo + 4 * (tokbase * T::Wlo + c);
    }
  }
  // LDS piece a lane stages its c-th 16-byte piece of a record to
  int kst[NKL];
#pragma unroll
  for (int c = 0; c < NKL; ++c) {
    int piece = c * 64 + lane;
    const int j = piece - (off_klo >> 4);
    if (SWZ && j >= 0 && j < 2 * R) piece = (off_klo >> 4) + (j ^ ((j >> 5) & 3));
    kst[c] = piece;
  }
  const int h4_word_off = off_k4 + 4 * (tokbase * T::W4 + (kg < T::W4 ? kg : 0));
  const int k16_off = off_k16 + 2 * (tokbase * K16 + (8 * kg < K16 ? 8 * kg : 0));

  // running state (log2 domain)
  float m_run = -INFINITY, l_run = 0.f;
  float zacc[NVG][4];   // sum p' z per register index; its position factor is a per-lane constant
  // position exponent of pair i in this lane half: step 0 (lanes 0..7 of a row) or step 1 (lanes 8..15)
  // p is rounded to fp16 once, as p' = p * 4^-sc * 2^kPBoost (p <= 1, so p' <= 2^kPBoost).  The boost keeps small
  // weights out of the fp16 subnormals: with it the weight of a token that meets a code at position 4 is resolved
  // down to 2^-25 of the wavefront's largest weight (2^-17 without).
  // (the variants with the highest register pressure, both side tiers and four value groups, do not keep these eight
  //  constants across the loop, where they would be spilled: they form them where they are used, two instructions each)
  constexpr bool kLeanConstants = NVG == 4 && K4 > 0 && K16 > 0;
  float sc2f[4];        // 2 sc - kPBoost: exponent offset of p' for pair i
  unsigned w4sc[4];     // fp16 pair (4^sc 2^-kPBoost, same): turns p' back into p for the sum l
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int sc = role ? sc2(4 + i) : i;
    sc2f[i] = 2.f * sc - (float)kPBoost;
    w4sc[i] = ((unsigned)(15 + 2 * sc - kPBoost) << 10) * 0x00010001u;
  }
  f32x4 O[2][4];   // [x'][q]: channels 64x' + 16kg + 4i + q
#pragma unroll
  for (int a = 0; a < NVG; ++a)
#pragma unroll
    for (int c = 0; c < 4; ++c) zacc[a][c] = 0.f;
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int c = 0; c < 4; ++c) O[a][c] = f32x4{0.f, 0.f, 0.f, 0.f};

  // q in slot order (rebuilt when the block's channel selection changes)
  unsigned qlo[2 * NU][4];            // [step][vgpr]: normalised q pairs of the 2-bit tier
  unsigned qh4[4];                    // 4-bit tier pairs
  // fp16-tier pairs, zero beyond the tier, as two small operands: q16a is zero in columns 8..15 and q16b in columns
  // 0..7.  A product of tile 0 (1) with q16a and one of tile 2 (3) with q16b into the SAME accumulator leave in
  // every lane the tile its half keeps (lanes 0..7 of a row keep tiles 0 and 1, lanes 8..15 tiles 2 and 3).
  unsigned q16a[4], q16b[4];
  constexpr int kSelWords = K4 + K16 > 0 ? (K4 + K16 + 3) / 4 : 1;
  unsigned sel_prev[kSelWords];     // wave-uniform: the selection q was last laid out for
#pragma unroll
  for (int i = 0; i < kSelWords; ++i) sel_prev[i] = 0xffffffffu;
#pragma unroll
  for (int s = 0; s < 2 * NU; ++s)
#pragma unroll
    for (int e = 0; e < 4; ++e) qlo[s][e] = 0u;
#pragma unroll
  for (int e = 0; e < 4; ++e) { qh4[e] = 0u; q16a[e] = 0u; q16b[e] = 0u; }

  // prefetch registers
  u32x4 kreg[NKL];
  constexpr int NVM = NVG == 4 ? 2 : 1;   // 1 KiB pieces of the value scale / zero-point planes
  u32x4 vmreg[NVM];
  u32x4 vreg[2][2];   // [h][x]

  // Where a record lives: block BLK of the pair in the contiguous layout, or with a block table the pair's record
  // in pool slot SLOT.  The slots of this wavefront's next two records are looked up ahead of time, so that no
  // record load ever waits for a table entry.
  // (PG = 0: instantiations for the contiguous layout, where all of this folds away)
  // PG = 2: either layout, decided by the table pointer at run time (1-2 % slower than a variant for one layout)
  const int32_t* const tab = (PG == 1 || (PG == 2 && cv.table)) ? cv.table + (size_t)b * NB : nullptr;
#define MIXKVQ_REC_INDEX(BLK, SLOT) \
  (tab ? (unsigned)(SLOT) * (unsigned)Hkv + (unsigned)jkv : (unsigned)p * (unsigned)NB + (unsigned)(BLK))
#define MIXKVQ_REC(IDX) (blocks + (size_t)(IDX) * rec_bytes)     // (fewer than 2^31 records: the host checks)
  int slot_cur = 0, slot_nx = 0;

  // Loads of one block.  A record's address is a scalar; every lane adds a 32-bit byte offset that is fixed for
  // the whole kernel (so the loop spends no vector instruction on addresses).  Chunk indices are clamped to the
  // record so that every lane loads and stores unconditionally (a clamped lane repeats the record's last chunk).
  // Variants that stage more than 8 KiB of key part, or have four value groups, or both side tiers with key groups of 32
  // tokens, have no registers to spare for one offset per piece (kept, they are
  // spilled and reloaded inside the loop, and a reload waits for every record load in flight before it): those form each
  // offset where it is used, with an add and a minimum, from a copy of the lane's first offset that the compiler
  // cannot see through (else it would hoist the ten to twelve results out of the loop again).
  constexpr bool kKeepOffsets = NKL <= 8 && NVG != 4 && !(G32 && K4 > 0 && K16 > 0);
  unsigned koff[kKeepOffsets ? NKL : 1], vmoff[NVM];
#pragma unroll
  for (int c = 0; c < (kKeepOffsets ? NKL : 1); ++c)
    koff[c] = 16u * (unsigned)(c * 64 + lane < rec_chunks ? c * 64 + lane : rec_chunks - 1);
  const unsigned koff_last = 16u * (unsigned)(rec_chunks - 1);
#pragma unroll
  for (int c = 0; c < NVM; ++c) vmoff[c] = (unsigned)off_v_s + 16u * (unsigned)(c * 64 + lane < nvm ? c * 64 + lane : nvm - 1);
  // byte offset of this lane's value words in token group 0 of a record: channels value_channel(0, 0..3, n) of row kgv
  const unsigned voff = (unsigned)off_v + 4u * (unsigned)(kgv * kD) + (NVG == 4 ? 8u : 16u) * (unsigned)n;
  /* RG variants split a record's key part in the pieces its first 64 tokens need (EARLY, with the value */       \
  /* metadata) and the rest (LATE); elsewhere everything is EARLY */
  using HS = HalfSplit<K4, K16, THR>;
#define MIXKVQ_IS_EARLY(C) (!RG || HS::early(C))
#define MIXKVQ_KOFF(C) (kKeepOffsets ? koff[kKeepOffsets ? (C) : 0] : min(lane16_ + 1024u * (unsigned)(C), koff_last))
#define MIXKVQ_ISSUE_K_EARLY(REC)                                                                           \
  {                                                                                                          \
    const unsigned char* rec_ = MIXKVQ_REC(REC);                                                             \
    unsigned lane16_ = koff[0];                                                                              \
    if (!kKeepOffsets) asm volatile("" : "+v"(lane16_));                                                     \
    _Pragma("unroll") for (int c = 0; c < NKL; ++c)                                                         \
        if (MIXKVQ_IS_EARLY(c)) kreg[c] = *reinterpret_cast<const u32x4*>(rec_ + MIXKVQ_KOFF(c));            \
    _Pragma("unroll") for (int c = 0; c < NVM; ++c)                                                         \
        vmreg[c] = *reinterpret_cast<const u32x4*>(rec_ + vmoff[c]);                                         \
  }
#define MIXKVQ_ISSUE_K_LATE(REC)                                                                            \
  {                                                                                                          \
    const unsigned char* rec_ = MIXKVQ_REC(REC);                                                             \
    unsigned lane16_ = koff[0];                                                                              \
    if (!kKeepOffsets) asm volatile("" : "+v"(lane16_));                                                     \
    _Pragma("unroll") for (int c = 0; c < NKL; ++c)                                                         \
        if (!MIXKVQ_IS_EARLY(c)) kreg[c] = *reinterpret_cast<const u32x4*>(rec_ + MIXKVQ_KOFF(c));           \
  }
  /* the four value words of vreg[.][X]: channels value_channel(X, 0..3, n) of the token group row at byte ROWB_ */
#define MIXKVQ_LOAD_VWORDS(DST, ROWB_, X)                                                                    \
  {                                                                                                          \
    if (NVG == 4) {                                                                                          \
      const uint2 lo_ = *reinterpret_cast<const uint2*>((ROWB_) + 256 * (X));                                \
      const uint2 hi_ = *reinterpret_cast<const uint2*>((ROWB_) + 256 * (X) + 128);                          \
      DST = u32x4{lo_.x, lo_.y, hi_.x, hi_.y};                                                               \
    } else {                                                                                                 \
      DST = *reinterpret_cast<const u32x4*>((ROWB_) + 256 * (X));                                            \
    }                                                                                                        \
  }
#define MIXKVQ_ISSUE_V_LOADS(REC)                                                                           \
  {                                                                                                          \
    const unsigned char* rec_ = MIXKVQ_REC(REC);                                                             \
    _Pragma("unroll") for (int h = 0; h < 2; ++h) _Pragma("unroll") for (int x = 0; x < 2; ++x)             \
        MIXKVQ_LOAD_VWORDS(vreg[h][x], rec_ + 2048 * (h * 64 < R ? h : 0) + voff, x)                        \
  }

  // The value words of one half (64 tokens) of a record: asked for as soon as the previous record's matrix
  // products have consumed the registers they land in, so that each half has most of a record's time to arrive.
#define MIXKVQ_ISSUE_V_HALF(REC, H)                                                                          \
  {                                                                                                          \
    const unsigned char* rec_ = MIXKVQ_REC(REC);                                                             \
    _Pragma("unroll") for (int x = 0; x < 2; ++x)                                                           \
        MIXKVQ_LOAD_VWORDS(vreg[H][x], rec_ + 2048 * (H) + voff, x)                                         \
  }

  // q in slot order from the selection words SELW (wave-uniform): a table [head][slot] in LDS, slots 0..127 for the
  // block's 2-bit channels in ascending order (zero past the last one), slots 128.. for the fp16 tier and then the
  // 4-bit tier.  Bitmaps of the two tiers are built with scalar arithmetic; every lane then knows the slots of its
  // two channels (lane, lane + 64) from population counts, reads their 8 heads from the transposed q (one 16-byte
  // read each) and scatters them into the table: no list of channels goes through memory.  Places no channel
  // claims are zeroed (FIRST_: the ones that never change; threshold policy: also the ones that depend on the block).
  // Every lane finally reads the 8 entries of each of its contraction steps with one 16-byte read.
#define MIXKVQ_BELOW(MASK_) \
  ((int)__builtin_amdgcn_mbcnt_hi((unsigned)((MASK_) >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)(MASK_), 0u)))
#define MIXKVQ_REBUILD_Q(SELW, FIRST_)                                                                         \
  {                                                                                                            \
    unsigned long long a0_ = 0, a1_ = 0, b0_ = 0, b1_ = 0;   /* fp16 tier / 4-bit tier, channels 0..63 / 64..127 */ \
    _Pragma("unroll") for (int i = 0; i < K4 + K16; ++i) {                                                     \
      const unsigned ch = (SELW[i >> 2] >> (8 * (i & 3))) & 0xffu;   /* >= 128: an unused entry */             \
      const unsigned long long lo_ = ch < 64u ? 1ull << (ch & 63u) : 0ull;                                     \
      const unsigned long long hi_ = (ch >= 64u && ch < 128u) ? 1ull << (ch & 63u) : 0ull;                     \
      if (i < K16) { a0_ |= lo_; a1_ |= hi_; } else { b0_ |= lo_; b1_ |= hi_; }                                \
    }                                                                                                          \
    const unsigned long long m0_ = a0_ | b0_, m1_ = a1_ | b1_;                                                 \
    const int n16_ = __popcll(a0_) + __popcll(a1_), n4_ = __popcll(b0_) + __popcll(b1_);                       \
    const int n_lo_ = kD - n16_ - n4_;                                                                         \
    int slot0_ = lane - MIXKVQ_BELOW(m0_), slot1_ = 64 + lane - __popcll(m0_) - MIXKVQ_BELOW(m1_);             \
    if (K16 > 0) {                                                                                             \
      if ((a0_ >> lane) & 1) slot0_ = 128 + MIXKVQ_BELOW(a0_);                                                 \
      if ((a1_ >> lane) & 1) slot1_ = 128 + __popcll(a0_) + MIXKVQ_BELOW(a1_);                                 \
    }                                                                                                          \
    if (K4 > 0) {                                                                                              \
      if ((b0_ >> lane) & 1) slot0_ = 128 + K16 + MIXKVQ_BELOW(b0_);                                           \
      if ((b1_ >> lane) & 1) slot1_ = 128 + K16 + __popcll(b0_) + MIXKVQ_BELOW(b1_);                           \
    }                                                                                                          \
    {                                                                                                          \
      const u32x4 h0_ = *reinterpret_cast<const u32x4*>(sQt + lane * 8);                                       \
      const u32x4 h1_ = *reinterpret_cast<const u32x4*>(sQt + (lane + 64) * 8);                                \
      _Pragma("unroll") for (int e = 0; e < 4; ++e) {                                                          \
        sQs[(2 * e) * kQsStride + slot0_] = (unsigned short)(h0_[e] & 0xffffu);                                \
        sQs[(2 * e + 1) * kQsStride + slot0_] = (unsigned short)(h0_[e] >> 16);                                \
        sQs[(2 * e) * kQsStride + slot1_] = (unsigned short)(h1_[e] & 0xffffu);                                \
        sQs[(2 * e + 1) * kQsStride + slot1_] = (unsigned short)(h1_[e] >> 16);                                \
      }                                                                                                        \
    }                                                                                                          \
    if (THR || (FIRST_)) {                                                                                     \
      /* 2-bit places past the block's last 2-bit channel; side places that are unused or beyond both tiers */ \
      const bool side_ = lane < 32 && (lane >= K16 + K4 || (lane < K16 ? lane >= n16_ : lane - K16 >= n4_));   \
      _Pragma("unroll") for (int h = 0; h < 8; ++h) {                                                          \
        if (lane < kD - n_lo_) sQs[h * kQsStride + n_lo_ + lane] = 0;                                          \
        if (side_) sQs[h * kQsStride + 128 + lane] = 0;                                                        \
      }                                                                                                        \
    }                                                                                                          \
    wave_lds_handoff();                                                                                        \
    const unsigned short* qrow = sQs + head * kQsStride;                                                       \
    _Pragma("unroll") for (int u = 0; u < NU; ++u) _Pragma("unroll") for (int x = 0; x < 2; ++x) {             \
      const u32x4 t_ = *reinterpret_cast<const u32x4*>(qrow + 16 * (4 * u + kg) + 8 * x);                      \
      _Pragma("unroll") for (int e = 0; e < 4; ++e) qlo[2 * u + x][e] = t_[e];                                 \
    }                                                                                                          \
    if (K4 > 0) {                                                                                              \
      unsigned t_[4];                                                                                          \
      __builtin_memcpy(t_, qrow + 128 + K16 + 8 * (kg < T::W4 ? kg : 0), 16);                                  \
      _Pragma("unroll") for (int e = 0; e < 4; ++e) qh4[e] = kg < T::W4 ? t_[e] : 0u;                          \
    }                                                                                                          \
    if (K16 > 0) {                                                                                             \
      const u32x4 t_ = *reinterpret_cast<const u32x4*>(qrow + 128 + (8 * kg < K16 ? 8 * kg : 0));              \
      _Pragma("unroll") for (int e = 0; e < 4; ++e) {                                                          \
        const unsigned v_ = 8 * kg + 2 * e < K16 ? t_[e] : 0u;   /* (the table goes on with the 4-bit tier) */ \
        q16a[e] = role ? 0u : v_;                                                                              \
        q16b[e] = role ? v_ : 0u;                                                                              \
      }                                                                                                        \
    }                                                                                                          \
  }

  MIXKVQ_PHASE(0)
  MIXKVQ_PHASE_CYCLES(12)
  // Loads go out in the order of use (they return in order): q, the first record's channel selection, the
  // residual sub-unit, the first record.
  int blk = blk_lo;
  // the pair's bookkeeping wavefront: old accumulator values and the new token's rows, first in the queue
  unsigned long long qacc_old[2] = {0ull, 0ull}, qcnt_old = 0ull;
  uint4 nt_row = make_uint4(0u, 0u, 0u, 0u);
  if (bookkeeper) {
    if (accumulate_q) {
      qacc_old[0] = cv.qacc[(size_t)p * kD + lane];
      qacc_old[1] = cv.qacc[(size_t)p * kD + lane + 64];
      if (lane == 0) qcnt_old = cv.qcnt[p];
    }
    if (nt.k && lane < 32) {
      const int64_t src = (int64_t)b * nt.st.b + (int64_t)jkv * nt.st.h + (lane & 15) * 8;
      nt_row = *reinterpret_cast<const uint4*>((lane < 16 ? nt.k : nt.v) + src);
    }
  }
  uint2 qraw = make_uint2(0u, 0u);
  {
    const int h = tid >> 5, l32 = tid & 31;
    if (h < g) qraw = *reinterpret_cast<const uint2*>(q + ((size_t)b * Hq + jkv * g + h) * kD + l32 * 4);
  }
  unsigned sel_first[kSelWords];
#pragma unroll
  for (int i = 0; i < kSelWords; ++i) sel_first[i] = 0u;
  if (tab) {
    if (blk < blk_hi) slot_cur = tab[blk];
    if (blk + blk_step < blk_hi) slot_nx = tab[blk + blk_step];
  }
  const unsigned rec_first = MIXKVQ_REC_INDEX(blk, slot_cur);
  if (K4 + K16 > 0 && blk < blk_hi) {
    const unsigned* recw = reinterpret_cast<const unsigned*>(MIXKVQ_REC(rec_first) + off_idx);
#pragma unroll
    for (int i = 0; i < kSelWords; ++i) sel_first[i] = recw[i];
  }
  // Residual sub-unit of this wavefront: 2 key tiles x 4 contraction steps, 32 value rows.  This step's new
  // token is read from the caller's tensors.
  const int sub_t0 = 32 * (my_sub > 0 ? my_sub : 0);
  const int tokb = 8 * (n >> 2) + 2 * (n & 3);      // A-row n of tile x: token sub_t0 + tokb + x
  u32x4 kr[2][4], vr[8];
  if (my_sub >= 0) {
    const __half* rk = cv.res_k + (size_t)p * cv.RW * kD;     // the pair's fp16 rows: sink, then residual window
    const __half* rv = cv.res_v + (size_t)p * cv.RW * kD;
    const int64_t nt_off = (int64_t)b * nt.st.b + (int64_t)jkv * nt.st.h;
#pragma unroll
    for (int x = 0; x < 2; ++x) {
      const int row = sub_t0 + tokb + x;
      const __half* src = (nt.k && row == nt.row) ? nt.k + nt_off : rk + (size_t)row * kD;
#pragma unroll
      for (int st = 0; st < 4; ++st) kr[x][st] = *reinterpret_cast<const u32x4*>(src + 8 * kg + 32 * st);
    }
#pragma unroll
    for (int it = 0; it < 8; ++it) {
      const int ci = it * 64 + lane, row = sub_t0 + (ci >> 4);
      const __half* src = (nt.k && row == nt.row) ? nt.v + nt_off : rv + (size_t)row * kD;
      vr[it] = *reinterpret_cast<const u32x4*>(src + 8 * (ci & 15));
    }
  }
  if (blk < blk_hi) MIXKVQ_ISSUE_K_EARLY(rec_first)

  // ---- normalise q per head: qn = q * 2^-Eq with max|qn| in [1/2, 1) ----
  {
    const int h = tid >> 5, l32 = tid & 31;
    if (cv.cfg.in_dtype) {      // bfloat16 queries enter as binary16
      qraw.x = bf16x2_to_f16x2(qraw.x);
      qraw.y = bf16x2_to_f16x2(qraw.y);
    }
    const h2 q01 = __builtin_bit_cast(h2, qraw.x), q23 = __builtin_bit_cast(h2, qraw.y);
    const float v[4] = {(float)q01[0], (float)q01[1], (float)q23[0], (float)q23[1]};
    float mx = fmaxf(fmaxf(fabsf(v[0]), fabsf(v[1])), fmaxf(fabsf(v[2]), fabsf(v[3])));
    for (int o = 16; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 32));
    int ef = (int)((__float_as_uint(mx) >> 23) & 0xff) - 127 + 15;   // fp16 exponent field of the maximum
    if (ef < 1) ef = 1;
    const int eq = ef - 14;
    uint2 qn;
    qn.x = cvt_pk(ldexpf(v[0], -eq), ldexpf(v[1], -eq));
    qn.y = cvt_pk(ldexpf(v[2], -eq), ldexpf(v[3], -eq));
    *reinterpret_cast<uint2*>(sQn + h * kD + l32 * 4) = qn;
    if (accumulate_q) *reinterpret_cast<uint2*>(sQraw + h * kD + l32 * 4) = qraw;
    unsigned short* qt = reinterpret_cast<unsigned short*>(sQt) + (l32 * 4) * 8 + h;
    qt[0] = (unsigned short)(qn.x & 0xffffu);
    qt[8] = (unsigned short)(qn.x >> 16);
    qt[16] = (unsigned short)(qn.y & 0xffffu);
    qt[24] = (unsigned short)(qn.y >> 16);
    if (l32 == 0) sEq[h] = eq;
  }
  __syncthreads();
  const int Eq = sEq[head];
  MIXKVQ_PHASE(1)
  if (bookkeeper) {   // the new token enters the window; |q| of this step joins the accumulator (one writer per pair)
    if (nt.k && lane < 32) {
      const size_t dst = ((size_t)p * cv.RW + nt.row) * kD + (lane & 15) * 8;
      *reinterpret_cast<uint4*>((lane < 16 ? cv.res_k : cv.res_v) + dst) = as_f16x8(nt_row, cv.cfg.in_dtype != 0);
    }
    if (accumulate_q) {
#pragma unroll
      for (int hc = 0; hc < 2; ++hc) {
        const int d = lane + 64 * hc;
        unsigned long long acc = qacc_old[hc];
        for (int h = 0; h < g; ++h) acc += fix24_abs(sQraw[h * kD + d]);
        cv.qacc[(size_t)p * kD + d] = acc;
      }
      if (lane == 0) cv.qcnt[p] = qcnt_old + (unsigned long long)g;
    }
  }
  // q in the slot order of the first record, while that record is still on its way (its value words are
  // asked for only now: the first answers come the sooner the less every wavefront asks for at once)
  if (blk < blk_hi) {
    if (RG) {      // in the order of use: first half of the values, rest of the keys, second half of the values
      MIXKVQ_ISSUE_V_HALF(rec_first, 0)
      MIXKVQ_ISSUE_K_LATE(rec_first)
      MIXKVQ_ISSUE_V_HALF(rec_first, 1)
    } else {
      MIXKVQ_ISSUE_V_LOADS(rec_first)
    }
#pragma unroll
    for (int i = 0; i < kSelWords; ++i) sel_prev[i] = __builtin_amdgcn_readfirstlane(sel_first[i]);
    MIXKVQ_REBUILD_Q(sel_prev, true)
  }

  // ---- residual window (fp16 keys/values): 32 tokens per wavefront, before its block records ----
  if (my_sub >= 0) {
    const int t0 = sub_t0;
    if (cv.cfg.in_dtype && nt.k) {     // the new token's rows came from the caller's bfloat16 tensors
#pragma unroll
      for (int x = 0; x < 2; ++x)
        if (sub_t0 + tokb + x == nt.row) {
#pragma unroll
          for (int st = 0; st < 4; ++st)
#pragma unroll
            for (int e = 0; e < 4; ++e) kr[x][st][e] = bf16x2_to_f16x2(kr[x][st][e]);
        }
#pragma unroll
      for (int it = 0; it < 8; ++it)
        if (sub_t0 + ((it * 64 + lane) >> 4) == nt.row) {
#pragma unroll
          for (int e = 0; e < 4; ++e) vr[it][e] = bf16x2_to_f16x2(vr[it][e]);
        }
    }
    constexpr int kVStride = 264;     // bytes per staged value row (+8 against bank conflicts)
    const float Cres = ldexpf(scale_log2e, Eq);
    f32x4 S0 = {0.f, 0.f, 0.f, 0.f}, S1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int st = 0; st < 4; ++st) {
      u32x4 bq;       // normalised q in natural channel order; columns 8..15 stay zero
#pragma unroll
      for (int e = 0; e < 4; ++e)
        bq[e] = (role == 0 && live) ? *reinterpret_cast<const unsigned*>(sQn + head * kD + 32 * st + 8 * kg + 2 * e) : 0u;
      S0 = mfma(kr[0][st], bq, S0);
      S1 = mfma(kr[1][st], bq, S1);
    }
    float xa[4], xb[4];
    float mx = -INFINITY;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int tok = t0 + 8 * kg + 2 * i;      // token of xa; xb is the next one
      xa[i] = (role == 0 && tok < n_res) ? S0[i] * Cres : -INFINITY;
      xb[i] = (role == 0 && tok + 1 < n_res) ? S1[i] * Cres : -INFINITY;
      mx = fmaxf(mx, fmaxf(xa[i], xb[i]));
    }
    mx = xkg_max(mx);
    mx = fmaxf(mx, row_ror8(mx));       // finite: token t0 is valid
    m_run = mx;                          // nothing has been accumulated yet
    u32x4 Bp;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      Bp[i] = cvt_pk(__builtin_amdgcn_exp2f(xa[i] - m_run), __builtin_amdgcn_exp2f(xb[i] - m_run));
      l_run = dot2(Bp[i], 0x3c003c00u, l_run);
    }
    // values through LDS (rows beyond the window are zeroed), read back transposed: A row = channel,
    // slot pair = adjacent tokens
#pragma unroll
    for (int it = 0; it < 8; ++it) {
      const int ci = it * 64 + lane, rowi = ci >> 4, c16 = ci & 15;
      u32x4 v = vr[it];
      if (t0 + rowi >= n_res) v = u32x4{0u, 0u, 0u, 0u};
      uint2* dst = reinterpret_cast<uint2*>(sK + rowi * kVStride + 16 * c16);
      dst[0] = make_uint2(v[0], v[1]);
      dst[1] = make_uint2(v[2], v[3]);
    }
    wave_lds_handoff();
#pragma unroll
    for (int xp = 0; xp < 2; ++xp)
#pragma unroll
      for (int qq = 0; qq < 4; ++qq) {
        u32x4 a;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const unsigned short* cp = reinterpret_cast<const unsigned short*>(sK + (8 * kg + 2 * e) * kVStride) +
                                     value_channel<NVG>(xp, qq, n);
          a[e] = (unsigned)cp[0] | ((unsigned)cp[kVStride / 2] << 16);
        }
        // the block loop accumulates sum p' c 4^sc 2^-24 = 2^(kPBoost-24) sum p c and is scaled back at the end
        const f32x4 t = mfma(a, Bp, f32x4{0.f, 0.f, 0.f, 0.f});
        O[xp][qq] = t * (5.9604644775390625e-8f * (float)(1 << kPBoost));
      }
    wave_lds_handoff();     // the staging area is the record buffer of the block loop
  }

  // The two pieces of a super-group's key work, written once and placed per key group (see the loop below).
#define MIXKVQ_GROUP_OPERANDS(GRP)                                                                                     \
  {                                                                                                                    \
    /* ---- small key operand of this group: Qs = q * s (head and tail), bias = sum q z ---- */                        \
    /* The bias runs on the matrix cores too: the zero-points of a step's 32 slots as every row of the */              \
    /* large operand, q as the small one; all 16 rows of the result hold sum q z of the lane's head. */                \
    unsigned sp[2 * NU][4], sp4[4];   /* scales of this lane's slots: adjacent pairs, as stored */                     \
    f32x4 zd4 = {0.f, 0.f, 0.f, 0.f};                                                                                  \
    _Pragma("unroll")                                                                                                  \
    for (int u = 0; u < NU; ++u) {                                                                                     \
      const int c = 4 * u + kg < T::Wlo ? 4 * u + kg : T::Wlo - 1;                                                     \
      const uint4* ps = reinterpret_cast<const uint4*>(sK + off_klo_s + 2 * ((GRP) * T::NLp + 16 * c));                \
      const uint4* pz = reinterpret_cast<const uint4*>(sK + off_klo_z + 2 * ((GRP) * T::NLp + 16 * c));                \
    _Pragma("unroll")                                                                                                  \
      for (int x = 0; x < 2; ++x) {                                                                                    \
        const uint4 sv = ps[x], zv = pz[x];                                                                            \
        const unsigned sw[4] = {sv.x, sv.y, sv.z, sv.w}, zw[4] = {zv.x, zv.y, zv.z, zv.w};                             \
    _Pragma("unroll")                                                                                                  \
        for (int e = 0; e < 4; ++e) sp[2 * u + x][e] = sw[e];                                                          \
        zd4 = mfma(u32x4{zw[0], zw[1], zw[2], zw[3]},                                                                  \
                   u32x4{qlo[2 * u + x][0], qlo[2 * u + x][1], qlo[2 * u + x][2], qlo[2 * u + x][3]}, zd4);            \
      }                                                                                                                \
    }                                                                                                                  \
    if (K4 > 0) {                                                                                                      \
      const int w = kg < T::W4 ? kg : 0;                                                                               \
      const uint4 sv = *reinterpret_cast<const uint4*>(sK + off_k4_s + 2 * ((GRP) * K4 + 8 * w));                      \
      const uint4 zv = *reinterpret_cast<const uint4*>(sK + off_k4_z + 2 * ((GRP) * K4 + 8 * w));                      \
      const unsigned sw[4] = {sv.x, sv.y, sv.z, sv.w}, zw[4] = {zv.x, zv.y, zv.z, zv.w};                               \
    _Pragma("unroll")                                                                                                  \
      for (int e = 0; e < 4; ++e) sp4[e] = sw[e];                                                                      \
      zd4 = mfma(u32x4{zw[0], zw[1], zw[2], zw[3]}, u32x4{qh4[0], qh4[1], qh4[2], qh4[3]}, zd4);                       \
    }                                                                                                                  \
    zdot = zd4[0];                                                                                                     \
    /* block exponent: scales are multiplied by 2^e0 so that the largest lands in [2^14, 2^15) (e0 <= 15), */          \
    /* and by 4^-sc, the position factor of the code they meet in the product */                                       \
    int efs = (int)(*reinterpret_cast<const unsigned short*>(sK + off_kmax + 2 * (GRP)) >> 10);   /* exponent field */ \
    if (efs < 1) efs = 1;                                                                                              \
    efs = __builtin_amdgcn_readfirstlane(efs);                                                                         \
    const int e0 = 29 - efs < 15 ? 29 - efs : 15;                                                                      \
    /* every lane forms the head fp16(q s); the lanes of the tail columns then replace it by the exact */              \
    /* remainder q s - head in ONE divergent region (cheaper than a select per register) */                            \
    _Pragma("unroll")                                                                                                  \
    for (int s = 0; s < 2 * NU; ++s)                                                                                   \
    _Pragma("unroll")                                                                                                  \
      for (int e = 0; e < 4; ++e) {                                                                                    \
        const unsigned mult = ((unsigned)(15 + e0 - 2 * sc2(4 * (s & 1) + e)) << 10) * 0x00010001u;                    \
        sp[s][e] = pk_mul(sp[s][e], mult);                 /* fp16 pair s * 2^(e0 - 2 sc) */                           \
        Blo[s][e] = pk_mul(qlo[s][e], sp[s][e]);                                                                       \
      }                                                                                                                \
    if (K4 > 0) {                                                                                                      \
    _Pragma("unroll")                                                                                                  \
      for (int e = 0; e < 4; ++e) {                                                                                    \
        const unsigned mult = ((unsigned)(15 + e0 - 2 * sc4(e)) << 10) * 0x00010001u;                                  \
        sp4[e] = pk_mul(sp4[e], mult);                                                                                 \
        Bh4[e] = pk_mul(qh4[e], sp4[e]);                                                                               \
      }                                                                                                                \
    }                                                                                                                  \
    if (role) {                                                                                                        \
    _Pragma("unroll")                                                                                                  \
      for (int s = 0; s < 2 * NU; ++s)                                                                                 \
    _Pragma("unroll")                                                                                                  \
        for (int e = 0; e < 4; ++e) Blo[s][e] = pk_fma_neg(qlo[s][e], sp[s][e], Blo[s][e]);                            \
      if (K4 > 0) {                                                                                                    \
    _Pragma("unroll")                                                                                                  \
        for (int e = 0; e < 4; ++e) Bh4[e] = pk_fma_neg(qh4[e], sp4[e], Bh4[e]);                                       \
      }                                                                                                                \
    }                                                                                                                  \
    /* logits in the log2 domain: x2 = S * C + Z * Cz */                                                               \
    Cz = ldexpf(scale_log2e, Eq);                                                                                      \
    C = ldexpf(scale_log2e, 24 - e0 + Eq);                                                                             \
    W = ldexpf(1.f, 24 - e0);                                                                                          \
    zc = zdot * Cz;                                                                                                    \
  }
#define MIXKVQ_KEY_TILES(X0, X1)                                                                         \
  {                                                                                                      \
    _Pragma("unroll")                                                                                    \
    for (int x = (X0); x < (X1); ++x) {                                                                  \
      const int tk = 64 * hsg + offx[x];                                                                 \
    _Pragma("unroll")                                                                                    \
      for (int u = 0; u < NU; ++u)                                                                       \
        wlo[u][x] = *reinterpret_cast<const unsigned*>(sK + lo_word_off[u][SWZ ? x : 0] + 4 * tk * T::Wlo); \
      if (K4 > 0) wh4[x] = *reinterpret_cast<const unsigned*>(sK + h4_word_off + 4 * tk * T::W4);        \
    }                                                                                                    \
    _Pragma("unroll")                                                                                    \
    for (int u = 0; u < NU; ++u) {                                                                       \
      u32x4 a0[4], a1[4];                                                                                \
    _Pragma("unroll")                                                                                    \
      for (int x = (X0); x < (X1); ++x) unpack2(wlo[u][x], a0[x], a1[x]);                                \
    _Pragma("unroll")                                                                                    \
      for (int x = (X0); x < (X1); ++x) S[x] = mfma(a0[x], Blo[2 * u], S[x]);                            \
    _Pragma("unroll")                                                                                    \
      for (int x = (X0); x < (X1); ++x) S[x] = mfma(a1[x], Blo[2 * u + 1], S[x]);                        \
    }                                                                                                    \
    if (K4 > 0) {                                                                                        \
    _Pragma("unroll")                                                                                    \
      for (int x = (X0); x < (X1); ++x) S[x] = mfma(unpack4(wh4[x]), Bh4, S[x]);                         \
    }                                                                                                    \
    if (K16 > 0) {                                                                                       \
      const u32x4 bqa = {q16a[0], q16a[1], q16a[2], q16a[3]}, bqb = {q16b[0], q16b[1], q16b[2], q16b[3]};   \
    _Pragma("unroll")                                                                                    \
      for (int x = (X0); x < (X1); ++x) {                                                                \
        const unsigned char* src = sK + k16_off + 2 * (64 * hsg + offx[x]) * K16;                        \
        const uint2 v0 = *reinterpret_cast<const uint2*>(src);                                           \
        const uint2 v1 = *reinterpret_cast<const uint2*>(src + 8);                                       \
        /* Entries beyond the tier meet zeros in the small operand; they are another token's finite */   \
        /* keys, except behind the last token of the plane (always in tile 3), where they are cleared */ \
        u32x4 a = {v0.x, v0.y, v1.x, v1.y};                                                              \
        if (x == 3 && K16 % 8 != 0) {                                                                    \
          a[0] = 8 * kg < K16 ? v0.x : 0u;                                                               \
          a[1] = 8 * kg + 2 < K16 ? v0.y : 0u;                                                           \
          a[2] = 8 * kg + 4 < K16 ? v1.x : 0u;                                                           \
          a[3] = 8 * kg + 6 < K16 ? v1.y : 0u;                                                           \
        }                                                                                                \
        /* tiles 0, 2 share one accumulator, tiles 1, 3 the other */                                     \
        S16[x & 1] = mfma(a, x < 2 ? bqa : bqb, S16[x & 1]);                                             \
      }                                                                                                  \
    }                                                                                                    \
  }

  MIXKVQ_PHASE(2)
  [[maybe_unused]] int phase_i = 3;
  [[maybe_unused]] int prio_iter = 0;
  for (; blk < blk_hi; blk += blk_step, ++prio_iter) {
    // ---- stage the key part and value metadata in LDS (wave-private: no barrier needed) ----
#pragma unroll
    for (int c = 0; c < NKL; ++c)
      if (MIXKVQ_IS_EARLY(c)) reinterpret_cast<u32x4*>(sK)[SWZ ? kst[c] : c * 64 + lane] = kreg[c];
#pragma unroll
    for (int c = 0; c < NVM; ++c) reinterpret_cast<u32x4*>(sVm)[c * 64 + lane < nvm ? c * 64 + lane : nvm - 1] = vmreg[c];
    wave_lds_handoff();
    const unsigned rec_nx = MIXKVQ_REC_INDEX(blk + blk_step, slot_nx);     // the next record of this wavefront
    if (blk + blk_step < blk_hi) MIXKVQ_ISSUE_K_EARLY(rec_nx)
    int slot_nn = 0;      // requested behind the record loads; needed only after they have arrived
    if (tab && blk + 2 * blk_step < blk_hi) slot_nn = tab[blk + 2 * blk_step];
    // Value scales above 255 (a group of values that spans more than 765) would overflow p' * s in fp16.  Such a
    // record (the record carries its largest value scale; wave-uniform, rare) is guarded: its scales are staged
    // 2^-kPBoost smaller, so its value products come out too small by that factor; the sums they join are taken
    // down by the same exact factor before the record and brought back after it.
    const bool big_s = (unsigned)__builtin_amdgcn_readfirstlane(
                           (int)reinterpret_cast<const unsigned short*>(sK + off_kmax)[cv.lay.NG]) > kBigScale;
    if (big_s) {
      constexpr unsigned kVsDown = ((unsigned)(15 - kPBoost) << 10) * 0x00010001u;   // fp16 pair (2^-kPBoost, same)
#pragma unroll
      for (int c = 0; c < NVM; ++c)
        if (c * 64 + lane < (nvm >> 1)) {     // the scales come first, then the zero-points
          u32x4 v = reinterpret_cast<const u32x4*>(sVm)[c * 64 + lane];
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = pk_mul(v[e], kVsDown);
          reinterpret_cast<u32x4*>(sVm)[c * 64 + lane] = v;
        }
#pragma unroll
      for (int xp = 0; xp < 2; ++xp)
#pragma unroll
        for (int qq = 0; qq < 4; ++qq) O[xp][qq] *= 1.f / (float)(1 << kPBoost);
      wave_lds_handoff();
    }

    // ---- channel selection of this block: rebuild q in slot order if it changed ----
    {
      bool rebuild = false;
      unsigned selw[kSelWords];
#pragma unroll
      for (int i = 0; i < kSelWords; ++i) {
        selw[i] = K4 + K16 > 0 ? __builtin_amdgcn_readfirstlane(reinterpret_cast<const unsigned*>(sK + off_idx)[i]) : 0u;
        rebuild |= selw[i] != sel_prev[i];
        sel_prev[i] = selw[i];
      }
      if (rebuild) MIXKVQ_REBUILD_Q(selw, false)
    }

    // operands that live across the super-groups of one key group
    u32x4 Blo[2 * NU], Bh4;
    float zdot = 0.f, C = 0.f, Cz = 0.f, zc = 0.f, W = 0.f;
#pragma unroll
    for (int hsg = 0; hsg < 2; ++hsg) {       // super-groups of 64 tokens
      if (RG && hsg == 1) {     // the pieces of the key part that only the second half needs
#pragma unroll
        for (int c = 0; c < NKL; ++c)
          if (!MIXKVQ_IS_EARLY(c)) reinterpret_cast<u32x4*>(sK)[SWZ ? kst[c] : c * 64 + lane] = kreg[c];
        wave_lds_handoff();
        if (blk + blk_step < blk_hi) MIXKVQ_ISSUE_K_LATE(rec_nx)
      }
      if (64 * hsg < R) {
        if (younger) {      // 5 of 8 half-records (measured: 4 of 8 nearly as good, 3 of 8 and 6 of 8 and more worse)
          if (hsg || (prio_iter & 3) == 0) __builtin_amdgcn_s_setprio(1);
          else __builtin_amdgcn_s_setprio(0);
        }
        // ---- S^T tiles: tile x holds tokens 64*hsg + tokbase(row) + offx[x] ----
        constexpr int offx[4] = {kOffx[0], kOffx[1], kOffx[2], kOffx[3]};
        unsigned wlo[NU][4], wh4[4];
        f32x4 S[4], S16[2];
#pragma unroll
        for (int x = 0; x < 4; ++x) S[x] = f32x4{0.f, 0.f, 0.f, 0.f};
        S16[0] = S16[1] = f32x4{0.f, 0.f, 0.f, 0.f};
        // logit constants of this lane's tiles.  With y the sum of the code products of a token (plus, with an
        // fp16 tier, its fp16 products brought to the same unit by the power of two Wx), the logit is
        // x = y * Mx + zcx with Mx > 0, so the maximum is taken over y and the subtraction of the running maximum is
        // folded into the constant of the fused multiply-add that feeds exp2.
        float Mx = 0.f, zcx = 0.f, Wx = 0.f;
        if (G32) {
          // two key groups per super-group: tiles 0, 1 with the first group's operands, tiles 2, 3 with the second's
          MIXKVQ_GROUP_OPERANDS(2 * hsg)
          MIXKVQ_KEY_TILES(0, 2)
          const float C0 = C, zc0 = zc, W0 = W;
          MIXKVQ_GROUP_OPERANDS(2 * hsg + 1)
          MIXKVQ_KEY_TILES(2, 4)
          Mx = K16 > 0 ? Cz : (role ? C : C0);      // lanes 0..7 of a row keep tiles 0, 1; lanes 8..15 tiles 2, 3
          zcx = role ? zc : zc0;
          Wx = role ? W : W0;
        } else {
          if ((64 * hsg) % Gk == 0) MIXKVQ_GROUP_OPERANDS((64 * hsg) / Gk)
          MIXKVQ_KEY_TILES(0, 4)
          Mx = K16 > 0 ? Cz : C;
          zcx = zc;
          Wx = W;
        }

        // ---- logits.  Only columns 0..7 carry heads, so two tiles share one register: lanes 0..7 of a
        // row of 16 keep tile 0 (resp. 1), lanes 8..15 take tile 2 (resp. 3).  ror8 adds head and tail. ----
        float ya[4], yb[4];     // packed: ya = tiles (0 | 2), yb = tiles (1 | 3)
        float ymax = -INFINITY;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float c0 = S[0][i] + row_ror8(S[0][i]), c2 = S[2][i] + row_ror8(S[2][i]);
          const float c1 = S[1][i] + row_ror8(S[1][i]), c3 = S[3][i] + row_ror8(S[3][i]);
          const float sa = role ? c2 : c0, sb = role ? c3 : c1;
          if (K16 > 0) {
            ya[i] = fmaf(sa, Wx, S16[0][i]);
            yb[i] = fmaf(sb, Wx, S16[1][i]);
          } else {
            ya[i] = sa;
            yb[i] = sb;
          }
          ymax = fmaxf(ymax, fmaxf(ya[i], yb[i]));
        }
        float mx = fmaf(ymax, Mx, zcx);
        if (RH && no_tokens) mx = -INFINITY;
        mx = xkg_max(mx);
        mx = fmaxf(mx, row_ror8(mx));
        const float m_new = fmaxf(m_run, mx);
        if (__builtin_amdgcn_readfirstlane((int)__any(m_new > m_run))) {
          const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);   // exp2(-inf) = 0 on the first block
          l_run *= alpha;
#pragma unroll
          for (int a = 0; a < NVG; ++a)
#pragma unroll
            for (int c = 0; c < 4; ++c) zacc[a][c] *= alpha;
#pragma unroll
          for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int c = 0; c < 4; ++c) O[a][c] *= alpha;
          m_run = m_new;
        }

        // ---- p in fp16 with the position factor 4^-sc of the value code it meets.  In lanes 0..7 pair i is
        // (token 2i, token 2i+1) of this lane group's 16 tokens = PV step 0; in lanes 8..15 it is (8+2i, 9+2i) = step 1.
        unsigned pk[4];
        const float zm = zcx - m_run;
        int role_here = role;
        if (kLeanConstants) asm volatile("" : "+v"(role_here));
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          float sc2f_i = sc2f[i];
          unsigned w4sc_i = w4sc[i];
          if (kLeanConstants) {      // formed here from an opaque copy of the lane's role (see kLeanConstants)
            const int sc_ = role_here ? sc2(4 + i) : i;
            sc2f_i = 2.f * sc_ - (float)kPBoost;
            w4sc_i = ((unsigned)(15 + 2 * sc_ - kPBoost) << 10) * 0x00010001u;
          }
          const float k = zm - sc2f_i;
          float ea = fmaf(ya[i], Mx, k), eb = fmaf(yb[i], Mx, k);
          if (RH && no_tokens) ea = eb = -INFINITY;
          pk[i] = cvt_pk(__builtin_amdgcn_exp2f(ea), __builtin_amdgcn_exp2f(eb));
          l_run = dot2(pk[i], w4sc_i, l_run);
        }
        // value scales / zero-points of the tokens this lane half pairs
        u32x4 Bp[NVG == 4 ? 2 : NVG][2];   // NVG = 4: the two value groups of one xp at a time
        {
          // the 8 tokens this lane half pairs: 16 kg + 8 role .. (G32: 32 role + 8 kg ..), pair i = tokens 2i, 2i + 1
          const int tv = 64 * hsg + (G32 ? 32 * role + 8 * kg : 16 * kgv + 8 * role);
          if (NVG == 1) {
            const uint4 sv = *reinterpret_cast<const uint4*>(sVm + 2 * tv);
            const uint4 zv = *reinterpret_cast<const uint4*>(sVm + 2 * R + 2 * tv);
            const unsigned sw[4] = {sv.x, sv.y, sv.z, sv.w}, zw[4] = {zv.x, zv.y, zv.z, zv.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              ps_operands(pk[i], sw[i], Bp[0][0], Bp[0][1], i);
              zacc[0][i] = dot2(pk[i], zw[i], zacc[0][i]);
            }
          } else if (NVG == 2) {
            // [token][2] layout: one dword per token, value group a in half a; tokens 8*role .. 8*role+7
            const uint4* ps = reinterpret_cast<const uint4*>(sVm + 4 * tv);
            const uint4* pz = reinterpret_cast<const uint4*>(sVm + 4 * R + 4 * tv);
            const uint4 s0 = ps[0], s1 = ps[1], z0 = pz[0], z1 = pz[1];
            const unsigned sw[8] = {s0.x, s0.y, s0.z, s0.w, s1.x, s1.y, s1.z, s1.w};
            const unsigned zw[8] = {z0.x, z0.y, z0.z, z0.w, z1.x, z1.y, z1.z, z1.w};
#pragma unroll
            for (int a = 0; a < NVG; ++a)
#pragma unroll
              for (int i = 0; i < 4; ++i) {
                const unsigned selb = a ? 0x07060302u : 0x05040100u;
                ps_operands(pk[i], __builtin_amdgcn_perm(sw[2 * i + 1], sw[2 * i], selb), Bp[a][0], Bp[a][1], i);
                zacc[a][i] = dot2(pk[i], __builtin_amdgcn_perm(zw[2 * i + 1], zw[2 * i], selb), zacc[a][i]);
              }
          }
        }

        // NVG = 4, [token][4] layout: 8 bytes per token, value groups (0, 1) in the first dword, (2, 3) in the second;
        // element i of s4 / z4 holds tokens 2i and 2i + 1 of this lane half
        uint4 s4[NVG == 4 ? 4 : 1], z4[NVG == 4 ? 4 : 1];
        if (NVG == 4) {
          const int tv = 64 * hsg + (G32 ? 32 * role + 8 * kg : 16 * kgv + 8 * role);
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            s4[i] = reinterpret_cast<const uint4*>(sVm + 8 * tv)[i];
            z4[i] = reinterpret_cast<const uint4*>(sVm + 8 * R + 8 * tv)[i];
          }
        }

        // ---- O^T += V_codes^T . Ps^T ----
#pragma unroll
        for (int xp = 0; xp < 2; ++xp) {
          const u32x4 vw = vreg[hsg][xp];
          if (NVG == 4) {      // small operands of value groups 2 xp and 2 xp + 1
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              const unsigned s_a = xp ? s4[i].y : s4[i].x, s_b = xp ? s4[i].w : s4[i].z;   // tokens 2i, 2i + 1
              const unsigned z_a = xp ? z4[i].y : z4[i].x, z_b = xp ? z4[i].w : z4[i].z;
#pragma unroll
              for (int cc = 0; cc < 2; ++cc) {
                const unsigned selb = cc ? 0x07060302u : 0x05040100u;
                ps_operands(pk[i], __builtin_amdgcn_perm(s_b, s_a, selb), Bp[cc][0], Bp[cc][1], i);
                zacc[2 * xp + cc][i] = dot2(pk[i], __builtin_amdgcn_perm(z_b, z_a, selb), zacc[2 * xp + cc][i]);
              }
            }
          }
#pragma unroll
          for (int qq = 0; qq < 4; ++qq) {
            const int a = NVG == 4 ? (qq >> 1) : value_group<NVG>(xp, qq);
            u32x4 a0, a1;
            unpack2(vw[qq], a0, a1);
            O[xp][qq] = mfma(a0, Bp[a][0], O[xp][qq]);
            O[xp][qq] = mfma(a1, Bp[a][1], O[xp][qq]);
          }
        }
        if (blk + blk_step < blk_hi) MIXKVQ_ISSUE_V_HALF(rec_nx, hsg)
      }
    }
    if (big_s) {
#pragma unroll
      for (int xp = 0; xp < 2; ++xp)
#pragma unroll
        for (int qq = 0; qq < 4; ++qq) O[xp][qq] *= (float)(1 << kPBoost);
    }
    slot_nx = slot_nn;
    MIXKVQ_PHASE(phase_i < 11 ? phase_i : 11)
    ++phase_i;
  }
  MIXKVQ_PHASE(14)
#undef MIXKVQ_ISSUE_K_EARLY
#undef MIXKVQ_ISSUE_K_LATE
#undef MIXKVQ_KOFF
#undef MIXKVQ_IS_EARLY
#undef MIXKVQ_REC
#undef MIXKVQ_REC_INDEX
#undef MIXKVQ_ISSUE_V_LOADS
#undef MIXKVQ_ISSUE_V_HALF
#undef MIXKVQ_LOAD_VWORDS
#undef MIXKVQ_REBUILD_Q
#undef MIXKVQ_BELOW
#undef MIXKVQ_GROUP_OPERANDS
#undef MIXKVQ_KEY_TILES

  // ---- wave results -> workgroup partial ------------------------------------------
  l_run = xkg_sum(l_run);
  l_run += row_ror8(l_run);          // the two lane halves hold different tokens of the same head
  float zsum[NVG];
#pragma unroll
  for (int a = 0; a < NVG; ++a) {
    float z = 0.f;
#pragma unroll
    for (int c = 0; c < 4; ++c) z = fmaf(zacc[a][c], __builtin_amdgcn_exp2f(sc2f[c]), z);
    z = xkg_sum(z);
    zsum[a] = z + row_ror8(z);
  }
  // each wavefront leaves its result in its own LDS region; after one barrier all threads merge the four
  // in a fixed order
  // columns 8..15 of the value products hold the part that came from the remainders of P*s
  f32x4 Ot[2][4];
#pragma unroll
  for (int xp = 0; xp < 2; ++xp)
#pragma unroll
    for (int qq = 0; qq < 4; ++qq)
#pragma unroll
      for (int i = 0; i < 4; ++i) Ot[xp][qq][i] = O[xp][qq][i] + row_ror8(O[xp][qq][i]);
  float* wO = reinterpret_cast<float*>(wbase);        // [8][128] O, then [8] l
  float* sM = reinterpret_cast<float*>(smem + 2048 + 64);          // [waves][8]
  if (role == 0 && live) {
#pragma unroll
    for (int xp = 0; xp < 2; ++xp)
#pragma unroll
      for (int qq = 0; qq < 4; ++qq)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int ch = value_channel<NVG>(xp, qq, 4 * kg + i);
          const int a = value_group<NVG>(xp, qq);
          wO[head * kD + ch] = fmaf(Ot[xp][qq][i], 16777216.f / (float)(1 << kPBoost), zsum[a]);
        }
    if (kg == 0) {
      wO[8 * kD + head] = l_run;
      sM[wave * 8 + head] = m_run;
    }
  }
  __syncthreads();
  // natural-log domain for the merge kernel: m_e = m2 * ln2
  float* out = part + ((size_t)p * n_splits + split) * g * kPartStrideM;
  const float* r0 = reinterpret_cast<const float*>(smem + kHdrLds);
  constexpr int kWaveF = kWaveLds / 4;
  for (int i = tid; i < g * (kD + 1); i += kMfmaThreads) {
    // elements g*kD .. are the l sums
    const int h = i < g * kD ? i / kD : i - g * kD;
    const int src = i < g * kD ? i : 8 * kD + h;
    float mw[kWaves], m_wg = -INFINITY;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      mw[w] = sM[w * 8 + h];
      m_wg = fmaxf(m_wg, mw[w]);
    }
    float acc = 0.f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w)
      acc += mw[w] == -INFINITY ? 0.f : r0[w * kWaveF + src] * __builtin_amdgcn_exp2f(mw[w] - m_wg);
    if (fin_out) {
      // the pair's only workgroup: the result is final (what the merge kernel would make of a single partial)
      float lw = 0.f;
#pragma unroll
      for (int w = 0; w < kWaves; ++w)
        lw += mw[w] == -INFINITY ? 0.f : r0[w * kWaveF + 8 * kD + h] * __builtin_amdgcn_exp2f(mw[w] - m_wg);
      const size_t bh = (size_t)b * Hq + (size_t)jkv * g + h;
      if (i < g * kD) {
        const float r = lw > 0.f ? acc / lw : 0.f;      // l == 0: a sequence without tokens
        reinterpret_cast<unsigned short*>(fin_out)[bh * kD + (i % kD)] =
            cv.cfg.in_dtype ? f32_to_bf16_bits(r) : __half_as_ushort(__float2half_rn(r));
      } else if (fin_lse) {
        fin_lse[bh] = lw > 0.f ? m_wg * 0.6931471805599453f + __logf(lw) : -INFINITY;
      }
    } else if (i < g * kD) {
      out[h * kPartStrideM + (i % kD)] = acc;
    } else {
      out[h * kPartStrideM + kD] = m_wg * 0.6931471805599453f;
      out[h * kPartStrideM + kD + 1] = acc;
    }
  }
  MIXKVQ_PHASE(15)
  MIXKVQ_PHASE_CYCLES(13)
}

// One launch per decode step: the workgroups (pair, split) share the pair's block records and its
// residual window.
template <int K4, int K16, int NVG, int NKL, int RG, int THR, int G32, int PG, int RH>
__global__ void __launch_bounds__(kMfmaThreads, 2)
decode_fused_kernel(CacheView cv, const __half* __restrict__ q, float scale, int n_blocks, int n_res, int n_splits,
                    float* __restrict__ part, int accumulate_q, NewToken nt, SeqCounts sc, __half* __restrict__ fin_out,
                    float* __restrict__ fin_lse) {
  extern __shared__ __align__(16) unsigned char smem[];
  mfma_part<K4, K16, NVG, NKL, RG, THR, G32, PG, RH>(cv, q, scale * 1.4426950408889634f, n_blocks, n_res, n_splits, part,
                                             accumulate_q, nt, sc, smem, fin_out, fin_lse);
}

template <int K4, int K16, int NVG, int NKL, int RG, int THR, int G32, int PG, int RH>
static hipError_t launch_one(const CacheView& v, const __half* q, float scale, int n_blocks, int n_res, int n_splits,
                             float* part, __half* out, float* lse, int accumulate_q, NewToken nt, const SeqCounts& sc,
                             hipStream_t s, hipEvent_t ev_start, hipEvent_t ev_stop) {
  auto kern = decode_fused_kernel<K4, K16, NVG, NKL, RG, THR, G32, PG, RH>;
  const size_t lds = kHdrLds + (size_t)kWaves * kWaveLds;
  // the kernel's LDS limit is raised once per device (a repeated call from another thread does no harm)
  static std::atomic<uint64_t> attr_set{0};
  int device = 0;
  if (hipError_t e = hipGetDevice(&device); e != hipSuccess) return e;
  const uint64_t bit = 1ull << (device & 63);
  if (!(attr_set.load(std::memory_order_acquire) & bit)) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_set.fetch_or(bit, std::memory_order_release);
  }
  // a pair with a single workgroup needs no merge: that workgroup writes the output itself
  __half* fin_out = n_splits == 1 ? out : nullptr;
  float* fin_lse = n_splits == 1 ? lse : nullptr;
  if (ev_start && ev_stop) {
    // profiling aid: the two events take the start and the end time of this kernel itself (not of the launch call)
    hipExtLaunchKernelGGL(kern, dim3(v.P, n_splits), dim3(kMfmaThreads), (uint32_t)lds, s, ev_start, ev_stop, 0u, v, q,
                          scale, n_blocks, n_res, n_splits, part, accumulate_q, nt, sc, fin_out, fin_lse);
  } else {
    kern<<<dim3(v.P, n_splits), dim3(kMfmaThreads), lds, s>>>(v, q, scale, n_blocks, n_res, n_splits, part, accumulate_q, nt, sc,
                                                             fin_out, fin_lse);
  }
  if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
  if (n_splits == 1) return hipSuccess;
  return launch_merge_pair(v, part, n_splits, out, lse, s);
}

}  // namespace mixkvq
