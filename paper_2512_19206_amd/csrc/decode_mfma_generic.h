// Wider tables of matrix-core variants: every tier combination below for the usual group sizes, so that a
// configuration outside the measured ones does not fall onto the vector-ALU kernel.  These variants take both the
// contiguous and the paged layout (PG = 2) and no compile-time R; each table is a translation unit of its own.
#pragma once
#include "decode_mfma_kernel.h"

namespace mixkvq {

// (k4, k16, policy): budgets of the top-k policy, capacities of the threshold policy
#define MIXKVQ_TIER_LIST(X)                                                                                   \
  X(0, 0, 0) X(8, 0, 0) X(16, 0, 0) X(24, 0, 0) X(32, 0, 0) X(0, 4, 0) X(0, 8, 0) X(0, 12, 0) X(0, 16, 0)      \
  X(0, 24, 0) X(0, 32, 0) X(8, 4, 0) X(8, 8, 0) X(16, 4, 0) X(16, 8, 0)                                        \
  X(8, 0, 1) X(16, 0, 1) X(0, 8, 1) X(0, 12, 1) X(0, 16, 1) X(8, 4, 1) X(16, 8, 1) X(16, 16, 1)

constexpr int al16c(int n) { return (n + 15) / 16 * 16; }
// 1-KiB pieces of the key part of a record of R tokens with NG key groups (the layout of mixkvq_block_layout)
constexpr int key_part_kib(int K4, int K16, int THR, int NG, int R) {
  const int ks = K4 + K16, NL = THR ? kD : kD - ks, Wlo = (NL + 15) / 16, NLp = 16 * Wlo;
  const int off_v = al16c(ks) + al16c((NG + 1) * 2) + 2 * al16c(NG * NLp * 2) + 2 * al16c(NG * K4 * 2) +
                    al16c(R * Wlo * 4) + al16c(R * (K4 / 8) * 4) + al16c(R * K16 * 2);
  return (off_v / 16 + 63) / 64;
}

struct GenericArgs {
  const CacheView& v;
  const __half* q;
  float scale;
  int n_blocks, n_res, n_splits;
  float* part;
  __half* out;
  float* lse;
  int accumulate_q;
  NewToken nt;
  const SeqCounts& sc;
  hipStream_t s;
  hipEvent_t ev_start, ev_stop;
  int nkl, g32, rh;     // of the cache: 1-KiB pieces of its key part, key groups of 32 tokens, records of 32 tokens
};

// Launches the variant <K4, K16, NVG, THR, G32, RH> if the cache is of that kind.  NG: the most key groups a
// record of that kind has (it sizes the staging loop).
template <int K4, int K16, int NVG, int THR, int G32, int RH>
static bool try_generic(const GenericArgs& a, hipError_t* err) {
  constexpr int NKL = key_part_kib(K4, K16, THR, G32 ? 4 : (RH ? 1 : 2), RH ? 32 : 128);
  if constexpr (NKL * 1024 <= kKPartMax) {
    const mixkvq_config& c = a.v.cfg;
    if (c.k4 == K4 && c.k16 == K16 && a.v.lay.NVG == NVG && c.policy == THR && a.g32 == G32 && a.rh == RH && a.nkl <= NKL) {
      *err = launch_one<K4, K16, NVG, NKL, 0, THR, G32, 2, RH>(a.v, a.q, a.scale, a.n_blocks, a.n_res, a.n_splits, a.part,
                                                              a.out, a.lse, a.accumulate_q, a.nt, a.sc, a.s, a.ev_start,
                                                              a.ev_stop);
      return true;
    }
  }
  return false;
}

bool try_launch_generic_plain(const GenericArgs& a, hipError_t* err);      // key groups of 64 or 128 tokens
bool try_launch_generic_g32(const GenericArgs& a, hipError_t* err);        // key groups of 32 tokens
bool try_launch_generic_rh(const GenericArgs& a, hipError_t* err);         // records of 32 tokens

}  // namespace mixkvq
