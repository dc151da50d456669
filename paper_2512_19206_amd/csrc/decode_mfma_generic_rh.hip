// Matrix-core variants for records of 32 tokens (R = 32, or R = 96 stored as three records) and value groups of
// 32, 128 or 64 channels.
#include "decode_mfma_generic.h"

namespace mixkvq {

bool try_launch_generic_rh(const GenericArgs& a, hipError_t* err) {
#define MIXKVQ_X(K4_, K16_, THR_) \
  if (try_generic<K4_, K16_, 4, THR_, 0, 1>(a, err) || try_generic<K4_, K16_, 1, THR_, 0, 1>(a, err) ||  \
      try_generic<K4_, K16_, 2, THR_, 0, 1>(a, err))                                                          \
    return true;
  MIXKVQ_TIER_LIST(MIXKVQ_X)
#undef MIXKVQ_X
  return false;
}

}  // namespace mixkvq
