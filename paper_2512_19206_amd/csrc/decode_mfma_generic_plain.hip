// Matrix-core variants for key groups of 64 or 128 tokens and value groups of 128, 64 or 32 channels.
#include "decode_mfma_generic.h"

namespace mixkvq {

bool try_launch_generic_plain(const GenericArgs& a, hipError_t* err) {
#define MIXKVQ_X(K4_, K16_, THR_) \
  if (try_generic<K4_, K16_, 1, THR_, 0, 0>(a, err) || try_generic<K4_, K16_, 2, THR_, 0, 0>(a, err) ||  \
      try_generic<K4_, K16_, 4, THR_, 0, 0>(a, err))                                                          \
    return true;
  MIXKVQ_TIER_LIST(MIXKVQ_X)
#undef MIXKVQ_X
  return false;
}

}  // namespace mixkvq
