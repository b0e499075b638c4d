// Rotary generation-phase attention over a pruned cache (explicit positions) in the form that also stores its
// scores, d_head = 128 instantiations.
#include "ea_decode_rope_dispatch.h"

namespace ea {

int decode_rope_pos_scores_bf16_d128(int ks, int ncb, const DecodeArgs& a, int32_t B, hipStream_t st) {
  return dispatch_ks_rope<4, true, true>(ks, ncb, a, B, st);
}

}  // namespace ea
