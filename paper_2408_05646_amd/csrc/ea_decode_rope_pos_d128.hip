// Rotary generation-phase attention over a pruned cache (explicit positions), d_head = 128 instantiations.
#include "ea_decode_rope_dispatch.h"

namespace ea {

int decode_rope_pos_bf16_d128(int ks, int ncb, const DecodeArgs& a, int32_t B, hipStream_t st) {
  return dispatch_ks_rope<4, false, true>(ks, ncb, a, B, st);
}

}  // namespace ea
