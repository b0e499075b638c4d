// Rotary generation-phase attention over a pruned cache (explicit positions), d_head = 64 instantiations.
#include "ea_decode_rope_dispatch.h"

namespace ea {

int decode_rope_pos_bf16_d64(int ks, int ncb, bool scores, const DecodeArgs& a, int32_t B, hipStream_t st) {
  return scores ? dispatch_ks_rope<2, true, true>(ks, ncb, a, B, st) : dispatch_ks_rope<2, false, true>(ks, ncb, a, B, st);
}

}  // namespace ea
