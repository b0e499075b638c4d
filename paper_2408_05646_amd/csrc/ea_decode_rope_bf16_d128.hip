// Rotary generation-phase attention, d_head = 128 instantiations (a file of their own: they compile in parallel
// with the d_head = 64 ones).
#include "ea_decode_rope_dispatch.h"

namespace ea {

int decode_rope_bf16_d128(int ks, int ncb, const DecodeArgs& a, int32_t B, hipStream_t st) {
  return dispatch_ks_rope<4>(ks, ncb, a, B, st);
}

}  // namespace ea
