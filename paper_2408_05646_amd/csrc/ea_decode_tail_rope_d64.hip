// One-launch back half of a generation step, rotary form, d_head = 64 instantiations (a file of their own: they
// compile in parallel with the others).
#include "ea_decode_tail_dispatch.h"

namespace ea {

int decode_tail_rope_d64(int ks, int ncb, const DecodeArgs& a, const TailArgs& t, int32_t B, hipStream_t st) {
  return dispatch_ks_tail<2>(ks, ncb, a, t, B, st);
}

}  // namespace ea
