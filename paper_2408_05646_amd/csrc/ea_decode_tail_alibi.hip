// Launch side of the one-launch back half of a generation step, ALiBi form (the MPT family of Sec. 5.1).
#include "ea_decode_tail_dispatch.h"

namespace ea {

int decode_tail_alibi(int ks, int ncb, const DecodeArgs& a, const TailArgs& t, int32_t B, hipStream_t st) {
  return dispatch_ks_tail<0, true>(ks, ncb, a, t, B, st);
}

}  // namespace ea
