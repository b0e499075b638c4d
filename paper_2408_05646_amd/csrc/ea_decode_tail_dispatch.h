// Template dispatch of the one-launch back half of a generation step over the (r_k, r_v) register shapes.
#pragma once
#include "ea_decode_tail.h"

namespace ea {

// NKK = 0: position-free form; NKK = d_head / 32: rotary form (half-tile iterations, as the rotary kernel alone).
template <int KS, int NCB, int NKK>
static void launch_tail(const DecodeArgs& a, const TailArgs& t, int32_t B, hipStream_t st) {
  dim3 grid(a.g.n_kv_heads, a.n_splits, B), block(256);
  constexpr int TBN = NKK > 0 ? 2 : ((KS * 4 + NCB * 2 > 22) ? 2 : 4);
  decode_layer_back_kernel<KS, NCB, TBN, NKK><<<grid, block, 0, st>>>(a, t);
}

template <int KS, int NKK>
static int dispatch_ncb_tail(int ncb, const DecodeArgs& a, const TailArgs& t, int32_t B, hipStream_t st) {
  switch (ncb) {
    case 1: launch_tail<KS, 1, NKK>(a, t, B, st); break;
    case 2: launch_tail<KS, 2, NKK>(a, t, B, st); break;
    case 3: launch_tail<KS, 3, NKK>(a, t, B, st); break;
    case 4: launch_tail<KS, 4, NKK>(a, t, B, st); break;
    case 5: launch_tail<KS, 5, NKK>(a, t, B, st); break;
    case 6: launch_tail<KS, 6, NKK>(a, t, B, st); break;
    case 7: launch_tail<KS, 7, NKK>(a, t, B, st); break;
    case 8: launch_tail<KS, 8, NKK>(a, t, B, st); break;
    default: return EA_ERR_SHAPE;
  }
  return launch_status();
}

template <int NKK>
static int dispatch_ks_tail(int ks, int ncb, const DecodeArgs& a, const TailArgs& t, int32_t B, hipStream_t st) {
  switch (ks) {
    case 1: return dispatch_ncb_tail<1, NKK>(ncb, a, t, B, st);
    case 2: return dispatch_ncb_tail<2, NKK>(ncb, a, t, B, st);
    case 3: return dispatch_ncb_tail<3, NKK>(ncb, a, t, B, st);
    case 4: return dispatch_ncb_tail<4, NKK>(ncb, a, t, B, st);
    default: return EA_ERR_SHAPE;
  }
}

}  // namespace ea
