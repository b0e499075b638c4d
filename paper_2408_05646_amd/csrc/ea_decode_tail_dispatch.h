// Template dispatch of the one-launch back half of a generation step over the (r_k, r_v) register shapes.
#pragma once
#include "ea_decode_tail.h"

namespace ea {

// NKK = 0: position-free form (ALIBI: with the per-head distance bias); NKK = d_head / 32: rotary form (half-tile
// iterations, as the rotary kernel alone).
template <int KS, int NCB, int NKK, bool ALIBI>
static void launch_tail(const DecodeArgs& a, const TailArgs& t, int32_t B, hipStream_t st) {
  dim3 grid(a.g.n_kv_heads, a.n_splits, B), block(256);
  constexpr int TBN = NKK > 0 ? 2 : ((KS * 4 + NCB * 2 > 22) ? 2 : 4);
  decode_layer_back_kernel<KS, NCB, TBN, NKK, ALIBI><<<grid, block, 0, st>>>(a, t);
}

template <int KS, int NKK, bool ALIBI>
static int dispatch_ncb_tail(int ncb, const DecodeArgs& a, const TailArgs& t, int32_t B, hipStream_t st) {
  switch (ncb) {
    case 1: launch_tail<KS, 1, NKK, ALIBI>(a, t, B, st); break;
    case 2: launch_tail<KS, 2, NKK, ALIBI>(a, t, B, st); break;
    case 3: launch_tail<KS, 3, NKK, ALIBI>(a, t, B, st); break;
    case 4: launch_tail<KS, 4, NKK, ALIBI>(a, t, B, st); break;
    case 5: launch_tail<KS, 5, NKK, ALIBI>(a, t, B, st); break;
    case 6: launch_tail<KS, 6, NKK, ALIBI>(a, t, B, st); break;
    case 7: launch_tail<KS, 7, NKK, ALIBI>(a, t, B, st); break;
    case 8: launch_tail<KS, 8, NKK, ALIBI>(a, t, B, st); break;
    default: return EA_ERR_SHAPE;
  }
  return launch_status();
}

template <int NKK, bool ALIBI = false>
static int dispatch_ks_tail(int ks, int ncb, const DecodeArgs& a, const TailArgs& t, int32_t B, hipStream_t st) {
  switch (ks) {
    case 1: return dispatch_ncb_tail<1, NKK, ALIBI>(ncb, a, t, B, st);
    case 2: return dispatch_ncb_tail<2, NKK, ALIBI>(ncb, a, t, B, st);
    case 3: return dispatch_ncb_tail<3, NKK, ALIBI>(ncb, a, t, B, st);
    case 4: return dispatch_ncb_tail<4, NKK, ALIBI>(ncb, a, t, B, st);
    default: return EA_ERR_SHAPE;
  }
}

}  // namespace ea
