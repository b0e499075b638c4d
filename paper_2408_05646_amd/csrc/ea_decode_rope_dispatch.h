// Template dispatch of the rotary generation-phase kernel over (r_k, r_v) register shapes.
#pragma once
#include "ea_decode_kernel.h"

namespace ea {

// SCORES / POS: the form that also stores its scores / takes the position of every cached token from an array.
template <int KS, int NCB, int NKK, bool SCORES, bool POS>
static void launch_decode_rope(const DecodeArgs& a, int32_t B, hipStream_t st) {
  dim3 grid(a.g.n_kv_heads, a.n_splits, B), block(256);
  // half-tile iterations keep the kernel within 256 registers, so two workgroups share a compute unit
  decode_bf16_kernel<KS, NCB, 2, 2, NKK, false, SCORES, POS><<<grid, block, 0, st>>>(a);
}

template <int KS, int NKK, bool SCORES, bool POS>
static int dispatch_ncb_rope(int ncb, const DecodeArgs& a, int32_t B, hipStream_t st) {
  switch (ncb) {
    case 1: launch_decode_rope<KS, 1, NKK, SCORES, POS>(a, B, st); break;
    case 2: launch_decode_rope<KS, 2, NKK, SCORES, POS>(a, B, st); break;
    case 3: launch_decode_rope<KS, 3, NKK, SCORES, POS>(a, B, st); break;
    case 4: launch_decode_rope<KS, 4, NKK, SCORES, POS>(a, B, st); break;
    case 5: launch_decode_rope<KS, 5, NKK, SCORES, POS>(a, B, st); break;
    case 6: launch_decode_rope<KS, 6, NKK, SCORES, POS>(a, B, st); break;
    case 7: launch_decode_rope<KS, 7, NKK, SCORES, POS>(a, B, st); break;
    case 8: launch_decode_rope<KS, 8, NKK, SCORES, POS>(a, B, st); break;
    default: return EA_ERR_SHAPE;
  }
  return launch_status();
}

template <int NKK, bool SCORES = false, bool POS = false>
static int dispatch_ks_rope(int ks, int ncb, const DecodeArgs& a, int32_t B, hipStream_t st) {
  switch (ks) {
    case 1: return dispatch_ncb_rope<1, NKK, SCORES, POS>(ncb, a, B, st);
    case 2: return dispatch_ncb_rope<2, NKK, SCORES, POS>(ncb, a, B, st);
    case 3: return dispatch_ncb_rope<3, NKK, SCORES, POS>(ncb, a, B, st);
    case 4: return dispatch_ncb_rope<4, NKK, SCORES, POS>(ncb, a, B, st);
    default: return EA_ERR_SHAPE;
  }
}

}  // namespace ea
