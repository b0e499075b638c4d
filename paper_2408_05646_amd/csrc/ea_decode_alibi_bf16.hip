// Launch side of the generation-phase attention kernel with the ALiBi position bias (the MPT family's scheme:
// every score gets -slope_h times the distance of its key to the query).
#include "ea_decode_kernel.h"

namespace ea {

template <int KS, int NCB>
static void launch_decode_alibi(const DecodeArgs& a, int32_t B, hipStream_t st) {
  dim3 grid(a.g.n_kv_heads, a.n_splits, B), block(256);
  constexpr int TBN = (KS * 4 + NCB * 2 > 22) ? 2 : 4;
  decode_bf16_kernel<KS, NCB, TBN, 2, 0, true><<<grid, block, 0, st>>>(a);
}

template <int KS>
static int dispatch_ncb_alibi(int ncb, const DecodeArgs& a, int32_t B, hipStream_t st) {
  switch (ncb) {
    case 1: launch_decode_alibi<KS, 1>(a, B, st); break;
    case 2: launch_decode_alibi<KS, 2>(a, B, st); break;
    case 3: launch_decode_alibi<KS, 3>(a, B, st); break;
    case 4: launch_decode_alibi<KS, 4>(a, B, st); break;
    case 5: launch_decode_alibi<KS, 5>(a, B, st); break;
    case 6: launch_decode_alibi<KS, 6>(a, B, st); break;
    case 7: launch_decode_alibi<KS, 7>(a, B, st); break;
    case 8: launch_decode_alibi<KS, 8>(a, B, st); break;
    default: return EA_ERR_SHAPE;
  }
  return launch_status();
}

int decode_alibi_bf16(const ea_layer_desc* d, const Geo& g, const float* q, const float* slopes, const void* k_pool,
                      const void* v_pool, const int32_t* page_table, const int32_t* seq_len, float* out, int32_t B,
                      int32_t n_splits, float* ws, hipStream_t st, int32_t seq_add, int32_t out_bf16) {
  if (B > 65535 || g.n_kv_heads > 65535) return EA_ERR_SHAPE;
  DecodeArgs a;
  a.q = q;
  a.k_pool = (const uint16_t*)k_pool;
  a.v_pool = (const uint16_t*)v_pool;
  a.page_table = page_table;
  a.seq_len = seq_len;
  a.out = out;
  a.ws = ws;
  a.g = g;
  a.n_splits = n_splits;
  a.scale_log2 = 1.4426950408889634f / sqrtf((float)d->d_head);
  a.u_k = nullptr;
  a.d_head = d->d_head;
  a.log2_base = 0.0;
  a.alibi = slopes;
  a.seq_add = seq_add;
  a.out_bf16 = out_bf16;
  const int ks = (g.r_k_pad + 31) / 32, ncb = g.r_v_pad / 16;
  switch (ks) {
    case 1: return dispatch_ncb_alibi<1>(ncb, a, B, st);
    case 2: return dispatch_ncb_alibi<2>(ncb, a, B, st);
    case 3: return dispatch_ncb_alibi<3>(ncb, a, B, st);
    case 4: return dispatch_ncb_alibi<4>(ncb, a, B, st);
    default: return EA_ERR_SHAPE;
  }
}

}  // namespace ea
