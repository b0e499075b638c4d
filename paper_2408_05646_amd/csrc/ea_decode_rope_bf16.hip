// Launch side of the generation-phase attention kernel for models with rotary position embedding
// (Sec. 4.3, Eq. 10): full-rank query, rank-r cached keys brought back to d_head channels tile by tile.
#include "ea_decode_rope_dispatch.h"

namespace ea {

int decode_rope_bf16_d128(int ks, int ncb, const DecodeArgs& a, int32_t B, hipStream_t st);   // in its own file

int decode_rope_bf16(const ea_layer_desc* d, const Geo& g, const float* q, const void* u_k, double rope_base,
                     const void* k_pool, const void* v_pool, const int32_t* page_table, const int32_t* seq_len,
                     float* out, int32_t B, int32_t n_splits, float* ws, hipStream_t st, int32_t ws_slots,
                     int32_t ws_slot0, int32_t seq_add, int32_t out_bf16) {
  if (B > 65535 || g.n_kv_heads > 65535) return EA_ERR_SHAPE;
  if (d->d_head != 64 && d->d_head != 128) return EA_ERR_SHAPE;
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
  a.u_k = (const uint16_t*)u_k;
  a.d_head = d->d_head;
  a.alibi = nullptr;
  a.log2_base = log2(rope_base);
  a.ws_slots = ws_slots;
  a.ws_slot0 = ws_slot0;
  a.seq_add = seq_add;
  a.out_bf16 = out_bf16;
  const int ks = (g.r_k_pad + 31) / 32, ncb = g.r_v_pad / 16;
  if (d->d_head == 128) return decode_rope_bf16_d128(ks, ncb, a, B, st);
  return dispatch_ks_rope<2>(ks, ncb, a, B, st);
}

}  // namespace ea
