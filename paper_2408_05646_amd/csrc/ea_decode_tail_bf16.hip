// Launch side of the one-launch back half of a generation step (attention, split merge, output projection),
// position-free form.
#include "ea_decode_tail_dispatch.h"

namespace ea {

int decode_tail_rope_d64(int ks, int ncb, const DecodeArgs& a, const TailArgs& t, int32_t B, hipStream_t st);
int decode_tail_rope_d128(int ks, int ncb, const DecodeArgs& a, const TailArgs& t, int32_t B, hipStream_t st);
int decode_tail_alibi(int ks, int ncb, const DecodeArgs& a, const TailArgs& t, int32_t B, hipStream_t st);

int decode_tail_bf16(const ea_layer_desc* d, const Geo& g, const float* q, const void* u_k, double rope_base,
                     const void* k_pool, const void* v_pool, const int32_t* page_table, const int32_t* seq_len,
                     int32_t B, int32_t n_splits, float* ws, int32_t seq_add, const TailArgs& t, hipStream_t st,
                     const float* slopes) {
  if (B > 16 || g.n_kv_heads > 65535) return EA_ERR_SHAPE;
  const bool rope = u_k != nullptr;
  if (rope && slopes) return EA_ERR_ARG;
  if (rope && d->d_head != 64 && d->d_head != 128) return EA_ERR_SHAPE;
  DecodeArgs a;
  a.q = q;
  a.k_pool = (const uint16_t*)k_pool;
  a.v_pool = (const uint16_t*)v_pool;
  a.page_table = page_table;
  a.seq_len = seq_len;
  a.out = nullptr;
  a.ws = ws;
  a.g = g;
  a.n_splits = n_splits;
  a.scale_log2 = 1.4426950408889634f / sqrtf((float)d->d_head);
  a.u_k = (const uint16_t*)u_k;
  a.d_head = d->d_head;
  a.alibi = slopes;
  a.log2_base = rope ? log2(rope_base) : 0.0;
  a.seq_add = seq_add;
  const int ks = (g.r_k_pad + 31) / 32, ncb = g.r_v_pad / 16;
  if (slopes) return decode_tail_alibi(ks, ncb, a, t, B, st);
  if (!rope) return dispatch_ks_tail<0>(ks, ncb, a, t, B, st);
  if (d->d_head == 128) return decode_tail_rope_d128(ks, ncb, a, t, B, st);
  return decode_tail_rope_d64(ks, ncb, a, t, B, st);
}

}  // namespace ea
