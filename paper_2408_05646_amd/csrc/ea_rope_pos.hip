// Rotary models after token pruning (results, "Eigen Attention with token pruning"; the paper's table is on Llama
// models, whose attention is the form of Sec. 4.3, Eq. 10): a token that stays in the cache keeps the position it
// had in the text, so the position of the key in cache slot t comes from an array instead of being t.  The cache
// itself does not change -- it holds rank-r keys that were never rotated -- so a freed slot is simply overwritten
// by ea_project_qkv_rope and the caller updates the slot's position.
//
//   ea_decode_attn_rope_pos        ea_decode_attn_rope with explicit positions
//   ea_decode_attn_mass_rope_pos   the same, and the attention probability every slot received is added to the
//                                  caller's accumulator (what an H2O-style policy ranks tokens by)
#include "ea_decode_kernel.h"

namespace ea {

int decode_rope_pos_bf16_d64(int ks, int ncb, bool scores, const DecodeArgs& a, int32_t B, hipStream_t st);
int decode_rope_pos_bf16_d128(int ks, int ncb, const DecodeArgs& a, int32_t B, hipStream_t st);
int decode_rope_pos_scores_bf16_d128(int ks, int ncb, const DecodeArgs& a, int32_t B, hipStream_t st);
int decode_rope_pos_f32(const ea_layer_desc* d, const Geo& g, const float* q, const float* u_k, double rope_base,
                        const float* k_pool, const float* v_pool, const int32_t* page_table, const int32_t* seq_len,
                        const int32_t* slot_pos, int32_t pos_stride, const int32_t* q_pos, float* out, int32_t B,
                        int32_t n_splits, float* ws, hipStream_t st);

// scores != nullptr: the score-storing form, which always leaves split partials for the merge
static int decode_rope_pos_bf16(const ea_layer_desc* d, const Geo& g, const float* q, const void* u_k, double rope_base,
                                const void* k_pool, const void* v_pool, const int32_t* page_table,
                                const int32_t* seq_len, const int32_t* slot_pos, int32_t pos_stride,
                                const int32_t* q_pos, float* out, int32_t B, int32_t n_splits, float* ws, float* scores,
                                int32_t s_row, hipStream_t st) {
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
  a.u_k = (const uint16_t*)u_k;
  a.d_head = d->d_head;
  a.alibi = nullptr;
  a.log2_base = log2(rope_base);
  a.slot_pos = slot_pos;
  a.q_pos = q_pos;
  a.pos_stride = pos_stride;
  if (scores) {
    a.ws_slots = n_splits;
    a.ws_slot0 = 0;
    a.scores = scores;
    a.s_row = s_row;
  }
  const int ks = (g.r_k_pad + 31) / 32, ncb = g.r_v_pad / 16;
  if (d->d_head == 64) return decode_rope_pos_bf16_d64(ks, ncb, scores != nullptr, a, B, st);
  return scores ? decode_rope_pos_scores_bf16_d128(ks, ncb, a, B, st) : decode_rope_pos_bf16_d128(ks, ncb, a, B, st);
}

static int check_rope_pos_args(const ea_layer_desc* desc, const void* dev_q, const void* dev_u_k, double rope_base,
                               const void* dev_k_pool, const void* dev_v_pool, const int32_t* dev_page_table,
                               const int32_t* dev_seq_len, const int32_t* dev_slot_pos, int32_t pos_stride,
                               const int32_t* dev_q_pos, const float* dev_out, int32_t B, int32_t max_pages,
                               int32_t pool_pages, int32_t n_splits) {
  const int rc = validate_desc(desc);
  if (rc != EA_OK) return rc;
  if (!dev_q || !dev_u_k || !dev_k_pool || !dev_v_pool || !dev_page_table || !dev_seq_len || !dev_slot_pos ||
      !dev_q_pos || !dev_out)
    return EA_ERR_ARG;
  if (B <= 0 || max_pages <= 0 || pool_pages <= 0 || n_splits < 0 || n_splits > 1024) return EA_ERR_ARG;
  if (!(rope_base > 1.0) || !(rope_base < 1e30)) return EA_ERR_ARG;
  // the kernels read the positions of whole 64-token tiles, up to the capacity of the page table
  if ((int64_t)pos_stride < (int64_t)max_pages * desc->page_tokens) return EA_ERR_ARG;
  if (desc->r_k > desc->d_head) return EA_ERR_SHAPE;
  if (desc->dtype == EA_BF16 ? (desc->d_head != 64 && desc->d_head != 128)
                             : (desc->d_head % 2 != 0 || desc->d_head > 256))
    return EA_ERR_SHAPE;
  if (!aligned16(dev_q) || !aligned16(dev_u_k) || !aligned16(dev_k_pool) || !aligned16(dev_v_pool) ||
      !aligned16(dev_out) || (reinterpret_cast<uintptr_t>(dev_slot_pos) & 3u) || (reinterpret_cast<uintptr_t>(dev_q_pos) & 3u))
    return EA_ERR_ALIGN;
  return EA_OK;
}

}  // namespace ea

using namespace ea;

extern "C" {

int ea_decode_attn_rope_pos(const ea_layer_desc* desc, const float* dev_q, const void* dev_u_k, double rope_base,
                            const void* dev_k_pool, const void* dev_v_pool, const int32_t* dev_page_table,
                            const int32_t* dev_seq_len, const int32_t* dev_slot_pos, int32_t pos_stride,
                            const int32_t* dev_q_pos, float* dev_out, int32_t B, int32_t max_pages, int32_t pool_pages,
                            int32_t n_splits, void* dev_ws, int64_t ws_bytes, void* stream) {
  int rc = check_rope_pos_args(desc, dev_q, dev_u_k, rope_base, dev_k_pool, dev_v_pool, dev_page_table, dev_seq_len,
                               dev_slot_pos, pos_stride, dev_q_pos, dev_out, B, max_pages, pool_pages, n_splits);
  if (rc != EA_OK) return rc;
  if (n_splits == 0) {
    const int64_t cap_tokens = (int64_t)max_pages * desc->page_tokens;
    n_splits = ea_decode_rope_auto_splits(desc, B, cap_tokens > INT32_MAX ? INT32_MAX : (int32_t)cap_tokens);
  }
  if (n_splits > 1) {
    if (!dev_ws || !aligned16(dev_ws)) return EA_ERR_WORKSPACE;
    if (ws_bytes < ea_decode_workspace_bytes(desc, B, n_splits)) return EA_ERR_WORKSPACE;
  }
  const Geo g = make_geo(desc, max_pages, pool_pages);
  hipStream_t st = (hipStream_t)stream;
  clear_stale_error();
  if (desc->dtype == EA_BF16)
    rc = decode_rope_pos_bf16(desc, g, dev_q, dev_u_k, rope_base, dev_k_pool, dev_v_pool, dev_page_table, dev_seq_len,
                              dev_slot_pos, pos_stride, dev_q_pos, dev_out, B, n_splits, (float*)dev_ws, nullptr, 0, st);
  else
    rc = decode_rope_pos_f32(desc, g, dev_q, (const float*)dev_u_k, rope_base, (const float*)dev_k_pool,
                             (const float*)dev_v_pool, dev_page_table, dev_seq_len, dev_slot_pos, pos_stride, dev_q_pos,
                             dev_out, B, n_splits, (float*)dev_ws, st);
  if (rc != EA_OK) return rc;
  if (n_splits > 1) rc = merge_splits(g, (const float*)dev_ws, dev_out, B, n_splits, st);
  return rc;
}

int ea_decode_attn_mass_rope_pos(const ea_layer_desc* desc, const float* dev_q, const void* dev_u_k, double rope_base,
                                 const void* dev_k_pool, const void* dev_v_pool, const int32_t* dev_page_table,
                                 const int32_t* dev_seq_len, const int32_t* dev_slot_pos, int32_t pos_stride,
                                 const int32_t* dev_q_pos, float* dev_out, float* dev_mass, int32_t B,
                                 int32_t max_pages, int32_t pool_pages, int32_t n_splits, void* dev_ws,
                                 int64_t ws_bytes, void* stream) {
  int rc = check_rope_pos_args(desc, dev_q, dev_u_k, rope_base, dev_k_pool, dev_v_pool, dev_page_table, dev_seq_len,
                               dev_slot_pos, pos_stride, dev_q_pos, dev_out, B, max_pages, pool_pages, n_splits);
  if (rc != EA_OK) return rc;
  if (!dev_mass) return EA_ERR_ARG;
  if (!aligned16(dev_mass)) return EA_ERR_ALIGN;
  if (desc->dtype != EA_BF16) return EA_ERR_SHAPE;
  const int64_t n_cap64 = (int64_t)max_pages * desc->page_tokens;
  if (n_cap64 > (int64_t)INT32_MAX - 2048) return EA_ERR_SHAPE;
  if (n_splits == 0) n_splits = ea_decode_rope_auto_splits(desc, B, (int32_t)n_cap64);
  if (!dev_ws || !aligned16(dev_ws) || ws_bytes < ea_decode_attn_mass_workspace_bytes(desc, B, max_pages, n_splits))
    return EA_ERR_WORKSPACE;
  const Geo g = make_geo(desc, max_pages, pool_pages);
  if (g.group > 16) return EA_ERR_SHAPE;
  const int32_t n_cap = (int32_t)n_cap64;
  const int32_t s_row = (int32_t)mass_row_floats(n_cap);
  float* partials = (float*)dev_ws;
  float* scores = partials + (ws_floats(B, g.n_heads, n_splits, g.r_v_pad) + 3) / 4 * 4;
  float* ml = scores + (int64_t)B * g.n_heads * s_row;
  hipStream_t st = (hipStream_t)stream;
  clear_stale_error();
  rc = decode_rope_pos_bf16(desc, g, dev_q, dev_u_k, rope_base, dev_k_pool, dev_v_pool, dev_page_table, dev_seq_len,
                            dev_slot_pos, pos_stride, dev_q_pos, nullptr, B, n_splits, partials, scores, s_row, st);
  if (rc != EA_OK) return rc;
  rc = merge_splits(g, partials, dev_out, B, n_splits, st, ml);
  if (rc != EA_OK) return rc;
  return mass_from_scores(g, scores, ml, dev_seq_len, dev_mass, B, n_cap, s_row, st);
}

}  // extern "C"
