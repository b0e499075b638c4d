// C ABI of the 4-bit group-quantised cache: layout reference functions, page quantisation, attention.
#include "ea_q4.h"
#include "ea_prefill_q4_staged.h"

using namespace ea;

static int validate_q4(const ea_layer_desc* desc) {
  int rc = validate_desc(desc);
  if (rc != EA_OK) return rc;
  return desc->dtype == EA_BF16 ? EA_OK : EA_ERR_SHAPE;
}

static Q4Geo q4_geo_of(const ea_layer_desc* desc) {
  return make_q4_geo(desc->r_k, desc->r_v, desc->n_kv_heads, desc->page_tokens, desc->q4_key_group, desc->q4_bits);
}

static bool q4_pos_args_ok(const ea_layer_desc* desc, int32_t page, int32_t kv_head, int32_t token_in_page,
                           int32_t channel, bool keys, int32_t bits = 4) {
  if (validate_q4(desc) != EA_OK) return false;
  if (bits != 0 && (desc->q4_bits == 3) != (bits == 3)) return false;      // the wrong family of position functions
  return page >= 0 && kv_head >= 0 && kv_head < desc->n_kv_heads && token_in_page >= 0 &&
         token_in_page < desc->page_tokens && channel >= 0 && channel < (keys ? desc->r_k : desc->r_v);
}

static int64_t k_tile0(const Q4Geo& q, int32_t page, int32_t kv_head, int32_t token_in_page) {
  return (int64_t)page * q.k_page + (int64_t)kv_head * q.k_slab + q4_k_tile_off(q, token_in_page / kTile);
}
static int64_t v_tile0(const Q4Geo& q, int32_t page, int32_t kv_head, int32_t token_in_page) {
  return (int64_t)page * q.v_page + ((int64_t)kv_head * q.tiles_per_page + token_in_page / kTile) * q.v_tile;
}

extern "C" {

int ea_q4_layout_query(const ea_layer_desc* desc, ea_q4_layout* out) {
  if (!out) return EA_ERR_ARG;
  int rc = validate_q4(desc);
  if (rc != EA_OK) return rc;
  const Q4Geo q = q4_geo_of(desc);
  out->r_k_pad = q.nch * 8;
  out->r_v_pad = q.ncb * 16;
  out->k_tile_bytes = q.k_tile;
  out->v_tile_bytes = q.v_tile;
  out->k_page_bytes = q.k_page;
  out->v_page_bytes = q.v_page;
  return EA_OK;
}

int64_t ea_q4_k_code_pos(const ea_layer_desc* desc, int32_t page, int32_t kv_head, int32_t token_in_page,
                         int32_t channel) {
  if (!q4_pos_args_ok(desc, page, kv_head, token_in_page, channel, true)) return -1;
  const Q4Geo q = q4_geo_of(desc);
  return (k_tile0(q, page, kv_head, token_in_page) + q4_k_dword_off(token_in_page % kTile, channel)) * 8 +
         q4_nibble_shift(channel & 7);
}

int ea_q3_k_code_pos(const ea_layer_desc* desc, int32_t page, int32_t kv_head, int32_t token_in_page, int32_t channel,
                     int64_t* bit_pos) {
  if (!bit_pos || !q4_pos_args_ok(desc, page, kv_head, token_in_page, channel, true, 3)) return EA_ERR_ARG;
  const Q4Geo q = q4_geo_of(desc);
  const Q3Pos p = q3_k_pos(token_in_page % kTile, channel);
  const int64_t t0 = k_tile0(q, page, kv_head, token_in_page);
  for (int b = 0; b < 3; ++b) bit_pos[b] = (t0 + p.byte[b]) * 8 + p.bit[b];
  return EA_OK;
}

int ea_q3_v_code_pos(const ea_layer_desc* desc, int32_t page, int32_t kv_head, int32_t token_in_page, int32_t channel,
                     int64_t* bit_pos) {
  if (!bit_pos || !q4_pos_args_ok(desc, page, kv_head, token_in_page, channel, false, 3)) return EA_ERR_ARG;
  const Q4Geo q = q4_geo_of(desc);
  const Q3Pos p = q3_v_pos(q, token_in_page % kTile, channel);
  const int64_t t0 = v_tile0(q, page, kv_head, token_in_page);
  for (int b = 0; b < 3; ++b) bit_pos[b] = (t0 + p.byte[b]) * 8 + p.bit[b];
  return EA_OK;
}

int64_t ea_q4_k_scale_pos(const ea_layer_desc* desc, int32_t page, int32_t kv_head, int32_t token_in_page,
                          int32_t channel) {
  if (!q4_pos_args_ok(desc, page, kv_head, token_in_page, channel, true, 0)) return -1;
  const Q4Geo q = q4_geo_of(desc);
  return (int64_t)page * q.k_page + (int64_t)kv_head * q.k_slab + q4_k_group_scales_off(q, token_in_page / kTile) +
         q4_k_scale_off(channel);
}

int64_t ea_q4_v_code_pos(const ea_layer_desc* desc, int32_t page, int32_t kv_head, int32_t token_in_page,
                         int32_t channel) {
  if (!q4_pos_args_ok(desc, page, kv_head, token_in_page, channel, false)) return -1;
  const Q4Geo q = q4_geo_of(desc);
  int32_t slot = 0;
  const int32_t off = q4_v_dword_off(q, token_in_page % kTile, channel, &slot);
  return (v_tile0(q, page, kv_head, token_in_page) + off) * 8 + q4_nibble_shift(slot);
}

int64_t ea_q4_v_scale_pos(const ea_layer_desc* desc, int32_t page, int32_t kv_head, int32_t token_in_page) {
  if (!q4_pos_args_ok(desc, page, kv_head, token_in_page, 0, false, 0)) return -1;
  const Q4Geo q = q4_geo_of(desc);
  return v_tile0(q, page, kv_head, token_in_page) + q4_v_scale_off(q, token_in_page % kTile);
}

int ea_quantize_pages_q4(const ea_layer_desc* desc, const void* dev_k_pool, const void* dev_v_pool,
                         const int32_t* dev_src_pages, void* dev_kq_pool, void* dev_vq_pool,
                         const int32_t* dev_dst_pages, int32_t n_pages, int32_t pool_pages, int32_t q4_pool_pages,
                         void* stream) {
  int rc = validate_q4(desc);
  if (rc != EA_OK) return rc;
  if (!dev_k_pool || !dev_v_pool || !dev_src_pages || !dev_kq_pool || !dev_vq_pool || !dev_dst_pages) return EA_ERR_ARG;
  if (n_pages < 0 || pool_pages <= 0 || q4_pool_pages <= 0) return EA_ERR_ARG;
  if (!aligned16(dev_k_pool) || !aligned16(dev_v_pool) || !aligned16(dev_kq_pool) || !aligned16(dev_vq_pool))
    return EA_ERR_ALIGN;
  if (n_pages == 0) return EA_OK;
  const Geo g = make_geo(desc, 1, pool_pages);
  clear_stale_error();
  return quantize_pages_q4(g, q4_geo_of(desc), dev_k_pool, dev_v_pool, dev_src_pages, dev_kq_pool, dev_vq_pool,
                           dev_dst_pages, n_pages, q4_pool_pages, (hipStream_t)stream);
}

int ea_dequantize_pages_q4(const ea_layer_desc* desc, const void* dev_kq_pool, const void* dev_vq_pool,
                           const int32_t* dev_src_pages, void* dev_k_pool, void* dev_v_pool,
                           const int32_t* dev_dst_pages, int32_t n_pages, int32_t q4_pool_pages, int32_t pool_pages,
                           void* stream) {
  int rc = validate_q4(desc);
  if (rc != EA_OK) return rc;
  if (!dev_k_pool || !dev_v_pool || !dev_src_pages || !dev_kq_pool || !dev_vq_pool || !dev_dst_pages) return EA_ERR_ARG;
  if (n_pages < 0 || pool_pages <= 0 || q4_pool_pages <= 0) return EA_ERR_ARG;
  if (!aligned16(dev_k_pool) || !aligned16(dev_v_pool) || !aligned16(dev_kq_pool) || !aligned16(dev_vq_pool))
    return EA_ERR_ALIGN;
  if (n_pages == 0) return EA_OK;
  const Geo g = make_geo(desc, 1, pool_pages);
  clear_stale_error();
  return dequantize_pages_q4(g, q4_geo_of(desc), dev_kq_pool, dev_vq_pool, dev_src_pages, dev_k_pool, dev_v_pool,
                             dev_dst_pages, n_pages, q4_pool_pages, (hipStream_t)stream);
}

int64_t ea_decode_q4_workspace_bytes(const ea_layer_desc* desc, int32_t B, int32_t n_splits) {
  if (validate_q4(desc) != EA_OK || B <= 0 || n_splits <= 0) return -1;
  return ws_floats(B, desc->n_heads, n_splits + 1, round_up(desc->r_v, 16)) * (int64_t)sizeof(float);
}

static int decode_attn_q4_impl(const ea_layer_desc* desc, const float* dev_q_r, const float* dev_slopes, bool alibi,
                      const void* dev_kq_pool, const void* dev_vq_pool,
                      const int32_t* dev_q4_page_table, const int32_t* dev_q4_len, int32_t max_q4_pages,
                      int32_t q4_pool_pages, const void* dev_k_pool, const void* dev_v_pool,
                      const int32_t* dev_tail_page_table, const int32_t* dev_tail_len, int32_t max_tail_pages,
                      int32_t pool_pages, float* dev_out, int32_t B, int32_t n_splits, void* dev_ws, int64_t ws_bytes,
                      void* stream) {
  int rc = validate_q4(desc);
  if (rc != EA_OK) return rc;
  if (!dev_q_r || !dev_kq_pool || !dev_vq_pool || !dev_q4_page_table || !dev_q4_len || !dev_out) return EA_ERR_ARG;
  if (alibi && !dev_slopes) return EA_ERR_ARG;
  const bool tail = dev_tail_page_table != nullptr || dev_tail_len != nullptr;
  if (tail && (!dev_tail_page_table || !dev_tail_len || !dev_k_pool || !dev_v_pool || max_tail_pages <= 0 ||
               pool_pages <= 0))
    return EA_ERR_ARG;
  if (B <= 0 || max_q4_pages <= 0 || q4_pool_pages <= 0 || n_splits < 0 || n_splits > 1024) return EA_ERR_ARG;
  if (!aligned16(dev_q_r) || !aligned16(dev_kq_pool) || !aligned16(dev_vq_pool) || !aligned16(dev_out) ||
      (tail && (!aligned16(dev_k_pool) || !aligned16(dev_v_pool))))
    return EA_ERR_ALIGN;
  if (n_splits == 0) {
    const int64_t cap_tokens = (int64_t)max_q4_pages * desc->page_tokens;
    n_splits = ea_decode_auto_splits(desc, B, cap_tokens > INT32_MAX ? INT32_MAX : (int32_t)cap_tokens);
  }
  if (!dev_ws || !aligned16(dev_ws)) return EA_ERR_WORKSPACE;
  if (ws_bytes < ea_decode_q4_workspace_bytes(desc, B, n_splits)) return EA_ERR_WORKSPACE;
  const int32_t slots = n_splits + (tail ? 1 : 0);
  const Geo gq = make_geo(desc, max_q4_pages, q4_pool_pages);
  hipStream_t st = (hipStream_t)stream;
  clear_stale_error();
  const Geo gt = make_geo(desc, tail ? max_tail_pages : 1, tail ? pool_pages : 1);
  rc = decode_q4(desc, gq, q4_geo_of(desc), dev_q_r, dev_kq_pool, dev_vq_pool, dev_q4_page_table, dev_q4_len,
                 max_q4_pages, q4_pool_pages, B, n_splits, slots, (float*)dev_ws, st, tail ? &gt : nullptr, dev_k_pool,
                 dev_v_pool, dev_tail_page_table, dev_tail_len, alibi ? dev_slopes : nullptr);
  if (rc != EA_OK) return rc;
  return merge_splits(gq, (const float*)dev_ws, dev_out, B, slots, st);
}

int ea_decode_attn_q4(const ea_layer_desc* desc, const float* dev_q_r, const void* dev_kq_pool, const void* dev_vq_pool,
                      const int32_t* dev_q4_page_table, const int32_t* dev_q4_len, int32_t max_q4_pages,
                      int32_t q4_pool_pages, const void* dev_k_pool, const void* dev_v_pool,
                      const int32_t* dev_tail_page_table, const int32_t* dev_tail_len, int32_t max_tail_pages,
                      int32_t pool_pages, float* dev_out, int32_t B, int32_t n_splits, void* dev_ws, int64_t ws_bytes,
                      void* stream) {
  return decode_attn_q4_impl(desc, dev_q_r, nullptr, false, dev_kq_pool, dev_vq_pool, dev_q4_page_table, dev_q4_len,
                             max_q4_pages, q4_pool_pages, dev_k_pool, dev_v_pool, dev_tail_page_table, dev_tail_len,
                             max_tail_pages, pool_pages, dev_out, B, n_splits, dev_ws, ws_bytes, stream);
}

int ea_decode_attn_alibi_q4(const ea_layer_desc* desc, const float* dev_q_r, const float* dev_slopes,
                            const void* dev_kq_pool, const void* dev_vq_pool, const int32_t* dev_q4_page_table,
                            const int32_t* dev_q4_len, int32_t max_q4_pages, int32_t q4_pool_pages,
                            const void* dev_k_pool, const void* dev_v_pool, const int32_t* dev_tail_page_table,
                            const int32_t* dev_tail_len, int32_t max_tail_pages, int32_t pool_pages, float* dev_out,
                            int32_t B, int32_t n_splits, void* dev_ws, int64_t ws_bytes, void* stream) {
  return decode_attn_q4_impl(desc, dev_q_r, dev_slopes, true, dev_kq_pool, dev_vq_pool, dev_q4_page_table, dev_q4_len,
                             max_q4_pages, q4_pool_pages, dev_k_pool, dev_v_pool, dev_tail_page_table, dev_tail_len,
                             max_tail_pages, pool_pages, dev_out, B, n_splits, dev_ws, ws_bytes, stream);
}

int64_t ea_prefill_q4_workspace_bytes(const ea_layer_desc* desc, int32_t B, int32_t n) {
  if (validate_q4(desc) != EA_OK || B <= 0 || n <= 0) return -1;
  return 2 * (int64_t)B * n * desc->n_heads * (desc->r_v + 2) * (int64_t)sizeof(float);
}

int ea_prefill_attn_q4(const ea_layer_desc* desc, const void* dev_q_r, const void* dev_kq_pool, const void* dev_vq_pool,
                       const int32_t* dev_q4_page_table, const int32_t* dev_q4_len, int32_t max_q4_pages,
                       int32_t q4_pool_pages, const void* dev_k_pool, const void* dev_v_pool,
                       const int32_t* dev_tail_page_table, const int32_t* dev_tail_len, int32_t max_tail_pages,
                       int32_t pool_pages, void* dev_out, int32_t B, int32_t n, void* dev_ws, int64_t ws_bytes,
                       void* stream) {
  int rc = validate_q4(desc);
  if (rc != EA_OK) return rc;
  if (!dev_q_r || !dev_kq_pool || !dev_vq_pool || !dev_q4_page_table || !dev_q4_len || !dev_k_pool || !dev_v_pool ||
      !dev_tail_page_table || !dev_tail_len || !dev_out)
    return EA_ERR_ARG;
  if (B <= 0 || n <= 0 || max_q4_pages <= 0 || q4_pool_pages <= 0 || max_tail_pages <= 0 || pool_pages <= 0)
    return EA_ERR_ARG;
  if (!aligned16(dev_q_r) || !aligned16(dev_kq_pool) || !aligned16(dev_vq_pool) || !aligned16(dev_k_pool) ||
      !aligned16(dev_v_pool) || !aligned16(dev_out))
    return EA_ERR_ALIGN;
  if (!dev_ws || !aligned16(dev_ws) || ws_bytes < ea_prefill_q4_workspace_bytes(desc, B, n)) return EA_ERR_WORKSPACE;
  const Geo gq = make_geo(desc, max_q4_pages, q4_pool_pages);
  const Geo gt = make_geo(desc, max_tail_pages, pool_pages);
  clear_stale_error();
  return prefill_q4(desc, gq, q4_geo_of(desc), dev_q_r, dev_kq_pool, dev_vq_pool, dev_q4_page_table, dev_q4_len, gt,
                    dev_k_pool, dev_v_pool, dev_tail_page_table, dev_tail_len, dev_out, B, n, (float*)dev_ws,
                    (hipStream_t)stream);
}

int64_t ea_prefill_q4_staged_workspace_bytes(const ea_layer_desc* desc, int32_t B, int32_t n, int32_t max_q4_pages,
                                             int32_t max_tail_pages) {
  if (validate_q4(desc) != EA_OK || B <= 0 || n <= 0 || max_q4_pages <= 0 || max_tail_pages <= 0) return -1;
  if ((int64_t)B * ((int64_t)max_q4_pages + max_tail_pages) > INT32_MAX) return -1;
  return prefill_staged_q4_ws_bytes(desc, B, n, max_q4_pages, max_tail_pages, false);
}

static int prefill_q4_staged_impl(const ea_layer_desc* desc, const void* dev_q_r, const float* dev_slopes,
                                  const void* dev_kq_pool, const void* dev_vq_pool, const int32_t* dev_q4_page_table,
                                  const int32_t* dev_q4_len, int32_t max_q4_pages, int32_t q4_pool_pages,
                                  const void* dev_k_pool, const void* dev_v_pool, const int32_t* dev_tail_page_table,
                                  const int32_t* dev_tail_len, int32_t max_tail_pages, int32_t pool_pages,
                                  void* dev_out, int32_t B, int32_t n, void* dev_ws, int64_t ws_bytes, void* stream) {
  int rc = validate_q4(desc);
  if (rc != EA_OK) return rc;
  if (!dev_q_r || !dev_kq_pool || !dev_vq_pool || !dev_q4_page_table || !dev_q4_len || !dev_k_pool || !dev_v_pool ||
      !dev_tail_page_table || !dev_tail_len || !dev_out)
    return EA_ERR_ARG;
  if (B <= 0 || n <= 0 || max_q4_pages <= 0 || q4_pool_pages <= 0 || max_tail_pages <= 0 || pool_pages <= 0)
    return EA_ERR_ARG;
  if ((int64_t)B * ((int64_t)max_q4_pages + max_tail_pages) > INT32_MAX) return EA_ERR_SHAPE;
  if (!aligned16(dev_q_r) || !aligned16(dev_kq_pool) || !aligned16(dev_vq_pool) || !aligned16(dev_k_pool) ||
      !aligned16(dev_v_pool) || !aligned16(dev_out))
    return EA_ERR_ALIGN;
  if (!dev_ws || (reinterpret_cast<uintptr_t>(dev_ws) & 255u) ||
      ws_bytes < prefill_staged_q4_ws_bytes(desc, B, n, max_q4_pages, max_tail_pages, false))
    return EA_ERR_WORKSPACE;
  clear_stale_error();
  return prefill_staged_q4(desc, q4_geo_of(desc), dev_q_r, nullptr, 0.0, dev_kq_pool, dev_vq_pool, dev_q4_page_table,
                           dev_q4_len, max_q4_pages, q4_pool_pages, dev_k_pool, dev_v_pool, dev_tail_page_table,
                           dev_tail_len, max_tail_pages, pool_pages, dev_out, B, n, dev_ws, (hipStream_t)stream,
                           dev_slopes);
}

int ea_prefill_attn_q4_staged(const ea_layer_desc* desc, const void* dev_q_r, const void* dev_kq_pool,
                              const void* dev_vq_pool, const int32_t* dev_q4_page_table, const int32_t* dev_q4_len,
                              int32_t max_q4_pages, int32_t q4_pool_pages, const void* dev_k_pool, const void* dev_v_pool,
                              const int32_t* dev_tail_page_table, const int32_t* dev_tail_len, int32_t max_tail_pages,
                              int32_t pool_pages, void* dev_out, int32_t B, int32_t n, void* dev_ws, int64_t ws_bytes,
                              void* stream) {
  return prefill_q4_staged_impl(desc, dev_q_r, nullptr, dev_kq_pool, dev_vq_pool, dev_q4_page_table, dev_q4_len,
                                max_q4_pages, q4_pool_pages, dev_k_pool, dev_v_pool, dev_tail_page_table, dev_tail_len,
                                max_tail_pages, pool_pages, dev_out, B, n, dev_ws, ws_bytes, stream);
}

int ea_prefill_attn_alibi_q4(const ea_layer_desc* desc, const void* dev_q_r, const float* dev_slopes,
                             const void* dev_kq_pool, const void* dev_vq_pool, const int32_t* dev_q4_page_table,
                             const int32_t* dev_q4_len, int32_t max_q4_pages, int32_t q4_pool_pages,
                             const void* dev_k_pool, const void* dev_v_pool, const int32_t* dev_tail_page_table,
                             const int32_t* dev_tail_len, int32_t max_tail_pages, int32_t pool_pages, void* dev_out,
                             int32_t B, int32_t n, void* dev_ws, int64_t ws_bytes, void* stream) {
  if (!dev_slopes) return EA_ERR_ARG;
  return prefill_q4_staged_impl(desc, dev_q_r, dev_slopes, dev_kq_pool, dev_vq_pool, dev_q4_page_table, dev_q4_len,
                                max_q4_pages, q4_pool_pages, dev_k_pool, dev_v_pool, dev_tail_page_table, dev_tail_len,
                                max_tail_pages, pool_pages, dev_out, B, n, dev_ws, ws_bytes, stream);
}

int64_t ea_prefill_rope_q4_workspace_bytes(const ea_layer_desc* desc, int32_t B, int32_t n, int32_t max_q4_pages,
                                           int32_t max_tail_pages) {
  if (validate_q4(desc) != EA_OK || B <= 0 || n <= 0 || max_q4_pages <= 0 || max_tail_pages <= 0) return -1;
  if ((int64_t)B * ((int64_t)max_q4_pages + max_tail_pages) > INT32_MAX) return -1;
  return prefill_staged_q4_ws_bytes(desc, B, n, max_q4_pages, max_tail_pages, true);
}

int ea_prefill_attn_rope_q4(const ea_layer_desc* desc, const void* dev_q, const void* dev_u_k, double rope_base,
                            const void* dev_kq_pool, const void* dev_vq_pool, const int32_t* dev_q4_page_table,
                            const int32_t* dev_q4_len, int32_t max_q4_pages, int32_t q4_pool_pages,
                            const void* dev_k_pool, const void* dev_v_pool, const int32_t* dev_tail_page_table,
                            const int32_t* dev_tail_len, int32_t max_tail_pages, int32_t pool_pages, void* dev_out,
                            int32_t B, int32_t n, void* dev_ws, int64_t ws_bytes, void* stream) {
  int rc = validate_q4(desc);
  if (rc != EA_OK) return rc;
  if (!dev_q || !dev_u_k || !dev_kq_pool || !dev_vq_pool || !dev_q4_page_table || !dev_q4_len || !dev_k_pool ||
      !dev_v_pool || !dev_tail_page_table || !dev_tail_len || !dev_out)
    return EA_ERR_ARG;
  if (B <= 0 || n <= 0 || max_q4_pages <= 0 || q4_pool_pages <= 0 || max_tail_pages <= 0 || pool_pages <= 0)
    return EA_ERR_ARG;
  if (!(rope_base > 1.0) || !(rope_base < 1e30)) return EA_ERR_ARG;
  if (desc->r_k > desc->d_head || (desc->d_head != 64 && desc->d_head != 128)) return EA_ERR_SHAPE;
  if ((int64_t)B * ((int64_t)max_q4_pages + max_tail_pages) > INT32_MAX) return EA_ERR_SHAPE;
  if (!aligned16(dev_q) || !aligned16(dev_u_k) || !aligned16(dev_kq_pool) || !aligned16(dev_vq_pool) ||
      !aligned16(dev_k_pool) || !aligned16(dev_v_pool) || !aligned16(dev_out))
    return EA_ERR_ALIGN;
  if (!dev_ws || (reinterpret_cast<uintptr_t>(dev_ws) & 255u) ||
      ws_bytes < prefill_staged_q4_ws_bytes(desc, B, n, max_q4_pages, max_tail_pages, true))
    return EA_ERR_WORKSPACE;
  clear_stale_error();
  return prefill_staged_q4(desc, q4_geo_of(desc), dev_q, dev_u_k, rope_base, dev_kq_pool, dev_vq_pool, dev_q4_page_table,
                         dev_q4_len, max_q4_pages, q4_pool_pages, dev_k_pool, dev_v_pool, dev_tail_page_table,
                         dev_tail_len, max_tail_pages, pool_pages, dev_out, B, n, dev_ws, (hipStream_t)stream);
}

int ea_decode_attn_rope_q4(const ea_layer_desc* desc, const float* dev_q, const void* dev_u_k, double rope_base,
                           const void* dev_kq_pool, const void* dev_vq_pool, const int32_t* dev_q4_page_table,
                           const int32_t* dev_q4_len, int32_t max_q4_pages, int32_t q4_pool_pages,
                           const void* dev_k_pool, const void* dev_v_pool, const int32_t* dev_tail_page_table,
                           const int32_t* dev_tail_len, int32_t max_tail_pages, int32_t pool_pages, float* dev_out,
                           int32_t B, int32_t n_splits, void* dev_ws, int64_t ws_bytes, void* stream) {
  int rc = validate_q4(desc);
  if (rc != EA_OK) return rc;
  if (!dev_q || !dev_u_k || !dev_kq_pool || !dev_vq_pool || !dev_q4_page_table || !dev_q4_len || !dev_out)
    return EA_ERR_ARG;
  const bool tail = dev_tail_page_table != nullptr || dev_tail_len != nullptr;
  if (tail && (!dev_tail_page_table || !dev_tail_len || !dev_k_pool || !dev_v_pool || max_tail_pages <= 0 ||
               pool_pages <= 0))
    return EA_ERR_ARG;
  if (B <= 0 || max_q4_pages <= 0 || q4_pool_pages <= 0 || n_splits < 0 || n_splits > 1024) return EA_ERR_ARG;
  if (!(rope_base > 1.0) || !(rope_base < 1e30)) return EA_ERR_ARG;
  if (desc->r_k > desc->d_head || (desc->d_head != 64 && desc->d_head != 128)) return EA_ERR_SHAPE;
  if (!aligned16(dev_q) || !aligned16(dev_u_k) || !aligned16(dev_kq_pool) || !aligned16(dev_vq_pool) ||
      !aligned16(dev_out) || (tail && (!aligned16(dev_k_pool) || !aligned16(dev_v_pool))))
    return EA_ERR_ALIGN;
  if (n_splits == 0) {
    const int64_t cap_tokens = (int64_t)max_q4_pages * desc->page_tokens;
    n_splits = ea_decode_rope_auto_splits(desc, B, cap_tokens > INT32_MAX ? INT32_MAX : (int32_t)cap_tokens);
  }
  if (!dev_ws || !aligned16(dev_ws)) return EA_ERR_WORKSPACE;
  if (ws_bytes < ea_decode_q4_workspace_bytes(desc, B, n_splits)) return EA_ERR_WORKSPACE;
  const int32_t slots = n_splits + (tail ? 1 : 0);
  const Geo gq = make_geo(desc, max_q4_pages, q4_pool_pages);
  hipStream_t st = (hipStream_t)stream;
  clear_stale_error();
  rc = decode_rope_q4(desc, gq, q4_geo_of(desc), dev_q, dev_u_k, rope_base, dev_kq_pool, dev_vq_pool,
                      dev_q4_page_table, dev_q4_len, tail ? dev_tail_len : nullptr, max_q4_pages, q4_pool_pages, B,
                      n_splits, slots, (float*)dev_ws, st);
  if (rc != EA_OK) return rc;
  if (tail) {
    const Geo gt = make_geo(desc, max_tail_pages, pool_pages);
    rc = decode_rope_bf16(desc, gt, dev_q, dev_u_k, rope_base, dev_k_pool, dev_v_pool, dev_tail_page_table,
                          dev_tail_len, dev_out, B, 1, (float*)dev_ws, st, slots, n_splits);
    if (rc != EA_OK) return rc;
  }
  return merge_splits(gq, (const float*)dev_ws, dev_out, B, slots, st);
}

}  // extern "C"
