// Host side of the C ABI: argument checks, layout reference functions, dispatch.
#include "ea_common.h"

using namespace ea;

extern "C" {

int ea_version(void) { return 101; }

const char* ea_strerror(int code) {
  switch (code) {
    case EA_OK: return "ok";
    case EA_ERR_ARG: return "invalid argument (null pointer, non-positive size or bad enum)";
    case EA_ERR_SHAPE: return "unsupported shape";
    case EA_ERR_ALIGN: return "pointer is not 16-byte aligned";
    case EA_ERR_WORKSPACE: return "workspace missing or too small";
    case EA_ERR_DEVICE: return "HIP launch error";
    case EA_ERR_SCRATCH_LIMIT: return "the call needs more than the library's built-in scratch buffer holds";
    default: return "unknown error code";
  }
}

int ea_cache_layout_query(const ea_layer_desc* desc, ea_cache_layout* out) {
  int rc = validate_desc(desc);
  if (rc != EA_OK) return rc;
  if (!out) return EA_ERR_ARG;
  Geo g = make_geo(desc, 0, 0);
  out->layout_id = desc->dtype == EA_BF16 ? 1 : 0;
  out->elem_bytes = desc->dtype == EA_BF16 ? 2 : 4;
  out->r_k_pad = g.r_k_pad;
  out->r_v_pad = g.r_v_pad;
  out->k_slab_elems = g.k_slab;
  out->v_slab_elems = g.v_slab;
  out->k_page_elems = g.k_page;
  out->v_page_elems = g.v_page;
  return EA_OK;
}

static int64_t cache_index(const ea_layer_desc* desc, bool is_k, int32_t page, int32_t kv_head, int32_t t, int32_t c) {
  if (validate_desc(desc) != EA_OK) return -1;
  Geo g = make_geo(desc, 0, 0);
  const int32_t r = is_k ? g.r_k : g.r_v;
  if (page < 0 || kv_head < 0 || kv_head >= g.n_kv_heads || t < 0 || t >= g.page_tokens || c < 0 || c >= r) return -1;
  const int32_t r_pad = is_k ? g.r_k_pad : g.r_v_pad;
  const int64_t base = (int64_t)page * (is_k ? g.k_page : g.v_page) + (int64_t)kv_head * (is_k ? g.k_slab : g.v_slab);
  if (desc->dtype == EA_F32) return base + f32_slab_off(t, c, r_pad);
  return base + (is_k ? bf16_k_slab_off(t, c, r_pad) : bf16_v_slab_off(t, c, r_pad));
}

int64_t ea_cache_k_index(const ea_layer_desc* desc, int32_t page, int32_t kv_head, int32_t token_in_page, int32_t channel) {
  return cache_index(desc, true, page, kv_head, token_in_page, channel);
}
int64_t ea_cache_v_index(const ea_layer_desc* desc, int32_t page, int32_t kv_head, int32_t token_in_page, int32_t channel) {
  return cache_index(desc, false, page, kv_head, token_in_page, channel);
}

int64_t ea_cache_slot(const ea_layer_desc* desc, const int32_t* page_table_row, int32_t max_pages, int32_t pos) {
  if (validate_desc(desc) != EA_OK || !page_table_row || pos < 0) return -1;
  const int32_t lp = pos / desc->page_tokens;
  if (lp >= max_pages) return -1;
  const int32_t page = page_table_row[lp];
  if (page < 0) return -1;
  return (int64_t)page * desc->page_tokens + pos % desc->page_tokens;
}

int ea_cache_scatter(const ea_layer_desc* desc, const void* dev_k_dense, const void* dev_v_dense, void* dev_k_pool,
                     void* dev_v_pool, const int32_t* dev_page_table, int32_t B, int32_t n, int32_t pos0,
                     int32_t max_pages, int32_t pool_pages, void* stream) {
  int rc = validate_desc(desc);
  if (rc != EA_OK) return rc;
  if (!dev_page_table || B <= 0 || n < 0 || pos0 < 0 || max_pages <= 0 || pool_pages <= 0) return EA_ERR_ARG;
  if ((dev_k_dense && !dev_k_pool) || (dev_v_dense && !dev_v_pool)) return EA_ERR_ARG;
  if (n == 0) return EA_OK;
  Geo g = make_geo(desc, max_pages, pool_pages);
  clear_stale_error();
  return cache_copy(desc, g, true, const_cast<void*>(dev_k_dense), const_cast<void*>(dev_v_dense), dev_k_pool,
                    dev_v_pool, dev_page_table, B, n, pos0, (hipStream_t)stream);
}

int ea_cache_gather(const ea_layer_desc* desc, void* dev_k_dense, void* dev_v_dense, const void* dev_k_pool,
                    const void* dev_v_pool, const int32_t* dev_page_table, int32_t B, int32_t n, int32_t pos0,
                    int32_t max_pages, int32_t pool_pages, void* stream) {
  int rc = validate_desc(desc);
  if (rc != EA_OK) return rc;
  if (!dev_page_table || B <= 0 || n < 0 || pos0 < 0 || max_pages <= 0 || pool_pages <= 0) return EA_ERR_ARG;
  if ((dev_k_dense && !dev_k_pool) || (dev_v_dense && !dev_v_pool)) return EA_ERR_ARG;
  if (n == 0) return EA_OK;
  Geo g = make_geo(desc, max_pages, pool_pages);
  clear_stale_error();
  return cache_copy(desc, g, false, dev_k_dense, dev_v_dense, const_cast<void*>(dev_k_pool),
                    const_cast<void*>(dev_v_pool), dev_page_table, B, n, pos0, (hipStream_t)stream);
}

int64_t ea_packed_weight_elems(int32_t N, int32_t K, int32_t dtype) {
  if (N <= 0 || K <= 0 || (dtype != EA_F32 && dtype != EA_BF16)) return -1;
  if (dtype == EA_F32) return (int64_t)N * K;
  if (K % 32 != 0) return -1;
  return (int64_t)round_up(N, 16) * K;
}

int ea_pack_weight(const void* dev_w_t, void* dev_packed, int32_t N, int32_t K, int32_t dtype, void* stream) {
  if (!dev_w_t || !dev_packed || ea_packed_weight_elems(N, K, dtype) < 0) return EA_ERR_ARG;
  if (!aligned16(dev_w_t) || !aligned16(dev_packed)) return EA_ERR_ALIGN;
  clear_stale_error();
  return pack_weight(dev_w_t, dev_packed, N, K, dtype == EA_BF16, (hipStream_t)stream);
}

static int project_qkv_impl(const ea_layer_desc* desc, int32_t q_dim, const void* dev_x, const void* dev_wqkv_t,
                            void* dev_q, int32_t q_dtype, void* dev_k_pool, void* dev_v_pool,
                            const int32_t* dev_page_table, const int32_t* dev_seq_len, int32_t B, int32_t T,
                            int32_t max_pages, int32_t pool_pages, int32_t* dev_status, void* stream,
                            uint32_t* dev_clear = nullptr, int32_t clear_words = 0) {
  if (!dev_x || !dev_wqkv_t || !dev_q || !dev_k_pool || !dev_v_pool || !dev_page_table || !dev_seq_len)
    return EA_ERR_ARG;
  if (B <= 0 || T <= 0 || max_pages <= 0 || pool_pages <= 0) return EA_ERR_ARG;
  if (q_dtype != EA_F32 && q_dtype != EA_BF16) return EA_ERR_ARG;
  if (desc->dtype == EA_F32 && q_dtype != EA_F32) return EA_ERR_ARG;
  if ((int64_t)B * T > INT32_MAX) return EA_ERR_SHAPE;
  if (!aligned16(dev_x) || !aligned16(dev_wqkv_t) || !aligned16(dev_q) || !aligned16(dev_k_pool) ||
      !aligned16(dev_v_pool))
    return EA_ERR_ALIGN;
  if (dev_status && (reinterpret_cast<uintptr_t>(dev_status) & 3u)) return EA_ERR_ALIGN;
  if (desc->d_model % (desc->dtype == EA_BF16 ? 32 : 4) != 0) return EA_ERR_SHAPE;
  clear_stale_error();
  QkvDest dst;
  dst.q = dev_q;
  dst.q_is_f32 = q_dtype == EA_F32;
  dst.k_pool = dev_k_pool;
  dst.v_pool = dev_v_pool;
  dst.page_table = dev_page_table;
  dst.seq_len = dev_seq_len;
  dst.T = T;
  dst.status = dev_status;
  dst.clear = dev_clear;
  dst.clear_words = clear_words;
  dst.g = make_geo(desc, max_pages, pool_pages);
  dst.g.q_dim = q_dim;
  const int32_t N = desc->n_heads * q_dim + desc->n_kv_heads * (desc->r_k + desc->r_v);
  if (desc->dtype == EA_BF16)
    return gemm_qkv_bf16(dev_x, dev_wqkv_t, B * T, N, desc->d_model, dst, (hipStream_t)stream);
  return gemm_qkv_f32((const float*)dev_x, (const float*)dev_wqkv_t, B * T, N, desc->d_model, dst, (hipStream_t)stream);
}

int ea_project_qkv(const ea_layer_desc* desc, const void* dev_x, const void* dev_wqkv_t, void* dev_q_r, int32_t q_dtype,
                   void* dev_k_pool, void* dev_v_pool, const int32_t* dev_page_table, const int32_t* dev_seq_len,
                   int32_t B, int32_t T, int32_t max_pages, int32_t pool_pages, int32_t* dev_status, void* stream) {
  int rc = validate_desc(desc);
  if (rc != EA_OK) return rc;
  return project_qkv_impl(desc, desc->r_k, dev_x, dev_wqkv_t, dev_q_r, q_dtype, dev_k_pool, dev_v_pool, dev_page_table,
                          dev_seq_len, B, T, max_pages, pool_pages, dev_status, stream);
}

int ea_project_qkv_rope(const ea_layer_desc* desc, const void* dev_x, const void* dev_wqkv_t, void* dev_q,
                        int32_t q_dtype, void* dev_k_pool, void* dev_v_pool, const int32_t* dev_page_table,
                        const int32_t* dev_seq_len, int32_t B, int32_t T, int32_t max_pages, int32_t pool_pages,
                        int32_t* dev_status, void* stream) {
  int rc = validate_desc(desc);
  if (rc != EA_OK) return rc;
  if (desc->r_k > desc->d_head) return EA_ERR_SHAPE;
  return project_qkv_impl(desc, desc->d_head, dev_x, dev_wqkv_t, dev_q, q_dtype, dev_k_pool, dev_v_pool,
                          dev_page_table, dev_seq_len, B, T, max_pages, pool_pages, dev_status, stream);
}

// Compute units of the current device, asked once per process; 256 (MI355X) when no device can be asked.
static int resident_compute_units() {
  static int n = 0;
  if (n == 0) {
    int dev = 0, cu = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&cu, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cu > 0)
      n = cu;
    else
      n = 256;
    (void)hipGetLastError();
  }
  return n;
}

int32_t ea_decode_auto_splits(const ea_layer_desc* desc, int32_t B, int32_t max_seq_len) {
  if (validate_desc(desc) != EA_OK || B <= 0 || max_seq_len <= 0) return 1;
  // One workgroup per resident slot (compute units x 2 workgroups: the attention kernels run two 4-wave workgroups
  // per compute unit) measured best on MI355X: more splits only add merge work, fewer leave compute units without
  // a stream.  Every workgroup keeps at least eight tiles.
  const int64_t streams = (int64_t)B * (desc->dtype == EA_BF16 ? desc->n_kv_heads : desc->n_heads);
  const int32_t tiles = (max_seq_len + kTile - 1) / kTile;
  const int64_t slots = 2 * (int64_t)resident_compute_units();
  int64_t want = (slots + streams - 1) / streams;
  int64_t cap = tiles / 8;
  if (cap < 1) cap = 1;
  if (want > cap) want = cap;
  if (want > 64) want = 64;
  if (want < 1) want = 1;
  return (int32_t)want;
}

int32_t ea_decode_rope_auto_splits(const ea_layer_desc* desc, int32_t B, int32_t max_seq_len) {
  if (validate_desc(desc) != EA_OK || B <= 0 || max_seq_len <= 0) return 1;
  // The rotary kernel builds tables before it streams: with a single workgroup per resident slot all of them
  // would do that at the same time and leave the memory idle meanwhile; at least four rounds of workgroups
  // measured best on MI355X.
  int32_t s = ea_decode_auto_splits(desc, B, max_seq_len);
  int32_t cap = ((max_seq_len + kTile - 1) / kTile) / 8;
  if (cap < 1) cap = 1;
  const int32_t want = cap < 4 ? cap : 4;
  return s > want ? s : want;
}

int64_t ea_decode_workspace_bytes(const ea_layer_desc* desc, int32_t B, int32_t n_splits) {
  if (validate_desc(desc) != EA_OK || B <= 0 || n_splits < 0) return -1;
  if (n_splits <= 1) return 0;
  Geo g = make_geo(desc, 0, 0);
  return ws_floats(B, g.n_heads, n_splits, g.r_v_pad) * (int64_t)sizeof(float);
}

int ea_decode_attn(const ea_layer_desc* desc, const void* dev_q_r, const void* dev_k_pool, const void* dev_v_pool,
                   const int32_t* dev_page_table, const int32_t* dev_seq_len, float* dev_out, int32_t B,
                   int32_t max_pages, int32_t pool_pages, int32_t n_splits, void* dev_ws, int64_t ws_bytes,
                   void* stream) {
  int rc = validate_desc(desc);
  if (rc != EA_OK) return rc;
  if (!dev_q_r || !dev_k_pool || !dev_v_pool || !dev_page_table || !dev_seq_len || !dev_out) return EA_ERR_ARG;
  if (B <= 0 || max_pages <= 0 || pool_pages <= 0 || n_splits < 0 || n_splits > 1024) return EA_ERR_ARG;
  if (!aligned16(dev_q_r) || !aligned16(dev_k_pool) || !aligned16(dev_v_pool) || !aligned16(dev_out))
    return EA_ERR_ALIGN;
  if (n_splits == 0) {
    const int64_t cap_tokens = (int64_t)max_pages * desc->page_tokens;
    n_splits = ea_decode_auto_splits(desc, B, cap_tokens > INT32_MAX ? INT32_MAX : (int32_t)cap_tokens);
  }
  if (n_splits > 1) {
    if (!dev_ws || !aligned16(dev_ws)) return EA_ERR_WORKSPACE;
    if (ws_bytes < ea_decode_workspace_bytes(desc, B, n_splits)) return EA_ERR_WORKSPACE;
  }
  Geo g = make_geo(desc, max_pages, pool_pages);
  hipStream_t st = (hipStream_t)stream;
  clear_stale_error();
  if (desc->dtype == EA_BF16)
    rc = decode_bf16(desc, g, (const float*)dev_q_r, dev_k_pool, dev_v_pool, dev_page_table, dev_seq_len, dev_out, B,
                     n_splits, (float*)dev_ws, st);
  else
    rc = decode_f32(desc, g, (const float*)dev_q_r, (const float*)dev_k_pool, (const float*)dev_v_pool, dev_page_table,
                    dev_seq_len, dev_out, B, n_splits, (float*)dev_ws, st);
  if (rc != EA_OK) return rc;
  if (n_splits > 1) rc = merge_splits(g, (const float*)dev_ws, dev_out, B, n_splits, st);
  return rc;
}

int ea_decode_attn_rope(const ea_layer_desc* desc, const float* dev_q, const void* dev_u_k, double rope_base,
                        const void* dev_k_pool, const void* dev_v_pool, const int32_t* dev_page_table,
                        const int32_t* dev_seq_len, float* dev_out, int32_t B, int32_t max_pages, int32_t pool_pages,
                        int32_t n_splits, void* dev_ws, int64_t ws_bytes, void* stream) {
  int rc = validate_desc(desc);
  if (rc != EA_OK) return rc;
  if (!dev_q || !dev_u_k || !dev_k_pool || !dev_v_pool || !dev_page_table || !dev_seq_len || !dev_out)
    return EA_ERR_ARG;
  if (B <= 0 || max_pages <= 0 || pool_pages <= 0 || n_splits < 0 || n_splits > 1024) return EA_ERR_ARG;
  if (!(rope_base > 1.0) || !(rope_base < 1e30)) return EA_ERR_ARG;
  if (desc->r_k > desc->d_head) return EA_ERR_SHAPE;
  if (desc->dtype == EA_BF16 ? (desc->d_head != 64 && desc->d_head != 128)
                             : (desc->d_head % 2 != 0 || desc->d_head > 256))
    return EA_ERR_SHAPE;
  if (!aligned16(dev_q) || !aligned16(dev_u_k) || !aligned16(dev_k_pool) || !aligned16(dev_v_pool) ||
      !aligned16(dev_out))
    return EA_ERR_ALIGN;
  if (n_splits == 0) {
    const int64_t cap_tokens = (int64_t)max_pages * desc->page_tokens;
    n_splits = ea_decode_rope_auto_splits(desc, B, cap_tokens > INT32_MAX ? INT32_MAX : (int32_t)cap_tokens);
  }
  if (n_splits > 1) {
    if (!dev_ws || !aligned16(dev_ws)) return EA_ERR_WORKSPACE;
    if (ws_bytes < ea_decode_workspace_bytes(desc, B, n_splits)) return EA_ERR_WORKSPACE;
  }
  Geo g = make_geo(desc, max_pages, pool_pages);
  hipStream_t st = (hipStream_t)stream;
  clear_stale_error();
  if (desc->dtype == EA_BF16)
    rc = decode_rope_bf16(desc, g, dev_q, dev_u_k, rope_base, dev_k_pool, dev_v_pool, dev_page_table, dev_seq_len,
                          dev_out, B, n_splits, (float*)dev_ws, st);
  else
    rc = decode_rope_f32(desc, g, dev_q, (const float*)dev_u_k, rope_base, (const float*)dev_k_pool, (const float*)dev_v_pool,
                         dev_page_table, dev_seq_len, dev_out, B, n_splits, (float*)dev_ws, st);
  if (rc != EA_OK) return rc;
  if (n_splits > 1) rc = merge_splits(g, (const float*)dev_ws, dev_out, B, n_splits, st);
  return rc;
}

int ea_prefill_attn(const ea_layer_desc* desc, const void* dev_q_r, const void* dev_k_pool, const void* dev_v_pool,
                    const int32_t* dev_page_table, const int32_t* dev_seq_len, void* dev_out, int32_t B, int32_t n,
                    int32_t max_pages, int32_t pool_pages, void* stream) {
  int rc = validate_desc(desc);
  if (rc != EA_OK) return rc;
  if (!dev_q_r || !dev_k_pool || !dev_v_pool || !dev_page_table || !dev_seq_len || !dev_out) return EA_ERR_ARG;
  if (B <= 0 || n <= 0 || max_pages <= 0 || pool_pages <= 0) return EA_ERR_ARG;
  if (!aligned16(dev_q_r) || !aligned16(dev_k_pool) || !aligned16(dev_v_pool) || !aligned16(dev_out))
    return EA_ERR_ALIGN;
  Geo g = make_geo(desc, max_pages, pool_pages);
  clear_stale_error();
  if (desc->dtype == EA_BF16)
    return prefill_bf16(desc, g, dev_q_r, dev_k_pool, dev_v_pool, dev_page_table, dev_seq_len, dev_out, B, n,
                        (hipStream_t)stream);
  return prefill_f32(desc, g, (const float*)dev_q_r, (const float*)dev_k_pool, (const float*)dev_v_pool,
                     dev_page_table, dev_seq_len, (float*)dev_out, B, n, (hipStream_t)stream);
}

int ea_decode_attn_alibi(const ea_layer_desc* desc, const void* dev_q_r, const float* dev_slopes, const void* dev_k_pool,
                         const void* dev_v_pool, const int32_t* dev_page_table, const int32_t* dev_seq_len,
                         float* dev_out, int32_t B, int32_t max_pages, int32_t pool_pages, int32_t n_splits,
                         void* dev_ws, int64_t ws_bytes, void* stream) {
  int rc = validate_desc(desc);
  if (rc != EA_OK) return rc;
  if (!dev_q_r || !dev_slopes || !dev_k_pool || !dev_v_pool || !dev_page_table || !dev_seq_len || !dev_out)
    return EA_ERR_ARG;
  if (B <= 0 || max_pages <= 0 || pool_pages <= 0 || n_splits < 0 || n_splits > 1024) return EA_ERR_ARG;
  if (!aligned16(dev_q_r) || !aligned16(dev_k_pool) || !aligned16(dev_v_pool) || !aligned16(dev_out))
    return EA_ERR_ALIGN;
  if (n_splits == 0) {
    const int64_t cap_tokens = (int64_t)max_pages * desc->page_tokens;
    n_splits = ea_decode_auto_splits(desc, B, cap_tokens > INT32_MAX ? INT32_MAX : (int32_t)cap_tokens);
  }
  if (n_splits > 1) {
    if (!dev_ws || !aligned16(dev_ws)) return EA_ERR_WORKSPACE;
    if (ws_bytes < ea_decode_workspace_bytes(desc, B, n_splits)) return EA_ERR_WORKSPACE;
  }
  Geo g = make_geo(desc, max_pages, pool_pages);
  hipStream_t st = (hipStream_t)stream;
  clear_stale_error();
  if (desc->dtype == EA_BF16)
    rc = decode_alibi_bf16(desc, g, (const float*)dev_q_r, dev_slopes, dev_k_pool, dev_v_pool, dev_page_table,
                           dev_seq_len, dev_out, B, n_splits, (float*)dev_ws, st);
  else
    rc = decode_alibi_f32(desc, g, (const float*)dev_q_r, dev_slopes, (const float*)dev_k_pool,
                          (const float*)dev_v_pool, dev_page_table, dev_seq_len, dev_out, B, n_splits, (float*)dev_ws,
                          st);
  if (rc != EA_OK) return rc;
  if (n_splits > 1) rc = merge_splits(g, (const float*)dev_ws, dev_out, B, n_splits, st);
  return rc;
}

int ea_prefill_attn_alibi(const ea_layer_desc* desc, const void* dev_q_r, const float* dev_slopes,
                          const void* dev_k_pool, const void* dev_v_pool, const int32_t* dev_page_table,
                          const int32_t* dev_seq_len, void* dev_out, int32_t B, int32_t n, int32_t max_pages,
                          int32_t pool_pages, void* stream) {
  int rc = validate_desc(desc);
  if (rc != EA_OK) return rc;
  if (!dev_q_r || !dev_slopes || !dev_k_pool || !dev_v_pool || !dev_page_table || !dev_seq_len || !dev_out)
    return EA_ERR_ARG;
  if (B <= 0 || n <= 0 || max_pages <= 0 || pool_pages <= 0) return EA_ERR_ARG;
  if (!aligned16(dev_q_r) || !aligned16(dev_k_pool) || !aligned16(dev_v_pool) || !aligned16(dev_out))
    return EA_ERR_ALIGN;
  Geo g = make_geo(desc, max_pages, pool_pages);
  clear_stale_error();
  if (desc->dtype == EA_BF16)
    return prefill_alibi_bf16(desc, g, dev_q_r, dev_slopes, dev_k_pool, dev_v_pool, dev_page_table, dev_seq_len,
                              dev_out, B, n, (hipStream_t)stream);
  return prefill_alibi_f32(desc, g, (const float*)dev_q_r, dev_slopes, (const float*)dev_k_pool,
                           (const float*)dev_v_pool, dev_page_table, dev_seq_len, (float*)dev_out, B, n,
                           (hipStream_t)stream);
}

int64_t ea_prefill_rope_workspace_bytes(const ea_layer_desc* desc, int32_t B, int32_t n, int32_t max_pages) {
  if (validate_desc(desc) != EA_OK || B <= 0 || n <= 0 || max_pages <= 0) return -1;
  return prefill_rope_ws_bytes(desc, B, n, max_pages);
}

int ea_prefill_attn_rope(const ea_layer_desc* desc, const void* dev_q, const void* dev_u_k, double rope_base,
                         const void* dev_k_pool, const void* dev_v_pool, const int32_t* dev_page_table,
                         const int32_t* dev_seq_len, void* dev_out, int32_t B, int32_t n, int32_t max_pages,
                         int32_t pool_pages, void* dev_ws, int64_t ws_bytes, void* stream) {
  int rc = validate_desc(desc);
  if (rc != EA_OK) return rc;
  if (!dev_q || !dev_u_k || !dev_k_pool || !dev_v_pool || !dev_page_table || !dev_seq_len || !dev_out)
    return EA_ERR_ARG;
  if (B <= 0 || n <= 0 || max_pages <= 0 || pool_pages <= 0) return EA_ERR_ARG;
  if (!(rope_base > 1.0) || !(rope_base < 1e30)) return EA_ERR_ARG;
  if (desc->r_k > desc->d_head) return EA_ERR_SHAPE;
  if (!aligned16(dev_q) || !aligned16(dev_u_k) || !aligned16(dev_k_pool) || !aligned16(dev_v_pool) ||
      !aligned16(dev_out))
    return EA_ERR_ALIGN;
  Geo g = make_geo(desc, max_pages, pool_pages);
  clear_stale_error();
  if (desc->dtype == EA_BF16) {
    if (desc->d_head != 64 && desc->d_head != 128) return EA_ERR_SHAPE;
    if (!dev_ws || !aligned16(dev_ws) || ws_bytes < prefill_rope_ws_bytes(desc, B, n, max_pages))
      return EA_ERR_WORKSPACE;
    return prefill_rope_bf16(desc, g, dev_q, dev_u_k, rope_base, dev_k_pool, dev_v_pool, dev_page_table, dev_seq_len,
                             dev_out, B, n, dev_ws, (hipStream_t)stream);
  }
  if (desc->d_head % 2 != 0 || desc->d_head > 256) return EA_ERR_SHAPE;
  return prefill_rope_f32(desc, g, (const float*)dev_q, (const float*)dev_u_k, rope_base, (const float*)dev_k_pool,
                          (const float*)dev_v_pool, dev_page_table, dev_seq_len, (float*)dev_out, B, n,
                          (hipStream_t)stream);
}

int ea_out_proj(const ea_layer_desc* desc, const void* dev_o, int32_t o_dtype, const void* dev_wo_t, void* dev_y,
                int32_t M, void* stream) {
  int rc = validate_desc(desc);
  if (rc != EA_OK) return rc;
  if (!dev_o || !dev_wo_t || !dev_y || M <= 0) return EA_ERR_ARG;
  if (o_dtype != EA_F32 && o_dtype != EA_BF16) return EA_ERR_ARG;
  if (desc->dtype == EA_F32 && o_dtype != EA_F32) return EA_ERR_ARG;
  if (!aligned16(dev_o) || !aligned16(dev_wo_t) || !aligned16(dev_y)) return EA_ERR_ALIGN;
  const int32_t K = desc->n_heads * desc->r_v;
  if (K % (desc->dtype == EA_BF16 ? 32 : 4) != 0) return EA_ERR_SHAPE;
  clear_stale_error();
  if (desc->dtype == EA_BF16)
    return gemm_out_bf16(dev_o, o_dtype == EA_F32, dev_wo_t, dev_y, M, desc->d_model, K, (hipStream_t)stream);
  return gemm_out_f32((const float*)dev_o, (const float*)dev_wo_t, (float*)dev_y, M, desc->d_model, K,
                      (hipStream_t)stream);
}


// ---- the whole generation step of a layer in one call ------------------------------------------------------

static int64_t align256(int64_t x) { return (x + 255) / 256 * 256; }

static int64_t layer_ws_bytes(const ea_layer_desc* desc, int32_t B, int32_t n_splits, int32_t q_dim) {
  return align256(ea_decode_workspace_bytes(desc, B, n_splits)) + align256((int64_t)B * desc->n_heads * q_dim * 4) +
         align256((int64_t)B * desc->n_heads * desc->r_v * 4);
}

int64_t ea_decode_layer_workspace_bytes(const ea_layer_desc* desc, int32_t B, int32_t n_splits, int32_t rotary) {
  if (validate_desc(desc) != EA_OK || B <= 0 || n_splits < 1 || n_splits > 1024) return -1;
  return layer_ws_bytes(desc, B, n_splits, rotary ? desc->d_head : desc->r_k);
}

// Polls of the arrival counter after which a waiting workgroup of the two-launch step gives up.
static uint32_t g_wait_limit = 1u << 20;

int ea_set_wait_limit(uint32_t polls) {
  if (polls == 0) return EA_ERR_ARG;
  g_wait_limit = polls;
  return EA_OK;
}

static int64_t fused_sync_bytes(const ea_layer_desc* desc, int32_t B) {
  return align256(4 * (1 + (int64_t)B * desc->n_kv_heads));
}

// Workgroups of the second launch that go on to the output projection.  They wait for the rest of the grid, so
// they may hold at most half of the chip's resident workgroup slots (2 per compute unit): then every workgroup
// they wait for finds a slot.  (Workgroups go to the chip's eight dies in turn and each die dispatches its share in
// order, so the bound holds per die as well: the waiting workgroups are the last of every die's share.)
int32_t ea_decode_layer_fused_workers(const ea_layer_desc* desc, int32_t B, int32_t n_splits) {
  if (validate_desc(desc) != EA_OK || B <= 0 || n_splits < 1) return -1;
  const int64_t n_wgs = (int64_t)desc->n_kv_heads * n_splits * B;
  int64_t n_work = desc->d_model / 16;
  if (n_work > n_wgs) n_work = n_wgs;
  if (n_work > resident_compute_units()) n_work = resident_compute_units();
  return (int32_t)(n_work < 1 ? 1 : n_work);
}

int64_t ea_decode_layer_fused_workspace_bytes(const ea_layer_desc* desc, int32_t B, int32_t n_splits, int32_t rotary) {
  if (validate_desc(desc) != EA_OK || B <= 0 || B > 16 || n_splits < 1 || n_splits > 1024) return -1;
  return layer_ws_bytes(desc, B, n_splits, rotary ? desc->d_head : desc->r_k) + fused_sync_bytes(desc, B);
}

static int decode_layer_impl(const ea_layer_desc* desc, bool rope, bool fused, const void* dev_x, const void* dev_wqkv,
                             const void* dev_wo, const void* dev_u_k, double rope_base, void* dev_k_pool,
                             void* dev_v_pool, const int32_t* dev_page_table, const int32_t* dev_seq_len, void* dev_y,
                             int32_t B, int32_t max_pages, int32_t pool_pages, int32_t n_splits, void* dev_ws,
                             int64_t ws_bytes, int32_t* dev_status, void* stream,
                             const float* dev_slopes = nullptr) {
  int rc = validate_desc(desc);
  if (rc != EA_OK) return rc;
  if (desc->dtype != EA_BF16) return EA_ERR_SHAPE;
  if (!dev_x || !dev_wqkv || !dev_wo || !dev_k_pool || !dev_v_pool || !dev_page_table || !dev_seq_len || !dev_y ||
      (rope && !dev_u_k))
    return EA_ERR_ARG;
  if (B <= 0 || B > 64 || max_pages <= 0 || pool_pages <= 0 || n_splits < 0 || n_splits > 1024) return EA_ERR_ARG;
  if (rope && (!(rope_base > 1.0) || !(rope_base < 1e30))) return EA_ERR_ARG;
  if (rope && (desc->r_k > desc->d_head || (desc->d_head != 64 && desc->d_head != 128))) return EA_ERR_SHAPE;
  if (!aligned16(dev_x) || !aligned16(dev_wqkv) || !aligned16(dev_wo) || !aligned16(dev_k_pool) ||
      !aligned16(dev_v_pool) || !aligned16(dev_y) || (rope && !aligned16(dev_u_k)))
    return EA_ERR_ALIGN;
  if ((desc->n_heads * desc->r_v) % 32 != 0 || desc->d_model % 32 != 0) return EA_ERR_SHAPE;
  if (n_splits == 0) {
    const int64_t cap_tokens = (int64_t)max_pages * desc->page_tokens;
    const int32_t cap32 = cap_tokens > INT32_MAX ? INT32_MAX : (int32_t)cap_tokens;
    n_splits = rope ? ea_decode_rope_auto_splits(desc, B, cap32) : ea_decode_auto_splits(desc, B, cap32);
  }
  const int32_t q_dim = rope ? desc->d_head : desc->r_k;
  if (!dev_ws || (reinterpret_cast<uintptr_t>(dev_ws) & 255u)) return EA_ERR_WORKSPACE;
  if (ws_bytes < layer_ws_bytes(desc, B, n_splits, q_dim) + (fused ? fused_sync_bytes(desc, B) : 0))
    return EA_ERR_WORKSPACE;
  if (fused) {
    if (B > 16 || desc->d_model % 16 != 0 || n_splits > kTailMaxSplits) return EA_ERR_SHAPE;
    if (ea_decode_workspace_bytes(desc, B, n_splits) >= (int64_t)1 << 31) return EA_ERR_SHAPE;   // 32-bit offsets into the partials
    if (dev_status && (reinterpret_cast<uintptr_t>(dev_status) & 3u)) return EA_ERR_ALIGN;
  }
  char* w = (char*)dev_ws;
  float* part = (float*)w;                                   // split partials (nothing when n_splits == 1)
  w += align256(ea_decode_workspace_bytes(desc, B, n_splits));
  float* q = (float*)w;
  w += align256((int64_t)B * desc->n_heads * q_dim * 4);
  float* o = (float*)w;
  w += align256((int64_t)B * desc->n_heads * desc->r_v * 4);
  uint32_t* sync = (uint32_t*)w;                             // two-launch form only
  hipStream_t st = (hipStream_t)stream;
  const int32_t sync_words = 1 + B * desc->n_kv_heads;
  // a1 + a2: projection and append (two-launch form: its first workgroup also clears the counters of the launch
  // that follows)
  rc = project_qkv_impl(desc, q_dim, dev_x, dev_wqkv, q, EA_F32, dev_k_pool, dev_v_pool, dev_page_table, dev_seq_len, B,
                        1, max_pages, pool_pages, dev_status, stream, fused ? sync : nullptr, fused ? sync_words : 0);
  if (rc != EA_OK) return rc;
  // a3 over the sequences including the token just appended (the kernels add one to the lengths they read)
  Geo g = make_geo(desc, max_pages, pool_pages);
  if (fused) {
    // a3 + merge + a5 in one launch
    TailArgs t;
    t.o = (uint16_t*)o;
    t.w_o = (const uint16_t*)dev_wo;
    t.y = (uint16_t*)dev_y;
    t.N = desc->d_model;
    t.K = desc->n_heads * desc->r_v;
    t.sync = sync;
    t.status = dev_status;
    t.spin_limit = g_wait_limit;
    t.ws_bytes = (uint32_t)ea_decode_workspace_bytes(desc, B, n_splits);
    // the workgroups that go on to the projection wait for the rest of the grid: they may hold at most half of
    // the chip's resident workgroup slots (2 per compute unit), so that everything they wait for can run
    t.n_work = ea_decode_layer_fused_workers(desc, B, n_splits);
    return decode_tail_bf16(desc, g, q, rope ? dev_u_k : nullptr, rope_base, dev_k_pool, dev_v_pool, dev_page_table,
                            dev_seq_len, B, n_splits, part, 1, t, st, dev_slopes);
  }
  // (o is this call's own intermediate: it is kept in bfloat16, rounded once, which the output projection reads
  // faster than float rows)
  if (rope)
    rc = decode_rope_bf16(desc, g, q, dev_u_k, rope_base, dev_k_pool, dev_v_pool, dev_page_table, dev_seq_len, o, B,
                          n_splits, part, st, 0, 0, 1, 1);
  else if (dev_slopes)
    rc = decode_alibi_bf16(desc, g, q, dev_slopes, dev_k_pool, dev_v_pool, dev_page_table, dev_seq_len, o, B, n_splits,
                           part, st, 1, 1);
  else
    rc = decode_bf16(desc, g, q, dev_k_pool, dev_v_pool, dev_page_table, dev_seq_len, o, B, n_splits, part, st, 0, 0, 1,
                     1);
  if (rc != EA_OK) return rc;
  if (n_splits > 1) {
    rc = merge_splits(g, part, o, B, n_splits, st, nullptr, 1);
    if (rc != EA_OK) return rc;
  }
  // a5
  return gemm_out_bf16(o, 0, dev_wo, dev_y, B, desc->d_model, desc->n_heads * desc->r_v, st);
}

int ea_decode_layer(const ea_layer_desc* desc, const void* dev_x, const void* dev_wqkv, const void* dev_wo,
                    void* dev_k_pool, void* dev_v_pool, const int32_t* dev_page_table, const int32_t* dev_seq_len,
                    void* dev_y, int32_t B, int32_t max_pages, int32_t pool_pages, int32_t n_splits, void* dev_ws,
                    int64_t ws_bytes, int32_t* dev_status, void* stream) {
  return decode_layer_impl(desc, false, false, dev_x, dev_wqkv, dev_wo, nullptr, 0.0, dev_k_pool, dev_v_pool,
                           dev_page_table, dev_seq_len, dev_y, B, max_pages, pool_pages, n_splits, dev_ws, ws_bytes,
                           dev_status, stream);
}

int ea_decode_layer_fused(const ea_layer_desc* desc, const void* dev_x, const void* dev_wqkv, const void* dev_wo,
                          void* dev_k_pool, void* dev_v_pool, const int32_t* dev_page_table,
                          const int32_t* dev_seq_len, void* dev_y, int32_t B, int32_t max_pages, int32_t pool_pages,
                          int32_t n_splits, void* dev_ws, int64_t ws_bytes, int32_t* dev_status, void* stream) {
  return decode_layer_impl(desc, false, true, dev_x, dev_wqkv, dev_wo, nullptr, 0.0, dev_k_pool, dev_v_pool,
                           dev_page_table, dev_seq_len, dev_y, B, max_pages, pool_pages, n_splits, dev_ws, ws_bytes,
                           dev_status, stream);
}

int ea_decode_layer_fused_rope(const ea_layer_desc* desc, const void* dev_x, const void* dev_wqkv, const void* dev_wo,
                               const void* dev_u_k, double rope_base, void* dev_k_pool, void* dev_v_pool,
                               const int32_t* dev_page_table, const int32_t* dev_seq_len, void* dev_y, int32_t B,
                               int32_t max_pages, int32_t pool_pages, int32_t n_splits, void* dev_ws, int64_t ws_bytes,
                               int32_t* dev_status, void* stream) {
  return decode_layer_impl(desc, true, true, dev_x, dev_wqkv, dev_wo, dev_u_k, rope_base, dev_k_pool, dev_v_pool,
                           dev_page_table, dev_seq_len, dev_y, B, max_pages, pool_pages, n_splits, dev_ws, ws_bytes,
                           dev_status, stream);
}

int ea_decode_layer_alibi(const ea_layer_desc* desc, const void* dev_x, const void* dev_wqkv, const void* dev_wo,
                          const float* dev_slopes, void* dev_k_pool, void* dev_v_pool, const int32_t* dev_page_table,
                          const int32_t* dev_seq_len, void* dev_y, int32_t B, int32_t max_pages, int32_t pool_pages,
                          int32_t n_splits, void* dev_ws, int64_t ws_bytes, int32_t* dev_status, void* stream) {
  if (!dev_slopes) return EA_ERR_ARG;
  return decode_layer_impl(desc, false, false, dev_x, dev_wqkv, dev_wo, nullptr, 0.0, dev_k_pool, dev_v_pool,
                           dev_page_table, dev_seq_len, dev_y, B, max_pages, pool_pages, n_splits, dev_ws, ws_bytes,
                           dev_status, stream, dev_slopes);
}

int ea_decode_layer_fused_alibi(const ea_layer_desc* desc, const void* dev_x, const void* dev_wqkv, const void* dev_wo,
                                const float* dev_slopes, void* dev_k_pool, void* dev_v_pool,
                                const int32_t* dev_page_table, const int32_t* dev_seq_len, void* dev_y, int32_t B,
                                int32_t max_pages, int32_t pool_pages, int32_t n_splits, void* dev_ws, int64_t ws_bytes,
                                int32_t* dev_status, void* stream) {
  if (!dev_slopes) return EA_ERR_ARG;
  return decode_layer_impl(desc, false, true, dev_x, dev_wqkv, dev_wo, nullptr, 0.0, dev_k_pool, dev_v_pool,
                           dev_page_table, dev_seq_len, dev_y, B, max_pages, pool_pages, n_splits, dev_ws, ws_bytes,
                           dev_status, stream, dev_slopes);
}

int ea_decode_layer_rope(const ea_layer_desc* desc, const void* dev_x, const void* dev_wqkv, const void* dev_wo,
                         const void* dev_u_k, double rope_base, void* dev_k_pool, void* dev_v_pool,
                         const int32_t* dev_page_table, const int32_t* dev_seq_len, void* dev_y, int32_t B,
                         int32_t max_pages, int32_t pool_pages, int32_t n_splits, void* dev_ws, int64_t ws_bytes,
                         int32_t* dev_status, void* stream) {
  return decode_layer_impl(desc, true, false, dev_x, dev_wqkv, dev_wo, dev_u_k, rope_base, dev_k_pool, dev_v_pool,
                           dev_page_table, dev_seq_len, dev_y, B, max_pages, pool_pages, n_splits, dev_ws, ws_bytes,
                           dev_status, stream);
}

}  // extern "C"
