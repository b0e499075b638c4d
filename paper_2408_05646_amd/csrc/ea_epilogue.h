// Where one element of the fused QKV projection goes: q to the dense q_r tensor,
// k and v to their slot of the rank-r paged cache (K <- Concat(K, k), paged).
#pragma once
#include "ea_common.h"

namespace ea {

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float x) {
  __bf16 h = (__bf16)x;   // round to nearest even
  return __builtin_bit_cast(uint16_t, h);
}

template <bool BF16_CACHE>
__device__ __forceinline__ void cache_put(void* pool, int64_t off, float v) {
  if (BF16_CACHE) reinterpret_cast<uint16_t*>(pool)[off] = f32_to_bf16_rne(v);
  else reinterpret_cast<float*>(pool)[off] = v;
}

// One (sequence, token) append could not be stored (its position lies beyond the page table, or the table
// names a page outside the pool): counted in the caller's status word, if there is one.
__device__ __forceinline__ void qkv_report_drop(const QkvDest& d) {
  if (d.status) atomicAdd(d.status, 1);
}

// Cache page and offset inside it of row (= b*T + t) of the projection; page -1 = the token cannot be stored.
struct QkvRow {
  int32_t page, tp;
};
__device__ __forceinline__ QkvRow qkv_row(const QkvDest& d, int32_t row) {
  const Geo& g = d.g;
  const int32_t b = row / d.T, t = row % d.T;
  const int64_t pos = (int64_t)d.seq_len[b] + t;
  QkvRow r{-1, 0};
  if (pos < 0) return r;
  const int64_t lp = pos / g.page_tokens;
  if (lp >= g.max_pages) return r;
  const int32_t page = d.page_table[(int64_t)b * g.max_pages + lp];
  if (page < 0 || page >= g.pool_pages) return r;
  r.page = page;
  r.tp = (int32_t)(pos % g.page_tokens);
  return r;
}

// Which part of the concatenated [q | k | v] projection an output channel belongs to.
struct QkvCol {
  int32_t kind;          // 0 = q, 1 = k, 2 = v
  int32_t kvh, c;        // kv head and channel inside it (k, v); for q: c = the column itself
  int32_t r, r_pad;
};
__device__ __forceinline__ QkvCol qkv_col(const QkvDest& d, int32_t col) {
  const Geo& g = d.g;
  const int32_t nq = g.n_heads * g.q_dim;
  if (col < nq) return QkvCol{0, 0, col, 0, 0};
  int32_t cc = col - nq;
  const int32_t nk = g.n_kv_heads * g.r_k;
  const bool is_k = cc < nk;
  if (!is_k) cc -= nk;
  const int32_t r = is_k ? g.r_k : g.r_v;
  return QkvCol{is_k ? 1 : 2, cc / r, cc % r, r, is_k ? g.r_k_pad : g.r_v_pad};
}

// Store one element given its row's place in the cache and its column's section.
template <bool BF16_CACHE>
__device__ __forceinline__ void qkv_put(const QkvDest& d, const QkvCol& cl, const QkvRow& rw, int32_t row, float val) {
  const Geo& g = d.g;
  if (cl.kind == 0) {
    const int64_t idx = (int64_t)row * (g.n_heads * g.q_dim) + cl.c;
    if (d.q_is_f32) reinterpret_cast<float*>(d.q)[idx] = val;
    else reinterpret_cast<uint16_t*>(d.q)[idx] = f32_to_bf16_rne(val);
    return;
  }
  if (rw.page < 0) return;
  const bool is_k = cl.kind == 1;
  void* pool = is_k ? d.k_pool : d.v_pool;
  const int64_t base = (int64_t)rw.page * (is_k ? g.k_page : g.v_page) + (int64_t)cl.kvh * (is_k ? g.k_slab : g.v_slab);
  auto off = [&](int32_t ch) -> int64_t {
    if (!BF16_CACHE) return base + f32_slab_off(rw.tp, ch, cl.r_pad);
    return base + (is_k ? bf16_k_slab_off(rw.tp, ch, cl.r_pad) : bf16_v_slab_off(rw.tp, ch, cl.r_pad));
  };
  cache_put<BF16_CACHE>(pool, off(cl.c), val);
  if (cl.c == cl.r - 1)
    for (int32_t ch = cl.r; ch < cl.r_pad; ++ch) cache_put<BF16_CACHE>(pool, off(ch), 0.f);   // padding channels stay zero
}

// row = b*T + t of x, col = output channel of the concatenated [q | k | v] projection.
// The lane that holds the first key channel of a token reports a dropped append (once per token).
template <bool BF16_CACHE>
__device__ __forceinline__ void qkv_store(const QkvDest& d, int32_t row, int32_t col, float val) {
  const QkvCol cl = qkv_col(d, col);
  if (cl.kind == 0) {
    qkv_put<BF16_CACHE>(d, cl, QkvRow{-1, 0}, row, val);
    return;
  }
  const QkvRow rw = qkv_row(d, row);
  if (rw.page < 0) {
    if (cl.kind == 1 && cl.kvh == 0 && cl.c == 0) qkv_report_drop(d);
    return;
  }
  qkv_put<BF16_CACHE>(d, cl, rw, row, val);
}

}  // namespace ea
