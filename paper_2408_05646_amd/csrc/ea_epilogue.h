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

// row = b*T + t of x, col = output channel of the concatenated [q | k | v] projection.
template <bool BF16_CACHE>
__device__ __forceinline__ void qkv_store(const QkvDest& d, int32_t row, int32_t col, float val) {
  const Geo& g = d.g;
  const int32_t nq = g.n_heads * g.q_dim;
  if (col < nq) {
    const int64_t idx = (int64_t)row * nq + col;
    if (d.q_is_f32) reinterpret_cast<float*>(d.q)[idx] = val;
    else reinterpret_cast<uint16_t*>(d.q)[idx] = f32_to_bf16_rne(val);
    return;
  }
  int32_t cc = col - nq;
  const int32_t nk = g.n_kv_heads * g.r_k;
  const bool is_k = cc < nk;
  if (!is_k) cc -= nk;
  const int32_t r = is_k ? g.r_k : g.r_v;
  const int32_t r_pad = is_k ? g.r_k_pad : g.r_v_pad;
  const int32_t kvh = cc / r, c = cc % r;
  const int32_t b = row / d.T, t = row % d.T;
  const int64_t pos = (int64_t)d.seq_len[b] + t;
  if (pos < 0) return;
  const int64_t lp = pos / g.page_tokens;
  if (lp >= g.max_pages) return;
  const int32_t page = d.page_table[(int64_t)b * g.max_pages + lp];
  if (page < 0 || page >= g.pool_pages) return;
  const int32_t tp = (int32_t)(pos % g.page_tokens);
  void* pool = is_k ? d.k_pool : d.v_pool;
  const int64_t base = (int64_t)page * (is_k ? g.k_page : g.v_page) + (int64_t)kvh * (is_k ? g.k_slab : g.v_slab);
  auto off = [&](int32_t ch) -> int64_t {
    if (!BF16_CACHE) return base + f32_slab_off(tp, ch, r_pad);
    return base + (is_k ? bf16_k_slab_off(tp, ch, r_pad) : bf16_v_slab_off(tp, ch, r_pad));
  };
  cache_put<BF16_CACHE>(pool, off(c), val);
  if (c == r - 1)
    for (int32_t ch = r; ch < r_pad; ++ch) cache_put<BF16_CACHE>(pool, off(ch), 0.f);   // padding channels stay zero
}

// Two-phase form of qkv_store for kernels that know early which elements they will write: qkv_locate does
// the dependent loads (sequence length, page table) and the integer arithmetic while the GEMM's operands
// are still in flight, qkv_commit only converts and stores.
struct QkvSlot {
  void* p;
  int32_t kind;   // 0 = nothing to write, 1 = float, 2 = bfloat16, 3 = take the one-phase path (padding channels)
};

template <bool BF16_CACHE>
__device__ __forceinline__ QkvSlot qkv_locate(const QkvDest& d, int32_t row, int32_t col) {
  const Geo& g = d.g;
  const int32_t nq = g.n_heads * g.q_dim;
  if (col < nq) {
    const int64_t idx = (int64_t)row * nq + col;
    if (d.q_is_f32) return QkvSlot{reinterpret_cast<float*>(d.q) + idx, 1};
    return QkvSlot{reinterpret_cast<uint16_t*>(d.q) + idx, 2};
  }
  int32_t cc = col - nq;
  const int32_t nk = g.n_kv_heads * g.r_k;
  const bool is_k = cc < nk;
  if (!is_k) cc -= nk;
  const int32_t r = is_k ? g.r_k : g.r_v;
  const int32_t r_pad = is_k ? g.r_k_pad : g.r_v_pad;
  const int32_t kvh = cc / r, c = cc % r;
  if (c == r - 1 && r != r_pad) return QkvSlot{nullptr, 3};
  const int32_t b = row / d.T, t = row % d.T;
  const int64_t pos = (int64_t)d.seq_len[b] + t;
  if (pos < 0) return QkvSlot{nullptr, 0};
  const int64_t lp = pos / g.page_tokens;
  if (lp >= g.max_pages) return QkvSlot{nullptr, 0};
  const int32_t page = d.page_table[(int64_t)b * g.max_pages + lp];
  if (page < 0 || page >= g.pool_pages) return QkvSlot{nullptr, 0};
  const int32_t tp = (int32_t)(pos % g.page_tokens);
  const int64_t off = (int64_t)page * (is_k ? g.k_page : g.v_page) + (int64_t)kvh * (is_k ? g.k_slab : g.v_slab) +
                      (!BF16_CACHE ? f32_slab_off(tp, c, r_pad)
                                   : (is_k ? bf16_k_slab_off(tp, c, r_pad) : bf16_v_slab_off(tp, c, r_pad)));
  void* pool = is_k ? d.k_pool : d.v_pool;
  if (BF16_CACHE) return QkvSlot{reinterpret_cast<uint16_t*>(pool) + off, 2};
  return QkvSlot{reinterpret_cast<float*>(pool) + off, 1};
}

template <bool BF16_CACHE>
__device__ __forceinline__ void qkv_commit(const QkvDest& d, const QkvSlot& s, int32_t row, int32_t col, float val) {
  if (s.kind == 1) *reinterpret_cast<float*>(s.p) = val;
  else if (s.kind == 2) *reinterpret_cast<uint16_t*>(s.p) = f32_to_bf16_rne(val);
  else if (s.kind == 3) qkv_store<BF16_CACHE>(d, row, col, val);
}

}  // namespace ea
