// Internal definitions shared by the HIP translation units of libeigenattn.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "eigenattn.h"

namespace ea {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

constexpr int kTile = 64;          // tokens per cache tile of the bf16 layout
constexpr float kLazy = 8.0f;      // the softmax reference exponent moves when the maximum grew by more than 2^kLazy

// Cache geometry, precomputed on the host and passed to kernels by value.
struct Geo {
  int32_t n_heads, n_kv_heads, group;   // group = n_heads / n_kv_heads
  int32_t r_k, r_v, r_k_pad, r_v_pad;
  int32_t q_dim;                        // channels per query head the projection writes: r_k, or d_head (rotary)
  int32_t page_tokens;
  int32_t max_pages, pool_pages;
  int64_t k_slab, v_slab, k_page, v_page;   // elements
};

__host__ __device__ inline int32_t round_up(int32_t x, int32_t m) { return (x + m - 1) / m * m; }

inline int validate_desc(const ea_layer_desc* d) {
  if (!d) return EA_ERR_ARG;
  if (d->dtype != EA_F32 && d->dtype != EA_BF16) return EA_ERR_ARG;
  if (d->d_model <= 0 || d->n_heads <= 0 || d->n_kv_heads <= 0 || d->d_head <= 0 || d->r_k <= 0 || d->r_v <= 0 ||
      d->page_tokens <= 0)
    return EA_ERR_ARG;
  if (d->n_heads % d->n_kv_heads != 0) return EA_ERR_SHAPE;
  if (d->dtype == EA_BF16) {
    if (d->r_k > 128 || d->r_v > 128) return EA_ERR_SHAPE;
    if (d->page_tokens % kTile != 0) return EA_ERR_SHAPE;
    if (d->n_heads / d->n_kv_heads > 16) return EA_ERR_SHAPE;
    if (d->q4_key_group != 0 && d->q4_key_group != 64 && d->q4_key_group != 128) return EA_ERR_ARG;
    if (d->q4_key_group == 128 && d->page_tokens % 128 != 0) return EA_ERR_SHAPE;
    if (d->q4_bits != 0 && d->q4_bits != 4 && d->q4_bits != 3) return EA_ERR_ARG;
  } else {
    if (d->r_k > 256 || d->r_v > 256) return EA_ERR_SHAPE;
    if (d->page_tokens % 16 != 0) return EA_ERR_SHAPE;
  }
  return EA_OK;
}

inline Geo make_geo(const ea_layer_desc* d, int32_t max_pages, int32_t pool_pages) {
  Geo g;
  g.n_heads = d->n_heads;
  g.n_kv_heads = d->n_kv_heads;
  g.group = d->n_heads / d->n_kv_heads;
  g.r_k = d->r_k;
  g.r_v = d->r_v;
  g.q_dim = d->r_k;
  if (d->dtype == EA_BF16) {
    g.r_k_pad = round_up(d->r_k, 8);
    g.r_v_pad = round_up(d->r_v, 16);
  } else {
    g.r_k_pad = round_up(d->r_k, 4);
    g.r_v_pad = round_up(d->r_v, 4);
  }
  g.page_tokens = d->page_tokens;
  g.max_pages = max_pages;
  g.pool_pages = pool_pages;
  g.k_slab = (int64_t)d->page_tokens * g.r_k_pad;
  g.v_slab = (int64_t)d->page_tokens * g.r_v_pad;
  g.k_page = g.k_slab * d->n_kv_heads;
  g.v_page = g.v_slab * d->n_kv_heads;
  return g;
}

// ---- element offsets inside one (page, kv head) slab ------------------------
// fp32 cache: token-major rows.
__host__ __device__ inline int64_t f32_slab_off(int32_t t, int32_t c, int32_t r_pad) { return (int64_t)t * r_pad + c; }

// bf16 K: tiles of 64 tokens; in a tile [4 blocks of 16 tokens][r_pad/8 chunks][16 tokens][8 channels].
__host__ __device__ inline int64_t bf16_k_slab_off(int32_t t, int32_t c, int32_t r_pad) {
  const int32_t tile = t >> 6, tt = t & 63, tb = tt >> 4, row = tt & 15;
  const int32_t nck = r_pad >> 3;
  return (int64_t)tile * (kTile * r_pad) + (((tb * nck + (c >> 3)) * 16 + row) << 3) + (c & 7);
}

// bf16 V: tiles of 64 tokens; in a tile [2 groups of 32 tokens][r_pad/16 blocks][4 quads][16 channels][8 slots],
// slot j of quad q <-> token 16*(j/4) + 4*q + j%4 of the group.
__host__ __device__ inline int64_t bf16_v_slab_off(int32_t t, int32_t c, int32_t r_pad) {
  const int32_t tile = t >> 6, tt = t & 63, grp = tt >> 5, t32 = tt & 31;
  const int32_t half = t32 >> 4, r16 = t32 & 15, quad = r16 >> 2, j = half * 4 + (r16 & 3);
  const int32_t ncb = r_pad >> 4;
  return (int64_t)tile * (kTile * r_pad) + (((((grp * ncb + (c >> 4)) * 4 + quad) * 16 + (c & 15)) << 3) + j);
}

// D[16x16] += A[16x32] . B[32x16] on the matrix cores.  Lane l holds, of A, row l%16 and
// k = 8*(l/16) .. +7; of B, column l%16 and the same k; of D, column l%16 and rows 4*(l/16) .. +3.
__device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ bf16x8 zero_frag() {
  u32x4 z = {0u, 0u, 0u, 0u};
  return __builtin_bit_cast(bf16x8, z);
}

// Maximum over the lanes l, l^16, l^32, l^48: the four register quads that hold one column of an MFMA
// result.  v_permlane16_swap exchanges the odd 16-lane rows of its first operand with the even rows of
// the second, v_permlane32_swap the upper half of the first with the lower half of the second; with both
// operands equal, the two results hold each lane's own value and its partner's.
__device__ __forceinline__ float quad_column_max(float x) {
  typedef __attribute__((ext_vector_type(2))) unsigned u2;
  unsigned xi = __builtin_bit_cast(unsigned, x);
  u2 a = __builtin_amdgcn_permlane16_swap(xi, xi, false, false);
  x = fmaxf(__builtin_bit_cast(float, (unsigned)a[0]), __builtin_bit_cast(float, (unsigned)a[1]));
  xi = __builtin_bit_cast(unsigned, x);
  u2 b = __builtin_amdgcn_permlane32_swap(xi, xi, false, false);
  return fmaxf(__builtin_bit_cast(float, (unsigned)b[0]), __builtin_bit_cast(float, (unsigned)b[1]));
}

// cos and sin of an angle given in REVOLUTIONS.  The whole turns are dropped in double precision (positions
// reach 10^5 and more radians, where single precision no longer resolves the angle); v_cos_f32 / v_sin_f32 take
// the remaining fraction of a turn directly.
__device__ __forceinline__ void rot_turns(double x, float& c, float& s) {
  const float f = (float)(x - rint(x));
  c = __builtin_amdgcn_cosf(f);
  s = __builtin_amdgcn_sinf(f);
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// The HIP runtime keeps the last error of ANY earlier call of the process (another library's
// event query that was not ready, for instance); drop it so launch_status() reports our launches only.
inline void clear_stale_error() { (void)hipGetLastError(); }

inline int launch_status() { return hipGetLastError() == hipSuccess ? EA_OK : EA_ERR_DEVICE; }

// ---- entry points implemented per translation unit --------------------------
int cache_copy(const ea_layer_desc* d, const Geo& g, bool scatter, void* k_dense, void* v_dense, void* k_pool,
               void* v_pool, const int32_t* page_table, int32_t B, int32_t n, int32_t pos0, hipStream_t st);

// ws_slots > 0: write split partials only, into slots ws_slot0 .. of a workspace laid out for ws_slots splits.
int decode_bf16(const ea_layer_desc* d, const Geo& g, const float* q, const void* k_pool, const void* v_pool,
                const int32_t* page_table, const int32_t* seq_len, float* out, int32_t B, int32_t n_splits, float* ws,
                hipStream_t st, int32_t ws_slots = 0, int32_t ws_slot0 = 0, int32_t seq_add = 0, int32_t out_bf16 = 0);
int decode_f32(const ea_layer_desc* d, const Geo& g, const float* q, const float* k_pool, const float* v_pool,
               const int32_t* page_table, const int32_t* seq_len, float* out, int32_t B, int32_t n_splits, float* ws,
               hipStream_t st);
int decode_rope_bf16(const ea_layer_desc* d, const Geo& g, const float* q, const void* u_k, double rope_base,
                     const void* k_pool, const void* v_pool, const int32_t* page_table, const int32_t* seq_len,
                     float* out, int32_t B, int32_t n_splits, float* ws, hipStream_t st, int32_t ws_slots = 0,
                     int32_t ws_slot0 = 0, int32_t seq_add = 0, int32_t out_bf16 = 0);
int decode_rope_f32(const ea_layer_desc* d, const Geo& g, const float* q, const float* u_k, double rope_base,
                    const float* k_pool, const float* v_pool, const int32_t* page_table, const int32_t* seq_len,
                    float* out, int32_t B, int32_t n_splits, float* ws, hipStream_t st);
int decode_alibi_bf16(const ea_layer_desc* d, const Geo& g, const float* q, const float* slopes, const void* k_pool,
                      const void* v_pool, const int32_t* page_table, const int32_t* seq_len, float* out, int32_t B,
                      int32_t n_splits, float* ws, hipStream_t st, int32_t seq_add = 0, int32_t out_bf16 = 0);
int decode_alibi_f32(const ea_layer_desc* d, const Geo& g, const float* q, const float* slopes, const float* k_pool,
                     const float* v_pool, const int32_t* page_table, const int32_t* seq_len, float* out, int32_t B,
                     int32_t n_splits, float* ws, hipStream_t st);
int prefill_alibi_bf16(const ea_layer_desc* d, const Geo& g, const void* q, const float* slopes, const void* k_pool,
                       const void* v_pool, const int32_t* page_table, const int32_t* seq_len, void* out, int32_t B,
                       int32_t n, hipStream_t st);
int prefill_alibi_f32(const ea_layer_desc* d, const Geo& g, const float* q, const float* slopes, const float* k_pool,
                      const float* v_pool, const int32_t* page_table, const int32_t* seq_len, float* out, int32_t B,
                      int32_t n, hipStream_t st);
// The position-free bf16 kernel in the form that also stores the scaled scores (log2 units) [B, H, s_row]; always
// leaves split partials in ws (n_splits slots) for merge_splits.
int decode_scores_bf16(const ea_layer_desc* d, const Geo& g, const float* q, const void* k_pool, const void* v_pool,
                       const int32_t* page_table, const int32_t* seq_len, int32_t B, int32_t n_splits, float* ws,
                       float* scores, int32_t s_row, hipStream_t st);
// The back half of a generation step in one launch (attention over seq_len + seq_add tokens, split merge, output
// projection); u_k = null: position-free form.
constexpr int32_t kStatusWaitExpired = 1 << 30;   // bit of the status word: a bounded wait ran out
constexpr int kTailMaxSplits = 64;                 // splits per sequence the one-launch back half merges
struct TailArgs {
  uint16_t* o;            // [B, H * r_v] bf16: merged attention output (workspace)
  const uint16_t* w_o;    // packed W^O': [N/16][K/32] fragments of 1 KiB
  uint16_t* y;            // [B, N] bf16
  int32_t N, K;           // d_model, H * r_v
  uint32_t* sync;         // [0]: arrivals; [1 + b * H_kv + kv head]: tickets
  int32_t* status;        // or null
  uint32_t spin_limit;
  int32_t n_work;         // workgroups that run the projection: <= N / 16, <= grid size
  uint32_t ws_bytes;      // of the split partials
};
int decode_tail_bf16(const ea_layer_desc* d, const Geo& g, const float* q, const void* u_k, double rope_base,
                     const void* k_pool, const void* v_pool, const int32_t* page_table, const int32_t* seq_len,
                     int32_t B, int32_t n_splits, float* ws, int32_t seq_add, const TailArgs& t, hipStream_t st,
                     const float* slopes = nullptr);   // slopes [H]: the ALiBi form (not with u_k)
int merge_splits(const Geo& g, const float* ws, float* out, int32_t B, int32_t n_splits, hipStream_t st,
                 float* ml_out = nullptr,    // ml_out [B, H, 2]: each row's reference exponent and normaliser, or null
                 int32_t out_bf16 = 0);      // out holds bfloat16 instead of float
// Row length (floats) of the per-head scratch rows e / scores for a cache of n_cap tokens: whole tiles, plus a pad
// of 17 * 256 bytes.  Without it the rows of long sequences start a power of two apart, and all the workgroups,
// which advance through their rows in step, would write to the same memory channel at the same time.
__host__ __device__ inline int64_t mass_row_floats(int64_t n_cap) { return (n_cap + kTile - 1) / kTile * kTile + 1088; }
// mass[b, kv head, t] += sum over the kv head's query heads of 2^(scores[b, head, t] - M) / L, (M, L) = ml[b, head]
int mass_from_scores(const Geo& g, const float* scores, const float* ml, const int32_t* seq_len, float* mass, int32_t B,
                     int32_t n_cap, int32_t s_row, hipStream_t st);

int prefill_bf16(const ea_layer_desc* d, const Geo& g, const void* q, const void* k_pool, const void* v_pool,
                 const int32_t* page_table, const int32_t* seq_len, void* out, int32_t B, int32_t n, hipStream_t st,
                 int32_t k_compact = 0, float* part_o = nullptr, float* part_ml = nullptr);   // part_*: see PrefillArgs
// Rotary prefill (bf16): rotated full-rank keys and rotated queries are written to the workspace, then the
// position-free prefill kernel runs at rank d_head on them.
int64_t prefill_rope_ws_bytes(const ea_layer_desc* d, int32_t B, int32_t n, int32_t max_pages);
int prefill_rope_bf16(const ea_layer_desc* d, const Geo& g, const void* q, const void* u_k, double rope_base,
                      const void* k_pool, const void* v_pool, const int32_t* page_table, const int32_t* seq_len,
                      void* out, int32_t B, int32_t n, void* ws, hipStream_t st);
int prefill_rope_f32(const ea_layer_desc* d, const Geo& g, const float* q, const float* u_k, double rope_base,
                     const float* k_pool, const float* v_pool, const int32_t* page_table, const int32_t* seq_len,
                     float* out, int32_t B, int32_t n, hipStream_t st);
int prefill_f32(const ea_layer_desc* d, const Geo& g, const float* q, const float* k_pool, const float* v_pool,
                const int32_t* page_table, const int32_t* seq_len, float* out, int32_t B, int32_t n, hipStream_t st);

// Destination of the fused QKV GEMM: q goes to a dense tensor, k and v to the paged cache.
struct QkvDest {
  void* q;
  int32_t q_is_f32;
  void* k_pool;
  void* v_pool;
  const int32_t* page_table;
  const int32_t* seq_len;
  int32_t T;
  Geo g;
  int32_t* status = nullptr;   // device word that counts the (sequence, token) appends that could not be stored, or null
  // Generation-phase kernels only (M <= 64): words the first workgroup sets to zero -- the counters of the launch that
  // follows in the same call (a kernel boundary lies between the two, so it finds them cleared).
  uint32_t* clear = nullptr;
  int32_t clear_words = 0;
};
int pack_weight(const void* w_t, void* packed, int32_t N, int32_t K, bool bf16, hipStream_t st);
int gemm_qkv_bf16(const void* x, const void* w_t, int32_t M, int32_t N, int32_t K, const QkvDest& dst, hipStream_t st);
int gemm_qkv_f32(const float* x, const float* w_t, int32_t M, int32_t N, int32_t K, const QkvDest& dst, hipStream_t st);
int gemm_out_bf16(const void* a, int32_t a_is_f32, const void* w_t, void* y, int32_t M, int32_t N, int32_t K,
                  hipStream_t st);
int gemm_out_f32(const float* a, const float* w_t, float* y, int32_t M, int32_t N, int32_t K, hipStream_t st);

// Workspace layout of the split partials: m [B,H,S], l [B,H,S], acc [B,H,S,r_v_pad].
__host__ __device__ inline int64_t ws_floats(int32_t B, int32_t H, int32_t S, int32_t r_v_pad) {
  return (int64_t)B * H * S * (2 + r_v_pad);
}

}  // namespace ea
