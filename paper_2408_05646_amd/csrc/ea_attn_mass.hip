// Attention mass per cached token: mass[b, g, t] += sum over the query heads i of kv head g of p_i[t], with
// p_i = Softmax(q_r,i . K_r[g]^T / sqrt(d_h)) of Eq. (3) in the rank-r space (Eq. 7).  This is the statistic
// H2O-style token eviction accumulates (results, "Eigen Attention with token pruning"); the policy itself (which
// token to drop, where the next one is written) is the caller's: a dropped token's slot is simply overwritten by
// the next append, because the position-free cache does not care where a token sits.
//
// Two kernels, one pass over the keys (the values are not touched):
//   tile kernel  : 64-token tiles of one (sequence, kv head), each on its own: scores on the matrix cores, the tile's
//                  own maximum m, e_t = 2^(s_t - m), l = sum_t e_t  ->  e [B, H, n_cap] and (m, l) [B, H, tiles]
//   finish kernel: 4096 tokens of one (sequence, kv head) per workgroup: M = max over tiles of m and
//                  L = sum_tiles l 2^(m - M) per head (every workgroup for itself), then
//                  mass[t] += sum_heads e_t 2^(m_tile(t) - M) / L
// Algorithmic bytes per (sequence, kv head, token): r_k * 2 (keys) + G * 8 (e written and read again) + 8 (mass).
#include "ea_common.h"

namespace ea {


struct MassArgs {
  const float* q;            // [B, H, r_k]
  const void* k_pool;
  const int32_t* page_table;
  const int32_t* seq_len;
  float* e;                  // [B, H, e_row]
  float* ml;                 // [B, H, tiles_cap, 2]
  float* mass;               // [B, H_kv, n_cap]
  Geo g;
  int32_t n_cap;             // max_pages * page_tokens: row length of mass, and the bound of seq_len
  int32_t e_row;             // row length of e: mass_row_floats(n_cap)
  int32_t tiles_cap;         // ceil(n_cap / 64)
  int32_t tiles_wg;          // tiles of one (sequence, kv head) per workgroup of the bf16 tile kernel
  float scale_log2;
};

__device__ __forceinline__ int mass_len(const MassArgs& a, int b) {
  int64_t n = a.seq_len[b];
  if (n > a.n_cap) n = a.n_cap;
  if (n < 0) n = 0;
  return (int)n;
}

// Sum over the lanes l, l^16, l^32, l^48 (the four register quads of one MFMA result column).
__device__ __forceinline__ float quad_column_sum(float x) {
  typedef __attribute__((ext_vector_type(2))) unsigned u2;
  unsigned xi = __builtin_bit_cast(unsigned, x);
  u2 a = __builtin_amdgcn_permlane16_swap(xi, xi, false, false);
  x = __builtin_bit_cast(float, (unsigned)a[0]) + __builtin_bit_cast(float, (unsigned)a[1]);
  xi = __builtin_bit_cast(unsigned, x);
  u2 b = __builtin_amdgcn_permlane32_swap(xi, xi, false, false);
  return __builtin_bit_cast(float, (unsigned)b[0]) + __builtin_bit_cast(float, (unsigned)b[1]);
}

// ---- bf16 cache: the same fragments and score products as the decode kernel.  A workgroup of four waves takes
// tiles_wg consecutive tiles of one (sequence, kv head); a wave walks every fourth of them and requests the keys
// of its next tile as soon as the score products have consumed the current one's.  Tiles are independent: no running state.

template <int KS>
__global__ __launch_bounds__(256, KS <= 3 ? 4 : 2) void mass_tile_bf16_kernel(MassArgs a) {
  const Geo& g = a.g;
  const int kvh = blockIdx.x, chunk = blockIdx.y, b = blockIdx.z;
  const int lane = threadIdx.x & 63, col = lane & 15, quad = lane >> 4;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int G = g.group;
  const int n = mass_len(a, b);
  const int n_tiles = (n + kTile - 1) / kTile;
  const int t_end = min(n_tiles, (chunk + 1) * a.tiles_wg);
  int tile = chunk * a.tiles_wg + wave;
  if (tile >= t_end) return;
  const int tiles_per_page = g.page_tokens / kTile;
  const int nck = g.r_k_pad >> 3;
  const int32_t* pt_row = a.page_table + (int64_t)b * g.max_pages;

  bf16x8 qhi[KS], qlo[KS];
  {
    const float* qrow = a.q + ((int64_t)b * g.n_heads + (int64_t)kvh * G + (col < G ? col : 0)) * g.r_k;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int k = ks * 32 + quad * 8 + j;
        const float v = (col < G && k < g.r_k) ? qrow[k < g.r_k ? k : 0] * a.scale_log2 : 0.f;
        const __bf16 hi = (__bf16)v;
        qhi[ks][j] = hi;
        qlo[ks][j] = (__bf16)(v - (float)hi);
      }
  }
  // a tile without a valid page is read from page 0 and masked
  auto page_of = [&](int t) -> int {
    const int page = pt_row[t / tiles_per_page];
    return (page >= 0 && page < g.pool_pages) ? page : -1;
  };
  auto load_k = [&](int t, int page, bf16x8 (&kf)[4][KS]) {
    const uint16_t* base = reinterpret_cast<const uint16_t*>(a.k_pool) + (int64_t)page * g.k_page +
                           (int64_t)kvh * g.k_slab + (int64_t)(t % tiles_per_page) * (kTile * g.r_k_pad);
#pragma unroll
    for (int tb = 0; tb < 4; ++tb)
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const bool past = ks == KS - 1 && ks * 4 + quad >= nck;    // chunks the rank does not have
        const int off = past ? (((tb + 1) * nck - 1) * 16 + col) << 3 : ((tb * nck * 16 + ks * 64) << 3) + (lane << 3);
        const bf16x8 got = __builtin_nontemporal_load(reinterpret_cast<const bf16x8*>(base + off));
        kf[tb][ks] = past ? zero_frag() : got;
      }
  };
  bf16x8 kf[4][KS];
  int page = page_of(tile);
  load_k(tile, max(page, 0), kf);
  while (true) {
    f32x4 s[4];
#pragma unroll
    for (int tb = 0; tb < 4; ++tb) {
      s[tb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        s[tb] = mfma16(kf[tb][ks], qhi[ks], s[tb]);
        s[tb] = mfma16(kf[tb][ks], qlo[ks], s[tb]);
      }
    }
    // the keys are used up: the next tile's may come in while this tile's softmax runs (the last tile asks for
    // itself again, which keeps the request out of a branch)
    const int t = tile, pg = page;
    const bool more = tile + 4 < t_end;
    tile = more ? tile + 4 : tile;
    page = page_of(tile);
    load_k(tile, max(page, 0), kf);

    // lane (col = head, quad): tokens 16*tb + 4*quad + i
    const int rem = pg >= 0 ? n - t * kTile : 0;
    float mx = -INFINITY;
#pragma unroll
    for (int tb = 0; tb < 4; ++tb)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if (tb * 16 + quad * 4 + i >= rem) s[tb][i] = -INFINITY;
        mx = fmaxf(mx, s[tb][i]);
      }
    mx = quad_column_max(mx);
    const float m_use = mx == -INFINITY ? 0.f : mx;
    float l = 0.f;
#pragma unroll
    for (int tb = 0; tb < 4; ++tb)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        s[tb][i] = __builtin_amdgcn_exp2f(s[tb][i] - m_use);
        l += s[tb][i];
      }
    l = quad_column_sum(l);
    if (col < G) {
      const int head = kvh * G + col;
      float* erow = a.e + ((int64_t)b * g.n_heads + head) * a.e_row + (int64_t)t * kTile;
#pragma unroll
      for (int tb = 0; tb < 4; ++tb) __builtin_nontemporal_store(s[tb], reinterpret_cast<f32x4*>(erow + tb * 16 + quad * 4));
      if (quad == 0) {
        float* p = a.ml + (((int64_t)b * g.n_heads + head) * a.tiles_cap + t) * 2;
        p[0] = mx;
        p[1] = l;
      }
    }
    if (!more) break;
  }
}

// ---- fp32 cache: one wave per 64 tokens, one token per lane, head after head
__global__ __launch_bounds__(64) void mass_tile_f32_kernel(MassArgs a) {
  const Geo& g = a.g;
  const int tile = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z;
  const int lane = threadIdx.x;
  const int n = mass_len(a, b);
  if (tile * kTile >= n) return;
  const int t = tile * kTile + lane;
  const float* krow = nullptr;
  if (t < n) {
    const int page = a.page_table[(int64_t)b * g.max_pages + t / g.page_tokens];
    if (page >= 0 && page < g.pool_pages)
      krow = reinterpret_cast<const float*>(a.k_pool) + (int64_t)page * g.k_page + (int64_t)kvh * g.k_slab +
             f32_slab_off(t % g.page_tokens, 0, g.r_k_pad);
  }
  for (int hd = 0; hd < g.group; ++hd) {
    const int head = kvh * g.group + hd;
    const float* qrow = a.q + ((int64_t)b * g.n_heads + head) * g.r_k;
    float s = -INFINITY;
    if (krow) {
      float dot = 0.f;
      for (int c = 0; c < g.r_k; ++c) dot = fmaf(qrow[c], krow[c], dot);
      s = dot * a.scale_log2;
    }
    float mx = s;
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
    const float e = __builtin_amdgcn_exp2f(s - (mx == -INFINITY ? 0.f : mx));
    float l = e;
    for (int o = 32; o > 0; o >>= 1) l += __shfl_xor(l, o);
    a.e[((int64_t)b * g.n_heads + head) * a.e_row + t] = e;      // rows of e hold whole tiles
    if (lane == 0) {
      float* p = a.ml + (((int64_t)b * g.n_heads + head) * a.tiles_cap + tile) * 2;
      p[0] = mx;
      p[1] = l;
    }
  }
}

// ---- finish: normalise across tiles and accumulate
constexpr int kFinishTokens = 4096;      // tokens of one (sequence, kv head) per workgroup of the finish kernel

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

// Every workgroup works out the row maximum and normaliser of its kv head's query heads for itself (two floats per
// tile and head: little next to the tokens it then walks) and adds its share of the tokens, four per thread and step.
__global__ __launch_bounds__(256) void mass_finish_kernel(MassArgs a) {
  __shared__ float red[2][16][4];
  const Geo& g = a.g;
  const int chunk = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, wave = tid >> 6;
  const int n = mass_len(a, b);
  const int t0 = chunk * kFinishTokens;
  if (t0 >= n) return;
  const int n_tiles = (n + kTile - 1) / kTile;
  const int G = g.group;
  const int64_t bh0 = (int64_t)b * g.n_heads + (int64_t)kvh * G;
  for (int hd = 0; hd < G; ++hd) {
    const float* ml = a.ml + (bh0 + hd) * a.tiles_cap * 2;
    float mx = -INFINITY;
    for (int t = tid; t < n_tiles; t += 256) mx = fmaxf(mx, ml[2 * t]);
    mx = wave_max(mx);
    if ((tid & 63) == 0) red[0][hd][wave] = mx;
  }
  __syncthreads();
  for (int hd = 0; hd < G; ++hd) {
    const float* ml = a.ml + (bh0 + hd) * a.tiles_cap * 2;
    const float M = fmaxf(fmaxf(red[0][hd][0], red[0][hd][1]), fmaxf(red[0][hd][2], red[0][hd][3]));
    float ls = 0.f;
    if (M != -INFINITY)
      for (int t = tid; t < n_tiles; t += 256) ls += ml[2 * t + 1] * __builtin_amdgcn_exp2f(ml[2 * t] - M);
    ls = wave_sum(ls);
    if ((tid & 63) == 0) red[1][hd][wave] = ls;
  }
  __syncthreads();
  float* mrow = a.mass + ((int64_t)b * g.n_kv_heads + kvh) * a.n_cap;
  const int t_end = min(n, t0 + kFinishTokens);
  for (int t = t0 + tid * 4; t < t_end; t += 1024) {
    const int tile = t >> 6;
    f32x4 w = {0.f, 0.f, 0.f, 0.f};
    for (int hd = 0; hd < G; ++hd) {
      const float M = fmaxf(fmaxf(red[0][hd][0], red[0][hd][1]), fmaxf(red[0][hd][2], red[0][hd][3]));
      const float L = (red[1][hd][0] + red[1][hd][1]) + (red[1][hd][2] + red[1][hd][3]);
      const float m = a.ml[((bh0 + hd) * a.tiles_cap + tile) * 2];
      if (m != -INFINITY && L > 0.f) {
        const float f = __builtin_amdgcn_exp2f(m - M) / L;
        const f32x4 ev = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(a.e + (bh0 + hd) * a.e_row + t));
        w += ev * f;
      }
    }
    // entries past the sequence's end are exp2(-inf) = 0 in e, but they are not this call's to touch
    if (t + 4 <= n) {
      f32x4* p = reinterpret_cast<f32x4*>(mrow + t);
      *p = *p + w;
    } else {
      for (int i = 0; t + i < n; ++i) mrow[t + i] += w[i];
    }
  }
}

// The finish of the fused form: the decode kernel has stored the scores s (log2 units, masked tokens -inf) and the
// split merge each row's reference exponent M and normaliser L;  mass[t] += sum_heads 2^(s_t - M) / L.
struct MassFromScoresArgs {
  const float* scores;       // [B, H, s_row]
  const float* ml;           // [B, H, 2]
  const int32_t* seq_len;
  float* mass;               // [B, H_kv, n_cap]
  int32_t n_heads, n_kv_heads, group, n_cap, s_row;
};

__global__ __launch_bounds__(256) void mass_from_scores_kernel(MassFromScoresArgs a) {
  const int chunk = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z;
  int n = a.seq_len[b];
  n = n < 0 ? 0 : (n > a.n_cap ? a.n_cap : n);
  const int t0 = chunk * kFinishTokens;
  if (t0 >= n) return;
  const int t_end = min(n, t0 + kFinishTokens);
  const int64_t bh0 = (int64_t)b * a.n_heads + (int64_t)kvh * a.group;
  float* mrow = a.mass + ((int64_t)b * a.n_kv_heads + kvh) * a.n_cap;
  for (int t = t0 + threadIdx.x * 4; t < t_end; t += 1024) {
    f32x4 w = {0.f, 0.f, 0.f, 0.f};
    for (int hd = 0; hd < a.group; ++hd) {
      const float M = a.ml[2 * (bh0 + hd)], L = a.ml[2 * (bh0 + hd) + 1];
      if (M != -INFINITY && L > 0.f) {
        const f32x4 sv = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(a.scores + (bh0 + hd) * a.s_row + t));
        const float inv = 1.0f / L;
#pragma unroll
        for (int i = 0; i < 4; ++i) w[i] += __builtin_amdgcn_exp2f(sv[i] - M) * inv;
      }
    }
    if (t + 4 <= n) {
      f32x4* p = reinterpret_cast<f32x4*>(mrow + t);
      *p = *p + w;
    } else {
      for (int i = 0; t + i < n; ++i) mrow[t + i] += w[i];
    }
  }
}

int mass_from_scores(const Geo& g, const float* scores, const float* ml, const int32_t* seq_len, float* mass, int32_t B,
                     int32_t n_cap, int32_t s_row, hipStream_t st) {
  MassFromScoresArgs a;
  a.scores = scores;
  a.ml = ml;
  a.seq_len = seq_len;
  a.mass = mass;
  a.n_heads = g.n_heads;
  a.n_kv_heads = g.n_kv_heads;
  a.group = g.group;
  a.n_cap = n_cap;
  a.s_row = s_row;
  mass_from_scores_kernel<<<dim3((uint32_t)((n_cap + kFinishTokens - 1) / kFinishTokens), g.n_kv_heads, B), dim3(256), 0,
                            st>>>(a);
  return launch_status();
}

static int64_t mass_ws_floats(const ea_layer_desc* d, int32_t B, int32_t max_pages) {
  const int64_t n_cap = (int64_t)max_pages * d->page_tokens;
  const int64_t tiles = (n_cap + kTile - 1) / kTile;
  // e is sized for whole tiles, so the tile kernels may write a full 64-token row at the end of a sequence
  return (int64_t)B * d->n_heads * (mass_row_floats(n_cap) + tiles * 2);
}

}  // namespace ea

using namespace ea;

extern "C" {

int64_t ea_attn_mass_workspace_bytes(const ea_layer_desc* desc, int32_t B, int32_t max_pages) {
  if (validate_desc(desc) != EA_OK || B <= 0 || max_pages <= 0) return -1;
  return mass_ws_floats(desc, B, max_pages) * (int64_t)sizeof(float);
}

int ea_attn_mass(const ea_layer_desc* desc, const float* dev_q_r, const void* dev_k_pool, const int32_t* dev_page_table,
                 const int32_t* dev_seq_len, float* dev_mass, int32_t B, int32_t max_pages, int32_t pool_pages,
                 void* dev_ws, int64_t ws_bytes, void* stream) {
  int rc = validate_desc(desc);
  if (rc != EA_OK) return rc;
  if (!dev_q_r || !dev_k_pool || !dev_page_table || !dev_seq_len || !dev_mass) return EA_ERR_ARG;
  if (B <= 0 || max_pages <= 0 || pool_pages <= 0) return EA_ERR_ARG;
  if (!aligned16(dev_q_r) || !aligned16(dev_k_pool) || !aligned16(dev_mass)) return EA_ERR_ALIGN;
  if (!dev_ws || !aligned16(dev_ws) || ws_bytes < ea_attn_mass_workspace_bytes(desc, B, max_pages))
    return EA_ERR_WORKSPACE;
  const int64_t n_cap64 = (int64_t)max_pages * desc->page_tokens;
  if (n_cap64 > (int64_t)INT32_MAX - 2048) return EA_ERR_SHAPE;
  const Geo g = make_geo(desc, max_pages, pool_pages);
  if (B > 65535 || g.n_kv_heads > 65535 || g.group > 16) return EA_ERR_SHAPE;
  MassArgs a;
  a.q = dev_q_r;
  a.k_pool = dev_k_pool;
  a.page_table = dev_page_table;
  a.seq_len = dev_seq_len;
  a.g = g;
  a.n_cap = (int32_t)n_cap64;
  a.tiles_cap = (a.n_cap + kTile - 1) / kTile;
  a.e_row = (int32_t)mass_row_floats(a.n_cap);
  a.e = (float*)dev_ws;
  a.ml = a.e + (int64_t)B * g.n_heads * a.e_row;
  a.mass = dev_mass;
  a.scale_log2 = 1.4426950408889634f / sqrtf((float)desc->d_head);
  hipStream_t st = (hipStream_t)stream;
  clear_stale_error();
  if (desc->dtype == EA_BF16) {
    // few enough workgroups that each wave walks a run of tiles, enough of them to fill the chip
    const int64_t all_tiles = (int64_t)a.tiles_cap * g.n_kv_heads * B;
    a.tiles_wg = 16;
    while (a.tiles_wg < 128 && all_tiles / a.tiles_wg > 1024) a.tiles_wg *= 2;
    if ((a.tiles_cap + a.tiles_wg - 1) / a.tiles_wg > 65535) return EA_ERR_SHAPE;
    const dim3 grid(g.n_kv_heads, (a.tiles_cap + a.tiles_wg - 1) / a.tiles_wg, B);
    switch ((g.r_k_pad + 31) / 32) {
      case 1: mass_tile_bf16_kernel<1><<<grid, dim3(256), 0, st>>>(a); break;
      case 2: mass_tile_bf16_kernel<2><<<grid, dim3(256), 0, st>>>(a); break;
      case 3: mass_tile_bf16_kernel<3><<<grid, dim3(256), 0, st>>>(a); break;
      case 4: mass_tile_bf16_kernel<4><<<grid, dim3(256), 0, st>>>(a); break;
      default: return EA_ERR_SHAPE;
    }
  } else {
    mass_tile_f32_kernel<<<dim3(a.tiles_cap, g.n_kv_heads, B), dim3(64), 0, st>>>(a);
  }
  rc = launch_status();
  if (rc != EA_OK) return rc;
  mass_finish_kernel<<<dim3((uint32_t)((a.n_cap + kFinishTokens - 1) / kFinishTokens), g.n_kv_heads, B), dim3(256), 0, st>>>(a);
  return launch_status();
}

int64_t ea_decode_attn_mass_workspace_bytes(const ea_layer_desc* desc, int32_t B, int32_t max_pages, int32_t n_splits) {
  if (validate_desc(desc) != EA_OK || B <= 0 || max_pages <= 0 || n_splits < 1 || n_splits > 1024) return -1;
  const int64_t n_cap = (int64_t)max_pages * desc->page_tokens;
  const int64_t s_row = mass_row_floats(n_cap);
  const int64_t partials = ws_floats(B, desc->n_heads, n_splits, round_up(desc->r_v, 16));
  return ((partials + 3) / 4 * 4 + (int64_t)B * desc->n_heads * (s_row + 2)) * (int64_t)sizeof(float);
}

int ea_decode_attn_mass(const ea_layer_desc* desc, const float* dev_q_r, const void* dev_k_pool, const void* dev_v_pool,
                        const int32_t* dev_page_table, const int32_t* dev_seq_len, float* dev_out, float* dev_mass,
                        int32_t B, int32_t max_pages, int32_t pool_pages, int32_t n_splits, void* dev_ws,
                        int64_t ws_bytes, void* stream) {
  int rc = validate_desc(desc);
  if (rc != EA_OK) return rc;
  if (!dev_q_r || !dev_k_pool || !dev_v_pool || !dev_page_table || !dev_seq_len || !dev_out || !dev_mass)
    return EA_ERR_ARG;
  if (B <= 0 || max_pages <= 0 || pool_pages <= 0 || n_splits < 0 || n_splits > 1024) return EA_ERR_ARG;
  if (desc->dtype != EA_BF16) return EA_ERR_SHAPE;      // fp32 layers: ea_decode_attn, then ea_attn_mass
  if (!aligned16(dev_q_r) || !aligned16(dev_k_pool) || !aligned16(dev_v_pool) || !aligned16(dev_out) ||
      !aligned16(dev_mass))
    return EA_ERR_ALIGN;
  const int64_t n_cap64 = (int64_t)max_pages * desc->page_tokens;
  if (n_cap64 > (int64_t)INT32_MAX - 2048) return EA_ERR_SHAPE;
  if (n_splits == 0) n_splits = ea_decode_auto_splits(desc, B, (int32_t)n_cap64);
  if (!dev_ws || !aligned16(dev_ws) || ws_bytes < ea_decode_attn_mass_workspace_bytes(desc, B, max_pages, n_splits))
    return EA_ERR_WORKSPACE;
  const Geo g = make_geo(desc, max_pages, pool_pages);
  if (B > 65535 || g.n_kv_heads > 65535 || g.group > 16) return EA_ERR_SHAPE;
  const int32_t n_cap = (int32_t)n_cap64;
  const int32_t s_row = (int32_t)mass_row_floats(n_cap);
  float* partials = (float*)dev_ws;
  float* scores = partials + (ws_floats(B, g.n_heads, n_splits, g.r_v_pad) + 3) / 4 * 4;   // rows of 16-byte units
  float* ml = scores + (int64_t)B * g.n_heads * s_row;
  hipStream_t st = (hipStream_t)stream;
  clear_stale_error();
  rc = decode_scores_bf16(desc, g, dev_q_r, dev_k_pool, dev_v_pool, dev_page_table, dev_seq_len, B, n_splits, partials,
                          scores, s_row, st);
  if (rc != EA_OK) return rc;
  rc = merge_splits(g, partials, dev_out, B, n_splits, st, ml);
  if (rc != EA_OK) return rc;
  return mass_from_scores(g, scores, ml, dev_seq_len, dev_mass, B, n_cap, s_row, st);
}


}  // extern "C"
