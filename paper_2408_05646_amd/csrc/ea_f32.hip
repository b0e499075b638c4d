// fp32 path: straightforward vector-ALU kernels for the reference-precision
// configuration (float cache, float weights).  Token-major cache rows.
#include "ea_common.h"
#include "ea_epilogue.h"

namespace ea {

constexpr int kChunk = 256;   // tokens per step = threads per workgroup

// Score of one cached key against the rank-r query (Eq. 7: q_r . k_r).
struct DotScore {
  const float* sq;   // the query's r_k channels, in LDS
  int r_k;
  __device__ __forceinline__ float operator()(int /*tok*/, const float* __restrict__ krow) const {
    float dot = 0.f;
    for (int c = 0; c < r_k; ++c) dot = fmaf(sq[c], krow[c], dot);
    return dot;
  }
  __device__ __forceinline__ float bias_log2(int /*tok*/) const { return 0.f; }
};

// The same with the ALiBi position bias: -slope * (query position - key position), here in log2 units.
struct AlibiScore {
  const float* sq;
  int r_k;
  float slope_log2;
  int pos_q;
  __device__ __forceinline__ float operator()(int /*tok*/, const float* __restrict__ krow) const {
    float dot = 0.f;
    for (int c = 0; c < r_k; ++c) dot = fmaf(sq[c], krow[c], dot);
    return dot;
  }
  __device__ __forceinline__ float bias_log2(int tok) const { return slope_log2 * (float)(tok - pos_q); }
};

// Score for models with rotary position embedding (Sec. 4.3, Eq. 10): the cached rank-r key is brought back to
// d_head channels with the shared basis U^K, rotated to its position, and multiplied with the query rotated to
// its own position.  Only the difference of the two positions enters, so the key pair is rotated by
// (tok - pos_q) theta_j and the query is left as it is.  After token pruning the key in slot tok is at position
// slot_pos[tok] of the text instead of tok.
struct RopeScore {
  const float* sq;      // the query's d_head channels, in LDS
  const float* u_k;     // [d_head, r_k]
  const double* theta;  // [d_head / 2], in LDS
  int r_k, d_head, pos_q;
  const int32_t* slot_pos = nullptr;   // this sequence's row of positions, or null: slot t holds position t
  __device__ __forceinline__ float operator()(int tok, const float* __restrict__ krow) const {
    float dot = 0.f;
    for (int j = 0; j < d_head / 2; ++j) {
      const float* u0 = u_k + (int64_t)(2 * j) * r_k;
      const float* u1 = u0 + r_k;
      float k0 = 0.f, k1 = 0.f;
      for (int c = 0; c < r_k; ++c) {
        k0 = fmaf(u0[c], krow[c], k0);
        k1 = fmaf(u1[c], krow[c], k1);
      }
      // reduce the angle modulo 2 pi in double precision: positions reach 10^5 radians and more
      const double x = (double)((slot_pos ? slot_pos[tok] : tok) - pos_q) * theta[j];
      const double kq = rint(x * 0.15915494309189535);
      double r = fma(-kq, 6.283185307179586, x);
      r = fma(-kq, 2.4492935982947064e-16, r);
      const float cs = cosf((float)r), sn = sinf((float)r);
      dot = fmaf(sq[2 * j], k0 * cs - k1 * sn, dot);
      dot = fmaf(sq[2 * j + 1], k0 * sn + k1 * cs, dot);
    }
    return dot;
  }
  __device__ __forceinline__ float bias_log2(int /*tok*/) const { return 0.f; }
};

// Online-softmax attention of one query over tokens [tok_begin, tok_end) of sequence b (Eq. 3 / Eq. 2 row).
// Thread t scores token chunk*256 + t; afterwards thread c accumulates value channel c.
// Returns through (m, l, acc): running max (log2 domain), denominator and numerator of channel threadIdx.x.
template <typename Score>
__device__ __forceinline__ void attend_f32(const Score& score, const float* __restrict__ k_pool,
                                           const float* __restrict__ v_pool, const int32_t* __restrict__ pt_row,
                                           const Geo& g, int kvh, int tok_begin, int tok_end, float scale_log2,
                                           float& m_out, float& l_out, float& acc_out) {
  __shared__ float sp[kChunk];
  __shared__ int64_t svoff[kChunk];
  __shared__ float sred[4];
  const int tid = threadIdx.x;
  __syncthreads();
  float m = -INFINITY, l = 0.f, acc = 0.f;
  for (int base = tok_begin; base < tok_end; base += kChunk) {
    const int tok = base + tid;
    float s = -INFINITY;
    int64_t voff = -1;
    if (tok < tok_end) {
      const int lp = tok / g.page_tokens;
      const int page = lp < g.max_pages ? pt_row[lp] : -1;
      if (page >= 0 && page < g.pool_pages) {
        const int tp = tok % g.page_tokens;
        const float* krow = k_pool + (int64_t)page * g.k_page + (int64_t)kvh * g.k_slab + (int64_t)tp * g.r_k_pad;
        s = fmaf(score(tok, krow), scale_log2, score.bias_log2(tok));
        voff = (int64_t)page * g.v_page + (int64_t)kvh * g.v_slab + (int64_t)tp * g.r_v_pad;
      }
    }
    float mx = s;
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
    if ((tid & 63) == 0) sred[tid >> 6] = mx;
    __syncthreads();
    mx = fmaxf(fmaxf(sred[0], sred[1]), fmaxf(sred[2], sred[3]));
    const float m_new = fmaxf(m, mx);
    const float m_use = m_new == -INFINITY ? 0.f : m_new;
    const float alpha = exp2f(m - m_use);
    m = m_new;
    sp[tid] = exp2f(s - m_use);
    svoff[tid] = voff;
    __syncthreads();
    const int cnt = min(kChunk, tok_end - base);
    float psum = 0.f, vsum = 0.f;
    for (int j = 0; j < cnt; ++j) {
      const float p = sp[j];
      psum += p;
      if (tid < g.r_v && svoff[j] >= 0) vsum = fmaf(p, v_pool[svoff[j] + tid], vsum);
    }
    l = l * alpha + psum;
    acc = acc * alpha + vsum;
    __syncthreads();
  }
  m_out = m;
  l_out = l;
  acc_out = acc;
}

struct AttnF32Args {
  const float* q;
  const float* k_pool;
  const float* v_pool;
  const int32_t* page_table;
  const int32_t* seq_len;
  float* out;
  float* ws;
  Geo g;
  int32_t n_splits;
  int32_t n_q;   // prefill: queries per sequence
  float scale_log2;
  // rotary variant only
  const float* u_k;
  int32_t d_head;
  double log2_base;
  // ALiBi variant only
  const float* alibi;
  // rotary variant over a pruned cache: positions of the cached tokens [B, pos_stride] and of the queries [B], or null
  const int32_t* slot_pos = nullptr;
  const int32_t* q_pos = nullptr;
  int32_t pos_stride = 0;
};

__device__ __forceinline__ int clamp_len(const AttnF32Args& a, int b) {
  int64_t n = a.seq_len[b];
  const int64_t cap = (int64_t)a.g.max_pages * a.g.page_tokens;
  if (n > cap) n = cap;
  if (n < 0) n = 0;
  return (int)n;
}

// MODE: 0 position-free, 1 rotary, 2 ALiBi
template <int MODE>
__global__ __launch_bounds__(256) void decode_f32_kernel(AttnF32Args a) {
  constexpr bool ROPE = MODE == 1;
  const Geo& g = a.g;
  const int split = blockIdx.x, head = blockIdx.y, b = blockIdx.z;
  const int kvh = head / g.group;
  const int n = clamp_len(a, b);
  const int chunks = (n + kChunk - 1) / kChunk;
  const int per = (chunks + a.n_splits - 1) / a.n_splits;
  const int tok_begin = min(n, split * per * kChunk);
  const int tok_end = min(n, (split + 1) * per * kChunk);
  float m, l, acc;
  __shared__ float sq[256];
  if (!ROPE) {
    if (threadIdx.x < g.r_k) sq[threadIdx.x] = a.q[((int64_t)b * g.n_heads + head) * g.r_k + threadIdx.x];
    __syncthreads();
    if (MODE == 2)
      attend_f32(AlibiScore{sq, g.r_k, a.alibi[head] * 1.4426950408889634f, n - 1}, a.k_pool, a.v_pool,
                 a.page_table + (int64_t)b * g.max_pages, g, kvh, tok_begin, tok_end, a.scale_log2, m, l, acc);
    else
      attend_f32(DotScore{sq, g.r_k}, a.k_pool, a.v_pool, a.page_table + (int64_t)b * g.max_pages, g, kvh, tok_begin,
                 tok_end, a.scale_log2, m, l, acc);
  } else {
    __shared__ double theta[128];
    if (threadIdx.x < a.d_head) sq[threadIdx.x] = a.q[((int64_t)b * g.n_heads + head) * a.d_head + threadIdx.x];
    if (threadIdx.x < a.d_head / 2)
      theta[threadIdx.x] = exp2(-(2.0 * (double)threadIdx.x / (double)a.d_head) * a.log2_base);
    __syncthreads();
    attend_f32(RopeScore{sq, a.u_k, theta, g.r_k, a.d_head, a.q_pos ? a.q_pos[b] : n - 1,
                         a.slot_pos ? a.slot_pos + (int64_t)b * a.pos_stride : nullptr},
               a.k_pool, a.v_pool, a.page_table + (int64_t)b * g.max_pages, g, kvh, tok_begin, tok_end, a.scale_log2, m,
               l, acc);
  }
  const int c = threadIdx.x;
  if (a.n_splits == 1) {
    if (c < g.r_v) a.out[((int64_t)b * g.n_heads + head) * g.r_v + c] = l > 0.f ? acc / l : 0.f;
  } else {
    const int64_t BHS = (int64_t)gridDim.z * g.n_heads * a.n_splits;
    const int64_t row = ((int64_t)b * g.n_heads + head) * a.n_splits + split;
    if (c == 0) {
      a.ws[row] = m;
      a.ws[BHS + row] = l;
    }
    if (c < g.r_v_pad) a.ws[2 * BHS + row * g.r_v_pad + c] = c < g.r_v ? acc : 0.f;
  }
}

// Causal prefill: one workgroup per (query, head, sequence); query j sits at position len - n_q + j.
template <int MODE>
__global__ __launch_bounds__(256) void prefill_f32_kernel(AttnF32Args a) {
  constexpr bool ROPE = MODE == 1;
  const Geo& g = a.g;
  const int j = blockIdx.x, head = blockIdx.y, b = blockIdx.z;
  const int kvh = head / g.group;
  const int n = clamp_len(a, b);
  const int pos = n - a.n_q + j;
  const int64_t row = (((int64_t)b * a.n_q + j) * g.n_heads + head);
  float m, l, acc;
  __shared__ float sq[256];
  if (!ROPE) {
    if (threadIdx.x < g.r_k) sq[threadIdx.x] = a.q[row * g.r_k + threadIdx.x];
    __syncthreads();
    if (MODE == 2)
      attend_f32(AlibiScore{sq, g.r_k, a.alibi[head] * 1.4426950408889634f, pos}, a.k_pool, a.v_pool,
                 a.page_table + (int64_t)b * g.max_pages, g, kvh, 0, pos >= 0 ? pos + 1 : 0, a.scale_log2, m, l, acc);
    else
      attend_f32(DotScore{sq, g.r_k}, a.k_pool, a.v_pool, a.page_table + (int64_t)b * g.max_pages, g, kvh, 0,
                 pos >= 0 ? pos + 1 : 0, a.scale_log2, m, l, acc);
  } else {
    __shared__ double theta[128];
    if (threadIdx.x < a.d_head) sq[threadIdx.x] = a.q[row * a.d_head + threadIdx.x];
    if (threadIdx.x < a.d_head / 2)
      theta[threadIdx.x] = exp2(-(2.0 * (double)threadIdx.x / (double)a.d_head) * a.log2_base);
    __syncthreads();
    attend_f32(RopeScore{sq, a.u_k, theta, g.r_k, a.d_head, pos}, a.k_pool, a.v_pool,
               a.page_table + (int64_t)b * g.max_pages, g, kvh, 0, pos >= 0 ? pos + 1 : 0, a.scale_log2, m, l, acc);
  }
  const int c = threadIdx.x;
  if (c < g.r_v) a.out[row * g.r_v + c] = l > 0.f ? acc / l : 0.f;
}

static AttnF32Args make_args(const ea_layer_desc* d, const Geo& g, const float* q, const float* k_pool,
                             const float* v_pool, const int32_t* page_table, const int32_t* seq_len, float* out,
                             float* ws, int32_t n_splits, int32_t n_q) {
  AttnF32Args a;
  a.q = q;
  a.k_pool = k_pool;
  a.v_pool = v_pool;
  a.page_table = page_table;
  a.seq_len = seq_len;
  a.out = out;
  a.ws = ws;
  a.g = g;
  a.n_splits = n_splits;
  a.n_q = n_q;
  a.scale_log2 = 1.4426950408889634f / sqrtf((float)d->d_head);
  a.u_k = nullptr;
  a.d_head = d->d_head;
  a.log2_base = 0.0;
  a.alibi = nullptr;
  return a;
}

int decode_f32(const ea_layer_desc* d, const Geo& g, const float* q, const float* k_pool, const float* v_pool,
               const int32_t* page_table, const int32_t* seq_len, float* out, int32_t B, int32_t n_splits, float* ws,
               hipStream_t st) {
  if (B > 65535 || g.n_heads > 65535) return EA_ERR_SHAPE;
  AttnF32Args a = make_args(d, g, q, k_pool, v_pool, page_table, seq_len, out, ws, n_splits, 1);
  decode_f32_kernel<0><<<dim3(n_splits, g.n_heads, B), dim3(256), 0, st>>>(a);
  return launch_status();
}

int decode_rope_f32(const ea_layer_desc* d, const Geo& g, const float* q, const float* u_k, double rope_base,
                    const float* k_pool, const float* v_pool, const int32_t* page_table, const int32_t* seq_len,
                    float* out, int32_t B, int32_t n_splits, float* ws, hipStream_t st) {
  if (B > 65535 || g.n_heads > 65535) return EA_ERR_SHAPE;
  if (d->d_head > 256 || d->d_head % 2 != 0) return EA_ERR_SHAPE;
  AttnF32Args a = make_args(d, g, q, k_pool, v_pool, page_table, seq_len, out, ws, n_splits, 1);
  a.u_k = u_k;
  a.log2_base = log2(rope_base);
  decode_f32_kernel<1><<<dim3(n_splits, g.n_heads, B), dim3(256), 0, st>>>(a);
  return launch_status();
}

int decode_rope_pos_f32(const ea_layer_desc* d, const Geo& g, const float* q, const float* u_k, double rope_base,
                        const float* k_pool, const float* v_pool, const int32_t* page_table, const int32_t* seq_len,
                        const int32_t* slot_pos, int32_t pos_stride, const int32_t* q_pos, float* out, int32_t B,
                        int32_t n_splits, float* ws, hipStream_t st) {
  if (B > 65535 || g.n_heads > 65535) return EA_ERR_SHAPE;
  if (d->d_head > 256 || d->d_head % 2 != 0) return EA_ERR_SHAPE;
  AttnF32Args a = make_args(d, g, q, k_pool, v_pool, page_table, seq_len, out, ws, n_splits, 1);
  a.u_k = u_k;
  a.log2_base = log2(rope_base);
  a.slot_pos = slot_pos;
  a.q_pos = q_pos;
  a.pos_stride = pos_stride;
  decode_f32_kernel<1><<<dim3(n_splits, g.n_heads, B), dim3(256), 0, st>>>(a);
  return launch_status();
}

int prefill_f32(const ea_layer_desc* d, const Geo& g, const float* q, const float* k_pool, const float* v_pool,
                const int32_t* page_table, const int32_t* seq_len, float* out, int32_t B, int32_t n, hipStream_t st) {
  if (B > 65535 || g.n_heads > 65535) return EA_ERR_SHAPE;
  AttnF32Args a = make_args(d, g, q, k_pool, v_pool, page_table, seq_len, out, nullptr, 1, n);
  prefill_f32_kernel<0><<<dim3(n, g.n_heads, B), dim3(256), 0, st>>>(a);
  return launch_status();
}

int prefill_rope_f32(const ea_layer_desc* d, const Geo& g, const float* q, const float* u_k, double rope_base,
                     const float* k_pool, const float* v_pool, const int32_t* page_table, const int32_t* seq_len,
                     float* out, int32_t B, int32_t n, hipStream_t st) {
  if (B > 65535 || g.n_heads > 65535) return EA_ERR_SHAPE;
  if (d->d_head > 256 || d->d_head % 2 != 0) return EA_ERR_SHAPE;
  AttnF32Args a = make_args(d, g, q, k_pool, v_pool, page_table, seq_len, out, nullptr, 1, n);
  a.u_k = u_k;
  a.log2_base = log2(rope_base);
  prefill_f32_kernel<1><<<dim3(n, g.n_heads, B), dim3(256), 0, st>>>(a);
  return launch_status();
}

int decode_alibi_f32(const ea_layer_desc* d, const Geo& g, const float* q, const float* slopes, const float* k_pool,
                     const float* v_pool, const int32_t* page_table, const int32_t* seq_len, float* out, int32_t B,
                     int32_t n_splits, float* ws, hipStream_t st) {
  if (B > 65535 || g.n_heads > 65535) return EA_ERR_SHAPE;
  AttnF32Args a = make_args(d, g, q, k_pool, v_pool, page_table, seq_len, out, ws, n_splits, 1);
  a.alibi = slopes;
  decode_f32_kernel<2><<<dim3(n_splits, g.n_heads, B), dim3(256), 0, st>>>(a);
  return launch_status();
}

int prefill_alibi_f32(const ea_layer_desc* d, const Geo& g, const float* q, const float* slopes, const float* k_pool,
                      const float* v_pool, const int32_t* page_table, const int32_t* seq_len, float* out, int32_t B,
                      int32_t n, hipStream_t st) {
  if (B > 65535 || g.n_heads > 65535) return EA_ERR_SHAPE;
  AttnF32Args a = make_args(d, g, q, k_pool, v_pool, page_table, seq_len, out, nullptr, 1, n);
  a.alibi = slopes;
  prefill_f32_kernel<2><<<dim3(n, g.n_heads, B), dim3(256), 0, st>>>(a);
  return launch_status();
}

// ---- C[M,N] = A[M,K] . Bt[N,K]^T, 64x64 tiles, 4x4 outputs per thread --------
template <typename Epilogue>
__global__ __launch_bounds__(256) void gemm_f32_kernel(const float* __restrict__ A, const float* __restrict__ Bt,
                                                       int32_t M, int32_t N, int32_t K, Epilogue ep) {
  constexpr int BM = 64, BN = 64, BK = 16;
  __shared__ float As[BK][BM + 4];
  __shared__ float Bs[BK][BN + 4];
  const int tid = threadIdx.x;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  const int tx = tid & 15, ty = tid >> 4;
  const int lr = tid >> 2, lk = (tid & 3) * 4;
  float c[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += BK) {
    float4 av = make_float4(0.f, 0.f, 0.f, 0.f), bv = av;
    if (m0 + lr < M && k0 + lk < K) av = *reinterpret_cast<const float4*>(A + (int64_t)(m0 + lr) * K + k0 + lk);
    if (n0 + lr < N && k0 + lk < K) bv = *reinterpret_cast<const float4*>(Bt + (int64_t)(n0 + lr) * K + k0 + lk);
    As[lk + 0][lr] = av.x; As[lk + 1][lr] = av.y; As[lk + 2][lr] = av.z; As[lk + 3][lr] = av.w;
    Bs[lk + 0][lr] = bv.x; Bs[lk + 1][lr] = bv.y; Bs[lk + 2][lr] = bv.z; Bs[lk + 3][lr] = bv.w;
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < BK; ++kk) {
      float a4[4], b4[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a4[i] = As[kk][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b4[j] = Bs[kk][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) c[i][j] = fmaf(a4[i], b4[j], c[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int r = m0 + ty * 4 + i, cc = n0 + tx * 4 + j;
      if (r < M && cc < N) ep(r, cc, c[i][j]);
    }
}

struct QkvEpF32 {
  QkvDest d;
  __device__ void operator()(int r, int c, float v) const { qkv_store<false>(d, r, c, v); }
};
struct PlainEpF32 {
  float* y;
  int32_t N;
  __device__ void operator()(int r, int c, float v) const { y[(int64_t)r * N + c] = v; }
};

int gemm_qkv_f32(const float* x, const float* w_t, int32_t M, int32_t N, int32_t K, const QkvDest& dst,
                 hipStream_t st) {
  dim3 grid((N + 63) / 64, (M + 63) / 64);
  if (grid.y > 65535) return EA_ERR_SHAPE;
  gemm_f32_kernel<<<grid, dim3(256), 0, st>>>(x, w_t, M, N, K, QkvEpF32{dst});
  return launch_status();
}

int gemm_out_f32(const float* a, const float* w_t, float* y, int32_t M, int32_t N, int32_t K, hipStream_t st) {
  dim3 grid((N + 63) / 64, (M + 63) / 64);
  if (grid.y > 65535) return EA_ERR_SHAPE;
  gemm_f32_kernel<<<grid, dim3(256), 0, st>>>(a, w_t, M, N, K, PlainEpF32{y, N});
  return launch_status();
}

}  // namespace ea
