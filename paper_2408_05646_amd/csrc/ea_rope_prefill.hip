// Prefill-phase attention for models with rotary position embedding (Sec. 4.3, Eq. 9-10), bf16 path.
//
// In the prefill every cached key meets many queries, so the keys are brought back to d_head channels and
// rotated ONCE (K'[t] = rot(U^K k_r[t], t), written in the K tile order of a rank-d_head cache), the queries
// are rotated once, and the position-free prefill kernel then runs at rank d_head on the two.  The rotated
// keys live in a workspace for the duration of the call; the cache keeps its rank-r keys.
#include "ea_common.h"

namespace ea {

struct RopeExpandArgs {
  const uint16_t* k_pool;     // rank-r cache
  uint16_t* k_rot;            // [B * max_pages pages][H_kv][page_tokens * d_head]: K tile order at rank d_head
  const uint16_t* u_k;        // [d_head, r_k] bf16
  const int32_t* page_table;
  const int32_t* seq_len;
  Geo g;                      // geometry of the rank-r cache
  int32_t d_head;
  double log2_base;
};

// One workgroup = one 64-token tile of one sequence; wave w = its 16-token block w, all kv heads in turn.
// Per block: K'^T = U^K . k_r^T on the matrix cores (basis in LDS in A-operand order, rows permuted so that both
// channels of a rotary pair land in one lane), rotation by the token's position in fp32, one 16-byte store of
// eight consecutive channels per lane.
template <int KS, int NKK>
__global__ __launch_bounds__(256) void rope_expand_kernel(RopeExpandArgs a) {
  const Geo& g = a.g;
  const int tile = blockIdx.x, b = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int col = lane & 15, quad = lane >> 4;
  int64_t n64 = a.seq_len[b];
  const int64_t cap = (int64_t)g.max_pages * g.page_tokens;
  if (n64 > cap) n64 = cap;
  if ((int64_t)tile * kTile >= n64) return;                     // nothing cached here (uniform for the workgroup)
  const int tiles_per_page = g.page_tokens / kTile;
  const int lp = tile / tiles_per_page, tin = tile % tiles_per_page;
  const int page = a.page_table[(int64_t)b * g.max_pages + lp];
  if (page < 0 || page >= g.pool_pages) return;                 // the attention kernel masks this page's tokens

  __shared__ bf16x8 uf[2 * NKK][KS][64];
  __shared__ double turns[NKK * 16];
  if (threadIdx.x < NKK * 16)
    turns[threadIdx.x] = exp2(-(2.0 * (double)threadIdx.x / (double)a.d_head) * a.log2_base) * 0.15915494309189535;
  for (int e = threadIdx.x; e < 2 * NKK * KS * 64; e += 256) {
    const int ln = e & 63, ks = (e >> 6) % KS, fb = e / (64 * KS);
    const uint16_t* urow = a.u_k + (int64_t)(2 * ((fb >> 1) * 16 + (ln & 15)) + (fb & 1)) * g.r_k;
    typedef __attribute__((ext_vector_type(8))) uint16_t u16x8;
    u16x8 w;
#pragma unroll
    for (int x = 0; x < 8; ++x) {
      const int rho = ks * 32 + (ln >> 4) * 8 + x;
      w[x] = rho < g.r_k ? urow[rho] : (uint16_t)0;
    }
    uf[fb][ks][ln] = __builtin_bit_cast(bf16x8, w);
  }
  __syncthreads();

  // this lane's token and the cos / sin of its 4*NKK pairs j = 16*kk + 4*quad + i
  const int tok = tile * kTile + wave * 16 + col;
  float cs[NKK][4], sn[NKK][4];
#pragma unroll
  for (int kk = 0; kk < NKK; ++kk)
#pragma unroll
    for (int i = 0; i < 4; ++i) rot_turns((double)tok * turns[kk * 16 + quad * 4 + i], cs[kk][i], sn[kk][i]);

  const int nck = g.r_k_pad >> 3, nck_dst = a.d_head >> 3;
  const int64_t dst_slab = (int64_t)g.page_tokens * a.d_head;
  for (int kvh = 0; kvh < g.n_kv_heads; ++kvh) {
    const uint16_t* src = a.k_pool + (int64_t)page * g.k_page + (int64_t)kvh * g.k_slab +
                          (int64_t)tin * (kTile * g.r_k_pad) + wave * (16 * g.r_k_pad);
    bf16x8 kf[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      kf[ks] = ks * 4 + quad < nck ? *reinterpret_cast<const bf16x8*>(src + (((ks * 4 + quad) * 16 + col) << 3))
                                   : zero_frag();
    uint16_t* dst = a.k_rot + (((int64_t)b * g.max_pages + lp) * g.n_kv_heads + kvh) * dst_slab +
                    (int64_t)tin * (kTile * a.d_head) + wave * (16 * a.d_head);
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk) {
      f32x4 x0 = {0.f, 0.f, 0.f, 0.f}, x1 = x0;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        x0 = mfma16(uf[2 * kk][ks][lane], kf[ks], x0);
        x1 = mfma16(uf[2 * kk + 1][ks][lane], kf[ks], x1);
      }
      // channels 2j, 2j+1 for j = 16*kk + 4*quad + 0..3: the eight channels of chunk 4*kk + quad of this token
      bf16x8 o;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        o[2 * i] = (__bf16)(x0[i] * cs[kk][i] - x1[i] * sn[kk][i]);
        o[2 * i + 1] = (__bf16)(x0[i] * sn[kk][i] + x1[i] * cs[kk][i]);
      }
      *reinterpret_cast<bf16x8*>(dst + (((kk * 4 + quad) * 16 + col) << 3)) = o;
    }
  }
  (void)nck_dst;
}

// q [B, n, H, d_head] bf16 -> the same rotated to position seq_len[b] - n + j and multiplied by `scale` (the
// softmax scale in log2 units, which the attention kernel expects inside the query); one thread per 8 channels.
__global__ void rope_rotate_q_kernel(const uint16_t* __restrict__ q, uint16_t* __restrict__ q_rot,
                                     const int32_t* __restrict__ seq_len, int32_t B, int32_t n, int32_t H,
                                     int32_t d_head, int32_t max_tokens, double log2_base, float scale) {
  __shared__ double turns_of[128];                               // theta_pair / (2 pi), once per workgroup
  if (threadIdx.x < (d_head >> 1))
    turns_of[threadIdx.x] = exp2(-(2.0 * (double)threadIdx.x / (double)d_head) * log2_base) * 0.15915494309189535;
  __syncthreads();
  const int units = d_head >> 3;
  const int64_t total = (int64_t)B * n * H * units;
  for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
       idx += (int64_t)gridDim.x * blockDim.x) {
    const int u = (int)(idx % units);
    const int64_t row = idx / units;                             // (b*n + j)*H + h
    const int64_t bj = row / H;
    const int b = (int)(bj / n), j = (int)(bj % n);
    int len = seq_len[b];
    len = len < 0 ? 0 : (len > max_tokens ? max_tokens : len);
    const int pos = len - n + j;
    const bf16x8 x = *reinterpret_cast<const bf16x8*>(q + row * d_head + u * 8);
    bf16x8 y;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      float c, s;
      rot_turns((double)pos * turns_of[u * 4 + i], c, s);
      const float x0 = (float)x[2 * i] * scale, x1 = (float)x[2 * i + 1] * scale;
      y[2 * i] = (__bf16)(x0 * c - x1 * s);
      y[2 * i + 1] = (__bf16)(x0 * s + x1 * c);
    }
    *reinterpret_cast<bf16x8*>(q_rot + row * d_head + u * 8) = y;
  }
}

static int64_t align256(int64_t x) { return (x + 255) / 256 * 256; }

int64_t prefill_rope_ws_bytes(const ea_layer_desc* d, int32_t B, int32_t n, int32_t max_pages) {
  if (d->dtype != EA_BF16) return 0;
  const int64_t k_rot = (int64_t)B * max_pages * d->n_kv_heads * d->page_tokens * d->d_head * 2;
  const int64_t q_rot = (int64_t)B * n * d->n_heads * d->d_head * 2;
  return align256(k_rot) + align256(q_rot);
}

template <int NKK>
static int launch_expand(int ks, const RopeExpandArgs& a, dim3 grid, hipStream_t st) {
  switch (ks) {
    case 1: rope_expand_kernel<1, NKK><<<grid, 256, 0, st>>>(a); break;
    case 2: rope_expand_kernel<2, NKK><<<grid, 256, 0, st>>>(a); break;
    case 3: rope_expand_kernel<3, NKK><<<grid, 256, 0, st>>>(a); break;
    case 4: rope_expand_kernel<4, NKK><<<grid, 256, 0, st>>>(a); break;
    default: return EA_ERR_SHAPE;
  }
  return launch_status();
}

int prefill_rope_bf16(const ea_layer_desc* d, const Geo& g, const void* q, const void* u_k, double rope_base,
                      const void* k_pool, const void* v_pool, const int32_t* page_table, const int32_t* seq_len,
                      void* out, int32_t B, int32_t n, void* ws, hipStream_t st) {
  if (d->d_head != 64 && d->d_head != 128) return EA_ERR_SHAPE;
  if (B > 65535) return EA_ERR_SHAPE;
  const int64_t tiles = (int64_t)g.max_pages * (g.page_tokens / kTile);
  if (tiles > INT32_MAX) return EA_ERR_SHAPE;
  uint16_t* k_rot = (uint16_t*)ws;
  uint16_t* q_rot = (uint16_t*)((char*)ws + align256((int64_t)B * g.max_pages * d->n_kv_heads * d->page_tokens *
                                                     d->d_head * 2));
  RopeExpandArgs a;
  a.k_pool = (const uint16_t*)k_pool;
  a.k_rot = k_rot;
  a.u_k = (const uint16_t*)u_k;
  a.page_table = page_table;
  a.seq_len = seq_len;
  a.g = g;
  a.d_head = d->d_head;
  a.log2_base = log2(rope_base);
  const int ks = (g.r_k_pad + 31) / 32;
  const dim3 grid((uint32_t)tiles, (uint32_t)B);
  int rc = d->d_head == 128 ? launch_expand<4>(ks, a, grid, st) : launch_expand<2>(ks, a, grid, st);
  if (rc != EA_OK) return rc;
  const int64_t units = (int64_t)B * n * d->n_heads * (d->d_head / 8);
  int64_t blocks = (units + 255) / 256;
  if (blocks > 65536) blocks = 65536;
  const int64_t cap = (int64_t)g.max_pages * g.page_tokens;
  rope_rotate_q_kernel<<<dim3((uint32_t)blocks), 256, 0, st>>>((const uint16_t*)q, q_rot, seq_len, B, n, d->n_heads,
                                                               d->d_head, cap > INT32_MAX ? INT32_MAX : (int32_t)cap,
                                                               a.log2_base,
                                                               1.4426950408889634f / sqrtf((float)d->d_head));
  rc = launch_status();
  if (rc != EA_OK) return rc;
  // the position-free kernel at rank d_head on the rotated operands; K pages are addressed without a lookup
  ea_layer_desc full = *d;
  full.r_k = d->d_head;
  Geo gf = make_geo(&full, g.max_pages, g.pool_pages);
  return prefill_bf16(&full, gf, q_rot, k_rot, v_pool, page_table, seq_len, out, B, n, st, 1);
}

}  // namespace ea
