// Generation-phase attention over the rank-r bf16 paged cache (Eq. 3 with the
// rank-r operands of Eq. 7): split-K flash-decode on the gfx950 matrix cores.
//
// One workgroup (4 waves) owns one (sequence, kv head, split).  Each wave streams
// whole 64-token tiles: the cache layout is the MFMA operand order, so every
// global load is one contiguous 1 KiB wave access and nothing is shuffled
// between lanes.  Per tile and wave:
//   S[64 tok x 16 head cols]  = K_tile . q^T        v_mfma_f32_16x16x32_bf16, q split in hi+lo bf16
//   online softmax in the D layout (lane = head column, 4 token rows per register quad)
//   O^T[r_v x 16 head cols]  += V_tile^T . P^T      P rounded to bf16, row sums by an all-ones MFMA
// The 16 head columns carry the G = H / H_kv query heads that share the kv head
// (unused columns hold zeros), so grouped-query attention costs no extra traffic.
#include "ea_common.h"

namespace ea {

constexpr float kLazy = 8.0f;

struct DecodeArgs {
  const float* q;
  const uint16_t* k_pool;
  const uint16_t* v_pool;
  const int32_t* page_table;
  const int32_t* seq_len;
  float* out;
  float* ws;
  Geo g;
  int32_t n_splits;
  float scale_log2;   // log2(e) / sqrt(d_head)
};

// TBN = 16-token blocks handled per loop iteration: 4 (a whole 64-token tile) or 2 (half a tile, for the
// large ranks whose fragments would not fit the register file otherwise).
template <int KS, int NCB, int TBN, int WPE>
__global__ __launch_bounds__(256, WPE) void decode_bf16_kernel(DecodeArgs a) {
  constexpr int UN = TBN / 2;            // 32-token groups per iteration
  constexpr int SUB = 4 / TBN;           // iterations per 64-token tile
  constexpr int TOK = TBN * 16;          // tokens per iteration
  const Geo& g = a.g;
  // neighbouring workgroups take neighbouring kv heads of the same pages: their slabs are adjacent in memory
  const int kvh = blockIdx.x, split = blockIdx.y, b = blockIdx.z;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int col = lane & 15, quad = lane >> 4;
  const int G = g.group;
  const int nck = g.r_k_pad >> 3;

  int64_t n64 = a.seq_len[b];
  const int64_t cap = (int64_t)g.max_pages * g.page_tokens;
  if (n64 > cap) n64 = cap;
  if (n64 < 0) n64 = 0;
  const int n = (int)n64;
  const int n_tiles = (n + kTile - 1) / kTile;
  const int per = (n_tiles + a.n_splits - 1) / a.n_splits;
  const int t_begin = split * per;
  const int t_end = min(n_tiles, t_begin + per);
  const int tiles_per_page = g.page_tokens / kTile;

  // B operand of the score MFMA: q^T, lane (col, quad) holds channels 32*ks + 8*quad .. +7 of head col.
  bf16x8 qhi[KS], qlo[KS];
  {
    const float* qrow = a.q + ((int64_t)b * g.n_heads + (int64_t)kvh * G + col) * g.r_k;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int k = ks * 32 + quad * 8 + j;
        const float v = (col < G && k < g.r_k) ? qrow[k] : 0.f;
        const __bf16 hi = (__bf16)v;
        qhi[ks][j] = hi;
        qlo[ks][j] = (__bf16)(v - (float)hi);
      }
    }
  }
  bf16x8 ones;
#pragma unroll
  for (int j = 0; j < 8; ++j) ones[j] = (__bf16)1.0f;

  f32x4 acc[NCB];
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb) acc[cb] = f32x4{0.f, 0.f, 0.f, 0.f};
  f32x4 lacc = {0.f, 0.f, 0.f, 0.f};
  float m = -INFINITY;

  bf16x8 kf[TBN][KS], vf[UN][NCB];

  // Physical page of tile t, or -1.
  auto tile_page = [&](int it) -> int {
    const int lp = (it / SUB) / tiles_per_page;
    const int page = a.page_table[(int64_t)b * g.max_pages + lp];
    return (page >= 0 && page < g.pool_pages) ? page : -1;
  };
  auto load_k = [&](int it, int page) {
    const uint16_t* base = a.k_pool + (int64_t)page * g.k_page + (int64_t)kvh * g.k_slab +
                           (int64_t)((it / SUB) % tiles_per_page) * (kTile * g.r_k_pad) +
                           (it % SUB) * (TOK * g.r_k_pad);
#pragma unroll
    for (int tb = 0; tb < TBN; ++tb) {
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const int chunk = ks * 4 + quad;
        if (chunk < nck)
          kf[tb][ks] = __builtin_nontemporal_load(reinterpret_cast<const bf16x8*>(base + (((tb * nck + chunk) * 16 + col) << 3)));
        else
          kf[tb][ks] = zero_frag();
      }
    }
  };
  auto load_v = [&](int it, int page) {
    const uint16_t* base = a.v_pool + (int64_t)page * g.v_page + (int64_t)kvh * g.v_slab +
                           (int64_t)((it / SUB) % tiles_per_page) * (kTile * g.r_v_pad) +
                           (it % SUB) * (TOK * g.r_v_pad);
#pragma unroll
    for (int u = 0; u < UN; ++u) {
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb)
        vf[u][cb] = __builtin_nontemporal_load(reinterpret_cast<const bf16x8*>(base + (((u * NCB + cb) * 64 + lane) << 3)));
    }
  };
  auto zero_kv = [&]() {
#pragma unroll
    for (int tb = 0; tb < TBN; ++tb)
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) kf[tb][ks] = zero_frag();
#pragma unroll
    for (int u = 0; u < UN; ++u)
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb) vf[u][cb] = zero_frag();
  };

  // the four waves interleave the iterations of the split (neighbouring waves read neighbouring memory)
  const int it_end = t_end * SUB;
  int t = t_begin * SUB + wave;
  bool have = t < it_end;
  int page = -1;
  if (have) {
    page = tile_page(t);
    if (page >= 0) {
      load_k(t, page);
      load_v(t, page);
    } else {
      zero_kv();
    }
  }

  while (have) {
    // ---- scores: S[tb] (16 tokens x 16 head columns) = K_block . q^T
    f32x4 s[TBN];
#pragma unroll
    for (int tb = 0; tb < TBN; ++tb) {
      s[tb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        s[tb] = mfma16(kf[tb][ks], qhi[ks], s[tb]);
        s[tb] = mfma16(kf[tb][ks], qlo[ks], s[tb]);
      }
    }
    const int rem = page >= 0 ? n - t * TOK : 0;   // valid tokens in this iteration (>= TOK: all)
    const int tn = t + 4;
    const bool have_n = tn < it_end;
    const int page_n = have_n ? tile_page(tn) : -1;
    if (have_n && page_n >= 0) load_k(tn, page_n);   // K registers are free again: prefetch the next tile

    // ---- online softmax on s (lane: head column `col`, tokens tb*16 + 4*quad + i)
    float mx = -INFINITY;
#pragma unroll
    for (int tb = 0; tb < TBN; ++tb) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if (rem < TOK && tb * 16 + quad * 4 + i >= rem) s[tb][i] = -INFINITY;
        mx = fmaxf(mx, s[tb][i]);
      }
    }
    mx = quad_column_max(mx) * a.scale_log2;                  // the scale is positive: max commutes with it
    // m is a reference exponent: it moves only when the max has grown by more than kLazy (log2 units), so
    // P stays <= 2^kLazy and the accumulators are rescaled a few times per stream, not at every tile.
    if (__any(mx > m + kLazy)) {
      const float m_new = fmaxf(m, mx);
      const float m_safe = m_new == -INFINITY ? 0.f : m_new;
      const float alpha = __builtin_amdgcn_exp2f(m - m_safe);  // m = -inf -> 0
      lacc *= alpha;
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb) acc[cb] *= alpha;
      m = m_new;
    }
    const float m_use = m == -INFINITY ? 0.f : m;
    bf16x8 pf[UN];
#pragma unroll
    for (int u = 0; u < UN; ++u) {
#pragma unroll
      for (int h = 0; h < 2; ++h) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
          pf[u][h * 4 + i] = (__bf16)__builtin_amdgcn_exp2f(fmaf(s[2 * u + h][i], a.scale_log2, -m_use));
      }
    }
    if (rem < TOK) {
      // Partial tile: cache slots past the sequence end hold arbitrary bits; clear them so 0 * x stays 0.
#pragma unroll
      for (int u = 0; u < UN; ++u) {
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) {
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            const int tok = u * 32 + (j >> 2) * 16 + quad * 4 + (j & 3);
            if (tok >= rem) vf[u][cb][j] = (__bf16)0.0f;
          }
        }
      }
    }
    // ---- O^T += V^T . P^T, row sums of P through the all-ones operand
#pragma unroll
    for (int u = 0; u < UN; ++u) lacc = mfma16(ones, pf[u], lacc);
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) {
#pragma unroll
      for (int u = 0; u < UN; ++u) acc[cb] = mfma16(vf[u][cb], pf[u], acc[cb]);
    }
    if (have_n) {
      if (page_n >= 0) load_v(tn, page_n);
      else zero_kv();
    }
    t = tn;
    have = have_n;
    page = page_n;
  }

  // ---- merge the four waves of the workgroup
  __shared__ float sm_m[4][16];
  __shared__ float sm_l[4][16];
  __shared__ float sm_acc[4][16][NCB * 16];
  if (quad == 0) {
    sm_m[wave][col] = m;
    sm_l[wave][col] = lacc[0];
  }
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
    for (int i = 0; i < 4; ++i) sm_acc[wave][col][cb * 16 + quad * 4 + i] = acc[cb][i];
  __syncthreads();

  const int r_v_pad = NCB * 16;
  for (int idx = threadIdx.x; idx < G * r_v_pad; idx += blockDim.x) {
    const int hd = idx / r_v_pad, c = idx % r_v_pad;
    float mm = sm_m[0][hd];
#pragma unroll
    for (int w = 1; w < 4; ++w) mm = fmaxf(mm, sm_m[w][hd]);
    float lsum = 0.f, val = 0.f;
    if (mm != -INFINITY) {
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const float wt = __builtin_amdgcn_exp2f(sm_m[w][hd] - mm);
        lsum += wt * sm_l[w][hd];
        val += wt * sm_acc[w][hd][c];
      }
    }
    const int head = kvh * G + hd;
    if (a.n_splits == 1) {
      if (c < g.r_v) a.out[((int64_t)b * g.n_heads + head) * g.r_v + c] = lsum > 0.f ? val / lsum : 0.f;
    } else {
      const int64_t BHS = (int64_t)gridDim.z * g.n_heads * a.n_splits;
      const int64_t row = ((int64_t)b * g.n_heads + head) * a.n_splits + split;
      if (c == 0) {
        a.ws[row] = mm;
        a.ws[BHS + row] = lsum;
      }
      a.ws[2 * BHS + row * r_v_pad + c] = val;
    }
  }
}

// out[b, h, :] = sum_s w_s acc_s / sum_s w_s l_s with w_s = 2^(m_s - max_s m_s).
__global__ void merge_splits_kernel(const float* __restrict__ ws, float* __restrict__ out, int32_t BH, int32_t S,
                                    int32_t r_v, int32_t r_v_pad) {
  const int64_t bh = blockIdx.x;
  const int64_t BHS = (int64_t)BH * S;
  const float* pm = ws + bh * S;
  const float* pl = ws + BHS + bh * S;
  const float* pa = ws + 2 * BHS + bh * S * r_v_pad;
  float mm = -INFINITY;
  for (int s = 0; s < S; ++s) mm = fmaxf(mm, pm[s]);
  for (int c = threadIdx.x; c < r_v; c += blockDim.x) {
    float lsum = 0.f, val = 0.f;
    if (mm != -INFINITY) {
      for (int s = 0; s < S; ++s) {
        const float wt = __builtin_amdgcn_exp2f(pm[s] - mm);
        lsum += wt * pl[s];
        val += wt * pa[(int64_t)s * r_v_pad + c];
      }
    }
    out[bh * r_v + c] = lsum > 0.f ? val / lsum : 0.f;
  }
}

int merge_splits(const Geo& g, const float* ws, float* out, int32_t B, int32_t n_splits, hipStream_t st) {
  merge_splits_kernel<<<dim3(B * g.n_heads), dim3(64), 0, st>>>(ws, out, B * g.n_heads, n_splits, g.r_v, g.r_v_pad);
  return launch_status();
}

template <int KS, int NCB>
static void launch_decode(const DecodeArgs& a, int32_t B, hipStream_t st) {
  dim3 grid(a.g.n_kv_heads, a.n_splits, B), block(256);
  constexpr int TBN = (KS * 4 + NCB * 2 > 22) ? 2 : 4;   // fragments of a whole tile: 16*KS + 8*NCB registers
  decode_bf16_kernel<KS, NCB, TBN, 2><<<grid, block, 0, st>>>(a);
}

template <int KS>
static int dispatch_ncb(int ncb, const DecodeArgs& a, int32_t B, hipStream_t st) {
  switch (ncb) {
    case 1: launch_decode<KS, 1>(a, B, st); break;
    case 2: launch_decode<KS, 2>(a, B, st); break;
    case 3: launch_decode<KS, 3>(a, B, st); break;
    case 4: launch_decode<KS, 4>(a, B, st); break;
    case 5: launch_decode<KS, 5>(a, B, st); break;
    case 6: launch_decode<KS, 6>(a, B, st); break;
    case 7: launch_decode<KS, 7>(a, B, st); break;
    case 8: launch_decode<KS, 8>(a, B, st); break;
    default: return EA_ERR_SHAPE;
  }
  return launch_status();
}

int decode_bf16(const ea_layer_desc* d, const Geo& g, const float* q, const void* k_pool, const void* v_pool,
                const int32_t* page_table, const int32_t* seq_len, float* out, int32_t B, int32_t n_splits, float* ws,
                hipStream_t st) {
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
  const int ks = (g.r_k_pad + 31) / 32, ncb = g.r_v_pad / 16;
  switch (ks) {
    case 1: return dispatch_ncb<1>(ncb, a, B, st);
    case 2: return dispatch_ncb<2>(ncb, a, B, st);
    case 3: return dispatch_ncb<3>(ncb, a, B, st);
    case 4: return dispatch_ncb<4>(ncb, a, B, st);
    default: return EA_ERR_SHAPE;
  }
}

}  // namespace ea
