// Prefill-phase attention in rank space (Eq. 2 with the rank-r operands of Eq. 7,
// causal): flash attention on the gfx950 matrix cores, K and V read straight from
// the paged cache in MFMA fragment order.
//
// One workgroup = 4 waves = 4 * QT * 16 consecutive queries of one (sequence, head).
// A wave keeps QT blocks of 16 queries as MFMA columns and walks the 64-token cache
// tiles up to its diagonal:
//   S[64 kv x 16 q]   = K_tile . Q^T              (A = K fragments, B = q rows)
//   online softmax per query column (rows = kv tokens: 16 registers + two cross-quad shuffles)
//   O^T[r_v x 16 q]  += V_tile^T . P^T            (P rounded to bf16; row sums by an all-ones MFMA)
// Every K / V fragment is loaded once per wave and reused for the QT query blocks.
#include "ea_common.h"
#include "ea_epilogue.h"

namespace ea {

struct PrefillArgs {
  const uint16_t* q;
  const uint16_t* k_pool;
  const uint16_t* v_pool;
  const int32_t* page_table;
  const int32_t* seq_len;
  uint16_t* out;
  Geo g;
  int32_t n_q;
  float scale_log2;
};

template <int KS, int NCB, int QT>
__global__ __launch_bounds__(256, 2) void prefill_bf16_kernel(PrefillArgs a) {
  const Geo& g = a.g;
  const int head = blockIdx.y, b = blockIdx.z;
  const int kvh = head / g.group;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int col = lane & 15, quad = lane >> 4;
  const int nck = g.r_k_pad >> 3;
  constexpr int QW = QT * 16;                                   // queries per wave
  const int q_tile = gridDim.x - 1 - blockIdx.x;                // longest (latest) query tiles first
  const int q0 = (q_tile * 4 + wave) * QW;                      // first query of this wave
  if (q0 >= a.n_q) return;

  int64_t n64 = a.seq_len[b];
  const int64_t cap = (int64_t)g.max_pages * g.page_tokens;
  if (n64 > cap) n64 = cap;
  if (n64 < 0) n64 = 0;
  const int len = (int)n64;
  const int pos0 = len - a.n_q;                                  // position of query 0 (may be < 0: such queries see nothing)
  const int tiles_per_page = g.page_tokens / kTile;

  // B operands: q rows of this wave's QT query blocks
  bf16x8 qf[QT][KS];
#pragma unroll
  for (int qb = 0; qb < QT; ++qb) {
    const int qi = q0 + qb * 16 + col;
    const uint16_t* qrow = a.q + (((int64_t)b * a.n_q + qi) * g.n_heads + head) * g.r_k;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const int k = ks * 32 + quad * 8;
      qf[qb][ks] = (qi < a.n_q && k < g.r_k) ? *reinterpret_cast<const bf16x8*>(qrow + k) : zero_frag();
    }
  }
  bf16x8 ones;
#pragma unroll
  for (int j = 0; j < 8; ++j) ones[j] = (__bf16)1.0f;

  f32x4 acc[QT][NCB], lacc[QT];
  float m[QT];
#pragma unroll
  for (int qb = 0; qb < QT; ++qb) {
    m[qb] = -INFINITY;
    lacc[qb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) acc[qb][cb] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  const int q_last = min(a.n_q, q0 + QW) - 1;
  const int pos_last = pos0 + q_last;                            // last position any query of this wave sees
  const int pos_first = pos0 + q0;                               // every query of this wave sees positions <= this
  const int t_end = pos_last >= 0 ? min(pos_last, len - 1) / kTile + 1 : 0;

  bf16x8 kf[4][KS], vf[2][NCB];
  auto tile_page = [&](int t) -> int {
    const int page = a.page_table[(int64_t)b * g.max_pages + t / tiles_per_page];
    return (page >= 0 && page < g.pool_pages) ? page : -1;
  };
  auto load_k = [&](int t, int page) {
    const uint16_t* base = a.k_pool + (int64_t)page * g.k_page + (int64_t)kvh * g.k_slab +
                           (int64_t)(t % tiles_per_page) * (kTile * g.r_k_pad);
#pragma unroll
    for (int tb = 0; tb < 4; ++tb)
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const int chunk = ks * 4 + quad;
        kf[tb][ks] = chunk < nck ? *reinterpret_cast<const bf16x8*>(base + (((tb * nck + chunk) * 16 + col) << 3))
                                 : zero_frag();
      }
  };
  auto load_v = [&](int t, int page) {
    const uint16_t* base = a.v_pool + (int64_t)page * g.v_page + (int64_t)kvh * g.v_slab +
                           (int64_t)(t % tiles_per_page) * (kTile * g.r_v_pad);
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb)
        vf[u][cb] = *reinterpret_cast<const bf16x8*>(base + (((u * NCB + cb) * 64 + lane) << 3));
  };
  auto zero_kv = [&]() {
#pragma unroll
    for (int tb = 0; tb < 4; ++tb)
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) kf[tb][ks] = zero_frag();
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb) vf[u][cb] = zero_frag();
  };

  int page = -1;
  if (t_end > 0) {
    page = tile_page(0);
    if (page >= 0) {
      load_k(0, page);
      load_v(0, page);
    } else {
      zero_kv();
    }
  }

  for (int t = 0; t < t_end; ++t) {
    const int tok0 = t * kTile;
    const bool full = page >= 0 && tok0 + kTile - 1 <= pos_first && tok0 + kTile <= len;   // no masking needed
    const int limit = page >= 0 ? len : 0;                       // tokens >= limit do not exist
    const bool have_n = t + 1 < t_end;
    const int page_n = have_n ? tile_page(t + 1) : -1;

    if (tok0 + kTile > limit) {
      // slots past the end of the sequence hold arbitrary bits: clear them so 0 * x stays 0
#pragma unroll
      for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            const int tok = tok0 + u * 32 + (j >> 2) * 16 + quad * 4 + (j & 3);
            if (tok >= limit) vf[u][cb][j] = (__bf16)0.0f;
          }
    }

#pragma unroll
    for (int qb = 0; qb < QT; ++qb) {
      f32x4 s[4];
#pragma unroll
      for (int tb = 0; tb < 4; ++tb) {
        s[tb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) s[tb] = mfma16(kf[tb][ks], qf[qb][ks], s[tb]);
      }
      if (qb == QT - 1 && have_n && page_n >= 0) load_k(t + 1, page_n);   // K registers are free: prefetch
      const int qpos = pos0 + q0 + qb * 16 + col;                // this lane's query position
      const int vis = min(qpos + 1, limit);                      // kv tokens < vis are visible
      float mx = -INFINITY;
#pragma unroll
      for (int tb = 0; tb < 4; ++tb)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          float v = s[tb][i] * a.scale_log2;
          if (!full && tok0 + tb * 16 + quad * 4 + i >= vis) v = -INFINITY;
          s[tb][i] = v;
          mx = fmaxf(mx, v);
        }
      mx = fmaxf(mx, __shfl_xor(mx, 16));
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float m_new = fmaxf(m[qb], mx);
      const float m_use = m_new == -INFINITY ? 0.f : m_new;
      const float alpha = __builtin_amdgcn_exp2f(m[qb] - m_use);
      m[qb] = m_new;
      bf16x8 pf[2];
#pragma unroll
      for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
          for (int i = 0; i < 4; ++i) pf[u][h * 4 + i] = (__bf16)__builtin_amdgcn_exp2f(s[2 * u + h][i] - m_use);
      lacc[qb] *= alpha;
      lacc[qb] = mfma16(ones, pf[0], lacc[qb]);
      lacc[qb] = mfma16(ones, pf[1], lacc[qb]);
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb) {
        acc[qb][cb] *= alpha;
        acc[qb][cb] = mfma16(vf[0][cb], pf[0], acc[qb][cb]);
        acc[qb][cb] = mfma16(vf[1][cb], pf[1], acc[qb][cb]);
      }
    }
    if (have_n) {
      if (page_n >= 0) load_v(t + 1, page_n);
      else zero_kv();
    }
    page = page_n;
  }

  // ---- write O: lane holds, for query `col` of each block, channels cb*16 + 4*quad .. +3
#pragma unroll
  for (int qb = 0; qb < QT; ++qb) {
    const int qi = q0 + qb * 16 + col;
    if (qi >= a.n_q) continue;
    const float l = lacc[qb][0];
    const float inv = l > 0.f ? 1.0f / l : 0.f;
    uint16_t* orow = a.out + (((int64_t)b * a.n_q + qi) * g.n_heads + head) * g.r_v;
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) {
      const int c = cb * 16 + quad * 4;
      if (c + 3 < g.r_v) {
        u32x2 w;
        w[0] = (uint32_t)f32_to_bf16_rne(acc[qb][cb][0] * inv) | ((uint32_t)f32_to_bf16_rne(acc[qb][cb][1] * inv) << 16);
        w[1] = (uint32_t)f32_to_bf16_rne(acc[qb][cb][2] * inv) | ((uint32_t)f32_to_bf16_rne(acc[qb][cb][3] * inv) << 16);
        *reinterpret_cast<u32x2*>(orow + c) = w;
      } else {
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (c + i < g.r_v) orow[c + i] = f32_to_bf16_rne(acc[qb][cb][i] * inv);
      }
    }
  }
}

template <int KS, int NCB>
static void launch_prefill(const PrefillArgs& a, int32_t B, hipStream_t st) {
  constexpr int QT = (KS <= 2 && NCB <= 4) ? 4 : 2;
  const int per_block = 4 * QT * 16;
  dim3 grid((a.n_q + per_block - 1) / per_block, a.g.n_heads, B), block(256);
  prefill_bf16_kernel<KS, NCB, QT><<<grid, block, 0, st>>>(a);
}

template <int KS>
static int dispatch_ncb(int ncb, const PrefillArgs& a, int32_t B, hipStream_t st) {
  switch (ncb) {
    case 1: launch_prefill<KS, 1>(a, B, st); break;
    case 2: launch_prefill<KS, 2>(a, B, st); break;
    case 3: launch_prefill<KS, 3>(a, B, st); break;
    case 4: launch_prefill<KS, 4>(a, B, st); break;
    case 5: launch_prefill<KS, 5>(a, B, st); break;
    case 6: launch_prefill<KS, 6>(a, B, st); break;
    case 7: launch_prefill<KS, 7>(a, B, st); break;
    case 8: launch_prefill<KS, 8>(a, B, st); break;
    default: return EA_ERR_SHAPE;
  }
  return launch_status();
}

int prefill_bf16(const ea_layer_desc* d, const Geo& g, const void* q, const void* k_pool, const void* v_pool,
                 const int32_t* page_table, const int32_t* seq_len, void* out, int32_t B, int32_t n, hipStream_t st) {
  if (B > 65535 || g.n_heads > 65535) return EA_ERR_SHAPE;
  if (g.r_k % 8 != 0 || g.r_v % 4 != 0) return EA_ERR_SHAPE;     // 16-byte q rows, 8-byte output stores
  PrefillArgs a;
  a.q = (const uint16_t*)q;
  a.k_pool = (const uint16_t*)k_pool;
  a.v_pool = (const uint16_t*)v_pool;
  a.page_table = page_table;
  a.seq_len = seq_len;
  a.out = (uint16_t*)out;
  a.g = g;
  a.n_q = n;
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
