// Prefill-phase attention in rank space (Eq. 2 with the rank-r operands of Eq. 7,
// causal): flash attention on the gfx950 matrix cores, K and V read straight from
// the paged cache in MFMA fragment order.
//
// One workgroup = 4 waves = 4 * QT * 16 consecutive queries of one (sequence, head).
// A wave keeps QT blocks of 16 queries as MFMA columns and walks the 64-token cache
// tiles up to its diagonal, a whole tile per step or (for the ranks whose whole-tile
// fragments do not fit beside the accumulators) half a tile:
//   S[64 kv x 16 q]   = K_tile . Q^T              (A = K fragments, B = q rows)
//   online softmax per query column (rows = kv tokens: 16 registers + two cross-quad shuffles)
//   O^T[r_v x 16 q]  += V_tile^T . P^T            (P rounded to bf16; row sums by an all-ones MFMA)
// Every K / V fragment is loaded once per wave and tile and reused for the QT query blocks.
// Tiles below the diagonal take an unmasked path that does not search for the tile's maximum (the row sums are
// inspected every few tiles instead, see the tile loop); the grid is ordered by work (longest query tiles first).
#pragma once
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
  int32_t batch;
  int32_t n_qtiles;   // query tiles per (sequence, head) = gridDim.x / (H * batch)
  // Operands prepared by the rotary path: K pages are not looked up (logical page lp of sequence b is page
  // b*max_pages + lp of k_pool) and the query already carries the factor log2(e)/sqrt(d_head).
  int32_t k_compact;
  const float* alibi; // [H] ALiBi slopes (natural-log units, >= 0), ALIBI kernels only
  float scale_log2;
  // When set, the kernel leaves its result as a PART of a softmax that another kernel continues (a cache whose older
  // tokens are held elsewhere): per (sequence, query, head) row the normalised output in float, its reference
  // exponent (log2 units) and its row sum.  `out` is not written then.
  float* part_o = nullptr;    // [B * n_q * H, r_v]
  float* part_ml = nullptr;   // [B * n_q * H, 2]
};

// The fragment type of the two matrix-core contractions: bfloat16 for the cache as it is, half precision for tiles
// that are expanded from 4-bit codes in registers (their format is free, and half precision keeps three more bits).
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
__device__ __forceinline__ f32x4 mfma16(f16x8 a, f16x8 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
}
template <class F> struct FragElem;
template <> struct FragElem<bf16x8> { using type = __bf16; };
template <> struct FragElem<f16x8> { using type = _Float16; };

// One 64-token tile against one block of 16 queries: scores, online softmax, P.V.
// MASKED = the tile is cut by the causal diagonal or by the end of the sequence (lane-wise limits);
// unmasked tiles run the lean path.  `vis` = number of kv positions this lane's query may see.
// ALIBI: every score gets slope * (key position - query position) (log2 units) before the softmax; `dist0` is
// the distance of this lane's query to the tile's first token of this register quad (tok0 + 4*quad - pos).
// RAWREF (ALiBi only): the tile's maximum is taken over the scores WITHOUT the bias.  The bias of a visible key is
// never positive, so a reference exponent that bounds the scores alone bounds the biased ones too, and the tiles
// that run without a maximum search can keep it although the bias of their keys grows from tile to tile.
template <int KS, int NCB, int TB, bool MASKED, bool ALIBI, class F = bf16x8, bool RAWREF = false>
__device__ __forceinline__ void attend_block(const F (&kf)[TB][KS], const F (&vf)[TB / 2][NCB],
                                             const F (&q)[KS], const F& ones, f32x4 (&acc)[NCB],
                                             f32x4& lacc, float& m, float scale_log2, int tok0, int vis, int quad,
                                             float slope, int dist0) {
  // The query arrives already multiplied by log2(e)/sqrt(d_head), and the score accumulators start at minus the
  // reference exponent: what the matrix cores return is the argument of exp2, no vector instruction in between.
  const float m_base = m == -INFINITY ? 0.f : m;
  f32x4 s[TB];
#pragma unroll
  for (int tb = 0; tb < TB; ++tb) {
    s[tb] = f32x4{-m_base, -m_base, -m_base, -m_base};
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) s[tb] = mfma16(kf[tb][ks], q[ks], s[tb]);
  }
  float mx = -INFINITY;
  if constexpr (ALIBI && RAWREF) {
    const float base = slope * (float)dist0;
#pragma unroll
    for (int tb = 0; tb < TB; ++tb)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const bool hidden = MASKED && tok0 + tb * 16 + quad * 4 + i >= vis;
        mx = fmaxf(mx, hidden ? -INFINITY : s[tb][i]);
        s[tb][i] = hidden ? -INFINITY : s[tb][i] + fmaf(slope, (float)(tb * 16 + i), base);
      }
  } else {
    if (ALIBI) {
      const float base = slope * (float)dist0;
#pragma unroll
      for (int tb = 0; tb < TB; ++tb)
#pragma unroll
        for (int i = 0; i < 4; ++i) s[tb][i] += fmaf(slope, (float)(tb * 16 + i), base);
    }
#pragma unroll
    for (int tb = 0; tb < TB; ++tb)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if (MASKED && tok0 + tb * 16 + quad * 4 + i >= vis) s[tb][i] = -INFINITY;
        mx = fmaxf(mx, s[tb][i]);
      }
  }
  mx = quad_column_max(mx);                                  // relative to m_base
  // m is a reference exponent, not the exact running max: it only moves when the max has grown by more
  // than kLazy (log2 units), so P stays <= 2^kLazy -- harmless in bf16 / fp32 -- and the accumulators are
  // rescaled a handful of times per query instead of at every tile.  The final o = acc / l is unchanged.
  if (__any(m == -INFINITY ? mx > -INFINITY : mx > kLazy)) {
    const float m_new = fmaxf(m, mx + m_base);
    const float m_safe = m_new == -INFINITY ? 0.f : m_new;
    const float alpha = __builtin_amdgcn_exp2f(m - m_safe);   // m = -inf -> 0
    const float delta = m_safe - m_base;
    lacc *= alpha;
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) acc[cb] *= alpha;
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) s[tb] -= delta;
    m = m_new;
  }
  F pf[TB / 2];
#pragma unroll
  for (int u = 0; u < TB / 2; ++u)
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
      for (int i = 0; i < 4; ++i) pf[u][h * 4 + i] = (typename FragElem<F>::type)__builtin_amdgcn_exp2f(s[2 * u + h][i]);
#pragma unroll
  for (int u = 0; u < TB / 2; ++u) lacc = mfma16(ones, pf[u], lacc);
#pragma unroll
  for (int u = 0; u < TB / 2; ++u)
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) acc[cb] = mfma16(vf[u][cb], pf[u], acc[cb]);
}

// The same tile against the same block when nothing is masked and the reference exponent m is already finite,
// without looking for the tile's maximum: the exponentials are taken against the reference as it stands and the
// caller inspects the row sums afterwards (see the tile loop).  Per score that leaves the exponential and half a
// conversion for the vector unit.
// ALIBI: the accumulators start at bias - m instead (one multiply-add per score, as the exact form pays for the bias
// alone); m must then bound the scores without the bias (RAWREF above).
template <int KS, int NCB, int TB, class F = bf16x8, bool ALIBI = false>
__device__ __forceinline__ void attend_block_optimistic(const F (&kf)[TB][KS], const F (&vf)[TB / 2][NCB],
                                                        const F (&q)[KS], const F& ones, f32x4 (&acc)[NCB],
                                                        f32x4& lacc, float m, float slope = 0.f, int dist0 = 0) {
  const f32x4 neg_m{-m, -m, -m, -m};
  f32x4 s[TB];
  if constexpr (ALIBI) {
    const float base = fmaf(slope, (float)dist0, -m);
#pragma unroll
    for (int tb = 0; tb < TB; ++tb)
#pragma unroll
      for (int i = 0; i < 4; ++i) s[tb][i] = fmaf(slope, (float)(tb * 16 + i), base);
  }
  // Two waves share a SIMD, and of two that are ready the older one issues.  Its run of exponentials would keep
  // the issue port for itself while the other wave's matrix instructions -- which need the port only half of
  // their time -- wait; with the matrix phases at the higher priority the wave that is multiplying goes first and
  // the other one's exponentials fill the gaps (3 % of the kernel's time at config 4; the reverse costs 2 %).
  __builtin_amdgcn_s_setprio(1);
#pragma unroll
  for (int tb = 0; tb < TB; ++tb) {
    if constexpr (ALIBI) s[tb] = mfma16(kf[tb][0], q[0], s[tb]);
    else s[tb] = mfma16(kf[tb][0], q[0], neg_m);
#pragma unroll
    for (int ks = 1; ks < KS; ++ks) s[tb] = mfma16(kf[tb][ks], q[ks], s[tb]);
  }
  __builtin_amdgcn_s_setprio(0);
  F pf[TB / 2];
#pragma unroll
  for (int u = 0; u < TB / 2; ++u)
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
      for (int i = 0; i < 4; ++i) pf[u][h * 4 + i] = (typename FragElem<F>::type)__builtin_amdgcn_exp2f(s[2 * u + h][i]);
  __builtin_amdgcn_s_setprio(1);
#pragma unroll
  for (int u = 0; u < TB / 2; ++u) lacc = mfma16(ones, pf[u], lacc);
#pragma unroll
  for (int u = 0; u < TB / 2; ++u)
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) acc[cb] = mfma16(vf[u][cb], pf[u], acc[cb]);
}

// Clears value slots of tokens >= limit (never written, arbitrary bits) so that 0 * x stays 0.
template <int NCB, int TB>
__device__ __forceinline__ void clear_tail(bf16x8 (&vf)[TB / 2][NCB], int tok0, int limit, int quad) {
#pragma unroll
  for (int u = 0; u < TB / 2; ++u)
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int tok = tok0 + u * 32 + (j >> 2) * 16 + quad * 4 + (j & 3);
        if (tok >= limit) vf[u][cb][j] = (__bf16)0.0f;
      }
}

template <int NCB, int QT>
__device__ __forceinline__ void write_out(const PrefillArgs& a, const f32x4 (&acc)[QT][NCB], const f32x4 (&lacc)[QT],
                                          const float (&m)[QT], int b, int head, int q0, int col, int quad) {
  const Geo& g = a.g;
#pragma unroll
  for (int qb = 0; qb < QT; ++qb) {
    const int qi = q0 + qb * 16 + col;
    const float l = lacc[qb][0];
    const float inv = l > 0.f ? 1.0f / l : 0.f;
    if (a.part_o) {
      if (qi < a.n_q) {
        const int64_t row = ((int64_t)b * a.n_q + qi) * g.n_heads + head;
        float* prow = a.part_o + row * g.r_v;
        if (quad == 0) {
          a.part_ml[2 * row] = m[qb];
          a.part_ml[2 * row + 1] = l;
        }
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int c = cb * 16 + quad * 4 + i;
            if (c < g.r_v) prow[c] = acc[qb][cb][i] * inv;
          }
      }
      continue;
    }
    uint16_t* orow = a.out + (((int64_t)b * a.n_q + qi) * g.n_heads + head) * g.r_v;
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) {
      const int c = cb * 16 + quad * 4;
      if (qi >= a.n_q) {
      } else if (c + 3 < g.r_v && (g.r_v & 3) == 0) {          // rows of whole 8-byte units
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

// Every wave reads its K / V fragments straight from global memory (the four waves of a workgroup walk
// the same tiles, so three of four reads hit in L1/L2); the next tile is requested into the registers the
// current one has just left.  (Staging the tiles through LDS was measured and is slower here.)
// TB = 16-token blocks per step of the walk: 4 (a whole 64-token cache tile per step) or 2 (half a tile: half the
// fragment registers, for the ranks whose whole tile does not fit beside the accumulators).
template <int KS, int NCB, int QT, int WPE, bool ALIBI, int TB>
__global__ __launch_bounds__(256, WPE) void prefill_bf16_direct_kernel(PrefillArgs a) {
  static_assert(TB == 4 || TB == 2, "a step is a whole or half a cache tile");
  constexpr int kStep = 16 * TB;                                // tokens per step
  constexpr int kSpt = 4 / TB;                                  // steps per cache tile
  const Geo& g = a.g;
  // 1-D grid ordered by work: the latest (longest) query tiles of every (sequence, head) come first
  const int hb = g.n_heads * a.batch;
  const int q_tile = a.n_qtiles - 1 - (int)(blockIdx.x / hb);
  const int head = (blockIdx.x % hb) % g.n_heads, b = (blockIdx.x % hb) / g.n_heads;
  const int kvh = head / g.group;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int col = lane & 15, quad = lane >> 4;
  const int nck = g.r_k_pad >> 3;
  constexpr int QW = QT * 16;                                   // queries per wave
  const int q0 = (q_tile * 4 + wave) * QW;                      // first query of this wave
  if (q0 >= a.n_q) return;

  // Sequence lengths and page ids are the same for every lane and do not change while the kernel runs: read
  // through the constant address space they arrive in scalar registers.
  typedef const int32_t __attribute__((address_space(4))) * const_i32_ptr;
  const const_i32_ptr pt_row = (const_i32_ptr)(a.page_table + (int64_t)b * g.max_pages);
  int64_t n64 = ((const_i32_ptr)a.seq_len)[b];
  const int64_t cap = (int64_t)g.max_pages * g.page_tokens;
  if (n64 > cap) n64 = cap;
  if (n64 < 0) n64 = 0;
  const int len = (int)n64;
  const int pos0 = len - a.n_q;                                  // position of query 0 (may be < 0: such queries see nothing)
  const int tiles_per_page = g.page_tokens / kTile;

  bf16x8 qf[QT][KS];
#pragma unroll
  for (int qb = 0; qb < QT; ++qb) {
    const int qi = q0 + qb * 16 + col;
    const uint16_t* qrow = a.q + (((int64_t)b * a.n_q + qi) * g.n_heads + head) * g.r_k;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const int k = ks * 32 + quad * 8;
      if ((g.r_k & 7) == 0) {                                     // rows of whole 16-byte units
        qf[qb][ks] = (qi < a.n_q && k < g.r_k) ? *reinterpret_cast<const bf16x8*>(qrow + k) : zero_frag();
      } else {                                                    // any rank: channel by channel, zero past the rank
        qf[qb][ks] = zero_frag();
        if (qi < a.n_q) {
#pragma unroll
          for (int j = 0; j < 8; ++j)
            if (k + j < g.r_k) qf[qb][ks][j] = __builtin_bit_cast(__bf16, qrow[k + j]);
        }
      }
      // the softmax scale goes into the query (one more rounding to bfloat16, of the size of P's own)
      if (!a.k_compact) {
#pragma unroll
        for (int j = 0; j < 8; ++j) qf[qb][ks][j] = (__bf16)((float)qf[qb][ks][j] * a.scale_log2);
      }
    }
  }
  bf16x8 ones;
#pragma unroll
  for (int j = 0; j < 8; ++j) ones[j] = (__bf16)1.0f;
  float slope = 0.f;                                            // this head's ALiBi slope in log2 units
  if (ALIBI) slope = a.alibi[head] * 1.4426950408889634f;

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
  const int t_end = pos_last >= 0 ? min(pos_last, len - 1) / kStep + 1 : 0;     // in steps

  bf16x8 kf[TB][KS], vf[TB / 2][NCB];
  // step st covers blocks (st % kSpt) * TB .. + TB - 1 of cache tile st / kSpt
  auto tile_page = [&](int st) -> int {
    const int page = pt_row[(st / kSpt) / tiles_per_page];
    return (page >= 0 && page < g.pool_pages) ? page : -1;
  };
  auto load_k = [&](int st, int page) __attribute__((always_inline)) {
    const int t = st / kSpt, tb0 = (st % kSpt) * TB;
    const int64_t kpage = a.k_compact ? (int64_t)b * g.max_pages + t / tiles_per_page : page;
    const uint16_t* base = a.k_pool + kpage * g.k_page + (int64_t)kvh * g.k_slab +
                           (int64_t)(t % tiles_per_page) * (kTile * g.r_k_pad);
#pragma unroll
    for (int tb = 0; tb < TB; ++tb)
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        // only the last k-step can run past the rank's nck chunks; its surplus lanes read the last real chunk
        // instead and drop what they read
        const bool past = ks == KS - 1 && ks * 4 + quad >= nck;
        const int chunk = past ? nck - 1 : ks * 4 + quad;
        const bf16x8 got = *reinterpret_cast<const bf16x8*>(base + ((((tb0 + tb) * nck + chunk) * 16 + col) << 3));
        kf[tb][ks] = past ? zero_frag() : got;
      }
  };
  auto load_v = [&](int st, int page) __attribute__((always_inline)) {
    const int t = st / kSpt, u0 = (st % kSpt) * (TB / 2);
    const uint16_t* base = a.v_pool + (int64_t)page * g.v_page + (int64_t)kvh * g.v_slab +
                           (int64_t)(t % tiles_per_page) * (kTile * g.r_v_pad);
#pragma unroll
    for (int u = 0; u < TB / 2; ++u)
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb)
        vf[u][cb] = *reinterpret_cast<const bf16x8*>(base + ((((u0 + u) * NCB + cb) * 64 + lane) << 3));
  };

  // Unmasked tiles after the first run optimistically: no search for the tile's maximum, the exponentials are
  // taken against the reference exponent the earlier tiles left (exact in floating point whatever the reference,
  // as long as nothing overflows).  Every eighth tile, and after the last, the row sums are looked at -- they only
  // grow between two looks, so nothing is missed: one that passed 2^kGrow moves its reference by kGrow
  // (accumulators scaled down, a handful of times per query at most); one that passed 2^kAbort, or is not a
  // number, means the scores rose by more than the headroom since the last look -- then the wave starts over and
  // takes every tile with the exact maximum (P <= row sum < 2^kAbort otherwise, so the output accumulators are as
  // far from overflow as the values allow).  With the ALiBi bias the reference bounds the scores without the bias
  // (which is never positive for a key a query may see), so the same holds; what the bias can do instead is push
  // every term of a row far below its reference, so a row sum that ends below 2^-kTiny also sends the wave into
  // the exact walk, whose reference follows the biased maximum.
  constexpr float kGrow = 32.0f, kAbort = 64.0f, kTiny = 64.0f;
  bool optimistic = true;
  for (;;) {                                                     // one walk; a second, exact one if the first was lost
    bool lost_walk = false;
    int page = -1;
    if (t_end > 0) {
      page = tile_page(0);
      // a tile without a valid page is still read -- from page 0, which exists -- and all of its tokens are masked
      // (limit = 0 below): no load sits behind a data-dependent branch
      load_k(0, max(page, 0));
      load_v(0, max(page, 0));
    }
    for (int t = 0; t < t_end; ++t) {
      const int tok0 = t * kStep;
      const bool full = page >= 0 && tok0 + kStep - 1 <= pos_first && tok0 + kStep <= len;   // no masking needed
      const int limit = page >= 0 ? len : 0;                       // tokens >= limit do not exist
      const bool have_n = t + 1 < t_end;
      const int page_n = have_n ? tile_page(t + 1) : -1;
      if (full && optimistic && t > 0) {
#pragma unroll
        for (int qb = 0; qb < QT; ++qb)
          attend_block_optimistic<KS, NCB, TB, bf16x8, ALIBI>(kf, vf, qf[qb], ones, acc[qb], lacc[qb], m[qb], slope,
                                                              tok0 + quad * 4 - (pos0 + q0 + qb * 16 + col));
      } else if (full) {
#pragma unroll
        for (int qb = 0; qb < QT; ++qb) {
          const int dist0 = tok0 + quad * 4 - (pos0 + q0 + qb * 16 + col);
          if (ALIBI && optimistic)
            attend_block<KS, NCB, TB, false, ALIBI, bf16x8, ALIBI>(kf, vf, qf[qb], ones, acc[qb], lacc[qb], m[qb],
                                                                   a.scale_log2, tok0, 0, quad, slope, dist0);
          else
            attend_block<KS, NCB, TB, false, ALIBI>(kf, vf, qf[qb], ones, acc[qb], lacc[qb], m[qb], a.scale_log2, tok0, 0,
                                                    quad, slope, dist0);
        }
      } else {
        if (tok0 + kStep > limit) clear_tail<NCB, TB>(vf, tok0, limit, quad);
#pragma unroll
        for (int qb = 0; qb < QT; ++qb) {
          const int vis = min(pos0 + q0 + qb * 16 + col + 1, limit);
          const int dist0 = tok0 + quad * 4 - (pos0 + q0 + qb * 16 + col);
          if (ALIBI && optimistic)
            attend_block<KS, NCB, TB, true, ALIBI, bf16x8, ALIBI>(kf, vf, qf[qb], ones, acc[qb], lacc[qb], m[qb],
                                                                  a.scale_log2, tok0, vis, quad, slope, dist0);
          else
            attend_block<KS, NCB, TB, true, ALIBI>(kf, vf, qf[qb], ones, acc[qb], lacc[qb], m[qb], a.scale_log2, tok0, vis,
                                                   quad, slope, dist0);
        }
      }
      if (ALIBI && optimistic && t + 1 == t_end) {
        bool tiny = false;
#pragma unroll
        for (int qb = 0; qb < QT; ++qb)
          tiny |= q0 + qb * 16 + col < a.n_q && min(pos0 + q0 + qb * 16 + col + 1, len) > 0 &&
                  !(lacc[qb][0] > __builtin_exp2f(-kTiny));
        if (__any(tiny)) {                                           // wave-uniform
          lost_walk = true;
          break;
        }
      }
      if (optimistic && ((t & 7) == 7 || t + 1 == t_end)) {
        bool grown = false;
#pragma unroll
        for (int qb = 0; qb < QT; ++qb) grown |= !(lacc[qb][0] < __builtin_exp2f(kGrow));
        if (__any(grown)) {
          bool lost = false;
#pragma unroll
          for (int qb = 0; qb < QT; ++qb) lost |= !(lacc[qb][0] < __builtin_exp2f(kAbort));
          if (__any(lost)) {                                       // wave-uniform
            lost_walk = true;
            break;
          } else {
#pragma unroll
            for (int qb = 0; qb < QT; ++qb) {
              const bool g_qb = !(lacc[qb][0] < __builtin_exp2f(kGrow));
              const float alpha = g_qb ? __builtin_exp2f(-kGrow) : 1.0f;
              m[qb] += g_qb ? kGrow : 0.0f;
              lacc[qb] *= alpha;
#pragma unroll
              for (int cb = 0; cb < NCB; ++cb) acc[qb][cb] *= alpha;
            }
          }
        }
      }
      // the next tile is requested into the registers the current one has just left; without the barrier the
      // scheduler would start these loads early into a second set of registers and spill
      __builtin_amdgcn_sched_barrier(0);
      if (have_n) {
        load_k(t + 1, max(page_n, 0));
        load_v(t + 1, max(page_n, 0));
      }
      page = page_n;
    }
    if (!lost_walk) break;
    optimistic = false;
#pragma unroll
    for (int qb = 0; qb < QT; ++qb) {
      m[qb] = -INFINITY;
      lacc[qb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb) acc[qb][cb] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
  }
  write_out<NCB, QT>(a, acc, lacc, m, b, head, q0, col, quad);
}

template <int KS, int NCB, bool ALIBI>
static void launch_prefill(const PrefillArgs& a_in, int32_t B, hipStream_t st) {
  // Queries per wave (QT blocks of 16) and tokens per step (TB blocks of 16) from a register estimate: QT
  // accumulator sets (output, row sum, query fragments), the K and V fragments of one step, scores and P, and about
  // 40 for addresses and the rest.  More queries per wave reuse each fragment more often; whole-tile steps have fewer,
  // longer MFMA runs.  A tile loop that spills costs far more than either, so the first shape that fits is taken.
  constexpr auto fits = [](int qt, int tb) {
    return qt * (4 * NCB + 4 + 4 * KS) + 4 * tb * KS + 2 * tb * NCB + 6 * tb + 40 <= 244;
  };
  constexpr int QT = (fits(4, 4) || fits(4, 2)) ? 4 : 2;
  constexpr int TB = fits(QT, 4) ? 4 : 2;
  constexpr int WPE = 2;
  PrefillArgs a = a_in;
  a.batch = B;
  a.n_qtiles = (a.n_q + 64 * QT - 1) / (64 * QT);
  const dim3 grid((uint32_t)(a.n_qtiles * a.g.n_heads * B));
  prefill_bf16_direct_kernel<KS, NCB, QT, WPE, ALIBI, TB><<<grid, 256, 0, st>>>(a);
}

template <int KS, bool ALIBI>
static int dispatch_ncb(int ncb, const PrefillArgs& a, int32_t B, hipStream_t st) {
  switch (ncb) {
    case 1: launch_prefill<KS, 1, ALIBI>(a, B, st); break;
    case 2: launch_prefill<KS, 2, ALIBI>(a, B, st); break;
    case 3: launch_prefill<KS, 3, ALIBI>(a, B, st); break;
    case 4: launch_prefill<KS, 4, ALIBI>(a, B, st); break;
    case 5: launch_prefill<KS, 5, ALIBI>(a, B, st); break;
    case 6: launch_prefill<KS, 6, ALIBI>(a, B, st); break;
    case 7: launch_prefill<KS, 7, ALIBI>(a, B, st); break;
    case 8: launch_prefill<KS, 8, ALIBI>(a, B, st); break;
    default: return EA_ERR_SHAPE;
  }
  return launch_status();
}

template <bool ALIBI>
static int prefill_bf16_launch(const ea_layer_desc* d, const Geo& g, const void* q, const void* k_pool,
                               const void* v_pool, const int32_t* page_table, const int32_t* seq_len, void* out,
                               int32_t B, int32_t n, hipStream_t st, int32_t k_compact, const float* alibi,
                               float* part_o = nullptr, float* part_ml = nullptr) {
  if ((int64_t)((n + 63) / 64) * g.n_heads * B > INT32_MAX) return EA_ERR_SHAPE;
  PrefillArgs a;
  a.q = (const uint16_t*)q;
  a.k_pool = (const uint16_t*)k_pool;
  a.v_pool = (const uint16_t*)v_pool;
  a.page_table = page_table;
  a.seq_len = seq_len;
  a.out = (uint16_t*)out;
  a.g = g;
  a.n_q = n;
  a.k_compact = k_compact;
  a.alibi = alibi;
  a.scale_log2 = 1.4426950408889634f / sqrtf((float)d->d_head);
  a.part_o = part_o;
  a.part_ml = part_ml;
  const int ks = (g.r_k_pad + 31) / 32, ncb = g.r_v_pad / 16;
  switch (ks) {
    case 1: return dispatch_ncb<1, ALIBI>(ncb, a, B, st);
    case 2: return dispatch_ncb<2, ALIBI>(ncb, a, B, st);
    case 3: return dispatch_ncb<3, ALIBI>(ncb, a, B, st);
    case 4: return dispatch_ncb<4, ALIBI>(ncb, a, B, st);
    default: return EA_ERR_SHAPE;
  }
}

}  // namespace ea
