// Prefill-phase attention over a cache whose older tokens are held as 4-bit codes (Eq. 2 in rank space, causal;
// quantisation paragraph of the results): what lets a long prompt be prefilled chunk by chunk with every finished
// chunk quantised at once, so that the prompt never exists in 16 bits as a whole.
//
// A sequence is q4_len[b] tokens in the 4-bit pools followed by tail_len[b] tokens in the bfloat16 pools; the n
// queries are its last n tokens and all lie in the bfloat16 part.  Three launches:
//   1. the bfloat16 prefill kernel over the tail (causal), leaving its result as a part (normalised output,
//      reference exponent, row sum per query row);
//   2. prefill_q4_kernel over the 4-bit part, which every query sees in full: the same two matrix-core
//      contractions, the tiles expanded from their codes in registers to half-precision fragments
//      (code -> scale * code + zero, one packed subtraction and one packed fma per two codes), leaving a part, too;
//   3. the merge of the two parts per query row.
#include "ea_prefill_kernel.h"
#include "ea_q4.h"

namespace ea {

struct PrefillQ4Args {
  const uint16_t* q;          // [B, n_q, H, r_k] bfloat16
  const uint8_t* kq_pool;
  const uint8_t* vq_pool;
  const int32_t* page_table;  // [B, max_pages] of the 4-bit pools
  const int32_t* q4_len;
  float* part_o;              // [B * n_q * H, r_v]
  float* part_ml;             // [B * n_q * H, 2]
  Geo g;                      // max_pages / pool_pages are those of the 4-bit pools
  Q4Geo qg;
  int32_t n_q, batch, n_qtiles;
  float scale_log2;
};

// One workgroup = 4 waves = 4 * QT * 16 consecutive queries of one (sequence, head); every wave walks all tiles of
// the 4-bit part, half a tile (32 tokens) per step, and keeps QT blocks of 16 queries as matrix-core columns.
// HALF: only half a tile is held expanded at a time (larger ranks: half the fragment registers; the next tile's codes
// are then requested after the second half has been expanded instead of before the first step).
// BITS = 4 or 3: the width of a code.
template <int KS, int NCB, int QT, bool HALF, int BITS>
__global__ __launch_bounds__(256, 2) void prefill_q4_kernel(PrefillQ4Args a) {
  typedef Codes<BITS> CD;
  constexpr int NVP = NCB / 2;          // 16-byte units of value codes per lane
  constexpr bool VODD = (NCB & 1) != 0; // ... plus one 8-byte unit
  const Geo& g = a.g;
  const Q4Geo& qg = a.qg;
  const int hb = g.n_heads * a.batch;
  const int q_tile = (int)(blockIdx.x / hb);
  const int head = (blockIdx.x % hb) % g.n_heads, b = (blockIdx.x % hb) / g.n_heads;
  const int kvh = head / g.group;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int col = lane & 15, quad = lane >> 4;
  constexpr int QW = QT * 16;
  const int q0 = (q_tile * 4 + wave) * QW;
  if (q0 >= a.n_q) return;

  typedef const int32_t __attribute__((address_space(4))) * const_i32_ptr;
  const const_i32_ptr pt_row = (const_i32_ptr)(a.page_table + (int64_t)b * g.max_pages);
  int64_t n64 = ((const_i32_ptr)a.q4_len)[b];
  const int64_t cap = (int64_t)g.max_pages * g.page_tokens;
  if (n64 > cap) n64 = cap;
  if (n64 < 0) n64 = 0;
  const int n_tiles = (int)(n64 / (kTile * qg.tpg)) * qg.tpg;      // whole key groups only
  const int tiles_per_page = qg.tiles_per_page;

  // B operand of the score product: q^T in half precision, times log2(e)/sqrt(d_head)
  f16x8 qf[QT][KS];
#pragma unroll
  for (int qb = 0; qb < QT; ++qb) {
    const int qi = q0 + qb * 16 + col;
    const uint16_t* qrow = a.q + (((int64_t)b * a.n_q + (qi < a.n_q ? qi : 0)) * g.n_heads + head) * g.r_k;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int k = ks * 32 + quad * 8 + j;
        const float v = (qi < a.n_q && k < g.r_k) ? __builtin_bit_cast(float, (uint32_t)qrow[k < g.r_k ? k : 0] << 16) : 0.f;
        qf[qb][ks][j] = (_Float16)(v * a.scale_log2);
      }
  }
  f16x8 ones, negoff;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    ones[j] = (_Float16)1.0f;
    negoff[j] = (j & 2) ? (_Float16)-CD::kOffLo : (_Float16)-1024.0f;     // what the unpacking adds to the codes
  }
  uint32_t magic1024 = 0x64006400u, magic64 = CD::kMagicLo;
  asm volatile("" : "+v"(magic1024), "+v"(magic64));

  f32x4 acc[QT][NCB], lacc[QT];
  float m[QT];
#pragma unroll
  for (int qb = 0; qb < QT; ++qb) {
    m[qb] = -INFINITY;
    lacc[qb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) acc[qb][cb] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  // the codes and scales of one tile, as they come from memory
  u32x4 kc[KS];
  f16x8 ksc[KS], kzr[KS];
  u32x4 vc[NVP > 0 ? NVP : 1];
  u32x2 vcl = {0u, 0u};
  f16x8 vsc[2], vzr[2];
  auto page_of = [&](int t) -> int {
    const int page = pt_row[t / tiles_per_page];
    return (page >= 0 && page < g.pool_pages) ? page : -1;
  };
  auto load_tile = [&](int t, int page) __attribute__((always_inline)) {
    const int tin = t % tiles_per_page;
    const uint8_t* slab = a.kq_pool + (int64_t)page * qg.k_page + (int64_t)kvh * qg.k_slab;
    const uint8_t* kbase = slab + q4_k_tile_off(qg, tin);
    const uint8_t* scales = slab + q4_k_group_scales_off(qg, tin);
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) {
      // lanes of a quad the last k-step does not have re-read quad 0's unit; their query channels are zero
      const bool past = kk == KS - 1 && kk * 4 + quad >= qg.nch;
      kc[kk] = CD::template load<false>(kbase + kk * CD::kRun + (past ? col : lane) * CD::kUnit);
      const uint8_t* sp = scales + (kk * 4 + (past ? 0 : quad)) * 32;
      ksc[kk] = *reinterpret_cast<const f16x8*>(sp);
      kzr[kk] = *reinterpret_cast<const f16x8*>(sp + 16);
    }
    const uint8_t* vbase = a.vq_pool + (int64_t)page * qg.v_page + ((int64_t)kvh * tiles_per_page + tin) * qg.v_tile;
#pragma unroll
    for (int pp = 0; pp < NVP; ++pp) vc[pp] = CD::template load<false>(vbase + pp * CD::kRun + lane * CD::kUnit);
    if constexpr (VODD) vcl = *reinterpret_cast<const u32x2*>(vbase + NVP * CD::kRun + lane * 8);
    const uint8_t* sp = vbase + (NVP * CD::kRun + (VODD ? 512 : 0));      // behind the codes
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      vsc[u] = *reinterpret_cast<const f16x8*>(sp + (u * 4 + quad) * 16);
      vzr[u] = *reinterpret_cast<const f16x8*>(sp + 128 + (u * 4 + quad) * 16);
    }
  };
  auto v_frag = [&](int cb, int u) -> f16x8 {
    if (VODD && cb == NCB - 1) return CD::frag2(vcl, u, magic1024, magic64);
    return CD::frag(vc[cb >> 1], (cb & 1) * 2 + u, magic1024, magic64);
  };

  // Tiles after the first run without a search for the tile's maximum, as in the bfloat16 kernel: the exponentials
  // are taken against the reference exponent the earlier tiles left, the row sums are looked at every eighth tile and
  // after the last -- above 2^kGrow the reference moves, above 2^kAbort (or not a number) the wave starts over and
  // takes every tile with the exact maximum.  Half precision ends at 2^16, hence the smaller headroom: P <= row sum
  // < 2^kAbort.
  constexpr float kGrow = 8.0f, kAbort = 15.0f;
  bool optimistic = true;
  for (;;) {
    bool lost_walk = false;
    int page = -1;
    if (n_tiles > 0) {
      page = page_of(0);
      load_tile(0, max(page, 0));        // a tile without a valid page is still read, from page 0, and skipped below
    }
    bool first = true;                   // no valid tile attended yet: the reference exponents are not set
    for (int t = 0; t < n_tiles; ++t) {
      // ---- expand the tile (or half of it): K fragments [16-token block][k-step], V fragments [channel block]
      constexpr int NH = HALF ? 1 : 2;                  // halves held at a time
      f16x8 kf[NH][2][KS], vf[NH][1][NCB];
      auto expand = [&](int half, int slot) __attribute__((always_inline)) {
#pragma unroll
        for (int kk = 0; kk < KS; ++kk)
#pragma unroll
          for (int tb = 0; tb < 2; ++tb)
            kf[slot][tb][kk] = (CD::frag(kc[kk], 2 * half + tb, magic1024, magic64) + negoff) * ksc[kk] + kzr[kk];
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb)
          vf[slot][0][cb] = (v_frag(cb, half) + negoff) * vsc[half] + vzr[half];
      };
      const bool valid = page >= 0;
      const bool lean = optimistic && !first;         // wave-uniform
      auto attend = [&](int slot, bool fast) __attribute__((always_inline)) {
        if (fast) {
#pragma unroll
          for (int qb = 0; qb < QT; ++qb)
            attend_block_optimistic<KS, NCB, 2, f16x8>(kf[slot], vf[slot], qf[qb], ones, acc[qb], lacc[qb], m[qb]);
        } else {
#pragma unroll
          for (int qb = 0; qb < QT; ++qb)
            attend_block<KS, NCB, 2, false, false, f16x8>(kf[slot], vf[slot], qf[qb], ones, acc[qb], lacc[qb], m[qb],
                                                          a.scale_log2, 0, 0, quad, 0.f, 0);
        }
      };
      const bool have_n = t + 1 < n_tiles;
      const int page_n = have_n ? page_of(t + 1) : -1;
      // (the scheduling barriers keep the phases apart: without them the compiler starts the next phase's loads and
      // expansions early, into registers it does not have)
      if constexpr (!HALF) {
        expand(0, 0);
        expand(1, 1);
        __builtin_amdgcn_sched_barrier(0);
        if (have_n) load_tile(t + 1, max(page_n, 0));   // the registers of the codes are free: request the next tile
        __builtin_amdgcn_sched_barrier(0);
        if (valid) {
          attend(0, lean);
          __builtin_amdgcn_sched_barrier(0);
          attend(1, optimistic);                        // the first half has set the references
        }
      } else {
        expand(0, 0);
        __builtin_amdgcn_sched_barrier(0);
        if (valid) attend(0, lean);
        __builtin_amdgcn_sched_barrier(0);
        expand(1, 0);
        __builtin_amdgcn_sched_barrier(0);
        if (have_n) load_tile(t + 1, max(page_n, 0));
        __builtin_amdgcn_sched_barrier(0);
        if (valid) attend(0, optimistic);
      }
      __builtin_amdgcn_sched_barrier(0);
      if (valid) first = false;
      if (optimistic && ((t & 7) == 7 || t + 1 == n_tiles)) {
        bool grown = false;
#pragma unroll
        for (int qb = 0; qb < QT; ++qb) grown |= !(lacc[qb][0] < __builtin_exp2f(kGrow));
        if (__any(grown)) {
          bool lost = false;
#pragma unroll
          for (int qb = 0; qb < QT; ++qb) lost |= !(lacc[qb][0] < __builtin_exp2f(kAbort));
          if (__any(lost)) {
            lost_walk = true;
            break;
          }
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
  // ---- the part this kernel contributes
#pragma unroll
  for (int qb = 0; qb < QT; ++qb) {
    const int qi = q0 + qb * 16 + col;
    if (qi >= a.n_q) continue;
    const float l = lacc[qb][0];
    const float inv = l > 0.f ? 1.0f / l : 0.f;
    const int64_t row = ((int64_t)b * a.n_q + qi) * g.n_heads + head;
    if (quad == 0) {
      a.part_ml[2 * row] = m[qb];
      a.part_ml[2 * row + 1] = l;
    }
    float* prow = a.part_o + row * g.r_v;
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int c = cb * 16 + quad * 4 + i;
        if (c < g.r_v) prow[c] = acc[qb][cb][i] * inv;
      }
  }
}

// out[row] = (w0 l0 o0 + w1 l1 o1) / (w0 l0 + w1 l1), w_i = 2^(m_i - max(m_0, m_1)); a part without tokens has l = 0.
__global__ __launch_bounds__(256) void merge_prefill_parts_kernel(const float* o0, const float* ml0, const float* o1,
                                                                  const float* ml1, uint16_t* out, int64_t rows,
                                                                  int32_t r_v) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= rows * r_v) return;
  const int64_t row = idx / r_v;
  const float m0 = ml0[2 * row], l0 = ml0[2 * row + 1], m1 = ml1[2 * row], l1 = ml1[2 * row + 1];
  const float M = fmaxf(l0 > 0.f ? m0 : -INFINITY, l1 > 0.f ? m1 : -INFINITY);
  float val = 0.f;
  if (M != -INFINITY) {
    const float w0 = l0 > 0.f ? __builtin_amdgcn_exp2f(m0 - M) * l0 : 0.f;
    const float w1 = l1 > 0.f ? __builtin_amdgcn_exp2f(m1 - M) * l1 : 0.f;
    val = (w0 * o0[idx] + w1 * o1[idx]) / (w0 + w1);
  }
  out[idx] = f32_to_bf16_rne(val);
}

template <int KS, int NCB>
static void launch_prefill_q4(PrefillQ4Args a, hipStream_t st) {
  // Queries per wave (QT blocks of 16) and how much of a tile is held expanded, from a register estimate: the
  // expanded fragments, the codes and scales of a tile as they come from memory, QT sets of accumulators and query
  // fragments, about 40 for scores, probabilities and addresses.  The first shape that fits is taken.
  constexpr auto fits = [](int qt, bool half) {
    const int frag = (half ? 2 : 4) * KS * 4 + (half ? 1 : 2) * NCB * 4;
    const int codes = KS * 4 + KS * 8 + NCB * 2 + 16;
    return frag + codes + qt * (NCB * 4 + 4 + KS * 4) + 6 * NCB + 40 <= 250;     // (6 * NCB: fitted to what spills)
  };
  constexpr int QT = (fits(2, false) || fits(2, true)) ? 2 : 1;
  constexpr bool HALF = !fits(QT, false);
  a.n_qtiles = (a.n_q + 64 * QT - 1) / (64 * QT);
  const dim3 grid((uint32_t)(a.n_qtiles * a.g.n_heads * a.batch));
  if (a.qg.bits == 3) prefill_q4_kernel<KS, NCB, QT, HALF, 3><<<grid, 256, 0, st>>>(a);
  else prefill_q4_kernel<KS, NCB, QT, HALF, 4><<<grid, 256, 0, st>>>(a);
}

template <int KS>
static int dispatch_ncb_prefill_q4(int ncb, const PrefillQ4Args& a, hipStream_t st) {
  switch (ncb) {
    case 1: launch_prefill_q4<KS, 1>(a, st); break;
    case 2: launch_prefill_q4<KS, 2>(a, st); break;
    case 3: launch_prefill_q4<KS, 3>(a, st); break;
    case 4: launch_prefill_q4<KS, 4>(a, st); break;
    case 5: launch_prefill_q4<KS, 5>(a, st); break;
    case 6: launch_prefill_q4<KS, 6>(a, st); break;
    case 7: launch_prefill_q4<KS, 7>(a, st); break;
    case 8: launch_prefill_q4<KS, 8>(a, st); break;
    default: return EA_ERR_SHAPE;
  }
  return launch_status();
}

int prefill_q4(const ea_layer_desc* d, const Geo& gq, const Q4Geo& qg, const void* q, const void* kq_pool,
               const void* vq_pool, const int32_t* q4_page_table, const int32_t* q4_len, const Geo& gt,
               const void* k_pool, const void* v_pool, const int32_t* tail_page_table, const int32_t* tail_len,
               void* out, int32_t B, int32_t n, float* ws, hipStream_t st) {
  const int64_t rows = (int64_t)B * n * gq.n_heads;
  if ((int64_t)((n + 63) / 64) * gq.n_heads * B > INT32_MAX || rows * gq.r_v > (int64_t)INT32_MAX * 256) return EA_ERR_SHAPE;
  float* o_tail = ws;
  float* ml_tail = o_tail + rows * gq.r_v;
  float* o_q4 = ml_tail + 2 * rows;
  float* ml_q4 = o_q4 + rows * gq.r_v;
  int rc = prefill_bf16(d, gt, q, k_pool, v_pool, tail_page_table, tail_len, nullptr, B, n, st, 0, o_tail, ml_tail);
  if (rc != EA_OK) return rc;
  PrefillQ4Args a;
  a.q = (const uint16_t*)q;
  a.kq_pool = (const uint8_t*)kq_pool;
  a.vq_pool = (const uint8_t*)vq_pool;
  a.page_table = q4_page_table;
  a.q4_len = q4_len;
  a.part_o = o_q4;
  a.part_ml = ml_q4;
  a.g = gq;
  a.qg = qg;
  a.n_q = n;
  a.batch = B;
  a.scale_log2 = 1.4426950408889634f / sqrtf((float)d->d_head);
  switch (qg.ks) {
    case 1: rc = dispatch_ncb_prefill_q4<1>(qg.ncb, a, st); break;
    case 2: rc = dispatch_ncb_prefill_q4<2>(qg.ncb, a, st); break;
    case 3: rc = dispatch_ncb_prefill_q4<3>(qg.ncb, a, st); break;
    case 4: rc = dispatch_ncb_prefill_q4<4>(qg.ncb, a, st); break;
    default: return EA_ERR_SHAPE;
  }
  if (rc != EA_OK) return rc;
  const int64_t total = rows * gq.r_v;
  merge_prefill_parts_kernel<<<dim3((uint32_t)((total + 255) / 256)), 256, 0, st>>>(o_tail, ml_tail, o_q4, ml_q4,
                                                                                   (uint16_t*)out, rows, gq.r_v);
  return launch_status();
}

}  // namespace ea
