// Generation-phase attention over the 4-bit group-quantised part of the rank-r cache (keys: scale and zero per
// channel and 64-token tile; values: per token).  The codes never become 16-bit values in memory:
//   scores   s[t,h] = sum_c (scale_c code[t,c] + zero_c) q[h,c]
//                   = sum_c (off_c + code[t,c]) (scale_c q[h,c]) + sum_c zero_c q[h,c] - sum_c off_c scale_c q[h,c]:
//            the scales go into the query once per tile, the nibbles become fp16 numbers "offset + code" with
//            one mask-and-or each (see unpack_q4), and the two constant terms are two more matrix-core products
//            whose result starts the score accumulators;
//   output   o[h,c] = sum_t p[h,t] (scale_t code[t,c] + zero_t)
//                   = sum_t (p scale)[h,t] (off_t + code[t,c]) + sum_t p[h,t] zero_t - sum_t off_t (p scale)[h,t]:
//            the scales go into the probabilities, the constant terms are matrix-core products again, beside
//            the one that makes the softmax denominators.
// The kernel always writes split partials (m, l, acc).  The 16-bit tail of the sequences is attended in the same
// launch: the workgroups of one more grid row run the bfloat16 kernel's body (half-tile form, which needs no more
// registers than the 4-bit path) into the last slot of the workspace; one merge finishes.
#include "ea_decode_kernel.h"
#include "ea_q4.h"

namespace ea {

struct DecodeQ4Args {
  const float* q;
  const uint8_t* kq_pool;
  const uint8_t* vq_pool;
  const int32_t* page_table;
  const int32_t* q4_len;
  float* ws;
  Geo g;            // max_pages / pool_pages are those of the 4-bit pools
  Q4Geo qg;
  int32_t n_splits;
  int32_t ws_slots;
  float scale_log2;
  int32_t n_batch;
  int32_t has_tail;     // further grid slices attend the bfloat16 tail described by `tail`
  DecodeArgs tail;
  // ALiBi variant only: slopes [H] (natural-log units, >= 0); the newest token (the query) is the last one of the
  // tail, or of the 4-bit part when there is no tail
  const float* alibi;
  const int32_t* tail_len;
};

// BITS = 4 or 3: the width of a code (see ea_q4.h for the two packings; everything after the unpacking is the same).
template <int KS, int NCB, bool ALIBI, int BITS = 4>
__global__ __launch_bounds__(256, 2) void decode_q4_kernel(DecodeQ4Args a) {
  typedef Codes<BITS> CD;
  __shared__ union {
    MergeSmemQ4<NCB> q4;
    DecodeSmem<KS, NCB, 2, 0> tail;
  } smu;
  constexpr int NVP = NCB / 2;          // 16-byte units of value codes per lane
  constexpr bool VODD = (NCB & 1) != 0; // ... plus one 8-byte unit
  const Geo& g = a.g;
  const Q4Geo& qg = a.qg;
  const int kvh = blockIdx.x, split = blockIdx.y, b = blockIdx.z;
  if (b >= a.n_batch) {
    // The grid's last slices (they are dispatched last, so they do not disturb the placement of the long
    // workgroups) attend the bfloat16 tails: one workgroup per (sequence, kv head).
    const int t = ((b - a.n_batch) * a.n_splits + split) * g.n_kv_heads + kvh;
    const int tb = t / g.n_kv_heads;
    if (tb < a.n_batch) decode_bf16_body<KS, NCB, 2, 2, 0, ALIBI>(a.tail, t % g.n_kv_heads, 0, tb, a.n_batch, smu.tail);
    return;
  }
  MergeSmemQ4<NCB>& sm = smu.q4;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int col = lane & 15, quad = lane >> 4;
  const int G = g.group;

  typedef const int32_t __attribute__((address_space(4))) * const_i32_ptr;
  const const_i32_ptr len_c = (const_i32_ptr)a.q4_len;
  const const_i32_ptr pt_row = (const_i32_ptr)(a.page_table + (int64_t)b * g.max_pages);
  int64_t n64 = len_c[b];
  const int64_t cap = (int64_t)g.max_pages * g.page_tokens;
  if (n64 > cap) n64 = cap;
  if (n64 < 0) n64 = 0;
  // whole key groups only: a ragged end is not part of the 4-bit cache
  const int n_tiles = (int)(n64 / (kTile * qg.tpg)) * qg.tpg;
  const int per = (n_tiles + a.n_splits - 1) / a.n_splits;
  const int t_begin = split * per;
  const int t_end = min(n_tiles, t_begin + per);
  const int tiles_per_page = qg.tiles_per_page;
  float alibi_slope = 0.f;       // this lane's head, log2 units
  int pos_q = 0;                 // position of the query
  if constexpr (ALIBI) {
    alibi_slope = col < G ? a.alibi[kvh * G + col] * 1.4426950408889634f : 0.f;
    int64_t tail = a.tail_len ? (int64_t)((const_i32_ptr)a.tail_len)[b] : 0;
    if (tail < 0) tail = 0;
    pos_q = (int)((int64_t)n_tiles * kTile + tail - 1);
  }

  // B operand of the score product: q^T in fp16, already times log2(e)/sqrt(d_head); lane (col, quad) holds
  // channels 32*ks + 8*quad .. +7 of head col.
  f16x8 q16[KS];
  {
    const float* qrow = a.q + ((int64_t)b * g.n_heads + (int64_t)kvh * G + (col < G ? col : 0)) * g.r_k;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int k = ks * 32 + quad * 8 + j;
        const float v = (col < G && k < g.r_k) ? qrow[k < g.r_k ? k : 0] * a.scale_log2 : 0.f;
        q16[ks][j] = (_Float16)v;
      }
    }
  }
  // minus the offsets the unpacked codes carry, and ones
  f16x8 negoff, ones;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    negoff[j] = (j & 2) ? (_Float16)-CD::kOffLo : (_Float16)-1024.0f;   // what the unpacking adds
    ones[j] = (_Float16)1.0f;
  }
  uint32_t magic1024 = 0x64006400u, magic64 = CD::kMagicLo;    // (3-bit codes: 128.0)
  asm volatile("" : "+v"(magic1024), "+v"(magic64));   // keep them in vector registers

  f32x4 acc[NCB];
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb) acc[cb] = f32x4{0.f, 0.f, 0.f, 0.f};
  f32x4 lacc = {0.f, 0.f, 0.f, 0.f};   // every row: sum_t p
  f32x4 corr = {0.f, 0.f, 0.f, 0.f};   // every row: sum_t p zero_t - sum_t offset (p scale)_t
  float m = -INFINITY;

  u32x4 kc[KS];                        // 3-bit codes: the unit's three dwords in [0..2], group 3's word in [3]
  f16x8 ksc[KS], kzr[KS];
  u32x4 vc[NVP > 0 ? NVP : 1];
  u32x2 vcl = {0u, 0u};
  f16x8 vsc[2], vzr[2];
  constexpr int kUnit = CD::kUnit, kRun = CD::kRun;   // bytes of a lane's unit and of a run of 64 of them

  struct Pos {
    int tile, lp, tin;
  };
  Pos cur;
  cur.tile = t_begin + wave;           // the four waves interleave tiles
  cur.lp = cur.tile / tiles_per_page;
  cur.tin = cur.tile % tiles_per_page;
  auto advance = [&](Pos p) -> Pos {
    p.tile += 4;
    p.tin += 4;
    while (p.tin >= tiles_per_page) {
      p.tin -= tiles_per_page;
      p.lp += 1;
    }
    return p;
  };
  auto page_of = [&](const Pos& p) -> int {
    const int page = pt_row[p.lp];
    return (page >= 0 && page < g.pool_pages) ? page : -1;
  };
  auto load_k = [&](const Pos& p, int page) {
    const uint8_t* slab = a.kq_pool + (int64_t)page * qg.k_page + (int64_t)kvh * qg.k_slab;
    const uint8_t* base = slab + q4_k_tile_off(qg, p.tin);
    const uint8_t* scales = slab + q4_k_group_scales_off(qg, p.tin);     // of the tile's key group
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) {
      // lanes of a quad the last k-step does not have re-read quad 0's unit; their query channels are zero
      const bool past = kk == KS - 1 && kk * 4 + quad >= qg.nch;
      const int off = kk * kRun + (past ? col : lane) * kUnit;
      kc[kk] = CD::template load<true>(base + off);
      const uint8_t* sp = scales + (kk * 4 + quad) * 32;
      ksc[kk] = *reinterpret_cast<const f16x8*>(sp);
      kzr[kk] = *reinterpret_cast<const f16x8*>(sp + 16);
    }
  };
  auto load_v = [&](const Pos& p, int page) {
    const uint8_t* base = a.vq_pool + (int64_t)page * qg.v_page + ((int64_t)kvh * tiles_per_page + p.tin) * qg.v_tile;
#pragma unroll
    for (int pp = 0; pp < NVP; ++pp) vc[pp] = CD::template load<true>(base + pp * kRun + lane * kUnit);
    if constexpr (VODD) vcl = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(base + NVP * kRun + lane * 8));
    const uint8_t* sp = base + qg.v_codes;
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      vsc[u] = *reinterpret_cast<const f16x8*>(sp + (u * 4 + quad) * 16);
      vzr[u] = *reinterpret_cast<const f16x8*>(sp + 128 + (u * 4 + quad) * 16);
    }
  };
  // the A operands "offset + code": 16-token block tb of k-step kk; 32-token group u of channel block cb
  auto k_frag = [&](int kk, int tb) -> f16x8 { return CD::frag(kc[kk], tb, magic1024, magic64); };
  auto v_frag = [&](int cb, int u) -> f16x8 {
    if (VODD && cb == NCB - 1) return CD::frag2(vcl, u, magic1024, magic64);
    return CD::frag(vc[cb >> 1], (cb & 1) * 2 + u, magic1024, magic64);
  };

  bool have = cur.tile < t_end;
  int page = -1;
  if (have) {
    page = page_of(cur);
    // a tile without a valid page is still read -- from page 0 -- and masked below
    load_k(cur, max(page, 0));
    load_v(cur, max(page, 0));
  }
  Pos nxt = advance(cur);
  bool have_n = have && nxt.tile < t_end;
  int page_n = have_n ? page_of(nxt) : -1;

  const f16x8 zero8 = __builtin_bit_cast(f16x8, u32x4{0u, 0u, 0u, 0u});

  while (have) {
    // ---- scores (log2 units) relative to the reference exponent: lane (col, quad) gets tokens
    //      16*tb + 4*quad + i of head col
    f16x8 qs[KS];
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) qs[kk] = q16[kk] * ksc[kk];
    const float m_base = m == -INFINITY ? 0.f : m;
    f32x4 sb = {-m_base, -m_base, -m_base, -m_base};
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) {
      sb = mfma16h(kzr[kk], q16[kk], sb);      // every row: sum_c zero_c q_c
      sb = mfma16h(negoff, qs[kk], sb);        // every row: - sum_c offset_c scale_c q_c
    }
    f32x4 s[4];
#pragma unroll
    for (int tb = 0; tb < 4; ++tb) {
      s[tb] = sb;
#pragma unroll
      for (int kk = 0; kk < KS; ++kk) s[tb] = mfma16h(k_frag(kk, tb), qs[kk], s[tb]);
    }
    // unconditional (a wave's last tile re-reads itself): a load behind a branch would cost a second copy of the
    // registers for the path on which nothing is loaded
    load_k(have_n ? nxt : cur, max(have_n ? page_n : page, 0));

    if constexpr (ALIBI) {
      // s <- s + slope * (t - pos_q) in log2 units
      const float base = alibi_slope * (float)(cur.tile * kTile + quad * 4 - pos_q);
#pragma unroll
      for (int tb = 0; tb < 4; ++tb)
#pragma unroll
        for (int i = 0; i < 4; ++i) s[tb][i] += fmaf(alibi_slope, (float)(tb * 16 + i), base);
    }
    if (page < 0) {
      // a page that is not there: its tokens do not take part, and the scales read from page 0 are dropped
      asm volatile("");
#pragma unroll
      for (int tb = 0; tb < 4; ++tb) s[tb] = f32x4{-INFINITY, -INFINITY, -INFINITY, -INFINITY};
#pragma unroll
      for (int u = 0; u < 2; ++u) vsc[u] = vzr[u] = zero8;
    }
    // ---- online softmax; m moves only when the maximum has grown by more than 2^kLazy
    float mx = -INFINITY;
#pragma unroll
    for (int tb = 0; tb < 4; ++tb) {
#pragma unroll
      for (int i = 0; i < 4; ++i) mx = fmaxf(mx, s[tb][i]);
    }
    mx = quad_column_max(mx);
    if (__any(m == -INFINITY ? mx > -INFINITY : mx > kLazy)) {
      const float m_new = fmaxf(m, mx + m_base);
      const float m_safe = m_new == -INFINITY ? 0.f : m_new;
      const float alpha = __builtin_amdgcn_exp2f(m - m_safe);
      const float delta = m_safe - m_base;
      lacc *= alpha;
      corr *= alpha;
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb) acc[cb] *= alpha;
#pragma unroll
      for (int tb = 0; tb < 4; ++tb) s[tb] -= delta;
      m = m_new;
    }
    f16x8 pf[2], ps[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
#pragma unroll
      for (int h = 0; h < 2; ++h) {
#pragma unroll
        for (int i = 0; i < 4; ++i) pf[u][h * 4 + i] = (_Float16)__builtin_amdgcn_exp2f(s[2 * u + h][i]);
      }
      ps[u] = pf[u] * vsc[u];
      lacc = mfma16h(ones, pf[u], lacc);
      corr = mfma16h(vzr[u], pf[u], corr);
      corr = mfma16h(negoff, ps[u], corr);
    }
    // ---- O^T += (offset + codes)^T . (p scale)^T
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) {
#pragma unroll
      for (int u = 0; u < 2; ++u) acc[cb] = mfma16h(v_frag(cb, u), ps[u], acc[cb]);
    }
    load_v(have_n ? nxt : cur, max(have_n ? page_n : page, 0));
    cur = nxt;
    have = have_n;
    page = page_n;
    nxt = advance(cur);
    have_n = have && nxt.tile < t_end;
    page_n = have_n ? page_of(nxt) : -1;
  }

  // ---- merge the four waves, fold the constant terms in, write the split's partial
  if (quad == 0) {
    sm.m[wave][col] = m;
    sm.l[wave][col] = lacc[0];
  }
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
    for (int i = 0; i < 4; ++i) sm.acc[wave][col][cb * 16 + quad * 4 + i] = acc[cb][i] + corr[i];
  __syncthreads();

  constexpr int r_v_pad = NCB * 16;
  for (int idx = threadIdx.x; idx < G * r_v_pad; idx += blockDim.x) {
    const int hd = idx / r_v_pad, c = idx % r_v_pad;
    float mm = sm.m[0][hd];
#pragma unroll
    for (int w = 1; w < 4; ++w) mm = fmaxf(mm, sm.m[w][hd]);
    float lsum = 0.f, val = 0.f;
    if (mm != -INFINITY) {
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const float wt = __builtin_amdgcn_exp2f(sm.m[w][hd] - mm);
        lsum += wt * sm.l[w][hd];
        val += wt * sm.acc[w][hd][c];
      }
    }
    const int head = kvh * G + hd;
    const int64_t BHS = (int64_t)a.n_batch * g.n_heads * a.ws_slots;
    const int64_t row = ((int64_t)b * g.n_heads + head) * a.ws_slots + split;
    if (c == 0) {
      a.ws[row] = mm;
      a.ws[BHS + row] = lsum;
    }
    a.ws[2 * BHS + row * r_v_pad + c] = val;
  }
}

template <int KS, int NCB>
static void launch_q4(const DecodeQ4Args& a, int32_t B, hipStream_t st) {
  const int extra = a.has_tail ? (B + a.n_splits - 1) / a.n_splits : 0;
  const dim3 grid(a.g.n_kv_heads, a.n_splits, B + extra);
  if (a.qg.bits == 3) {
    if (a.alibi) decode_q4_kernel<KS, NCB, true, 3><<<grid, dim3(256), 0, st>>>(a);
    else decode_q4_kernel<KS, NCB, false, 3><<<grid, dim3(256), 0, st>>>(a);
  } else if (a.alibi) {
    decode_q4_kernel<KS, NCB, true><<<grid, dim3(256), 0, st>>>(a);
  } else {
    decode_q4_kernel<KS, NCB, false><<<grid, dim3(256), 0, st>>>(a);
  }
}

template <int KS>
static int dispatch_ncb_q4(int ncb, const DecodeQ4Args& a, int32_t B, hipStream_t st) {
  switch (ncb) {
    case 1: launch_q4<KS, 1>(a, B, st); break;
    case 2: launch_q4<KS, 2>(a, B, st); break;
    case 3: launch_q4<KS, 3>(a, B, st); break;
    case 4: launch_q4<KS, 4>(a, B, st); break;
    case 5: launch_q4<KS, 5>(a, B, st); break;
    case 6: launch_q4<KS, 6>(a, B, st); break;
    case 7: launch_q4<KS, 7>(a, B, st); break;
    case 8: launch_q4<KS, 8>(a, B, st); break;
    default: return EA_ERR_SHAPE;
  }
  return launch_status();
}

int decode_q4(const ea_layer_desc* d, const Geo& g, const Q4Geo& qg, const float* q, const void* kq_pool,
              const void* vq_pool, const int32_t* q4_page_table, const int32_t* q4_len, int32_t max_q4_pages,
              int32_t q4_pool_pages, int32_t B, int32_t n_splits, int32_t ws_slots, float* ws, hipStream_t st,
              const Geo* tail_geo, const void* k_pool, const void* v_pool, const int32_t* tail_page_table,
              const int32_t* tail_len, const float* alibi_slopes) {
  if (2 * B > 65535 || g.n_kv_heads > 65535) return EA_ERR_SHAPE;
  DecodeQ4Args a;
  a.q = q;
  a.kq_pool = (const uint8_t*)kq_pool;
  a.vq_pool = (const uint8_t*)vq_pool;
  a.page_table = q4_page_table;
  a.q4_len = q4_len;
  a.ws = ws;
  a.g = g;
  a.g.max_pages = max_q4_pages;
  a.g.pool_pages = q4_pool_pages;
  a.qg = qg;
  a.n_splits = n_splits;
  a.ws_slots = ws_slots;
  a.scale_log2 = 1.4426950408889634f / sqrtf((float)d->d_head);
  a.has_tail = tail_geo != nullptr;
  a.n_batch = B;
  a.alibi = alibi_slopes;
  a.tail_len = tail_geo ? tail_len : nullptr;
  a.tail = DecodeArgs{};
  if (tail_geo) {
    a.tail.q = q;
    a.tail.k_pool = (const uint16_t*)k_pool;
    a.tail.v_pool = (const uint16_t*)v_pool;
    a.tail.page_table = tail_page_table;
    a.tail.seq_len = tail_len;
    a.tail.out = nullptr;
    a.tail.ws = ws;
    a.tail.g = *tail_geo;
    a.tail.n_splits = 1;
    a.tail.scale_log2 = a.scale_log2;
    a.tail.u_k = nullptr;
    a.tail.d_head = d->d_head;
    a.tail.log2_base = 0.0;
    a.tail.alibi = alibi_slopes;
    a.tail.ws_slots = ws_slots;
    a.tail.ws_slot0 = n_splits;
  }
  switch (qg.ks) {
    case 1: return dispatch_ncb_q4<1>(qg.ncb, a, B, st);
    case 2: return dispatch_ncb_q4<2>(qg.ncb, a, B, st);
    case 3: return dispatch_ncb_q4<3>(qg.ncb, a, B, st);
    case 4: return dispatch_ncb_q4<4>(qg.ncb, a, B, st);
    default: return EA_ERR_SHAPE;
  }
}

}  // namespace ea
