// Generation-phase attention for models with rotary position embedding (Sec. 4.3, Eq. 9-10) over the 4-bit
// group-quantised part of the rank-r cache.  The cached keys are the rank-r keys k_r = k U^K of the one shared basis,
// quantised per channel; per 32 tokens the kernel
//   - expands their codes to fp16 (unpack_q4), takes the offsets off again and applies scale and zero of the
//     tile's channels (packed fp16: the dequantised k_r, rounded once to fp16),
//   - brings them back to d_head channels on the matrix cores (U^K as A operand from LDS, fp16),
//   - rotates the result by the keys' positions (packed fp16, cos/sin table of the offsets inside a tile in LDS)
//     and contracts it with the query, which is rotated to the tile's first position once per tile (in float,
//     stepped from tile to tile and re-computed exactly every kReseedQ4 tiles),
//   - and treats the values exactly as the position-free 4-bit kernel does (scales into the probabilities,
//     constants through the matrix cores).
// Always writes split partials; the bfloat16 tail is attended by the bfloat16 rotary kernel (rotary scores depend
// on position differences only, so the tail may count its positions from its own first token).
#include "ea_q4.h"

namespace ea {

struct DecodeRopeQ4Args {
  const float* q;            // [B, H, d_head], not rotated
  const uint16_t* u_k;       // [d_head, r_k] bf16
  const uint8_t* kq_pool;
  const uint8_t* vq_pool;
  const int32_t* page_table;
  const int32_t* q4_len;
  const int32_t* tail_len;   // may be null: no tokens after the 4-bit part
  float* ws;
  Geo g;                     // max_pages / pool_pages are those of the 4-bit pools
  Q4Geo qg;
  int32_t n_splits;
  int32_t ws_slots;
  int32_t d_head;
  float scale_log2;
  double log2_base;
};

template <int NKK, int KS>
struct RopeQ4Smem {
  // A operand of the up-projection: row m of block 2*kk + comp is channel 2*(16*kk + m) + comp of the basis
  f16x8 uf[2 * NKK][KS][64];
  f16x8 tcs[4][NKK][64];             // cos (slots 0-3) and sin (4-7) of (16*tb + col) * theta_j: a key's offset in its tile
  f32x4 sc[NKK][64], ss[NKK][64];    // angle -(4 * 64) * theta_j: from one tile of a wave to its next
  double turns[NKK * 16];            // theta_j / (2 pi)
};

constexpr int kReseedQ4 = 32;   // tiles between exact re-computations of the rotated query

// BITS = 4 or 3: the width of a code (everything after the unpacking is the same).
template <int KS, int NCB, int NKK, int BITS>
__global__ __launch_bounds__(256, 2) void decode_rope_q4_kernel(DecodeRopeQ4Args a) {
  typedef Codes<BITS> CD;
  __shared__ union {
    MergeSmemQ4<NCB> mg;
    RopeQ4Smem<NKK, KS> rp;
  } sm;
  constexpr int NVP = NCB / 2;
  constexpr bool VODD = (NCB & 1) != 0;
  const Geo& g = a.g;
  const Q4Geo& qg = a.qg;
  const int kvh = blockIdx.x, split = blockIdx.y, b = blockIdx.z;
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
  const int n_tiles = (int)(n64 / (kTile * qg.tpg)) * qg.tpg;      // whole key groups only
  const int per = (n_tiles + a.n_splits - 1) / a.n_splits;
  const int t_begin = split * per;
  const int t_end = min(n_tiles, t_begin + per);
  const int tiles_per_page = qg.tiles_per_page;
  // the query is the newest token: the last one of the bfloat16 tail, or of the 4-bit part if there is no tail
  int64_t tail = a.tail_len ? (int64_t)((const_i32_ptr)a.tail_len)[b] : 0;
  if (tail < 0) tail = 0;
  const int64_t pos_q = (int64_t)n_tiles * kTile + tail - 1;

  f16x8 negoff, ones;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    negoff[j] = (j & 2) ? (_Float16)-CD::kOffLo : (_Float16)-1024.0f;
    ones[j] = (_Float16)1.0f;
  }
  uint32_t magic1024 = 0x64006400u, magic64 = CD::kMagicLo;
  asm volatile("" : "+v"(magic1024), "+v"(magic64));

  f32x4 acc[NCB];
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb) acc[cb] = f32x4{0.f, 0.f, 0.f, 0.f};
  f32x4 lacc = {0.f, 0.f, 0.f, 0.f};
  f32x4 corr = {0.f, 0.f, 0.f, 0.f};
  float m = -INFINITY;

  u32x4 kc[KS];
  f16x8 ksc[KS], kzr[KS];
  u32x4 vc[NVP > 0 ? NVP : 1];
  u32x2 vcl = {0u, 0u};
  f16x8 vsc[2], vzr[2];

  // ---- the query's pairs j = 16*kk + 4*quad + i, times log2(e)/sqrt(d_head), rotated to the current tile
  float qa[NKK][4], qb[NKK][4];
  f16x8 qf[NKK];                 // ... as B operand of the score product: slot 4*comp + i of k-step kk
  auto seed_q = [&](int tile) {
    const float* qrow = a.q + ((int64_t)b * g.n_heads + (int64_t)kvh * G + (col < G ? col : 0)) * a.d_head;
    const double rel = (double)(pos_q - (int64_t)tile * kTile);
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int j = kk * 16 + quad * 4 + i;
        const float g0 = qrow[2 * j] * a.scale_log2, g1 = qrow[2 * j + 1] * a.scale_log2;
        const float q0 = col < G ? g0 : 0.f, q1 = col < G ? g1 : 0.f;
        float c, sn;
        rot_turns(rel * sm.rp.turns[j], c, sn);
        qa[kk][i] = q0 * c - q1 * sn;
        qb[kk][i] = q0 * sn + q1 * c;
      }
    }
  };
  auto step_q = [&](int tl) {
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk) {
      const f32x4 c4 = sm.rp.sc[kk][tl], s4 = sm.rp.ss[kk][tl];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float x0 = qa[kk][i], x1 = qb[kk][i];
        qa[kk][i] = x0 * c4[i] - x1 * s4[i];
        qb[kk][i] = x0 * s4[i] + x1 * c4[i];
      }
    }
  };
  auto pack_q = [&]() {
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        qf[kk][i] = (_Float16)qa[kk][i];
        qf[kk][4 + i] = (_Float16)qb[kk][i];
      }
    }
  };

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
      // lanes of a quad the last k-step does not have re-read quad 0's unit; the basis is zero in their channels
      const bool past = kk == KS - 1 && kk * 4 + quad >= qg.nch;
      const int off = kk * CD::kRun + (past ? col : lane) * CD::kUnit;
      kc[kk] = CD::template load<true>(base + off);
      const uint8_t* sp = scales + (kk * 4 + quad) * 32;
      ksc[kk] = *reinterpret_cast<const f16x8*>(sp);
      kzr[kk] = *reinterpret_cast<const f16x8*>(sp + 16);
    }
  };
  auto load_v = [&](const Pos& p, int page) {
    const uint8_t* base = a.vq_pool + (int64_t)page * qg.v_page + ((int64_t)kvh * tiles_per_page + p.tin) * qg.v_tile;
#pragma unroll
    for (int pp = 0; pp < NVP; ++pp) vc[pp] = CD::template load<true>(base + pp * CD::kRun + lane * CD::kUnit);
    if constexpr (VODD) vcl = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(base + NVP * CD::kRun + lane * 8));
    const uint8_t* sp = base + (NVP * CD::kRun + (VODD ? 512 : 0));      // behind the codes
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

  bool have = cur.tile < t_end;
  int page = -1;
  if (have) {
    page = page_of(cur);
    load_k(cur, max(page, 0));      // a tile without a valid page is still read -- from page 0 -- and masked below
    load_v(cur, max(page, 0));
  }
  Pos nxt = advance(cur);
  bool have_n = have && nxt.tile < t_end;
  int page_n = have_n ? page_of(nxt) : -1;

  // ---- the rotary tables are built while the first tile is on its way
  if (threadIdx.x < NKK * 16)
    sm.rp.turns[threadIdx.x] = exp2(-(2.0 * (double)threadIdx.x / (double)a.d_head) * a.log2_base) * 0.15915494309189535;
  for (int e = threadIdx.x; e < 2 * NKK * KS * 64; e += 256) {
    const int ln = e & 63, ks = (e >> 6) % KS, fb = e / (64 * KS);
    const uint16_t* urow = a.u_k + (int64_t)(2 * ((fb >> 1) * 16 + (ln & 15)) + (fb & 1)) * g.r_k;
    const int rho0 = ks * 32 + (ln >> 4) * 8;
    f16x8 w;
#pragma unroll
    for (int x = 0; x < 8; ++x)
      w[x] = rho0 + x < g.r_k ? (_Float16)__builtin_bit_cast(float, (uint32_t)urow[rho0 + x] << 16) : (_Float16)0.f;
    sm.rp.uf[fb][ks][ln] = w;
  }
  __syncthreads();
  for (int e = threadIdx.x; e < 4 * NKK * 64; e += 256) {
    const int ln = e & 63, kk = (e >> 6) % NKK, tb = e / (64 * NKK);
    f16x8 cs;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      float c, sn;
      rot_turns((double)(tb * 16 + (ln & 15)) * sm.rp.turns[kk * 16 + (ln >> 4) * 4 + i], c, sn);
      cs[i] = (_Float16)c;
      cs[4 + i] = (_Float16)sn;
    }
    sm.rp.tcs[tb][kk][ln] = cs;
  }
  for (int e = threadIdx.x; e < NKK * 64; e += 256) {
    const int ln = e & 63, kk = e >> 6;
    f32x4 c4, s4;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      float c, sn;
      rot_turns(-(double)(4 * kTile) * sm.rp.turns[kk * 16 + (ln >> 4) * 4 + i], c, sn);
      c4[i] = c;
      s4[i] = sn;
    }
    sm.rp.sc[kk][ln] = c4;
    sm.rp.ss[kk][ln] = s4;
  }
  __syncthreads();
  if (have) {
    seed_q(cur.tile);
    pack_q();
  }
  int since_seed = 0;
  const f16x8 zero8 = __builtin_bit_cast(f16x8, u32x4{0u, 0u, 0u, 0u});

  while (have) {
    // The tables never change, so the compiler would keep all of them in registers across the loop; an index
    // it cannot see through makes it read them where they are used.
    int tl = lane;
    asm volatile("" : "+v"(tl));
    if (page < 0) {
      asm volatile("");
#pragma unroll
      for (int u = 0; u < 2; ++u) vsc[u] = vzr[u] = zero8;
    }
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
      // ---- the 32 keys of this half tile, dequantised: lane (col, quad) holds channels 32*ks + 8*quad .. of
      //      token 16*tb + col
      f16x8 kf[2][KS];
#pragma unroll
      for (int tb = 0; tb < 2; ++tb)
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
          kf[tb][ks] = (CD::frag(kc[ks], 2 * sub + tb, magic1024, magic64) + negoff) * ksc[ks] + kzr[ks];
      // the key registers are free again; the load is unconditional (a wave's last tile re-reads itself), so that
      // the registers need no second copy for the path on which nothing is loaded
      if (sub == 1) load_k(have_n ? nxt : cur, max(have_n ? page_n : page, 0));

      // ---- scores (log2 units) relative to the reference exponent
      const float m_base = m == -INFINITY ? 0.f : m;
      f32x4 s[2];
#pragma unroll
      for (int tb = 0; tb < 2; ++tb) s[tb] = f32x4{-m_base, -m_base, -m_base, -m_base};
#pragma unroll
      for (int kk = 0; kk < NKK; ++kk) {
        // K'^T (32 of the d_head channels x 16 tokens) = U^K . k_r^T: lane (col, quad) receives, of token col,
        // the channels 2j + comp with j = 16*kk + 4*quad + i in up[comp][tb][i]
        f32x4 up[2][2];
#pragma unroll
        for (int tb = 0; tb < 2; ++tb) up[0][tb] = up[1][tb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          const f16x8 u0 = sm.rp.uf[2 * kk][ks][tl], u1 = sm.rp.uf[2 * kk + 1][ks][tl];
#pragma unroll
          for (int tb = 0; tb < 2; ++tb) {
            up[0][tb] = mfma16h(u0, kf[tb][ks], up[0][tb]);
            up[1][tb] = mfma16h(u1, kf[tb][ks], up[1][tb]);
          }
        }
#pragma unroll
        for (int tb = 0; tb < 2; ++tb) {
          const f16x8 cs = sm.rp.tcs[2 * sub + tb][kk][tl];
          const f16x4 c4 = cs.lo, s4 = cs.hi;
          const f16x4 x0 = __builtin_convertvector(up[0][tb], f16x4), x1 = __builtin_convertvector(up[1][tb], f16x4);
          const f16x4 r0 = x0 * c4 - x1 * s4, r1 = x0 * s4 + x1 * c4;
          const f16x8 kr = __builtin_shufflevector(r0, r1, 0, 1, 2, 3, 4, 5, 6, 7);
          s[tb] = mfma16h(kr, qf[kk], s[tb]);
        }
      }
      if (page < 0) {
        asm volatile("");
#pragma unroll
        for (int tb = 0; tb < 2; ++tb) s[tb] = f32x4{-INFINITY, -INFINITY, -INFINITY, -INFINITY};
      }

      // ---- online softmax; m moves only when the maximum has grown by more than 2^kLazy
      float mx = -INFINITY;
#pragma unroll
      for (int tb = 0; tb < 2; ++tb) {
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
        for (int tb = 0; tb < 2; ++tb) s[tb] -= delta;
        m = m_new;
      }
      f16x8 pf;
#pragma unroll
      for (int h = 0; h < 2; ++h) {
#pragma unroll
        for (int i = 0; i < 4; ++i) pf[h * 4 + i] = (_Float16)__builtin_amdgcn_exp2f(s[h][i]);
      }
      const f16x8 ps = pf * vsc[sub];
      lacc = mfma16h(ones, pf, lacc);
      corr = mfma16h(vzr[sub], pf, corr);
      corr = mfma16h(negoff, ps, corr);
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb)
        acc[cb] = mfma16h(v_frag(cb, sub), ps, acc[cb]);
    }
    load_v(have_n ? nxt : cur, max(have_n ? page_n : page, 0));
    if (have_n) {
      if (++since_seed == kReseedQ4) {
        since_seed = 0;
        seed_q(nxt.tile);
      } else {
        step_q(tl);
      }
      pack_q();
    }
    cur = nxt;
    have = have_n;
    page = page_n;
    nxt = advance(cur);
    have_n = have && nxt.tile < t_end;
    page_n = have_n ? page_of(nxt) : -1;
  }

  // ---- merge the four waves, fold the constant terms in, write the split's partial
  __syncthreads();   // the tables share their memory with the merge buffers
  if (quad == 0) {
    sm.mg.m[wave][col] = m;
    sm.mg.l[wave][col] = lacc[0];
  }
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
    for (int i = 0; i < 4; ++i) sm.mg.acc[wave][col][cb * 16 + quad * 4 + i] = acc[cb][i] + corr[i];
  __syncthreads();

  constexpr int r_v_pad = NCB * 16;
  for (int idx = threadIdx.x; idx < G * r_v_pad; idx += blockDim.x) {
    const int hd = idx / r_v_pad, c = idx % r_v_pad;
    float mm = sm.mg.m[0][hd];
#pragma unroll
    for (int w = 1; w < 4; ++w) mm = fmaxf(mm, sm.mg.m[w][hd]);
    float lsum = 0.f, val = 0.f;
    if (mm != -INFINITY) {
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const float wt = __builtin_amdgcn_exp2f(sm.mg.m[w][hd] - mm);
        lsum += wt * sm.mg.l[w][hd];
        val += wt * sm.mg.acc[w][hd][c];
      }
    }
    const int head = kvh * G + hd;
    const int64_t BHS = (int64_t)gridDim.z * g.n_heads * a.ws_slots;
    const int64_t row = ((int64_t)b * g.n_heads + head) * a.ws_slots + split;
    if (c == 0) {
      a.ws[row] = mm;
      a.ws[BHS + row] = lsum;
    }
    a.ws[2 * BHS + row * r_v_pad + c] = val;
  }
}

template <int KS, int NCB, int NKK>
static void launch_rope_q4(const DecodeRopeQ4Args& a, int32_t B, hipStream_t st) {
  const dim3 grid(a.g.n_kv_heads, a.n_splits, B);
  if (a.qg.bits == 3) decode_rope_q4_kernel<KS, NCB, NKK, 3><<<grid, dim3(256), 0, st>>>(a);
  else decode_rope_q4_kernel<KS, NCB, NKK, 4><<<grid, dim3(256), 0, st>>>(a);
}

template <int KS, int NKK>
static int dispatch_ncb_rope_q4(int ncb, const DecodeRopeQ4Args& a, int32_t B, hipStream_t st) {
  switch (ncb) {
    case 1: launch_rope_q4<KS, 1, NKK>(a, B, st); break;
    case 2: launch_rope_q4<KS, 2, NKK>(a, B, st); break;
    case 3: launch_rope_q4<KS, 3, NKK>(a, B, st); break;
    case 4: launch_rope_q4<KS, 4, NKK>(a, B, st); break;
    case 5: launch_rope_q4<KS, 5, NKK>(a, B, st); break;
    case 6: launch_rope_q4<KS, 6, NKK>(a, B, st); break;
    case 7: launch_rope_q4<KS, 7, NKK>(a, B, st); break;
    case 8: launch_rope_q4<KS, 8, NKK>(a, B, st); break;
    default: return EA_ERR_SHAPE;
  }
  return launch_status();
}

template <int NKK>
static int dispatch_ks_rope_q4(int ks, int ncb, const DecodeRopeQ4Args& a, int32_t B, hipStream_t st) {
  switch (ks) {
    case 1: return dispatch_ncb_rope_q4<1, NKK>(ncb, a, B, st);
    case 2: return dispatch_ncb_rope_q4<2, NKK>(ncb, a, B, st);
    case 3: return dispatch_ncb_rope_q4<3, NKK>(ncb, a, B, st);
    case 4: return dispatch_ncb_rope_q4<4, NKK>(ncb, a, B, st);
    default: return EA_ERR_SHAPE;
  }
}

int decode_rope_q4(const ea_layer_desc* d, const Geo& g, const Q4Geo& qg, const float* q, const void* u_k,
                   double rope_base, const void* kq_pool, const void* vq_pool, const int32_t* q4_page_table,
                   const int32_t* q4_len, const int32_t* tail_len, int32_t max_q4_pages, int32_t q4_pool_pages,
                   int32_t B, int32_t n_splits, int32_t ws_slots, float* ws, hipStream_t st) {
  if (B > 65535 || g.n_kv_heads > 65535 || n_splits > 65535) return EA_ERR_SHAPE;
  if (d->d_head != 64 && d->d_head != 128) return EA_ERR_SHAPE;
  DecodeRopeQ4Args a;
  a.q = q;
  a.u_k = (const uint16_t*)u_k;
  a.kq_pool = (const uint8_t*)kq_pool;
  a.vq_pool = (const uint8_t*)vq_pool;
  a.page_table = q4_page_table;
  a.q4_len = q4_len;
  a.tail_len = tail_len;
  a.ws = ws;
  a.g = g;
  a.g.max_pages = max_q4_pages;
  a.g.pool_pages = q4_pool_pages;
  a.qg = qg;
  a.n_splits = n_splits;
  a.ws_slots = ws_slots;
  a.d_head = d->d_head;
  a.scale_log2 = 1.4426950408889634f / sqrtf((float)d->d_head);
  a.log2_base = log2(rope_base);
  if (d->d_head == 128) return dispatch_ks_rope_q4<4>(qg.ks, qg.ncb, a, B, st);
  return dispatch_ks_rope_q4<2>(qg.ks, qg.ncb, a, B, st);
}

}  // namespace ea
