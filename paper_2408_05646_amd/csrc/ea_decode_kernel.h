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
//
// NKK > 0 selects the variant for models with rotary position embedding (Sec. 4.3, Eq. 10): the query
// arrives with all d_head = 32*NKK channels, and each 16-token block of cached rank-r keys is first
// brought back to d_head channels on the matrix cores (K' = U^K k_r, the basis shared by all heads kept
// in LDS in MFMA operand order), rotated to its position in packed half precision and only then multiplied
// with the query on the fp16 matrix-core path (11 significant bits on both operands, against 8 of bf16: the
// rotated keys exist in registers only, so their format is free; their magnitude is bounded by the cached
// key's norm, far inside the fp16 range for attention keys).  Only the position DIFFERENCE enters a score, so the rotation is split: the query is
// rotated (in fp32, once per tile of a wave) by the distance between its own position and the first
// token of the tile, each key by its offset inside the tile (a constant table in LDS).
//
// POS (rotary only) is the form for a cache from which tokens have been dropped (the token-pruning experiment of the
// results; a kept token keeps the position it had in the text): the position of the token in every cache slot comes
// from an array, so the split above no longer works -- the query is rotated once to its own position, each key to
// its own, with cos and sin computed where they are used (angle in turns, reduced exactly in two single-precision
// steps; v_sin_f32 / v_cos_f32 on the remaining fraction).  With SCORES the kernel also stores its scores, as the
// position-free form does.
#pragma once
#include <type_traits>
#include "ea_common.h"

namespace ea {

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
  // rotary variant only
  const uint16_t* u_k;   // [d_head, r_k] bf16 basis shared by all heads
  int32_t d_head;
  double log2_base;   // log2 of the rotary base
  // ALiBi variant only
  const float* alibi;  // [H] slopes (natural-log units, >= 0)
  // When ws_slots > 0 the kernel always writes split partials, into slots ws_slot0 .. ws_slot0 + n_splits - 1
  // of a workspace laid out for ws_slots splits (another kernel fills the other slots).
  int32_t ws_slots = 0;
  int32_t ws_slot0 = 0;
  // SCORES variant only: the scaled scores (log2 units) of every (sequence, head, token) are written here as well
  float* scores = nullptr;   // [B, H, s_row]
  int32_t s_row = 0;         // row length: the cache capacity rounded up to whole tiles
  int32_t seq_add = 0;       // added to seq_len[b]: 1 when seq_len holds the lengths BEFORE the token this step appends
  // POS variant only: positions in the text
  const int32_t* slot_pos = nullptr;   // [B, pos_stride]: of the token in logical cache slot t (0 <= value < 2^24)
  const int32_t* q_pos = nullptr;      // [B]: of the query
  int32_t pos_stride = 0;              // >= max_pages * page_tokens
  int32_t out_bf16 = 0;                // `out` holds bfloat16 instead of float (the layer step's own intermediate)
};

typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(4))) _Float16 f16x4;

template <int NCB>
struct MergeSmem {
  float m[4][16];
  float l[4][16];
  float acc[4][16][NCB * 16];
};

// Rotation tables of the rotary variant.  Pair j = 16*kk + 4*quad + i of lane (col, quad) rotates by
// theta_j = base^(-2j/d_head) per position.
template <int TBN, int NKK, int KS, bool POS>
struct RopeSmem {
  // A operand of the up-projection: row m of block 2*kk + comp is channel 2*(16*kk + m) + comp of the basis
  bf16x8 uf[2 * NKK][KS][64];
  // (not in the POS form, which has no use for tables over offsets)
  f16x8 tcs[POS ? 1 : 4][POS ? 1 : NKK][POS ? 1 : 64];   // cos (slots 0-3) and sin (4-7) of (16*tb + col) * theta_j: a key's offset in its tile
  f32x4 sc[POS ? 1 : NKK][POS ? 1 : 64], ss[POS ? 1 : NKK][POS ? 1 : 64];    // angle -(4 * 64) * theta_j: from one tile of a wave to its next
  double turns[NKK * 16];                     // theta_j / (2 pi)
  f32x4 thi[NKK][4], tlo[NKK][4];             // POS: the same as single-precision hi + lo, [kk][quad] = pairs 16*kk + 4*quad ..+3
};
struct NoSmem {};

constexpr int kReseed = 32;   // iterations between exact re-computations of the rotated query

// TBN = 16-token blocks handled per loop iteration: 4 (a whole 64-token tile) or 2 (half a tile, for the
// large ranks whose fragments would not fit the register file otherwise).
// ALIBI adds the linear position bias of the ALiBi scheme to the scores: -slope_h * (distance of the key to
// the query), in the position-free form only.
// SCORES also stores the scores (log2 units): what a caller that accumulates attention probabilities per cached
// token needs, without a second pass over the keys.  A wave collects the scores of several iterations in LDS and
// writes them out 2048 floats at a time with full-width stores (a store per tile from the four lanes that hold a
// head's scores measured slower: one counter covers loads and stores, so the next wait for loaded data also
// waits for the store).
// LDS of one workgroup: the rotary tables while the cache streams, the merge buffers afterwards.
constexpr int kScoreStage = 2048;      // floats of staged scores per wave (SCORES form)
struct ScoreSmem {
  float s[4][kScoreStage];
};
template <int KS, int NCB, int TBN, int NKK, bool SCORES, bool POS>
struct StreamSmem {    // what is live while the cache streams
  std::conditional_t<(NKK > 0), RopeSmem<TBN, (NKK > 0) ? NKK : 1, KS, POS>, NoSmem> rp;
  std::conditional_t<SCORES, ScoreSmem, NoSmem> sc;
};
template <int KS, int NCB, int TBN, int NKK, bool SCORES = false, bool POS = false>
union DecodeSmem {
  MergeSmem<NCB> mg;
  StreamSmem<KS, NCB, TBN, NKK, SCORES, POS> st;
};

// What becomes of one (head, channel) of a workgroup's merged result -- reference exponent mm, row sum lsum,
// weighted value sum val: the output element when the sequence is not split, else the split partials.  The
// default uses plain stores (visible to the kernel that comes next); a kernel that goes on to consume the
// values itself passes an emitter of its own.
struct PlainEmit {
  __device__ __forceinline__ void operator()(const DecodeArgs& a, int b, int n_batch, int split, int head, int c,
                                             int r_v_pad, float mm, float lsum, float val) const {
    const Geo& g = a.g;
    if (a.n_splits == 1 && a.ws_slots == 0) {
      if (c < g.r_v) {
        const int64_t idx = ((int64_t)b * g.n_heads + head) * g.r_v + c;
        const float o = lsum > 0.f ? val / lsum : 0.f;
        if (a.out_bf16) reinterpret_cast<__bf16*>(a.out)[idx] = (__bf16)o;
        else a.out[idx] = o;
      }
    } else {
      const int slots = a.ws_slots > 0 ? a.ws_slots : a.n_splits;
      const int64_t BHS = (int64_t)n_batch * g.n_heads * slots;
      const int64_t row = ((int64_t)b * g.n_heads + head) * slots + a.ws_slot0 + split;
      if (c == 0) {
        a.ws[row] = mm;
        a.ws[BHS + row] = lsum;
      }
      a.ws[2 * BHS + row * r_v_pad + c] = val;
    }
  }
};

template <int KS, int NCB, int TBN, int WPE, int NKK, bool ALIBI = false, bool SCORES = false, bool POS = false,
          typename Emit = PlainEmit>
__device__ __forceinline__ void decode_bf16_body(const DecodeArgs& a, const int kvh, const int split, const int b,
                                                 const int n_batch, DecodeSmem<KS, NCB, TBN, NKK, SCORES, POS>& sm,
                                                 const Emit& emit = Emit{}) {
  constexpr bool ROPE = NKK > 0;
  static_assert(!(ROPE && ALIBI), "a model has one position scheme");
  static_assert(!POS || ROPE, "explicit positions matter to the rotary form only");
  constexpr int UN = TBN / 2;            // 32-token groups per iteration
  constexpr int SUB = 4 / TBN;           // iterations per 64-token tile
  constexpr int TOK = TBN * 16;          // tokens per iteration
  const Geo& g = a.g;
  // neighbouring workgroups take neighbouring kv heads of the same pages: their slabs are adjacent in memory
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform, so is all that follows from it
  const int col = lane & 15, quad = lane >> 4;
  const int G = g.group;
  const int nck = g.r_k_pad >> 3;

  // Sequence lengths and page ids are the same for every lane and do not change while the kernel runs: read
  // through the constant address space they arrive in scalar registers, and their loads do not queue up
  // behind the cache tiles in flight.
  typedef const int32_t __attribute__((address_space(4))) * const_i32_ptr;
  const const_i32_ptr seq_len_c = (const_i32_ptr)a.seq_len;
  const const_i32_ptr pt_row = (const_i32_ptr)(a.page_table + (int64_t)b * g.max_pages);
  int64_t n64 = (int64_t)seq_len_c[b] + a.seq_add;
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
  bf16x8 qhi[ROPE ? 1 : KS], qlo[ROPE ? 1 : KS];
  if constexpr (!ROPE) {
    const float* qrow = a.q + ((int64_t)b * g.n_heads + (int64_t)kvh * G + col) * g.r_k;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int k = ks * 32 + quad * 8 + j;
        // times log2(e)/sqrt(d_head): the scores then come out of the matrix cores in log2 units
        const float v = (col < G && k < g.r_k) ? qrow[k] * a.scale_log2 : 0.f;
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

  // The rotary variant keeps TWO key buffers: its iterations are long, and a key tile requested only after the
  // previous one's scores would be in flight for less than the memory latency.
  constexpr bool KDB = ROPE;
  bf16x8 kfA[TBN][KS], kfB[KDB ? TBN : 1][KDB ? KS : 1], vf[UN][NCB];

  // ---- rotary variant: basis fragments, rotation tables, rotated query
  constexpr int NK1 = ROPE ? NKK : 1;
  float qa[NK1][4], qb[NK1][4];  // the query's pairs j = 16*kk + 4*quad + i, rotated to the current iteration
  f16x8 qf[NK1];                 // ... as B operand of the score MFMA: slot 4*comp + i of k-step kk
  int pos_q = n - 1;             // the query is the token appended last
  if constexpr (POS) pos_q = ((const_i32_ptr)a.q_pos)[b];
  float alibi_slope = 0.f;       // this lane's head, log2 units
  if constexpr (ALIBI) alibi_slope = col < G ? a.alibi[kvh * G + col] * 1.4426950408889634f : 0.f;
  auto seed_q = [&](int tile) {
    if constexpr (ROPE) {
    // head columns past the group read head 0 of the group (always there) and are zeroed
    const float* qrow = a.q + ((int64_t)b * g.n_heads + (int64_t)kvh * G + (col < G ? col : 0)) * a.d_head;
    // POS: keys are rotated to their absolute positions, so the query is, too (once)
    const double rel = POS ? (double)pos_q : (double)(pos_q - tile * kTile);
#pragma unroll
    for (int kk = 0; kk < NK1; ++kk) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int j = kk * 16 + quad * 4 + i;
        const float g0 = qrow[2 * j] * a.scale_log2, g1 = qrow[2 * j + 1] * a.scale_log2;
        const float q0 = col < G ? g0 : 0.f, q1 = col < G ? g1 : 0.f;
        float c, sn;
        rot_turns(rel * sm.st.rp.turns[j], c, sn);
        qa[kk][i] = q0 * c - q1 * sn;
        qb[kk][i] = q0 * sn + q1 * c;
      }
    }
    }
  };
  auto step_q = [&](int tl) {
    if constexpr (ROPE) {
#pragma unroll
    for (int kk = 0; kk < NK1; ++kk) {
      const f32x4 c4 = sm.st.rp.sc[kk][tl], s4 = sm.st.rp.ss[kk][tl];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float x0 = qa[kk][i], x1 = qb[kk][i];
        qa[kk][i] = x0 * c4[i] - x1 * s4[i];
        qb[kk][i] = x0 * s4[i] + x1 * c4[i];
      }
    }
    }
  };
  auto pack_q = [&]() {
    if constexpr (ROPE) {
#pragma unroll
    for (int kk = 0; kk < NK1; ++kk) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        qf[kk][i] = (_Float16)qa[kk][i];
        qf[kk][4 + i] = (_Float16)qb[kk][i];
      }
    }
    }
  };

  // Where a wave stands in its split.  Everything here is wave-uniform and lives in scalar registers; the
  // logical page and the tile's place inside it are stepped along, not divided out, per iteration.
  struct Pos {
    int tile, sub, lp, tin;
  };
  // waves of the position-free kernel interleave iterations (half tiles when SUB = 2), those of the rotary
  // variant whole tiles, so that a wave re-rotates its query once per 64 tokens
  constexpr int kStride = ROPE ? 4 : 4 / SUB;
  Pos cur;
  cur.tile = t_begin + (ROPE ? wave : wave / SUB);
  cur.sub = ROPE ? 0 : wave % SUB;
  cur.lp = cur.tile / tiles_per_page;
  cur.tin = cur.tile % tiles_per_page;
  auto advance = [&](Pos p) -> Pos {
    if (ROPE && p.sub + 1 < SUB) {
      p.sub += 1;
      return p;
    }
    if (ROPE) p.sub = 0;
    p.tile += kStride;
    p.tin += kStride;
    while (p.tin >= tiles_per_page) {
      p.tin -= tiles_per_page;
      p.lp += 1;
    }
    return p;
  };
  // Physical page of a position, or -1.
  auto page_of = [&](const Pos& p) -> int {
    const int page = pt_row[p.lp];
    return (page >= 0 && page < g.pool_pages) ? page : -1;
  };
  const int lane_off = lane << 3;
  auto load_k = [&](const Pos& p, int page, auto& kf) {
    const uint16_t* base = a.k_pool + (int64_t)page * g.k_page + (int64_t)kvh * g.k_slab +
                           (int64_t)p.tin * (kTile * g.r_k_pad) + p.sub * (TOK * g.r_k_pad);
#pragma unroll
    for (int tb = 0; tb < TBN; ++tb) {
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        // chunk ks*4 + quad of token row col: element ((tb*nck + ks*4 + quad)*16 + col)*8 = (tb*nck*16 + ks*64 + lane)*8.
        // Only the last k-step can run past the nck chunks the rank has (r_k_pad > 32*(KS-1)); its surplus
        // lanes read the last real chunk instead and drop what they read, so no load sits behind a branch.
        const bool past = ks == KS - 1 && ks * 4 + quad >= nck;
        const int off = past ? (((tb + 1) * nck - 1) * 16 + col) << 3 : ((tb * nck * 16 + ks * 64) << 3) + lane_off;
        const bf16x8 got = __builtin_nontemporal_load(reinterpret_cast<const bf16x8*>(base + off));
        kf[tb][ks] = past ? zero_frag() : got;
      }
    }
  };
  // POS: the positions of the tokens this lane's keys belong to (token col of each 16-token block)
  int kpA[POS ? TBN : 1], kpB[POS ? TBN : 1];
  auto load_pos = [&](const Pos& p, auto& kp) {
    if constexpr (POS) {
      const int32_t* prow = a.slot_pos + (int64_t)b * a.pos_stride + p.tile * kTile + p.sub * TOK + col;
#pragma unroll
      for (int tb = 0; tb < TBN; ++tb) kp[tb] = prow[tb * 16];
    }
  };
  auto load_v = [&](const Pos& p, int page) {
    const uint16_t* base = a.v_pool + (int64_t)page * g.v_page + (int64_t)kvh * g.v_slab +
                           (int64_t)p.tin * (kTile * g.r_v_pad) + p.sub * (TOK * g.r_v_pad);
#pragma unroll
    for (int u = 0; u < UN; ++u) {
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb)
        vf[u][cb] = __builtin_nontemporal_load(
            reinterpret_cast<const bf16x8*>(base + (((u * NCB + cb) * 64) << 3) + lane_off));
    }
  };

  bool have = cur.tile < t_end;
  int page = -1;
  if (have) {
    page = page_of(cur);
    // A tile without a valid page is still read -- from page 0, which exists -- and all of its tokens are
    // masked below: the loads never depend on the page table's contents, only their address does.
    load_k(cur, max(page, 0), kfA);
    load_pos(cur, kpA);
    load_v(cur, max(page, 0));
  }
  // the position after the current one (with two key buffers its keys are requested one iteration ahead)
  Pos nxt = advance(cur);
  bool have_n = have && nxt.tile < t_end;
  int page_n = have_n ? page_of(nxt) : -1;
  if constexpr (KDB) {
    if (have_n) {
      load_k(nxt, max(page_n, 0), kfB);
      load_pos(nxt, kpB);
    }
  }
  // the rotary tables are built while the first tile is on its way
  if constexpr (ROPE) {
    if (threadIdx.x < NKK * 16)
      sm.st.rp.turns[threadIdx.x] =
          exp2(-(2.0 * (double)threadIdx.x / (double)a.d_head) * a.log2_base) * 0.15915494309189535;
    for (int e = threadIdx.x; e < 2 * NKK * KS * 64; e += 256) {
      const int ln = e & 63, ks = (e >> 6) % KS, fb = e / (64 * KS);
      const uint16_t* urow = a.u_k + (int64_t)(2 * ((fb >> 1) * 16 + (ln & 15)) + (fb & 1)) * g.r_k;
      typedef __attribute__((ext_vector_type(8))) uint16_t u16x8;
      u16x8 w;
      const int rho0 = ks * 32 + (ln >> 4) * 8;
      if ((g.r_k & 7) == 0 && (reinterpret_cast<uintptr_t>(a.u_k) & 15) == 0) {   // rows are whole 16-byte units
        w = rho0 < g.r_k ? *reinterpret_cast<const u16x8*>(urow + rho0) : u16x8{0, 0, 0, 0, 0, 0, 0, 0};
      } else {
#pragma unroll
        for (int x = 0; x < 8; ++x) w[x] = rho0 + x < g.r_k ? urow[rho0 + x] : (uint16_t)0;
      }
      sm.st.rp.uf[fb][ks][ln] = __builtin_bit_cast(bf16x8, w);
    }
    __syncthreads();
    if constexpr (POS) {
      if (threadIdx.x < NKK * 16) {
        const double t = sm.st.rp.turns[threadIdx.x];
        const float hi = (float)t;
        sm.st.rp.thi[threadIdx.x >> 4][(threadIdx.x >> 2) & 3][threadIdx.x & 3] = hi;
        sm.st.rp.tlo[threadIdx.x >> 4][(threadIdx.x >> 2) & 3][threadIdx.x & 3] = (float)(t - (double)hi);
      }
    }
    for (int e = threadIdx.x; !POS && e < 4 * NKK * 64; e += 256) {
      const int ln = e & 63, kk = (e >> 6) % NKK, tb = e / (64 * NKK);
      f16x8 cs;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        float c, sn;
        rot_turns((double)(tb * 16 + (ln & 15)) * sm.st.rp.turns[kk * 16 + (ln >> 4) * 4 + i], c, sn);
        cs[i] = (_Float16)c;
        cs[4 + i] = (_Float16)sn;
      }
      sm.st.rp.tcs[tb][kk][ln] = cs;
    }
    for (int e = threadIdx.x; !POS && e < NKK * 64; e += 256) {
      const int ln = e & 63, kk = e >> 6;
      f32x4 c4, s4;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        float c, sn;
        rot_turns(-(double)(4 * kTile) * sm.st.rp.turns[kk * 16 + (ln >> 4) * 4 + i], c, sn);
        c4[i] = c;
        s4[i] = sn;
      }
      sm.st.rp.sc[kk][ln] = c4;
      sm.st.rp.ss[kk][ln] = s4;
    }
    __syncthreads();
  }
  if constexpr (ROPE) {
    if (have) {
      seed_q(cur.tile);
      pack_q();
    }
  }
  int since_seed = 0;

  // SCORES: iterations staged so far, the tile of the first of them, and how many fit
  static_assert(!(SCORES && ROPE && !POS), "the rotary score-storing form is built with explicit positions only");
  int stage_n = 0, stage_tile0 = cur.tile;
  const int cur_sub_tokens = ROPE ? 0 : cur.sub * TOK;     // position-free form: a wave keeps its half of the tiles
  // G <= 16, TOK <= 64: at least 2; the rotary form stages whole tiles (SUB iterations each)
  const int stage_cap = SCORES ? (kScoreStage / (G * TOK)) / (ROPE ? SUB : 1) * (ROPE ? SUB : 1) : 0;
  auto flush_scores = [&]() {
    if constexpr (SCORES) {
      // staged order: [iteration f][head hd][TOK tokens]; iteration f of this wave is tile stage_tile0 + f * kStride
      // (rotary form: tile stage_tile0 + (f / SUB) * kStride, part f % SUB of it)
      const int per_it = G * TOK, total = stage_n * per_it;
      float* rows = a.scores + ((int64_t)b * g.n_heads + (int64_t)kvh * G) * a.s_row + cur_sub_tokens;
      for (int i = lane * 4; i < total; i += 256) {
        const int f = i / per_it, r = i - f * per_it, hd = r / TOK, off = r - hd * TOK;
        const f32x4 v = *reinterpret_cast<const f32x4*>(&sm.st.sc.s[wave][i]);
        const int first = ROPE ? (stage_tile0 + (f / SUB) * kStride) * kTile + (f % SUB) * TOK : (stage_tile0 + f * kStride) * kTile;
        __builtin_nontemporal_store(v, reinterpret_cast<f32x4*>(rows + (int64_t)hd * a.s_row + first + off));
      }
      stage_n = 0;
    }
  };

  // One iteration; kf holds the current keys, kf_free is the buffer the keys after the next go to.
  auto iteration = [&](auto& kf, auto& kf_free, auto& kp, auto& kp_free) __attribute__((always_inline)) {
    // ---- scores: S[tb] (16 tokens x 16 head columns) = K_block . q^T
    f32x4 s[TBN];
    // The rotation tables never change, so the compiler would keep all of them in registers across the
    // loop; an index it cannot see through makes it read them where they are used.
    int tl = lane;
    if constexpr (ROPE) asm volatile("" : "+v"(tl));
    // the accumulators start at minus the reference exponent: what comes out is the argument of exp2
    const float m_base = m == -INFINITY ? 0.f : m;
    if constexpr (!ROPE) {
#pragma unroll
      for (int tb = 0; tb < TBN; ++tb) {
        s[tb] = f32x4{-m_base, -m_base, -m_base, -m_base};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          s[tb] = mfma16(kf[tb][ks], qhi[ks], s[tb]);
          s[tb] = mfma16(kf[tb][ks], qlo[ks], s[tb]);
        }
      }
    } else {
#pragma unroll
      for (int tb = 0; tb < TBN; ++tb) s[tb] = f32x4{-m_base, -m_base, -m_base, -m_base};
#pragma unroll
      for (int kk = 0; kk < NK1; ++kk) {
        // K'^T (32 of the d_head channels x 16 tokens) = U^K . k_r^T: lane (col, quad) receives, of token col,
        // the channels 2j + comp with j = 16*kk + 4*quad + i in up[comp][tb][i]
        f32x4 up[2][TBN];
#pragma unroll
        for (int tb = 0; tb < TBN; ++tb) up[0][tb] = up[1][tb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          const bf16x8 u0 = sm.st.rp.uf[2 * kk][ks][tl], u1 = sm.st.rp.uf[2 * kk + 1][ks][tl];
#pragma unroll
          for (int tb = 0; tb < TBN; ++tb) {
            up[0][tb] = mfma16(u0, kf[tb][ks], up[0][tb]);
            up[1][tb] = mfma16(u1, kf[tb][ks], up[1][tb]);
          }
        }
#pragma unroll
        for (int tb = 0; tb < TBN; ++tb) {
          f16x4 c4, s4;
          if constexpr (POS) {
            // angle of pair j at position p, in turns: p * (hi_j + lo_j).  p * hi_j is split exactly into its
            // rounded value and the rounding error (fma), the whole turns leave with v_fract_f32
            const float p = (float)kp[tb];
            const f32x4 hi = sm.st.rp.thi[kk][tl >> 4], lo = sm.st.rp.tlo[kk][tl >> 4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              const float t = p * hi[i];
              const float err = __builtin_fmaf(p, hi[i], -t);
              const float f = __builtin_fmaf(p, lo[i], __builtin_amdgcn_fractf(t) + err);
              c4[i] = (_Float16)__builtin_amdgcn_cosf(f);
              s4[i] = (_Float16)__builtin_amdgcn_sinf(f);
            }
          } else {
            const f16x8 cs = sm.st.rp.tcs[cur.sub * TBN + tb][kk][tl];
            c4 = cs.lo;
            s4 = cs.hi;
          }
          const f16x4 x0 = __builtin_convertvector(up[0][tb], f16x4), x1 = __builtin_convertvector(up[1][tb], f16x4);
          const f16x4 r0 = x0 * c4 - x1 * s4, r1 = x0 * s4 + x1 * c4;
          const f16x8 kr = __builtin_shufflevector(r0, r1, 0, 1, 2, 3, 4, 5, 6, 7);
          s[tb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(kr, qf[kk], s[tb], 0, 0, 0);
        }
      }
    }
    const int rem = page >= 0 ? n - (cur.tile * kTile + cur.sub * TOK) : 0;   // valid tokens here (>= TOK: all)
    if constexpr (SCORES) {
      // tokens past the sequence's end are never read back; a tile without a page must read as "no probability"
      if (col < G) {
        float* dst = &sm.st.sc.s[wave][(stage_n * G + col) * TOK + quad * 4];
        const float add = page >= 0 ? m_base : -INFINITY;
#pragma unroll
        for (int tb = 0; tb < TBN; ++tb) *reinterpret_cast<f32x4*>(dst + tb * 16) = s[tb] + add;
      }
    }
    // the registers of the current keys are free again: request the next keys (one buffer) or the ones after
    // the next (two buffers)
    Pos nn = nxt;
    bool have_nn = false;
    int page_nn = -1;
    if constexpr (KDB) {
      nn = advance(nxt);
      have_nn = have_n && nn.tile < t_end;
      page_nn = have_nn ? page_of(nn) : -1;
      if (have_nn) {
        load_k(nn, max(page_nn, 0), kf_free);
        load_pos(nn, kp_free);
      }
    } else {
      if (have_n) load_k(nxt, max(page_n, 0), kf_free);
    }
    if constexpr (ROPE && !POS) {
      if (have_n && nxt.sub == 0) {
        if (++since_seed == kReseed) {
          since_seed = 0;
          seed_q(nxt.tile);
        } else {
          step_q(tl);
        }
        pack_q();
      }
    }

    // ---- online softmax on s (lane: head column `col`, tokens tb*16 + 4*quad + i)
    if constexpr (ALIBI) {
      // s <- s + slope * (t - pos_q) in log2 units
      const float base = alibi_slope * (float)(cur.tile * kTile + cur.sub * TOK + quad * 4 - pos_q);
#pragma unroll
      for (int tb = 0; tb < TBN; ++tb)
#pragma unroll
        for (int i = 0; i < 4; ++i) s[tb][i] += fmaf(alibi_slope, (float)(tb * 16 + i), base);
    }
    float mx = -INFINITY;
#pragma unroll
    for (int tb = 0; tb < TBN; ++tb) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if (rem < TOK && tb * 16 + quad * 4 + i >= rem) s[tb][i] = -INFINITY;
        mx = fmaxf(mx, s[tb][i]);
      }
    }
    mx = quad_column_max(mx);                                 // relative to m_base
    // m is a reference exponent: it moves only when the max has grown by more than kLazy (log2 units), so
    // P stays <= 2^kLazy and the accumulators are rescaled a few times per stream, not at every tile.
    if (__any(m == -INFINITY ? mx > -INFINITY : mx > kLazy)) {
      const float m_new = fmaxf(m, mx + m_base);
      const float m_safe = m_new == -INFINITY ? 0.f : m_new;
      const float alpha = __builtin_amdgcn_exp2f(m - m_safe);  // m = -inf -> 0
      const float delta = m_safe - m_base;
      lacc *= alpha;
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb) acc[cb] *= alpha;
#pragma unroll
      for (int tb = 0; tb < TBN; ++tb) s[tb] -= delta;
      m = m_new;
    }
    bf16x8 pf[UN];
#pragma unroll
    for (int u = 0; u < UN; ++u) {
#pragma unroll
      for (int h = 0; h < 2; ++h) {
#pragma unroll
        for (int i = 0; i < 4; ++i) pf[u][h * 4 + i] = (__bf16)__builtin_amdgcn_exp2f(s[2 * u + h][i]);
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
    if (have_n) load_v(nxt, max(page_n, 0));
    cur = nxt;
    have = have_n;
    page = page_n;
    if constexpr (KDB) {
      nxt = nn;
      have_n = have_nn;
      page_n = page_nn;
    } else {
      nxt = advance(cur);
      have_n = have && nxt.tile < t_end;
      page_n = have_n ? page_of(nxt) : -1;
    }
  };
  auto staged = [&]() {
    if constexpr (SCORES) {
      if (++stage_n == stage_cap) {
        flush_scores();
        stage_tile0 = cur.tile;      // the iteration that comes next
      }
    }
  };
  if constexpr (KDB) {
    while (have) {
      iteration(kfA, kfA, kpA, kpA);       // scores from A, then A takes the keys two iterations ahead
      staged();
      if (!have) break;
      iteration(kfB, kfB, kpB, kpB);
      staged();
    }
  } else {
    while (have) {
      iteration(kfA, kfA, kpA, kpA);
      staged();
    }
  }
  if constexpr (SCORES) {
    if (stage_n > 0) flush_scores();
    if constexpr (!ROPE) __syncthreads();   // the staging buffers share their memory with the merge buffers
  }

  // ---- merge the four waves of the workgroup
  if constexpr (ROPE) __syncthreads();   // the tables share their memory with the merge buffers
  auto& sm_m = sm.mg.m;
  auto& sm_l = sm.mg.l;
  auto& sm_acc = sm.mg.acc;
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
    emit(a, b, n_batch, split, kvh * G + hd, c, r_v_pad, mm, lsum, val);
  }
}

// The kernel: one workgroup per (kv head, split, sequence).  (The body is a function of its own because the
// kernel over the 4-bit cache runs it, too, for the bfloat16 tail of the sequences.)
template <int KS, int NCB, int TBN, int WPE, int NKK, bool ALIBI = false, bool SCORES = false, bool POS = false>
__global__ __launch_bounds__(256, WPE) void decode_bf16_kernel(DecodeArgs a) {
  __shared__ DecodeSmem<KS, NCB, TBN, NKK, SCORES, POS> sm;
  decode_bf16_body<KS, NCB, TBN, WPE, NKK, ALIBI, SCORES, POS>(a, blockIdx.x, blockIdx.y, blockIdx.z, gridDim.z, sm);
}

}  // namespace ea
