// The 4-bit group-quantised form of the rank-r cache (keys per channel over the 64 tokens of a tile -- or over the
// 128 tokens of two neighbouring tiles --, values per token; results paragraph on quantisation): geometry and the
// position of every code and scale.
//
// A page of the 4-bit pools holds the same tokens as a page of the bfloat16 pools: kv head after kv head,
// tile after tile; one tile block is 64 tokens of one kv head.
//
// K tile block  = codes, then scales.
//   codes : for k-step kk (32 channels) a run of 16-byte units, one per lane l = 16*quad + t of the quads that
//           exist in this step (4*kk + quad < r_k_pad/8); the unit's dword tb holds the 8 channels
//           32*kk + 8*quad .. +7 of token 16*tb + t.          -> 64 * r_k_pad / 2 bytes
//   scales: [k-step][quad][scale x8, zero x8] fp16, channel 32*kk + 8*quad + e at slot e.   -> KS * 128 bytes
// V tile block  = codes, then scales.
//   codes : dword (cb, u) of lane l = 16*quad + ch holds channel 16*cb + ch of the 8 tokens
//           32*u + 16*(j/4) + 4*quad + j%4, j = 0..7.  Dwords are stored four to a 16-byte unit per lane:
//           unit p = (cb = 2p, u = 0), (2p, 1), (2p+1, 0), (2p+1, 1); an odd last cb has 8-byte units.
//                                                             -> 64 * r_v_pad / 2 bytes
//   scales: [scale, zero][u][quad][8 token slots] fp16.       -> 256 bytes
// Key groups of 128 tokens (tpg = 2 tiles per group): the tile blocks of a kv head still follow each other, but only
// the first block of every pair carries scales -- the pair's -- and the second is codes only:
//   [codes 0][scales 0+1][codes 1] [codes 2][scales 2+3][codes 3] ...
// Inside a dword, element e (channel / token slot e of the 8) sits in nibble e/2 if e is even, 4 + e/2 if odd:
// the kernel's unpacking puts nibbles i and i+4 into the two halves of one register.
//
// 3-bit codes (bits = 3): the same order of tokens, channels and lanes, but a lane's unit holds its four groups of
// eight codes (K: the four 16-token blocks tb; V: the fragments (cb = 2p, u = 0), (2p, 1), (2p+1, 0), (2p+1, 1)) in
// 12 bytes instead of 16.  Dword k (k = 0, 1, 2) holds group k: element e = 2i + h in bits 3i .. 3i+2 of half word h
// (twelve bits per half word).  The four bits that are left in every half word hold group 3: its half word h (again
// twelve bits, element 2i + h at bits 3i .. 3i+2) is cut into three nibbles, nibble j stored in bits 12 .. 15 of half
// word h of dword j.  So three of the four groups unpack exactly like 4-bit codes (one shift, four mask-and-or
// operations: a field at bit s of a half word under the exponent of 2^(10-s) reads 2^(10-s) + its value), and the
// fourth takes six operations more to collect.  An odd last value channel block has units of two groups: two dwords.
//   K codes: 48 * r_k_pad / 2 bytes;  V codes: 768 per pair of channel blocks + 512 for an odd last one.
#pragma once
#include "ea_common.h"

namespace ea {

struct Q4Geo {
  int32_t nch;             // 8-channel chunks of a key row: r_k_pad / 8
  int32_t ks;              // 32-channel k-steps: ceil(nch / 4)
  int32_t ncb;             // 16-channel blocks of a value row: r_v_pad / 16
  int32_t tiles_per_page;
  int32_t tpg;             // tiles per key group: 1 (64 tokens) or 2 (128 tokens)
  int32_t bits;            // 4 or 3
  int32_t v_codes;         // bytes of the codes of a V tile block
  int32_t k_codes;         // bytes of the codes of a K tile block: nch * 256 (4 bits), nch * 192 (3 bits)
  int32_t k_scales;        // bytes of the scales and zeros of a key group: ks * 128
  int64_t k_tile, v_tile;  // bytes of a tile block (K: of one that carries scales)
  int64_t k_slab;          // bytes of the K tile blocks of one kv head in a page
  int64_t k_page, v_page;  // bytes of a page (all kv heads)
};

__host__ __device__ inline Q4Geo make_q4_geo(int32_t r_k, int32_t r_v, int32_t n_kv_heads, int32_t page_tokens,
                                             int32_t key_group, int32_t bits = 4) {
  Q4Geo q;
  q.nch = (r_k + 7) / 8;
  q.ks = (q.nch + 3) / 4;
  q.ncb = (r_v + 15) / 16;
  q.tiles_per_page = page_tokens / kTile;
  q.tpg = key_group == 128 ? 2 : 1;
  q.bits = bits == 3 ? 3 : 4;
  q.k_codes = q.nch * (q.bits == 3 ? 192 : 256);
  q.v_codes = q.bits == 3 ? (q.ncb / 2) * 768 + (q.ncb & 1) * 512 : q.ncb * 512;
  q.k_scales = q.ks * 128;
  q.k_tile = (int64_t)q.k_codes + q.k_scales;
  q.v_tile = (int64_t)q.v_codes + 256;
  q.k_slab = (int64_t)q.tiles_per_page * q.k_codes + (int64_t)(q.tiles_per_page / q.tpg) * q.k_scales;
  q.k_page = q.k_slab * n_kv_heads;
  q.v_page = q.v_tile * q.tiles_per_page * n_kv_heads;
  return q;
}

// Byte offset, inside a kv head's part of a K page, of tile `tin`'s block, and of the scales that belong to it
// (those of its group: right behind the codes of the group's first tile).
__host__ __device__ inline int64_t q4_k_tile_off(const Q4Geo& q, int32_t tin) {
  return (int64_t)tin * q.k_codes + (int64_t)((tin + q.tpg - 1) / q.tpg) * q.k_scales;
}
__host__ __device__ inline int64_t q4_k_group_scales_off(const Q4Geo& q, int32_t tin) {
  return q4_k_tile_off(q, tin - tin % q.tpg) + q.k_codes;
}

__host__ __device__ inline int32_t q4_nibble_shift(int32_t e) { return 4 * ((e & 1) ? 4 + (e >> 1) : (e >> 1)); }

// Byte offset inside a K tile block of the dword holding (token tt of the tile, channel c); c < 8 * nch.
__host__ __device__ inline int32_t q4_k_dword_off(int32_t tt, int32_t c) {
  const int32_t kk = c >> 5, quad = (c >> 3) & 3, tb = tt >> 4, t = tt & 15;
  return kk * 1024 + (quad * 16 + t) * 16 + tb * 4;
}
// Byte offset inside a group's block of scales of channel c's scale; the zero is 16 bytes further.
__host__ __device__ inline int32_t q4_k_scale_off(int32_t c) {
  return ((c >> 5) * 4 + ((c >> 3) & 3)) * 32 + (c & 7) * 2;
}
// Byte offset inside a V tile block of the dword holding (token tt, channel c), and the element slot of the token.
__host__ __device__ inline int32_t q4_v_dword_off(const Q4Geo& q, int32_t tt, int32_t c, int32_t* slot) {
  const int32_t u = tt >> 5, t32 = tt & 31, half = t32 >> 4, quad = (t32 & 15) >> 2;
  *slot = half * 4 + (t32 & 3);
  const int32_t cb = c >> 4, lane = quad * 16 + (c & 15), p = cb >> 1;
  if ((q.ncb & 1) && cb == q.ncb - 1) return p * 1024 + lane * 8 + u * 4;
  return p * 1024 + lane * 16 + ((cb & 1) * 2 + u) * 4;
}
__host__ __device__ inline int32_t q4_v_scale_off(const Q4Geo& q, int32_t tt) {
  const int32_t u = tt >> 5, t32 = tt & 31, half = t32 >> 4, quad = (t32 & 15) >> 2;
  return q.v_codes + ((u * 4 + quad) * 8 + half * 4 + (t32 & 3)) * 2;            // the zero is 128 bytes further
}

// ---- 3-bit codes: where the three bits of a code sit (byte offset of a dword inside the tile block, bit in it).
struct Q3Pos {
  int32_t byte[3], bit[3];
};
__host__ __device__ inline Q3Pos q3_in_unit(int32_t unit_off, int32_t group, int32_t e, bool two_groups) {
  const int32_t h = e & 1, i = e >> 1;
  Q3Pos p;
  for (int32_t b = 0; b < 3; ++b) {
    const int32_t s = 3 * i + b;                        // bit of the group's twelve-bit half word
    if (group < 3 || two_groups) {
      p.byte[b] = unit_off + 4 * group;
      p.bit[b] = 16 * h + s;
    } else {
      p.byte[b] = unit_off + 4 * (s >> 2);
      p.bit[b] = 16 * h + 12 + (s & 3);
    }
  }
  return p;
}
__host__ __device__ inline Q3Pos q3_k_pos(int32_t tt, int32_t c) {
  const int32_t kk = c >> 5, quad = (c >> 3) & 3, tb = tt >> 4, t = tt & 15;
  return q3_in_unit(kk * 768 + (quad * 16 + t) * 12, tb, c & 7, false);
}
__host__ __device__ inline Q3Pos q3_v_pos(const Q4Geo& q, int32_t tt, int32_t c) {
  const int32_t u = tt >> 5, t32 = tt & 31, half = t32 >> 4, quad = (t32 & 15) >> 2;
  const int32_t slot = half * 4 + (t32 & 3);
  const int32_t cb = c >> 4, lane = quad * 16 + (c & 15), p = cb >> 1;
  if ((q.ncb & 1) && cb == q.ncb - 1) return q3_in_unit(p * 768 + lane * 8, u, slot, true);
  return q3_in_unit(p * 768 + lane * 12, (cb & 1) * 2 + u, slot, false);
}
// the code at a position (host and device: the reference readers), and its bits spread to their places
__host__ __device__ inline uint32_t q3_read(const uint8_t* block, const Q3Pos& p) {
  uint32_t code = 0;
  for (int32_t b = 0; b < 3; ++b) code |= ((*reinterpret_cast<const uint32_t*>(block + p.byte[b]) >> p.bit[b]) & 1u) << b;
  return code;
}

typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(4))) _Float16 f16x4;

template <int NCB>
struct MergeSmemQ4 {
  float m[4][16];
  float l[4][16];
  float acc[4][16][NCB * 16];
};

__device__ __forceinline__ f32x4 mfma16h(f16x8 a, f16x8 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
}

// Eight nibbles -> eight fp16 numbers offset + code; element 2i is nibble i, element 2i+1 nibble i+4.
// A nibble in bits 0-3 of a half word, under the exponent of 1024.0 (0x6400, one unit per mantissa step), reads
// 1024 + code; one in bits 4-7 under the exponent of 64.0 (0x5400, sixteen steps per unit) reads 64 + code.  So
// the nibbles 0,1 (and 4,5) of the dword need no shift at all and the other four share one: elements 0,1,4,5
// carry the offset 1024, elements 2,3,6,7 the offset 64.  The two magic words come in registers (a mask-and-or
// takes one of its two constants from a vector register).
__device__ __forceinline__ f16x8 unpack_q4(uint32_t w, uint32_t magic1024, uint32_t magic64) {
  const uint32_t w8 = w >> 8;
  u32x4 r;
  r[0] = (w & 0x000f000fu) | magic1024;
  r[1] = (w & 0x00f000f0u) | magic64;
  r[2] = (w8 & 0x000f000fu) | magic1024;
  r[3] = (w8 & 0x00f000f0u) | magic64;
  return __builtin_bit_cast(f16x8, r);
}

// 3-bit codes: a word with element 2i + h in bits 3i .. 3i+2 of half word h -> eight fp16 numbers offset + code, the
// offsets 1024 (element pairs 0 and 2) and 128 (pairs 1 and 3): bits 0-2 under the exponent of 1024.0 (0x6400), bits
// 3-5 under that of 128.0 (0x5800, eight mantissa steps per unit).  Bits 12-15 of the half words are ignored.
__device__ __forceinline__ f16x8 unpack_q3(uint32_t w, uint32_t magic1024, uint32_t magic128) {
  const uint32_t w6 = w >> 6;
  u32x4 r;
  r[0] = (w & 0x00070007u) | magic1024;
  r[1] = (w & 0x00380038u) | magic128;
  r[2] = (w6 & 0x00070007u) | magic1024;
  r[3] = (w6 & 0x00380038u) | magic128;
  return __builtin_bit_cast(f16x8, r);
}
// the word of group 3, collected from the upper nibbles of the unit's three dwords
__device__ __forceinline__ uint32_t q3_group3(uint32_t d0, uint32_t d1, uint32_t d2) {
  return ((d0 >> 12) & 0x000f000fu) | ((d1 >> 8) & 0x00f000f0u) | ((d2 >> 4) & 0x0f000f00u);
}

// What the kernels that read codes share, for BITS = 4 or 3: a lane's unit of four groups of eight codes as it comes
// from memory (16 bytes, or 12 in the first three dwords), the A operand "offset + code" of one group, and what the
// unpacking added: elements 0,1,4,5 carry 1024, elements 2,3,6,7 carry kOffLo.
template <int BITS>
struct Codes {
  static constexpr int kUnit = BITS == 3 ? 12 : 16;       // bytes of a lane's unit
  static constexpr int kRun = 64 * kUnit;                 // ... of a wave's run of units
  static constexpr float kOffLo = BITS == 3 ? 128.0f : 64.0f;
  static constexpr uint32_t kMagicLo = BITS == 3 ? 0x58005800u : 0x54005400u;
  template <bool NT>
  __device__ static __forceinline__ u32x4 load(const uint8_t* p) {
    if constexpr (BITS == 3) {
      const uint32_t* w = reinterpret_cast<const uint32_t*>(p);
      if constexpr (NT)
        return u32x4{__builtin_nontemporal_load(w), __builtin_nontemporal_load(w + 1), __builtin_nontemporal_load(w + 2), 0u};
      else
        return u32x4{w[0], w[1], w[2], 0u};
    } else {
      if constexpr (NT) return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
      else return *reinterpret_cast<const u32x4*>(p);
    }
  }
  // group k (0..3) of a unit; group u (0..1) of the 8-byte unit of an odd last channel block
  __device__ static __forceinline__ f16x8 frag(const u32x4& un, int k, uint32_t magic1024, uint32_t magic_lo) {
    if constexpr (BITS == 3) return unpack_q3(k < 3 ? un[k] : q3_group3(un[0], un[1], un[2]), magic1024, magic_lo);
    else return unpack_q4(un[k], magic1024, magic_lo);
  }
  __device__ static __forceinline__ f16x8 frag2(const u32x2& un, int u, uint32_t magic1024, uint32_t magic_lo) {
    if constexpr (BITS == 3) return unpack_q3(un[u], magic1024, magic_lo);
    else return unpack_q4(un[u], magic1024, magic_lo);
  }
};

int quantize_pages_q4(const Geo& g, const Q4Geo& qg, const void* k_pool, const void* v_pool, const int32_t* src_pages,
                      void* kq_pool, void* vq_pool, const int32_t* dst_pages, int32_t n_pages, int32_t q4_pool_pages,
                      hipStream_t st);
int dequantize_pages_q4(const Geo& g, const Q4Geo& qg, const void* kq_pool, const void* vq_pool, const int32_t* src_pages,
                        void* k_pool, void* v_pool, const int32_t* dst_pages, int32_t n_pages, int32_t q4_pool_pages,
                        hipStream_t st);
int decode_q4(const ea_layer_desc* d, const Geo& g, const Q4Geo& qg, const float* q, const void* kq_pool,
              const void* vq_pool, const int32_t* q4_page_table, const int32_t* q4_len, int32_t max_q4_pages,
              int32_t q4_pool_pages, int32_t B, int32_t n_splits, int32_t ws_slots, float* ws, hipStream_t st,
              const Geo* tail_geo, const void* k_pool, const void* v_pool, const int32_t* tail_page_table,
              const int32_t* tail_len,      // tail_geo == nullptr: no bfloat16 tail
              const float* alibi_slopes = nullptr);
// Causal prefill attention of the last n tokens over q4_len 4-bit tokens followed by tail_len bfloat16 tokens; ws:
// 2 * B * n * H * (r_v + 2) floats.
int prefill_q4(const ea_layer_desc* d, const Geo& gq, const Q4Geo& qg, const void* q, const void* kq_pool,
               const void* vq_pool, const int32_t* q4_page_table, const int32_t* q4_len, const Geo& gt,
               const void* k_pool, const void* v_pool, const int32_t* tail_page_table, const int32_t* tail_len,
               void* out, int32_t B, int32_t n, float* ws, hipStream_t st);
int decode_rope_q4(const ea_layer_desc* d, const Geo& g, const Q4Geo& qg, const float* q, const void* u_k,
                   double rope_base, const void* kq_pool, const void* vq_pool, const int32_t* q4_page_table,
                   const int32_t* q4_len, const int32_t* tail_len, int32_t max_q4_pages, int32_t q4_pool_pages,
                   int32_t B, int32_t n_splits, int32_t ws_slots, float* ws, hipStream_t st);

}  // namespace ea
