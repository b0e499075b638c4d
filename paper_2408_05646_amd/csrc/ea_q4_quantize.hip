// Quantises whole pages of the bfloat16 rank-r cache to the 4-bit group form (keys: one scale per channel and
// 64-token tile, or per pair of tiles; values: one scale per token).  A group with minimum lo and maximum hi gets
// zero = fp16(lo), scale = fp16((hi - lo) / 15) and codes clip(rint((x - zero) / scale), 0, 15), all in float
// (7 in place of 15 for 3-bit codes); a scale that rounds to 0 gives code 0.  Not a hot kernel: it runs once per page, when the page is full.
#include "ea_q4.h"

namespace ea {

struct QuantArgs {
  const uint16_t* k_pool;
  const uint16_t* v_pool;
  const int32_t* src_pages;
  uint8_t* kq_pool;
  uint8_t* vq_pool;
  const int32_t* dst_pages;
  Geo g;
  Q4Geo qg;
  int32_t q4_pool_pages;
};

__device__ __forceinline__ float bf16_bits_to_float(uint16_t b) { return __builtin_bit_cast(float, (uint32_t)b << 16); }

// scale and zero of a group, as the fp16 values they are stored as
__device__ __forceinline__ void group_scale_zero(float lo, float hi, float levels, _Float16& s, _Float16& z) {
  lo = fminf(fmaxf(lo, -65504.f), 65504.f);
  hi = fminf(fmaxf(hi, -65504.f), 65504.f);
  s = (_Float16)fminf((hi - lo) / levels, 65504.f);
  z = (_Float16)lo;
}

__device__ __forceinline__ uint32_t code_of(float x, float s, float z, float levels) {
  if (!(s > 0.f)) return 0u;
  return (uint32_t)fminf(fmaxf(rintf((x - z) / s), 0.f), levels);
}

__global__ __launch_bounds__(256) void quantize_q4_kernel(QuantArgs a) {
  __shared__ float x[kTile][129];
  __shared__ float sc[128], zr[128];
  const Geo& g = a.g;
  const Q4Geo& qg = a.qg;
  const int tile = blockIdx.x, kvh = blockIdx.y;
  const int src = a.src_pages[blockIdx.z], dst = a.dst_pages[blockIdx.z];
  if (src < 0 || src >= g.pool_pages || dst < 0 || dst >= a.q4_pool_pages) return;   // the whole workgroup leaves
  const int tid = threadIdx.x;
  const float levels = qg.bits == 3 ? 7.0f : 15.0f;

  // ---- keys: x[token][channel] <- the tile in its fragment order [4 blocks][nch chunks][16 tokens][8 channels]
  {
    auto load_tile = [&](int tl) {
      const uint16_t* kb = a.k_pool + (int64_t)src * g.k_page + (int64_t)kvh * g.k_slab + (int64_t)tl * (kTile * g.r_k_pad);
      for (int u = tid; u < kTile * qg.nch; u += 256) {           // 16-byte units: 8 channels of one token
        const int t = u & 15, rest = u >> 4;
        const int chunk = rest % qg.nch, tb = rest / qg.nch;
        const u32x4 w = *reinterpret_cast<const u32x4*>(kb + (u << 3));
        float* dst = &x[tb * 16 + t][chunk * 8];
#pragma unroll
        for (int p = 0; p < 4; ++p) {
          dst[2 * p] = __builtin_bit_cast(float, w[p] << 16);
          dst[2 * p + 1] = __builtin_bit_cast(float, w[p] & 0xffff0000u);
        }
      }
    };
    // A key group of two tiles: this workgroup quantises its own tile, but the extremes are the pair's, so it first
    // looks at the other tile of the pair (a second read of it; this kernel runs once per page).
    float lo = INFINITY, hi = -INFINITY;
    if (qg.tpg == 2) {
      load_tile(tile ^ 1);
      __syncthreads();
      if (tid < g.r_k) {
        for (int t = 0; t < kTile; ++t) {
          lo = fminf(lo, x[t][tid]);
          hi = fmaxf(hi, x[t][tid]);
        }
      }
      __syncthreads();
    }
    load_tile(tile);
    __syncthreads();
    if (tid < 128) {
      _Float16 s = (_Float16)0.f, z = (_Float16)0.f;
      if (tid < g.r_k) {
        for (int t = 0; t < kTile; ++t) {
          lo = fminf(lo, x[t][tid]);
          hi = fmaxf(hi, x[t][tid]);
        }
        group_scale_zero(lo, hi, levels, s, z);
      }
      sc[tid] = (float)s;
      zr[tid] = (float)z;
    }
    __syncthreads();
    uint8_t* slab = a.kq_pool + (int64_t)dst * qg.k_page + (int64_t)kvh * qg.k_slab;
    uint8_t* ko = slab + q4_k_tile_off(qg, tile);
    if (tile % qg.tpg == 0) {                                   // the group's first tile carries the scales
      uint8_t* so = slab + q4_k_group_scales_off(qg, tile);
      for (int c = tid; c < qg.ks * 32; c += 256) {
        _Float16* p = reinterpret_cast<_Float16*>(so + q4_k_scale_off(c));
        p[0] = (_Float16)sc[c];
        p[8] = (_Float16)zr[c];
      }
    }
    if (qg.bits == 3) {
      // one 12-byte unit per (token of a block, 8-channel chunk): the four blocks' codes in three dwords
      for (int e = tid; e < qg.nch * 16; e += 256) {
        const int t = e & 15, chunk = e >> 4;
        uint32_t w[3] = {0u, 0u, 0u};
        const int unit = (chunk >> 2) * 768 + ((chunk & 3) * 16 + t) * 12;
        for (int tb = 0; tb < 4; ++tb)
#pragma unroll
          for (int ce = 0; ce < 8; ++ce) {
            const int c = chunk * 8 + ce;
            const uint32_t code = code_of(x[tb * 16 + t][c], sc[c], zr[c], levels);
            const Q3Pos p = q3_in_unit(0, tb, ce, false);
#pragma unroll
            for (int b = 0; b < 3; ++b) w[p.byte[b] >> 2] |= ((code >> b) & 1u) << p.bit[b];
          }
        uint32_t* dst = reinterpret_cast<uint32_t*>(ko + unit);
        dst[0] = w[0];
        dst[1] = w[1];
        dst[2] = w[2];
      }
    } else {
      for (int e = tid; e < qg.nch * 64; e += 256) {
        const int tb = e & 3, t = (e >> 2) & 15, chunk = e >> 6;
        uint32_t w = 0;
#pragma unroll
        for (int ce = 0; ce < 8; ++ce) {
          const int c = chunk * 8 + ce;
          w |= code_of(x[tb * 16 + t][c], sc[c], zr[c], levels) << q4_nibble_shift(ce);
        }
        *reinterpret_cast<uint32_t*>(ko + q4_k_dword_off(tb * 16 + t, chunk * 8)) = w;
      }
    }
    __syncthreads();
  }

  // ---- values: fragment order [2 groups][ncb blocks][4 quads][16 channels][8 token slots]
  {
    const uint16_t* vb = a.v_pool + (int64_t)src * g.v_page + (int64_t)kvh * g.v_slab + (int64_t)tile * (kTile * g.r_v_pad);
    for (int un = tid; un < kTile * g.r_v_pad / 8; un += 256) {  // 16-byte units: 8 token slots of one channel
      const int ch = un & 15, quad = (un >> 4) & 3, rest = un >> 6;
      const int cb = rest % qg.ncb, u = rest / qg.ncb;
      const u32x4 w = *reinterpret_cast<const u32x4*>(vb + (un << 3));
#pragma unroll
      for (int p = 0; p < 4; ++p) {
        const int j0 = 2 * p, j1 = 2 * p + 1;
        x[u * 32 + (j0 >> 2) * 16 + quad * 4 + (j0 & 3)][cb * 16 + ch] = __builtin_bit_cast(float, w[p] << 16);
        x[u * 32 + (j1 >> 2) * 16 + quad * 4 + (j1 & 3)][cb * 16 + ch] = __builtin_bit_cast(float, w[p] & 0xffff0000u);
      }
    }
    __syncthreads();
    uint8_t* vo = a.vq_pool + (int64_t)dst * qg.v_page + ((int64_t)kvh * qg.tiles_per_page + tile) * qg.v_tile;
    if (tid < kTile) {
      float lo = x[tid][0], hi = lo;
      for (int c = 1; c < g.r_v; ++c) {
        lo = fminf(lo, x[tid][c]);
        hi = fmaxf(hi, x[tid][c]);
      }
      _Float16 s, z;
      group_scale_zero(lo, hi, levels, s, z);
      sc[tid] = (float)s;
      zr[tid] = (float)z;
      _Float16* p = reinterpret_cast<_Float16*>(vo + q4_v_scale_off(qg, tid));
      p[0] = s;
      p[64] = z;
    }
    __syncthreads();
    auto v_code = [&](int cb, int u, int lane, int j) -> uint32_t {
      const int quad = lane >> 4, c = cb * 16 + (lane & 15);
      const int tt = u * 32 + (j >> 2) * 16 + quad * 4 + (j & 3);
      return c < g.r_v ? code_of(x[tt][c], sc[tt], zr[tt], levels) : 0u;
    };
    if (qg.bits == 3) {
      // one unit per (pair of channel blocks, lane): four groups (cb, u) in three dwords; an odd last block: two in two
      const int units = (qg.ncb + 1) / 2;
      for (int e = tid; e < units * 64; e += 256) {
        const int lane = e & 63, p = e >> 6;
        const bool two = (qg.ncb & 1) && p == units - 1;
        uint32_t w[3] = {0u, 0u, 0u};
        for (int k = 0; k < (two ? 2 : 4); ++k) {
          const int cb = two ? 2 * p : 2 * p + (k >> 1), u = two ? k : (k & 1);
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            const uint32_t code = v_code(cb, u, lane, j);
            const Q3Pos pp = q3_in_unit(0, k, j, two);
#pragma unroll
            for (int b = 0; b < 3; ++b) w[pp.byte[b] >> 2] |= ((code >> b) & 1u) << pp.bit[b];
          }
        }
        uint32_t* dst = reinterpret_cast<uint32_t*>(vo + p * 768 + lane * (two ? 8 : 12));
        dst[0] = w[0];
        dst[1] = w[1];
        if (!two) dst[2] = w[2];
      }
    } else {
      for (int e = tid; e < qg.ncb * 128; e += 256) {
        const int lane = e & 63, u = (e >> 6) & 1, cb = e >> 7;
        uint32_t w = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) w |= v_code(cb, u, lane, j) << q4_nibble_shift(j);
        int slot;
        *reinterpret_cast<uint32_t*>(vo + q4_v_dword_off(qg, u * 32 + (lane >> 4) * 4, cb * 16 + (lane & 15), &slot)) = w;
      }
    }
  }
}

// The inverse direction, for export and inspection: value = scale * code + zero in float, rounded once to bfloat16,
// written in the bfloat16 pools' fragment order (padding channels zero).
__global__ __launch_bounds__(256) void dequantize_q4_kernel(QuantArgs a) {
  const Geo& g = a.g;
  const Q4Geo& qg = a.qg;
  const int tile = blockIdx.x, kvh = blockIdx.y;
  const int src = a.src_pages[blockIdx.z], dst = a.dst_pages[blockIdx.z];      // src: 4-bit page, dst: bfloat16 page
  if (src < 0 || src >= a.q4_pool_pages || dst < 0 || dst >= g.pool_pages) return;
  const int tid = threadIdx.x;
  const uint8_t* k_slab = a.kq_pool + (int64_t)src * qg.k_page + (int64_t)kvh * qg.k_slab;
  const uint8_t* kb = k_slab + q4_k_tile_off(qg, tile);
  const uint8_t* ks_grp = k_slab + q4_k_group_scales_off(qg, tile);
  const uint8_t* vb = a.vq_pool + (int64_t)src * qg.v_page + ((int64_t)kvh * qg.tiles_per_page + tile) * qg.v_tile;
  uint16_t* ko = const_cast<uint16_t*>(a.k_pool) + (int64_t)dst * g.k_page + (int64_t)kvh * g.k_slab;
  uint16_t* vo = const_cast<uint16_t*>(a.v_pool) + (int64_t)dst * g.v_page + (int64_t)kvh * g.v_slab;
  auto to_bf16 = [](float f) -> uint16_t {
    uint32_t u = __builtin_bit_cast(uint32_t, f);
    u += 0x7fffu + ((u >> 16) & 1u);                       // round to nearest even (finite inputs)
    return (uint16_t)(u >> 16);
  };
  auto pack2 = [&](float lo, float hi) -> uint32_t { return (uint32_t)to_bf16(lo) | ((uint32_t)to_bf16(hi) << 16); };
  // keys: one 16-byte unit of the bfloat16 tile = the 8 channels of one code dword
  for (int u = tid; u < kTile * qg.nch; u += 256) {
    const int t = u & 15, rest = u >> 4;
    const int chunk = rest % qg.nch, tb = rest / qg.nch;
    const int tt = tb * 16 + t, c0 = chunk * 8;
    // the 8 scales and the 8 zeros of these channels: two 16-byte units, 16 bytes apart
    typedef __attribute__((ext_vector_type(8))) _Float16 half8;
    const half8 sc8 = *reinterpret_cast<const half8*>(ks_grp + q4_k_scale_off(c0));
    const half8 zr8 = *reinterpret_cast<const half8*>(ks_grp + q4_k_scale_off(c0) + 16);
    _Float16 sp[16];
#pragma unroll
    for (int ce = 0; ce < 8; ++ce) {
      sp[ce] = sc8[ce];
      sp[8 + ce] = zr8[ce];
    }
    float val[8];
    if (qg.bits == 3) {
#pragma unroll
      for (int ce = 0; ce < 8; ++ce) {
        const uint32_t code = q3_read(kb, q3_k_pos(tt, c0 + ce));
        val[ce] = c0 + ce < g.r_k ? fmaf((float)sp[ce], (float)code, (float)sp[8 + ce]) : 0.f;
      }
    } else {
      const uint32_t w = *reinterpret_cast<const uint32_t*>(kb + q4_k_dword_off(tt, c0));
#pragma unroll
      for (int ce = 0; ce < 8; ++ce)
        val[ce] = c0 + ce < g.r_k ? fmaf((float)sp[ce], (float)((w >> q4_nibble_shift(ce)) & 15u), (float)sp[8 + ce]) : 0.f;
    }
    *reinterpret_cast<u32x4*>(ko + bf16_k_slab_off(tile * kTile + tt, c0, g.r_k_pad)) =
        u32x4{pack2(val[0], val[1]), pack2(val[2], val[3]), pack2(val[4], val[5]), pack2(val[6], val[7])};
  }
  // values: one 16-byte unit = the 8 token slots of one channel, one code dword
  for (int un = tid; un < kTile * g.r_v_pad / 8; un += 256) {
    const int ch = un & 15, quad = (un >> 4) & 3, rest = un >> 6;
    const int cb = rest % qg.ncb, u = rest / qg.ncb;
    const int c = cb * 16 + ch, tt0 = u * 32 + quad * 4;
    float val[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (c < g.r_v) {
      // the scales of the unit's 8 token slots and, 128 bytes further, their zeros: one 16-byte unit each
      typedef __attribute__((ext_vector_type(8))) _Float16 half8;
      const half8 sc8 = *reinterpret_cast<const half8*>(vb + q4_v_scale_off(qg, tt0));
      const half8 zr8 = *reinterpret_cast<const half8*>(vb + q4_v_scale_off(qg, tt0) + 128);
      if (qg.bits == 3) {
#pragma unroll
        for (int jj = 0; jj < 8; ++jj) {
          // token slot jj of this unit: token tt0 + 16 * (jj / 4) + jj % 4
          const uint32_t code = q3_read(vb, q3_v_pos(qg, tt0 + (jj >> 2) * 16 + (jj & 3), c));
          val[jj] = fmaf((float)sc8[jj], (float)code, (float)zr8[jj]);
        }
      } else {
        int slot0;
        const uint32_t w = *reinterpret_cast<const uint32_t*>(vb + q4_v_dword_off(qg, tt0, c, &slot0));
#pragma unroll
        for (int jj = 0; jj < 8; ++jj)
          val[jj] = fmaf((float)sc8[jj], (float)((w >> q4_nibble_shift(jj)) & 15u), (float)zr8[jj]);
      }
    }
    *reinterpret_cast<u32x4*>(vo + bf16_v_slab_off(tile * kTile + tt0, c, g.r_v_pad)) =
        u32x4{pack2(val[0], val[1]), pack2(val[2], val[3]), pack2(val[4], val[5]), pack2(val[6], val[7])};
  }
}

int dequantize_pages_q4(const Geo& g, const Q4Geo& qg, const void* kq_pool, const void* vq_pool, const int32_t* src_pages,
                        void* k_pool, void* v_pool, const int32_t* dst_pages, int32_t n_pages, int32_t q4_pool_pages,
                        hipStream_t st) {
  if (g.n_kv_heads > 65535) return EA_ERR_SHAPE;
  QuantArgs a;
  a.k_pool = (const uint16_t*)k_pool;
  a.v_pool = (const uint16_t*)v_pool;
  a.kq_pool = (uint8_t*)const_cast<void*>(kq_pool);
  a.vq_pool = (uint8_t*)const_cast<void*>(vq_pool);
  a.g = g;
  a.qg = qg;
  a.q4_pool_pages = q4_pool_pages;
  for (int32_t done = 0; done < n_pages; done += 65535) {
    const int32_t now = n_pages - done < 65535 ? n_pages - done : 65535;
    a.src_pages = src_pages + done;
    a.dst_pages = dst_pages + done;
    dequantize_q4_kernel<<<dim3(qg.tiles_per_page, g.n_kv_heads, now), dim3(256), 0, st>>>(a);
  }
  return launch_status();
}

int quantize_pages_q4(const Geo& g, const Q4Geo& qg, const void* k_pool, const void* v_pool, const int32_t* src_pages,
                      void* kq_pool, void* vq_pool, const int32_t* dst_pages, int32_t n_pages, int32_t q4_pool_pages,
                      hipStream_t st) {
  if (g.n_kv_heads > 65535) return EA_ERR_SHAPE;
  QuantArgs a;
  a.k_pool = (const uint16_t*)k_pool;
  a.v_pool = (const uint16_t*)v_pool;
  a.src_pages = src_pages;
  a.kq_pool = (uint8_t*)kq_pool;
  a.vq_pool = (uint8_t*)vq_pool;
  a.dst_pages = dst_pages;
  a.g = g;
  a.qg = qg;
  a.q4_pool_pages = q4_pool_pages;
  for (int32_t done = 0; done < n_pages; done += 65535) {        // grid.z is limited to 65535
    const int32_t now = n_pages - done < 65535 ? n_pages - done : 65535;
    QuantArgs b = a;
    b.src_pages = src_pages + done;
    b.dst_pages = dst_pages + done;
    quantize_q4_kernel<<<dim3(qg.tiles_per_page, g.n_kv_heads, now), dim3(256), 0, st>>>(b);
  }
  return launch_status();
}

}  // namespace ea
