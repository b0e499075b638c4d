// Launch side of the bf16 generation-phase attention kernel (position-free form) and the split merge.
#include "ea_decode_kernel.h"

namespace ea {

// out[b, h, :] = sum_s w_s acc_s / sum_s w_s l_s with w_s = 2^(m_s - max_s m_s).  With ml_out, the row's
// reference exponent max_s m_s and normaliser sum_s w_s l_s are stored too, as ml_out[2 (b H + h)], [.. + 1].
// The loads of up to eight splits are requested together (a split past the last reads the last one again and is
// ignored), so a row with at most eight splits costs one round trip to memory, not one per split.
__global__ void merge_splits_kernel(const float* __restrict__ ws, float* __restrict__ out, int32_t BH, int32_t S,
                                    int32_t r_v, int32_t r_v_pad, float* __restrict__ ml_out, int32_t out_bf16) {
  const int64_t bh = blockIdx.x;
  const int64_t BHS = (int64_t)BH * S;
  const float* pm = ws + bh * S;
  const float* pl = ws + BHS + bh * S;
  const float* pa = ws + 2 * BHS + bh * S * r_v_pad;
  for (int c0 = 0; c0 < r_v; c0 += blockDim.x) {
    const int c = min(c0 + (int)threadIdx.x, r_v - 1);      // surplus threads repeat the last channel and store nothing
    float mm = -INFINITY, lsum = 0.f, val = 0.f;
    if (S <= 8) {
      float m8[8], l8[8], a8[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int s = min(u, S - 1);
        m8[u] = pm[s];
        l8[u] = pl[s];
        a8[u] = pa[(int64_t)s * r_v_pad + c];
      }
#pragma unroll
      for (int u = 0; u < 8; ++u)
        if (u < S) mm = fmaxf(mm, m8[u]);
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        if (u < S && mm != -INFINITY) {
          const float wt = __builtin_amdgcn_exp2f(m8[u] - mm);
          lsum += wt * l8[u];
          val += wt * a8[u];
        }
      }
    } else {
      for (int s0 = 0; s0 < S; s0 += 8) {
        float m8[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) m8[u] = pm[min(s0 + u, S - 1)];
#pragma unroll
        for (int u = 0; u < 8; ++u) mm = fmaxf(mm, m8[u]);
      }
      for (int s0 = 0; s0 < S && mm != -INFINITY; s0 += 8) {
        float m8[8], l8[8], a8[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int s = min(s0 + u, S - 1);
          m8[u] = pm[s];
          l8[u] = pl[s];
          a8[u] = pa[(int64_t)s * r_v_pad + c];
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          if (s0 + u < S) {
            const float wt = __builtin_amdgcn_exp2f(m8[u] - mm);
            lsum += wt * l8[u];
            val += wt * a8[u];
          }
        }
      }
    }
    if (ml_out && c0 == 0 && threadIdx.x == 0) {
      ml_out[2 * bh] = mm;
      ml_out[2 * bh + 1] = lsum;
    }
    if (c0 + (int)threadIdx.x < r_v) {
      const float o = lsum > 0.f ? val / lsum : 0.f;
      if (out_bf16) reinterpret_cast<__bf16*>(out)[bh * r_v + c] = (__bf16)o;
      else out[bh * r_v + c] = o;
    }
  }
}

int merge_splits(const Geo& g, const float* ws, float* out, int32_t B, int32_t n_splits, hipStream_t st, float* ml_out,
                 int32_t out_bf16) {
  merge_splits_kernel<<<dim3(B * g.n_heads), dim3(64), 0, st>>>(ws, out, B * g.n_heads, n_splits, g.r_v, g.r_v_pad,
                                                               ml_out, out_bf16);
  return launch_status();
}

template <int KS, int NCB>
static void launch_decode(const DecodeArgs& a, int32_t B, hipStream_t st) {
  dim3 grid(a.g.n_kv_heads, a.n_splits, B), block(256);
  constexpr int TBN = (KS * 4 + NCB * 2 > 22) ? 2 : 4;   // fragments of a whole tile: 16*KS + 8*NCB registers
  decode_bf16_kernel<KS, NCB, TBN, 2, 0><<<grid, block, 0, st>>>(a);
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
                hipStream_t st, int32_t ws_slots, int32_t ws_slot0, int32_t seq_add, int32_t out_bf16) {
  if (B > 65535 || g.n_kv_heads > 65535) return EA_ERR_SHAPE;
  DecodeArgs a;
  a.out_bf16 = out_bf16;
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
  a.u_k = nullptr;
  a.d_head = d->d_head;
  a.alibi = nullptr;
  a.log2_base = 0.0;
  a.ws_slots = ws_slots;
  a.ws_slot0 = ws_slot0;
  a.seq_add = seq_add;
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
