// bf16 matrix-core GEMMs for the low-rank projections (Eq. 1 with the folded
// weights of Eq. 8, and the output projection of Eq. 2):
//   C[M,N] = A[M,K] . Wt[N,K]^T,  bf16 operands, fp32 accumulation.
// Both operands are K-contiguous, so MFMA fragments are plain 16-byte loads.
//  - tiled kernel (M > 64): 128x128x64 workgroup tiles staged through LDS,
//    2x2 waves of 64x64, v_mfma_f32_16x16x32_bf16;
//  - skinny kernel (M <= 64, the generation phase): one workgroup per 16 output
//    channels, the four waves split K and stream the weight rows straight from
//    HBM (the weights are read exactly once; x stays in L2).
#include "ea_common.h"
#include "ea_epilogue.h"

namespace ea {

// 8 consecutive K elements of a row as a bf16 fragment (float input is rounded to nearest even).
template <bool F32>
__device__ __forceinline__ bf16x8 load_frag(const void* base, int64_t elem_off) {
  if (!F32) return *reinterpret_cast<const bf16x8*>(reinterpret_cast<const uint16_t*>(base) + elem_off);
  const float4* p = reinterpret_cast<const float4*>(reinterpret_cast<const float*>(base) + elem_off);
  const float4 lo = p[0], hi = p[1];
  bf16x8 r;
  r[0] = (__bf16)lo.x; r[1] = (__bf16)lo.y; r[2] = (__bf16)lo.z; r[3] = (__bf16)lo.w;
  r[4] = (__bf16)hi.x; r[5] = (__bf16)hi.y; r[6] = (__bf16)hi.z; r[7] = (__bf16)hi.w;
  return r;
}

// ---------------------------------------------------------------------------
// Tiled kernel
// ---------------------------------------------------------------------------
template <typename Epilogue, bool A_F32>
__global__ __launch_bounds__(256, 2) void gemm_bf16_tiled_kernel(const void* __restrict__ A,
                                                                 const uint16_t* __restrict__ Wt, int32_t M, int32_t N,
                                                                 int32_t K, Epilogue ep) {
  constexpr int BM = 128, BN = 128, BK = 64, LDK = BK + 8;   // +8 elements: rows 144 B apart, conflict-free b128 reads
  __shared__ __attribute__((aligned(16))) uint16_t As[BM * LDK];
  __shared__ __attribute__((aligned(16))) uint16_t Bs[BN * LDK];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int col = lane & 15, quad = lane >> 4;
  const int wm = wave >> 1, wn = wave & 1;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;

  f32x4 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  bf16x8 ga[4], gb[4];
  auto gload = [&](int k0) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int chunk = tid + 256 * i, row = chunk >> 3, kc = (chunk & 7) * 8;
      const bool kin = k0 + kc < K;
      ga[i] = (kin && m0 + row < M) ? load_frag<A_F32>(A, (int64_t)(m0 + row) * K + k0 + kc) : zero_frag();
      gb[i] = (kin && n0 + row < N) ? load_frag<false>(Wt, (int64_t)(n0 + row) * K + k0 + kc) : zero_frag();
    }
  };
  gload(0);
  for (int k0 = 0; k0 < K; k0 += BK) {
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int chunk = tid + 256 * i, row = chunk >> 3, kc = (chunk & 7) * 8;
      *reinterpret_cast<bf16x8*>(&As[row * LDK + kc]) = ga[i];
      *reinterpret_cast<bf16x8*>(&Bs[row * LDK + kc]) = gb[i];
    }
    __syncthreads();
    if (k0 + BK < K) gload(k0 + BK);
#pragma unroll
    for (int ks = 0; ks < BK / 32; ++ks) {
      bf16x8 af[4], bfr[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        af[i] = *reinterpret_cast<const bf16x8*>(&As[(wm * 64 + i * 16 + col) * LDK + ks * 32 + quad * 8]);
        bfr[i] = *reinterpret_cast<const bf16x8*>(&Bs[(wn * 64 + i * 16 + col) * LDK + ks * 32 + quad * 8]);
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = mfma16(af[i], bfr[j], acc[i][j]);
    }
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int r = m0 + wm * 64 + i * 16 + quad * 4 + e, c = n0 + wn * 64 + j * 16 + col;
        if (r < M && c < N) ep(r, c, acc[i][j][e]);
      }
}

// ---------------------------------------------------------------------------
// Skinny kernel: M <= 16*MT rows, 16 output channels per workgroup, K split over 4 waves.
// A float A operand is split in hi + lo bf16 halves so it loses no precision.
// ---------------------------------------------------------------------------
template <typename Epilogue, bool A_F32, int MT>
__global__ __launch_bounds__(256) void gemm_bf16_skinny_kernel(const void* __restrict__ A,
                                                               const uint16_t* __restrict__ Wt, int32_t M, int32_t N,
                                                               int32_t K, Epilogue ep) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int col = lane & 15, quad = lane >> 4;
  const int n0 = blockIdx.x * 16;
  const bool n_ok = n0 + col < N;
  const uint16_t* wrow = Wt + (int64_t)(n_ok ? n0 + col : 0) * K + quad * 8;

  f32x4 acc[MT];
#pragma unroll
  for (int i = 0; i < MT; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};

  const int steps = K / 32;
  constexpr int UN = 4;
  for (int s0 = wave * UN; s0 < steps; s0 += 4 * UN) {
    bf16x8 bw[UN];
#pragma unroll
    for (int u = 0; u < UN; ++u)
      bw[u] = (n_ok && s0 + u < steps) ? *reinterpret_cast<const bf16x8*>(wrow + (int64_t)(s0 + u) * 32) : zero_frag();
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      if (s0 + u >= steps) break;
      const int64_t koff = (int64_t)(s0 + u) * 32 + quad * 8;
#pragma unroll
      for (int i = 0; i < MT; ++i) {
        const int row = i * 16 + col;
        if (!A_F32) {
          const bf16x8 af = row < M ? load_frag<false>(A, (int64_t)row * K + koff) : zero_frag();
          acc[i] = mfma16(af, bw[u], acc[i]);
        } else {
          bf16x8 hi = zero_frag(), lo = zero_frag();
          if (row < M) {
            const float4* p = reinterpret_cast<const float4*>(reinterpret_cast<const float*>(A) + (int64_t)row * K + koff);
            const float4 v0 = p[0], v1 = p[1];
            const float f[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
#pragma unroll
            for (int j = 0; j < 8; ++j) {
              const __bf16 h = (__bf16)f[j];
              hi[j] = h;
              lo[j] = (__bf16)(f[j] - (float)h);
            }
          }
          acc[i] = mfma16(hi, bw[u], acc[i]);
          acc[i] = mfma16(lo, bw[u], acc[i]);
        }
      }
    }
  }
  __shared__ f32x4 red[4][MT][64];
#pragma unroll
  for (int i = 0; i < MT; ++i) red[wave][i][lane] = acc[i];
  __syncthreads();
  for (int idx = tid; idx < MT * 64; idx += 256) {
    const int i = idx >> 6, ln = idx & 63;
    const f32x4 v = red[0][i][ln] + red[1][i][ln] + red[2][i][ln] + red[3][i][ln];
    const int c = n0 + (ln & 15);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int r = i * 16 + (ln >> 4) * 4 + e;
      if (r < M && c < N) ep(r, c, v[e]);
    }
  }
}

struct QkvEpBf16 {
  QkvDest d;
  __device__ void operator()(int r, int c, float v) const { qkv_store<true>(d, r, c, v); }
};
struct PlainEpBf16 {
  uint16_t* y;
  int32_t N;
  __device__ void operator()(int r, int c, float v) const { y[(int64_t)r * N + c] = f32_to_bf16_rne(v); }
};

template <typename Epilogue, bool A_F32>
static int launch_gemm(const void* A, const void* Wt, int32_t M, int32_t N, int32_t K, const Epilogue& ep,
                       hipStream_t st) {
  const uint16_t* w = (const uint16_t*)Wt;
  if (M <= 64) {
    dim3 grid((N + 15) / 16), block(256);
    const int mt = (M + 15) / 16;
    switch (mt) {
      case 1: gemm_bf16_skinny_kernel<Epilogue, A_F32, 1><<<grid, block, 0, st>>>(A, w, M, N, K, ep); break;
      case 2: gemm_bf16_skinny_kernel<Epilogue, A_F32, 2><<<grid, block, 0, st>>>(A, w, M, N, K, ep); break;
      case 3: gemm_bf16_skinny_kernel<Epilogue, A_F32, 3><<<grid, block, 0, st>>>(A, w, M, N, K, ep); break;
      default: gemm_bf16_skinny_kernel<Epilogue, A_F32, 4><<<grid, block, 0, st>>>(A, w, M, N, K, ep); break;
    }
  } else {
    dim3 grid((N + 127) / 128, (M + 127) / 128), block(256);
    if (grid.y > 65535) return EA_ERR_SHAPE;
    gemm_bf16_tiled_kernel<Epilogue, A_F32><<<grid, block, 0, st>>>(A, w, M, N, K, ep);
  }
  return launch_status();
}

int gemm_qkv_bf16(const void* x, const void* w_t, int32_t M, int32_t N, int32_t K, const QkvDest& dst,
                  hipStream_t st) {
  return launch_gemm<QkvEpBf16, false>(x, w_t, M, N, K, QkvEpBf16{dst}, st);
}

int gemm_out_bf16(const void* a, int32_t a_is_f32, const void* w_t, void* y, int32_t M, int32_t N, int32_t K,
                  hipStream_t st) {
  PlainEpBf16 ep{(uint16_t*)y, N};
  if (a_is_f32) return launch_gemm<PlainEpBf16, true>(a, w_t, M, N, K, ep, st);
  return launch_gemm<PlainEpBf16, false>(a, w_t, M, N, K, ep, st);
}

}  // namespace ea
