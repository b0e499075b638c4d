// bf16 matrix-core GEMMs for the low-rank projections (Eq. 1 with the folded
// weights of Eq. 8, and the output projection of Eq. 2):
//   C[M,N] = A[M,K] . W[N,K]^T,  bf16 operands, fp32 accumulation.
// A is row-major (K contiguous).  W is packed in MFMA fragment order
// [N/16][K/32][4 quads][16 channels][8 k]: the B operand of one (channel block, k step) is one
// contiguous 1 KiB wave load, and a channel block's K range is one contiguous stream.
//  - asynchronous kernel (M >= 2048, bf16 activations: the prefill): 256x256x64 workgroup tiles, eight waves,
//    global tiles loaded straight into LDS, two stages;
//  - tiled kernel (other M > 64): 128x128x64 (256x128x64 for M >= 2048 with float activations) workgroup tiles
//    staged through registers and LDS, 2x2 waves, v_mfma_f32_16x16x32_bf16, XCD-aware banded tile order;
//  - skinny kernel (M <= 64, the generation phase): one workgroup per 16 output
//    channels, the four waves split K and stream the weight rows straight from
//    HBM (the weights are read exactly once; x stays in L2).
#include "ea_common.h"
#include "ea_epilogue.h"
#include <type_traits>
#include <utility>

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
// Tiled kernel.  A wave owns a 64x64 output tile as 4x4 MFMA blocks.  With SWAP the operands
// are exchanged (D^T = W_blk . A_blk^T), so a lane holds 4 CONSECUTIVE OUTPUT CHANNELS of one
// row (an 8-byte bf16 store) instead of one channel of 4 rows; the epilogue picks per wave.
// ---------------------------------------------------------------------------
template <typename Epilogue, bool A_F32, int MI>
__global__ __launch_bounds__(256, 2) void gemm_bf16_tiled_kernel(const void* __restrict__ A,
                                                                 const uint16_t* __restrict__ Wt, int32_t M, int32_t N,
                                                                 int32_t K, Epilogue ep) {
  // The W tile sits in LDS in MFMA fragment order [8 blocks of 16 rows][2 k steps][64 lanes][8 elements]
  // (the order it has in memory); the A tile is row-major with padded rows.
  constexpr int BM = 32 * MI, BN = 128, BK = 64, LDK = BK + 8;   // A rows 144 B apart: conflict-free 16-byte reads
  __shared__ __attribute__((aligned(16))) uint16_t As[BM * LDK];
  __shared__ __attribute__((aligned(16))) uint16_t Bs[BN * BK];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int col = lane & 15, quad = lane >> 4;
  const int wm = wave >> 1, wn = wave & 1;
  // Tile order.  Workgroups go round-robin to the 8 XCDs (each with its own L2): give every XCD a contiguous
  // range of the tile sequence, and walk that sequence in bands of kGroupM row tiles so that the workgroups
  // running together on an XCD share a few A row tiles and W column tiles.
  const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
  const int total = tiles_m * tiles_n;
  int pid = blockIdx.x;
  {
    const int per_xcd = (total + 7) / 8;
    const int remapped = (pid % 8) * per_xcd + pid / 8;
    if (per_xcd * 8 == total) pid = remapped;          // only when the tiles divide evenly over the XCDs
  }
  constexpr int kGroupM = 8;
  const int band = pid / (kGroupM * tiles_n);
  const int band_rows = min(kGroupM, tiles_m - band * kGroupM);
  const int in_band = pid - band * kGroupM * tiles_n;
  const int tm = band * kGroupM + in_band % band_rows, tn = in_band / band_rows;
  const int m0 = tm * BM, n0 = tn * BN;
  const int r0 = m0 + wm * (16 * MI), c0 = n0 + wn * 64;
  const bool swap = ep.swap_for(c0);          // wave-uniform

  f32x4 acc[MI][4];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  bf16x8 ga[MI], gb[4];
  const int ksteps = K >> 5;
  const int nblks = (N + 15) >> 4;
  // Global tiles come through buffer loads: one scalar descriptor per operand and tile (rows / channel blocks
  // past the matrix read as zero, no branches), loop-invariant 32-bit lane offsets, and the K position in the
  // instruction's scalar offset -- no per-load 64-bit address arithmetic in the loop.
  constexpr int kEsz = A_F32 ? 4 : 2;
  constexpr uint32_t kOob = 0x7ffffff0u;     // beyond any descriptor's size: reads as zero
  const __amdgpu_buffer_rsrc_t a_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<char*>(reinterpret_cast<const char*>(A)) + (int64_t)m0 * K * kEsz, 0,
      (int)((int64_t)min(BM, M - m0) * K * kEsz), 0x00020000);
  const __amdgpu_buffer_rsrc_t w_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint16_t*>(Wt) + (((int64_t)(n0 >> 4) * ksteps) << 9), 0,
      (int)((int64_t)min(BN / 16, nblks - (n0 >> 4)) * ksteps * 1024), 0x00020000);
  uint32_t a_off[MI], w_off[4];
#pragma unroll
  for (int i = 0; i < MI; ++i) {
    const int chunk = tid + 256 * i, row = chunk >> 3, kc = (chunk & 7) * 8;     // A: 8 threads read 128 B of a row
    a_off[i] = (uint32_t)((row * K + kc) * kEsz);
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    // W: this thread's 16-byte unit of fragment (channel block nb, k step kst): 64 threads read 1 KiB contiguous
    const int chunk = tid + 256 * i;
    const int frag = chunk >> 6, ln = chunk & 63, nb = frag >> 1, kst = frag & 1;
    w_off[i] = (uint32_t)(((nb * ksteps + kst) << 10) + (ln << 4));
  }
  const bool k_even = (K & 63) == 0;          // otherwise the last step holds one 32-wide k step only
  auto gload = [&](int k0) __attribute__((always_inline)) {
    const bool tail = !k_even && k0 + BK > K;
#pragma unroll
    for (int i = 0; i < MI; ++i) {
      const int kc = ((tid + 256 * i) & 7) * 8;
      const uint32_t off = (tail && kc >= 32) ? kOob : a_off[i];
      if (!A_F32) {
        ga[i] = __builtin_bit_cast(bf16x8, __builtin_amdgcn_raw_buffer_load_b128(a_rsrc, off, k0 * kEsz, 0));
      } else {
        const f32x4 lo = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(a_rsrc, off, k0 * kEsz, 0));
        const f32x4 hi =
            __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(a_rsrc, off + 16, k0 * kEsz, 0));
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          ga[i][e] = (__bf16)lo[e];
          ga[i][4 + e] = (__bf16)hi[e];
        }
      }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int kst = ((tid + 256 * i) >> 6) & 1;
      const uint32_t off = (tail && kst == 1) ? kOob : w_off[i];
      gb[i] = __builtin_bit_cast(bf16x8, __builtin_amdgcn_raw_buffer_load_b128(w_rsrc, off, (k0 >> 5) << 10, 0));
    }
  };
  auto mainloop = [&](auto swap_tag) __attribute__((always_inline)) {
    constexpr bool SWAP = decltype(swap_tag)::value;
    gload(0);
    for (int k0 = 0; k0 < K; k0 += BK) {
      __syncthreads();
#pragma unroll
      for (int i = 0; i < MI; ++i) {
        const int chunk = tid + 256 * i, row = chunk >> 3, kc = (chunk & 7) * 8;
        *reinterpret_cast<bf16x8*>(&As[row * LDK + kc]) = ga[i];
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) *reinterpret_cast<bf16x8*>(&Bs[(tid + 256 * i) << 3]) = gb[i];
      __syncthreads();
      __builtin_amdgcn_s_setprio(1);
      if (k0 + BK < K) gload(k0 + BK);
      // One straight pipeline over the two k steps of the tile: while the four MFMAs of one A fragment run, the
      // next A fragment (and, during the first k step, the W fragments of the second) come from LDS.
      auto read_a = [&](int ks, int i) __attribute__((always_inline)) {
        return *reinterpret_cast<const bf16x8*>(&As[(wm * (16 * MI) + i * 16 + col) * LDK + ks * 32 + quad * 8]);
      };
      auto read_w = [&](int ks, int j) __attribute__((always_inline)) {
        return *reinterpret_cast<const bf16x8*>(&Bs[((((wn * 4 + j) * 2 + ks) * 64) + lane) << 3]);
      };
      bf16x8 w0[4], w1[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) w0[j] = read_w(0, j);
      bf16x8 af = read_a(0, 0);
#pragma unroll
      for (int i = 0; i < MI; ++i) {
        bf16x8 af_next = i + 1 < MI ? read_a(0, i + 1) : read_a(1, 0);
        if (i < 4) w1[i] = read_w(1, i);
#pragma unroll
        for (int j = 0; j < 4; ++j)
          acc[i][j] = SWAP ? mfma16(w0[j], af, acc[i][j]) : mfma16(af, w0[j], acc[i][j]);
        af = af_next;
      }
#pragma unroll
      for (int j = MI; j < 4; ++j) w1[j] = read_w(1, j);     // (tiles lower than 128 rows: the loop above took MI of them)
#pragma unroll
      for (int i = 0; i < MI; ++i) {
        bf16x8 af_next = af;
        if (i + 1 < MI) af_next = read_a(1, i + 1);
#pragma unroll
        for (int j = 0; j < 4; ++j)
          acc[i][j] = SWAP ? mfma16(w1[j], af, acc[i][j]) : mfma16(af, w1[j], acc[i][j]);
        af = af_next;
      }
      // instruction order for the scheduler (LDS latency hides behind matrix-core work instead of in front of it)
      __builtin_amdgcn_sched_group_barrier(0x100, 5, 0);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
      }
#pragma unroll
      for (int i = 4; i < MI; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
      }
#pragma unroll
      for (int i = 0; i < MI - 1; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
      __builtin_amdgcn_s_setprio(0);
    }
  };
  if (swap) mainloop(std::true_type{});
  else mainloop(std::false_type{});
  ep.template store<MI>(swap, r0, c0, acc, M, N, col, quad);
}

typedef int i32x4 __attribute__((ext_vector_type(4)));

// A raw buffer descriptor over n_bytes at base (reads past the end return zero).
__device__ __forceinline__ i32x4 raw_buffer(const void* base, int64_t n_bytes) {
  const uint64_t a = reinterpret_cast<uint64_t>(base);
  return i32x4{(int)(a & 0xffffffffu), (int)((a >> 32) & 0xffffu), (int)n_bytes, 0x00020000};
}

// One 16-byte-per-lane buffer load whose data goes to LDS instead of registers: lane l's 16 bytes land at
// lds_addr + 16 l (lds_addr wave-uniform), read from the descriptor at voff (per lane) + soff (uniform).
// Written as an instruction rather than through the compiler's builtin: the compiler would otherwise make every
// later LDS read wait for ALL such loads in flight, the prefetched stages included.  The waits are placed by hand.
// The instruction takes its LDS base from M0, which this statement overwrites; the compiler keeps M0 reserved and does not
// hold values in it (the kernel using this has no other M0 consumer: no LDS-direct builtins, no sendmsg, no movrel).
__device__ __forceinline__ void load_to_lds_b128(i32x4 rsrc, uint32_t lds_addr, uint32_t voff, uint32_t soff) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
               :
               : "s"(lds_addr), "v"(voff), "s"(rsrc), "s"(soff)
               : "memory");
}

// ---------------------------------------------------------------------------
// Tiled kernel, asynchronous form (bf16 activations): 256x256 output tiles, eight waves of 128x64 each, and the global
// tiles go straight into LDS (buffer loads with the LDS flag: lane l of a wave lands 16 bytes at base + 16 l, wherever
// it read them from) -- two 64-wide stages, one barrier per stage, no staging registers and no LDS stores.
//   A stage: 256 rows x 128 bytes, a 1 KiB unit = 8 rows; the eight 16-byte k chunks of a row sit at position
//            chunk ^ ((row >> 1) & 7), so the 16 rows a fragment read touches fall into 16 different bank groups;
//   W stage: 16 channel blocks x 2 k steps x 1 KiB in fragment order, as in memory.
// ---------------------------------------------------------------------------
constexpr int kAsyncLds = 2 * (256 * 64 + 256 * 64) * 2;      // bytes of dynamic LDS: two stages of A and W

template <typename Epilogue>
__global__ __launch_bounds__(512, 1) void gemm_bf16_async_kernel(const uint16_t* __restrict__ A,
                                                                 const uint16_t* __restrict__ Wt, int32_t M, int32_t N,
                                                                 int32_t K, Epilogue ep) {
  constexpr int MI = 8, BM = 256, BN = 256, BK = 64;
  extern __shared__ __attribute__((aligned(1024))) uint16_t smem[];
  // stage s: A at s * 32768 elements (A then W, 16384 elements each)
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int col = lane & 15, quad = lane >> 4;
  const int wm = wave >> 2, wn = wave & 3;
  const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
  const int total = tiles_m * tiles_n;
  int pid = blockIdx.x;
  {
    const int per_xcd = (total + 7) / 8;
    const int remapped = (pid % 8) * per_xcd + pid / 8;
    if (per_xcd * 8 == total) pid = remapped;
  }
  constexpr int kGroupM = 8;
  const int band = pid / (kGroupM * tiles_n);
  const int band_rows = min(kGroupM, tiles_m - band * kGroupM);
  const int in_band = pid - band * kGroupM * tiles_n;
  const int tm = band * kGroupM + in_band % band_rows, tn = in_band / band_rows;
  const int m0 = tm * BM, n0 = tn * BN;
  const int r0 = m0 + wm * (16 * MI), c0 = n0 + wn * 64;
  const bool swap = ep.swap_for(c0);

  f32x4 acc[MI][4];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  const int ksteps = K >> 5;                 // 32-wide k steps of the packed weights
  const int nst = (K + BK - 1) / BK;         // 64-wide stages (the last may hold one k step only)
  const int nblks = (N + 15) >> 4;
  const i32x4 a_rsrc = raw_buffer(A + (int64_t)m0 * K, (int64_t)min(BM, M - m0) * K * 2);
  const i32x4 w_rsrc = raw_buffer(Wt + (((int64_t)(n0 >> 4) * ksteps) << 9),
                                  (int64_t)min(BN / 16, nblks - (n0 >> 4)) * ksteps * 1024);
  // this wave's units of a stage: A units 4 wave .. + 3 (8 rows each), W units 4 wave .. + 3
  // (unit = channel block 2 wave + i / 2, k step i % 2)
  constexpr uint32_t kOob = 0x7ffffff0u;     // beyond any descriptor: reads as zero
  uint32_t a_off[4], w_off[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row = (wave * 4 + i) * 8 + (lane >> 3);
    const int chunk = (lane & 7) ^ ((row >> 1) & 7);           // the k chunk that belongs at this lane's LDS position
    a_off[i] = (uint32_t)((row * K + chunk * 8) * 2);
    const int nb = wave * 2 + (i >> 1), kst = i & 1;
    w_off[i] = (uint32_t)(((nb * ksteps + kst) << 10) + (lane << 4));
  }
  const bool k_even = (K & 63) == 0;
  const uint32_t lds0 = (uint32_t)reinterpret_cast<uintptr_t>((__attribute__((address_space(3))) const uint16_t*)smem);
  auto issue = [&](int buf, int s) __attribute__((always_inline)) {
    const bool tail = !k_even && s == nst - 1;                 // only the first 32 of this stage's 64 columns exist
    const uint32_t a_dst = lds0 + buf * 65536 + wave * 4096, w_dst = lds0 + buf * 65536 + 32768 + wave * 4096;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int chunk = (lane & 7) ^ ((((wave * 4 + i) * 8 + (lane >> 3)) >> 1) & 7);
      load_to_lds_b128(a_rsrc, a_dst + i * 1024, (tail && chunk >= 4) ? kOob : a_off[i], s * 128);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
      load_to_lds_b128(w_rsrc, w_dst + i * 1024, (tail && (i & 1)) ? kOob : w_off[i], s << 11);
  };
  // fragment reads: row wm*128 + 16 i + col, k chunk 4 ks + quad at its swizzled place
  const int a_lane0 = (wm * 128 + col) * BK + ((quad ^ ((col >> 1) & 7)) << 3);
  const int a_lane1 = (wm * 128 + col) * BK + (((4 + quad) ^ ((col >> 1) & 7)) << 3);
  const int w_lane = (wn * 4 * 2 * 64 + lane) << 3;            // unit (channel block 4 wn + j, k step ks) = 2 (4 wn + j) + ks

  auto mainloop = [&](auto swap_tag) __attribute__((always_inline)) {
    constexpr bool SWAP = decltype(swap_tag)::value;
    issue(0, 0);
    for (int s = 0; s < nst; ++s) {
      const int buf = s & 1;
      __builtin_amdgcn_s_waitcnt(0x0f70);                           // vmcnt(0): this wave's loads of stage s landed
      __builtin_amdgcn_s_barrier();                                 // ... so have everybody's, and stage s-1 is left
      asm volatile("" ::: "memory");                                // (no LDS read may move above the barrier)
      __builtin_amdgcn_s_setprio(1);
      if (s + 1 < nst) issue(buf ^ 1, s + 1);
      const uint16_t* as = smem + buf * 32768;
      const uint16_t* bs = as + 16384;
      bf16x8 w0[4], w1[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) w0[j] = *reinterpret_cast<const bf16x8*>(bs + w_lane + j * 1024);
      bf16x8 af[3];
      af[0] = *reinterpret_cast<const bf16x8*>(as + a_lane0);
      af[1] = *reinterpret_cast<const bf16x8*>(as + a_lane0 + 16 * BK);
#pragma unroll
      for (int x = 0; x < 2 * MI; ++x) {
        const int ks = x / MI, i = x % MI;
        if (x + 2 < 2 * MI) {
          const int ks2 = (x + 2) / MI, i2 = (x + 2) % MI;
          af[(x + 2) % 3] = *reinterpret_cast<const bf16x8*>(as + (ks2 ? a_lane1 : a_lane0) + i2 * 16 * BK);
        }
        if (x < 4) w1[x] = *reinterpret_cast<const bf16x8*>(bs + w_lane + x * 1024 + 512);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const bf16x8 w = ks == 0 ? w0[j] : w1[j];
          acc[i][j] = SWAP ? mfma16(w, af[x % 3], acc[i][j]) : mfma16(af[x % 3], w, acc[i][j]);
        }
      }
      __builtin_amdgcn_sched_group_barrier(0x100, 6, 0);
#pragma unroll
      for (int x = 0; x < 4; ++x) {
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
      }
#pragma unroll
      for (int x = 4; x < 2 * MI - 2; ++x) {
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);
      __builtin_amdgcn_s_setprio(0);
    }
  };
  if (swap) mainloop(std::true_type{});
  else mainloop(std::false_type{});
  ep.template store<MI>(swap, r0, c0, acc, M, N, col, quad);
}

// ---------------------------------------------------------------------------
// Skinny kernel: M <= 16*MT rows (the generation phase).  One workgroup owns NB blocks of 16 output channels; its
// eight waves interleave the 32-wide K steps and each requests all the weight fragments of a round at once (for
// K <= 4096 and M <= 16 that is the whole job: one memory round trip; nontemporal, the weights are streamed exactly
// once); the partial sums meet in LDS.  Every load goes through a buffer descriptor (the workgroup's channel blocks
// of W; the M rows of A), so rows past M, channel blocks past N and k steps past K read as zero and no load sits
// behind a branch: all of a wave's requests are out within a few dozen cycles of its start.  What the epilogue has
// to look up per row (the cache slot of the appended token) is fetched by M threads AFTER the loads are issued.
// A float A operand is split in hi + lo bf16 halves so it loses no precision.
// ---------------------------------------------------------------------------
constexpr int kSkinnyWaves = 8;

template <typename Epilogue, bool A_F32, int MT, int NB>
__global__ __launch_bounds__(512) void gemm_bf16_skinny_kernel(const void* __restrict__ A,
                                                               const uint16_t* __restrict__ Wt, int32_t M, int32_t N,
                                                               int32_t K, Epilogue ep) {
  constexpr int WAVES = kSkinnyWaves;
  constexpr int UN = 16 / MT;                              // k steps per wave and round, all requested up front
  constexpr int kEsz = A_F32 ? 4 : 2;
  constexpr uint32_t kOob = 0x7ffffff0u;                   // beyond any descriptor's size: reads as zero
  constexpr int kNt = 2;                                   // cache policy of the weight loads: nontemporal
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int col = lane & 15, quad = lane >> 4;
  const int n0 = blockIdx.x * (16 * NB);
  const int steps = K / 32;
  const int nblks = (N + 15) >> 4;
  // this workgroup's channel blocks: [NB][steps] fragments of 1 KiB, contiguous in the packed weights
  const int my_blks = min(NB, nblks - (n0 >> 4));
  const __amdgpu_buffer_rsrc_t w_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint16_t*>(Wt) + (((int64_t)(n0 >> 4) * steps) << 9), 0, (int)((int64_t)my_blks * steps * 1024),
      0x00020000);
  const __amdgpu_buffer_rsrc_t a_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<char*>(reinterpret_cast<const char*>(A)), 0, (int)((int64_t)M * K * kEsz), 0x00020000);

  f32x4 acc[MT][NB];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) acc[i][nb] = f32x4{0.f, 0.f, 0.f, 0.f};

  __shared__ typename Epilogue::Row rows[64];
  __shared__ f32x4 red[WAVES][MT][NB][64];
  // The epilogue's per-row lookup is a chain of two dependent loads (sequence length, then page id).  Loads return in
  // order, so the first is issued before the weight requests (waiting for it then waits for nothing younger) and the
  // second right behind them; its value is needed only after the matrix products.
  // (Every thread goes through the lookup, the ones past M for row 0: a branch around a load would make the
  // compiler wait for it on the spot.)
  typename Epilogue::RowLookup look = ep.lookup_begin(tid < M ? tid : 0);
  bool looked = false;
  if (blockIdx.x == 0) ep.clear(tid, 512);

  // the waves interleave the k steps (neighbouring waves stream neighbouring kilobytes of the weights)
  for (int s0 = wave; s0 < steps; s0 += WAVES * UN) {     // this wave: steps s0, s0 + WAVES, ...
    bf16x8 bw[UN][NB];
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const int s = s0 + WAVES * u;
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        const uint32_t off = s < steps ? (uint32_t)(((nb * steps + s) << 10) + (lane << 4)) : kOob;
        bw[u][nb] = __builtin_bit_cast(bf16x8, __builtin_amdgcn_raw_buffer_load_b128(w_rsrc, off, 0, kNt));
      }
    }
    // activations: a few rows, shared by every workgroup (L2 hits); float input is kept whole until it is split
    bf16x8 ab[A_F32 ? 1 : UN][MT];
    f32x4 af32[A_F32 ? UN : 1][MT][2];
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const int s = s0 + WAVES * u;
#pragma unroll
      for (int i = 0; i < MT; ++i) {
        const int row = i * 16 + col;                      // rows >= M lie beyond the descriptor
        const uint32_t off = s < steps ? (uint32_t)((row * K + s * 32 + quad * 8) * kEsz) : kOob;
        if (!A_F32) {
          ab[u][i] = __builtin_bit_cast(bf16x8, __builtin_amdgcn_raw_buffer_load_b128(a_rsrc, off, 0, 0));
        } else {
          af32[u][i][0] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(a_rsrc, off, 0, 0));
          af32[u][i][1] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(a_rsrc, off, 16, 0));
        }
      }
    }
    __builtin_amdgcn_sched_barrier(0);                     // every request of the round goes out before anything else
    if (!looked) {                                         // (first round only)
      ep.lookup_next(look);
      looked = true;
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < UN; ++u) {
#pragma unroll
      for (int i = 0; i < MT; ++i) {
        if (!A_F32) {
#pragma unroll
          for (int nb = 0; nb < NB; ++nb) acc[i][nb] = mfma16(ab[u][i], bw[u][nb], acc[i][nb]);
        } else {
          bf16x8 hi, lo;
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            const float f = af32[u][i][j >> 2][j & 3];
            const __bf16 h = (__bf16)f;
            hi[j] = h;
            lo[j] = (__bf16)(f - (float)h);
          }
#pragma unroll
          for (int nb = 0; nb < NB; ++nb) {
            acc[i][nb] = mfma16(hi, bw[u][nb], acc[i][nb]);
            acc[i][nb] = mfma16(lo, bw[u][nb], acc[i][nb]);
          }
        }
      }
    }
  }
  if (!looked) ep.lookup_next(look);                     // (a wave without a k step: K < 256)
  if (tid < M) rows[tid] = ep.lookup_end(look, blockIdx.x == 0);
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) red[wave][i][nb][lane] = acc[i][nb];
  __syncthreads();
  static_assert(MT * NB * 64 <= 64 * WAVES, "one output quad per thread");
  if (tid < MT * NB * 64) {
    const int nb = (tid >> 6) % NB, i = (tid >> 6) / NB;
    f32x4 v = red[0][i][nb][lane];
#pragma unroll
    for (int w = 1; w < WAVES; ++w) v += red[w][i][nb][lane];
    const int c = n0 + nb * 16 + col;
    if (c < N) {
      const typename Epilogue::Col cl = ep.column(c);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int r = i * 16 + quad * 4 + e;
        if (r < M) ep.put(cl, rows[r], r, v[e]);
      }
    }
  }
}

// ---------------------------------------------------------------------------
// Skinny kernel, pipelined form: M <= 16 rows of bf16 activations, K <= 4096 -- the fused QKV projection of a
// generation step.  One workgroup per compute unit walks the 16-channel blocks blk = blockIdx.x, + gridDim.x, ...:
// the weights of the block after the current one are requested before the current block's matrix products, so a
// compute unit always has one or two blocks (K * 32 bytes each) in flight, however many blocks there are per
// workgroup; the activations (this wave's 16 k steps of all rows) are fetched once and stay in registers.  Results
// are collected in LDS and stored after the last block: with no store between the loads, waiting for one block's
// weights never has to wait for the next block's.
// ---------------------------------------------------------------------------
constexpr int kPipeMaxUnits = 16;       // channel blocks per workgroup (the launch grows the grid beyond one per CU if needed)

template <typename Epilogue>
__global__ __launch_bounds__(512) void gemm_bf16_skinny_pipe_kernel(const uint16_t* __restrict__ A,
                                                                    const uint16_t* __restrict__ Wt, int32_t M,
                                                                    int32_t N, int32_t K, Epilogue ep) {
  constexpr int WAVES = kSkinnyWaves, UN = 16;
  constexpr uint32_t kOob = 0x7ffffff0u;
  constexpr int kNt = 2;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int col = lane & 15, quad = lane >> 4;
  const int steps = K / 32;                                  // <= WAVES * UN
  const int nblks = (N + 15) >> 4;
  const int stride = gridDim.x;

  __shared__ typename Epilogue::Row rows[16];
  __shared__ f32x4 red[2][WAVES][64];
  __shared__ f32x4 stage[kPipeMaxUnits][64];

  typename Epilogue::RowLookup look = ep.lookup_begin(tid < M ? tid : 0);
  if (blockIdx.x == 0) ep.clear(tid, 512);
  // this lane's part of the weight / activation fragment of its wave's u-th k step, or beyond every descriptor
  uint32_t w_off[UN], a_off[UN];
#pragma unroll
  for (int u = 0; u < UN; ++u) {
    const int s = wave + WAVES * u;
    w_off[u] = s < steps ? (uint32_t)((s << 10) + (lane << 4)) : kOob;
    a_off[u] = s < steps ? (uint32_t)((col * K + s * 32 + quad * 8) * 2) : kOob;      // rows >= M: beyond the descriptor
  }
  auto load_w = [&](int blk, bf16x8 (&bw)[UN]) __attribute__((always_inline)) {
    // a block past the last reads through an empty descriptor: zeros, no memory traffic, no branch around the loads
    const bool real = blk < nblks;
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t*>(Wt) + (((int64_t)(real ? blk : 0) * steps) << 9), 0, real ? steps * 1024 : 0, 0x00020000);
#pragma unroll
    for (int u = 0; u < UN; ++u)
      bw[u] = __builtin_bit_cast(bf16x8, __builtin_amdgcn_raw_buffer_load_b128(rsrc, w_off[u], 0, kNt));
  };
  bf16x8 w0[UN], w1[UN], af[UN];
  int blk = blockIdx.x;
  load_w(blk, w0);
  {
    const __amdgpu_buffer_rsrc_t a_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t*>(A), 0, (int)((int64_t)M * K * 2), 0x00020000);
#pragma unroll
    for (int u = 0; u < UN; ++u)
      af[u] = __builtin_bit_cast(bf16x8, __builtin_amdgcn_raw_buffer_load_b128(a_rsrc, a_off[u], 0, 0));
  }
  __builtin_amdgcn_sched_barrier(0);
  ep.lookup_next(look);
  __builtin_amdgcn_sched_barrier(0);

  int it = 0;
  auto unit = [&](bf16x8 (&wc)[UN], bf16x8 (&wn)[UN]) __attribute__((always_inline)) {
    load_w(blk + stride, wn);
    __builtin_amdgcn_sched_barrier(0);
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int u = 0; u < UN; ++u) acc = mfma16(af[u], wc[u], acc);
    red[it & 1][wave][lane] = acc;
    __syncthreads();
    if (wave == (it & 7)) {                                  // the waves take turns at summing up a block
      f32x4 v = red[it & 1][0][lane];
#pragma unroll
      for (int w = 1; w < WAVES; ++w) v += red[it & 1][w][lane];
      stage[it][lane] = v;
    }
    ++it;
    blk += stride;
  };
  while (true) {
    unit(w0, w1);
    if (blk >= nblks) break;
    unit(w1, w0);
    if (blk >= nblks) break;
  }
  if (tid < M) rows[tid] = ep.lookup_end(look, blockIdx.x == 0);
  __syncthreads();
  // stores: wave w writes the blocks it summed up (lane = column, 4 rows per lane)
  for (int j = wave; j < it; j += WAVES) {
    const f32x4 v = stage[j][lane];
    const int c = (blockIdx.x + j * stride) * 16 + col;
    if (c < N) {
      const typename Epilogue::Col cl = ep.column(c);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int r = quad * 4 + e;
        if (r < M) ep.put(cl, rows[r], r, v[e]);
      }
    }
  }
}

__device__ __forceinline__ u32x2 pack4_bf16(f32x4 v) {
  u32x2 w;
  w[0] = (uint32_t)f32_to_bf16_rne(v[0]) | ((uint32_t)f32_to_bf16_rne(v[1]) << 16);
  w[1] = (uint32_t)f32_to_bf16_rne(v[2]) | ((uint32_t)f32_to_bf16_rne(v[3]) << 16);
  return w;
}

// Element (row, column) of accumulator register e of block (i, j) of a wave tile at (r0, c0).
//   not swapped: lane = column, registers = 4 rows;   swapped: lane = row, registers = 4 columns.
__device__ __forceinline__ void acc_coord(bool swap, int r0, int c0, int i, int j, int e, int col, int quad, int& r,
                                          int& c) {
  r = swap ? r0 + i * 16 + col : r0 + i * 16 + quad * 4 + e;
  c = swap ? c0 + j * 16 + quad * 4 + e : c0 + j * 16 + col;
}

// Fused QKV destination.  When every section (q | k | v) is a multiple of 64 columns and the ranks are
// multiples of 16, a wave tile lies in one section and 16-row blocks that start on a 16-token boundary
// of the cache are stored as whole fragments of the cache layout:
//   q, k (swapped): a lane holds 4 consecutive channels of one token -> one 8-byte store;
//   v (not swapped): a lane holds one channel of 4 consecutive tokens = 4 consecutive slots of the V layout.
// Everything else falls back to element-wise stores.
struct QkvEpBf16 {
  QkvDest d;
  int32_t fast_cols;
  // generation-phase kernel: a row's cache slot is looked up once (and a dropped append reported once), a
  // column's section once, then elements are stored
  typedef QkvRow Row;
  typedef QkvCol Col;
  struct RowLookup {
    int32_t b, t, len, page, tp;
    bool ok;
  };
  __device__ __forceinline__ RowLookup lookup_begin(int r) const {
    RowLookup l;
    l.b = r / d.T;
    l.t = r % d.T;
    l.len = d.seq_len[l.b];
    l.page = -1;
    l.tp = 0;
    l.ok = false;
    return l;
  }
  __device__ __forceinline__ void lookup_next(RowLookup& l) const {
    int32_t len = l.len;
    asm volatile("" : "+v"(len));            // the loaded length is first looked at HERE (not where it was requested)
    const int64_t p64 = (int64_t)len + l.t;
    l.ok = p64 >= 0 && p64 <= (int64_t)INT32_MAX;
    const uint32_t pos = l.ok ? (uint32_t)p64 : 0u, P = (uint32_t)d.g.page_tokens;
    const uint32_t lp = pos / P;
    l.tp = (int32_t)(pos - lp * P);
    l.ok = l.ok && lp < (uint32_t)d.g.max_pages;
    l.page = d.page_table[(int64_t)l.b * d.g.max_pages + (l.ok ? lp : 0u)];     // (no branch around the load)
  }
  __device__ __forceinline__ Row lookup_end(const RowLookup& l, bool report) const {
    Row rw{-1, 0};
    if (l.ok && l.page >= 0 && l.page < d.g.pool_pages) {
      rw.page = l.page;
      rw.tp = l.tp;
    } else if (report) {
      qkv_report_drop(d);
    }
    return rw;
  }
  __device__ __forceinline__ Col column(int c) const { return qkv_col(d, c); }
  __device__ __forceinline__ void clear(int tid, int nthreads) const {
    for (int i = tid; i < d.clear_words; i += nthreads) d.clear[i] = 0u;
  }
  __device__ __forceinline__ void put(const Col& cl, const Row& rw, int r, float v) const { qkv_put<true>(d, cl, rw, r, v); }
  __device__ __forceinline__ bool swap_for(int c0) const {
    const Geo& g = d.g;
    return fast_cols && c0 < g.n_heads * g.q_dim + g.n_kv_heads * g.r_k;
  }
  // I is a compile-time index: the accumulators must stay in registers (no dynamic indexing).
  template <int I, int MI>
  __device__ __forceinline__ void store_slow(bool swap, int r0, int c0, const f32x4 (&acc)[MI][4], int M, int N,
                                             int col, int quad) const {
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        int r, c;
        acc_coord(swap, r0, c0, I, j, e, col, quad, r, c);
        if (r < M && c < N) qkv_store<true>(d, r, c, acc[I][j][e]);
      }
  }
  template <int I, int MI>
  __device__ __forceinline__ void store_block(bool swap, bool is_k, int sec0, int r, int r0, int c0,
                                              const f32x4 (&acc)[MI][4], int M, int N, int col, int quad) const {
    const Geo& g = d.g;
    const int row0 = r0 + I * 16;                  // wave-uniform
    bool fast = row0 + 16 <= M && d.T % 16 == 0;
    int page = -1, tp0 = 0;
    if (fast) {
      const int b = row0 / d.T;
      const int64_t pos0 = (int64_t)d.seq_len[b] + row0 % d.T;
      const int64_t lp = pos0 / g.page_tokens;
      fast = pos0 >= 0 && (pos0 & 15) == 0 && lp < g.max_pages;
      if (fast) {
        page = d.page_table[(int64_t)b * g.max_pages + lp];
        tp0 = (int)(pos0 % g.page_tokens);
        fast = page >= 0 && page < g.pool_pages;
      }
    }
    if (!fast) {
      store_slow<I, MI>(swap, r0, c0, acc, M, N, col, quad);
      return;
    }
    const int tile = tp0 >> 6, tb = (tp0 & 63) >> 4;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int cc0 = sec0 + j * 16;               // first channel of this 16-column block, wave-uniform
      const int kvh = cc0 / r, ch0 = cc0 % r;      // ch0 is a multiple of 16
      if (is_k) {
        const int ch = ch0 + quad * 4;             // this lane: channels ch .. ch+3 of token tp0 + col
        uint16_t* dst = reinterpret_cast<uint16_t*>(d.k_pool) + (int64_t)page * g.k_page + (int64_t)kvh * g.k_slab +
                        (int64_t)tile * (kTile * g.r_k_pad) +
                        ((((tb * (g.r_k_pad >> 3) + (ch >> 3)) * 16 + col) << 3) + (ch & 7));
        *reinterpret_cast<u32x2*>(dst) = pack4_bf16(acc[I][j]);
      } else {
        const int grp = tb >> 1, half = tb & 1;    // this lane: channel ch0 + col, tokens tp0 + 4*quad .. +3
        uint16_t* dst = reinterpret_cast<uint16_t*>(d.v_pool) + (int64_t)page * g.v_page + (int64_t)kvh * g.v_slab +
                        (int64_t)tile * (kTile * g.r_v_pad) +
                        ((((((grp * (g.r_v_pad >> 4) + (ch0 >> 4)) * 4 + quad) * 16 + col) << 3) + half * 4));
        *reinterpret_cast<u32x2*>(dst) = pack4_bf16(acc[I][j]);
      }
    }
  }
  template <int MI, int... Is>
  __device__ __forceinline__ void store_slow_all(std::integer_sequence<int, Is...>, bool swap, int r0, int c0,
                                                 const f32x4 (&acc)[MI][4], int M, int N, int col, int quad) const {
    (store_slow<Is, MI>(swap, r0, c0, acc, M, N, col, quad), ...);
  }
  template <int MI, int... Is>
  __device__ __forceinline__ void store_block_all(std::integer_sequence<int, Is...>, bool swap, bool is_k, int sec0,
                                                  int r, int r0, int c0, const f32x4 (&acc)[MI][4], int M, int N,
                                                  int col, int quad) const {
    (store_block<Is, MI>(swap, is_k, sec0, r, r0, c0, acc, M, N, col, quad), ...);
  }
  template <int MI>
  __device__ __forceinline__ void store(bool swap, int r0, int c0, const f32x4 (&acc)[MI][4], int M, int N, int col,
                                        int quad) const {
    const Geo& g = d.g;
    const int nq = g.n_heads * g.q_dim, nk = g.n_kv_heads * g.r_k;
    if (!fast_cols || c0 + 64 > N) {
      store_slow_all<MI>(std::make_integer_sequence<int, MI>{}, swap, r0, c0, acc, M, N, col, quad);
      return;
    }
    if (c0 < nq) {                                   // ---- q section: dense [M, nq]
#pragma unroll
      for (int i = 0; i < MI; ++i) {
        const int r = r0 + i * 16 + col;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int64_t idx = (int64_t)r * nq + c0 + j * 16 + quad * 4;
          if (r < M) {
            if (d.q_is_f32) *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(d.q) + idx) = acc[i][j];
            else *reinterpret_cast<u32x2*>(reinterpret_cast<uint16_t*>(d.q) + idx) = pack4_bf16(acc[i][j]);
          }
        }
      }
      return;
    }
    const bool is_k = c0 < nq + nk;
    const int sec0 = is_k ? c0 - nq : c0 - nq - nk;  // first column of the wave tile inside its section
    const int r = is_k ? g.r_k : g.r_v;
    store_block_all<MI>(std::make_integer_sequence<int, MI>{}, swap, is_k, sec0, r, r0, c0, acc, M, N, col, quad);
  }
};

struct PlainEpBf16 {
  uint16_t* y;
  int32_t N;
  struct Row {};
  struct RowLookup {};
  typedef int Col;
  __device__ __forceinline__ RowLookup lookup_begin(int) const { return RowLookup{}; }
  __device__ __forceinline__ void lookup_next(RowLookup&) const {}
  __device__ __forceinline__ Row lookup_end(const RowLookup&, bool) const { return Row{}; }
  __device__ __forceinline__ Col column(int c) const { return c; }
  __device__ __forceinline__ void clear(int, int) const {}
  __device__ __forceinline__ void put(const Col& c, const Row&, int r, float v) const { y[(int64_t)r * N + c] = f32_to_bf16_rne(v); }
  __device__ __forceinline__ bool swap_for(int) const { return true; }
  template <int MI>
  __device__ __forceinline__ void store(bool, int r0, int c0, const f32x4 (&acc)[MI][4], int M, int Ncols, int col,
                                        int quad) const {
#pragma unroll
    for (int i = 0; i < MI; ++i) {
      const int r = r0 + i * 16 + col;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int c = c0 + j * 16 + quad * 4;
        uint16_t* dst = y + (int64_t)r * Ncols + c;
        if (r >= M) {
        } else if (c + 3 < Ncols && (Ncols & 3) == 0) {
          *reinterpret_cast<u32x2*>(dst) = pack4_bf16(acc[i][j]);
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (c + e < Ncols) dst[e] = f32_to_bf16_rne(acc[i][j][e]);
        }
      }
    }
  }
};

// Compute units of the current device (asked once per process; 256 on MI355X, which is also the fallback).
static int compute_units() {
  static int n = 0;
  if (n == 0) {
    int dev = 0, cu = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&cu, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cu > 0)
      n = cu;
    else
      n = 256;
    (void)hipGetLastError();
  }
  return n;
}

template <typename Epilogue, bool A_F32>
static int launch_gemm(const void* A, const void* Wt, int32_t M, int32_t N, int32_t K, const Epilogue& ep,
                       hipStream_t st) {
  const uint16_t* w = (const uint16_t*)Wt;
  if constexpr (!A_F32) {
    if (M <= 16 && K <= 32 * kSkinnyWaves * 16) {
      // one workgroup per compute unit (more only when a workgroup would otherwise get more blocks than it can stage)
      const int nblks = (N + 15) / 16;
      int grid = nblks < compute_units() ? nblks : compute_units();
      if ((nblks + grid - 1) / grid > kPipeMaxUnits) grid = (nblks + kPipeMaxUnits - 1) / kPipeMaxUnits;
      gemm_bf16_skinny_pipe_kernel<Epilogue><<<dim3(grid), dim3(512), 0, st>>>((const uint16_t*)A, w, M, N, K, ep);
      return launch_status();
    }
  }
  if (M <= 64) {
    // two channel blocks per workgroup when that still leaves about one workgroup per compute unit
    const int nb = (!A_F32 && N / 32 >= 200) ? 2 : 1;     // (float activations need the registers themselves)
    dim3 grid((N + 16 * nb - 1) / (16 * nb)), block(512);
    const int mt = (M + 15) / 16;
#define EA_SKINNY(MT_, NB_) gemm_bf16_skinny_kernel<Epilogue, A_F32, MT_, NB_><<<grid, block, 0, st>>>(A, w, M, N, K, ep)
    if (nb == 2) {
      if constexpr (!A_F32) {                 // (never instantiated for float activations: it would spill)
        switch (mt) {
          case 1: EA_SKINNY(1, 2); break;
          case 2: EA_SKINNY(2, 2); break;
          case 3: EA_SKINNY(3, 2); break;
          default: EA_SKINNY(4, 2); break;
        }
      }
    } else {
      switch (mt) {
        case 1: EA_SKINNY(1, 1); break;
        case 2: EA_SKINNY(2, 1); break;
        case 3: EA_SKINNY(3, 1); break;
        default: EA_SKINNY(4, 1); break;
      }
    }
#undef EA_SKINNY
  } else {
    // taller tiles re-read the weights half as often, but only pay once there are enough of them for the chip:
    // below about 3/4 of the compute units' worth of 256x256 tiles the 128-row kernel's finer grid is faster
    const int64_t tiles256 = (int64_t)((N + 255) / 256) * ((M + 255) / 256);
    const int bm = (M >= 2048 && tiles256 >= 192) ? 256 : 128;
    const int64_t tiles = (int64_t)((N + 127) / 128) * ((M + bm - 1) / bm);
    if (tiles > INT32_MAX) return EA_ERR_SHAPE;
    dim3 grid((uint32_t)tiles), block(256);
    if constexpr (!A_F32) {
      if (bm == 256 && N > 128) {
        // bf16 activations, many rows (and more than one 128-wide column tile): the asynchronous 256x256 kernel (128 KiB of dynamic LDS, one workgroup per CU)
        const int64_t t2 = tiles256;
        if (t2 > INT32_MAX) return EA_ERR_SHAPE;
        static bool attr_set = false;      // (a benign race: the attribute is idempotent)
        if (!attr_set) {
          if (hipFuncSetAttribute((const void*)gemm_bf16_async_kernel<Epilogue>,
                                  hipFuncAttributeMaxDynamicSharedMemorySize, kAsyncLds) != hipSuccess)
            return EA_ERR_DEVICE;
          attr_set = true;
        }
        gemm_bf16_async_kernel<Epilogue><<<dim3((uint32_t)t2), dim3(512), kAsyncLds, st>>>((const uint16_t*)A, w, M, N, K, ep);
        return launch_status();
      }
    }
    if (bm == 256) {
      gemm_bf16_tiled_kernel<Epilogue, A_F32, 8><<<grid, block, 0, st>>>(A, w, M, N, K, ep);
    } else {
      // a few hundred rows: 128-row tiles would leave most compute units idle (32 tiles at M = 128, N = 4096), so
      // the tile height is halved until there are about as many tiles as compute units
      const int64_t tiles_n = (N + 127) / 128;
      int rows = 128;
      while (rows > 32 && tiles_n * ((M + rows - 1) / rows) < 200) rows >>= 1;
      const dim3 g2((uint32_t)(tiles_n * ((M + rows - 1) / rows)));
      if (rows == 128) gemm_bf16_tiled_kernel<Epilogue, A_F32, 4><<<g2, block, 0, st>>>(A, w, M, N, K, ep);
      else if (rows == 64) gemm_bf16_tiled_kernel<Epilogue, A_F32, 2><<<g2, block, 0, st>>>(A, w, M, N, K, ep);
      else gemm_bf16_tiled_kernel<Epilogue, A_F32, 1><<<g2, block, 0, st>>>(A, w, M, N, K, ep);
    }
  }
  return launch_status();
}

int gemm_qkv_bf16(const void* x, const void* w_t, int32_t M, int32_t N, int32_t K, const QkvDest& dst,
                  hipStream_t st) {
  const Geo& g = dst.g;
  const int nq = g.n_heads * g.q_dim, nk = g.n_kv_heads * g.r_k, nv = g.n_kv_heads * g.r_v;
  const int32_t fast_cols = nq % 64 == 0 && nk % 64 == 0 && nv % 64 == 0 && g.r_k % 16 == 0 && g.r_v % 16 == 0;
  return launch_gemm<QkvEpBf16, false>(x, w_t, M, N, K, QkvEpBf16{dst, fast_cols}, st);
}

int gemm_out_bf16(const void* a, int32_t a_is_f32, const void* w_t, void* y, int32_t M, int32_t N, int32_t K,
                  hipStream_t st) {
  PlainEpBf16 ep{(uint16_t*)y, N};
  if (a_is_f32) return launch_gemm<PlainEpBf16, true>(a, w_t, M, N, K, ep, st);
  return launch_gemm<PlainEpBf16, false>(a, w_t, M, N, K, ep, st);
}

}  // namespace ea
