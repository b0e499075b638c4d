// The back half of a generation step in ONE launch: attention over the rank-r cache (Eq. 3 with the operands of
// Eq. 7), the merge of the split partials and the output projection y = [o_1 .. o_H] W^O' (Eq. 8's folded W^O').
//
// The attention part is the generation-phase kernel body as it stands; its results leave the workgroup through
// stores that write through to memory.  What follows needs values from other workgroups, so it is ordered by two
// kinds of counters in the caller's workspace (cleared by the projection launch of the same call):
//   * one ticket per (sequence, kv head), taken by each of its splits when its partials are out: the workgroup
//     that takes the last one merges the partials of that (sequence, kv head) into the output row o;
//   * one arrival count for the whole grid, raised by every workgroup when it has nothing more to write to o.
// Only the LAST n_work workgroups of the grid (in dispatch order) go on to the projection: each requests the
// weights of its first block of 16 output channels, THEN waits for the arrival count to reach the grid size, and
// multiplies.  No other workgroup ever waits, workgroups are dispatched in order (to the chip's dies in turn, in
// order on each die), and the waiting ones fill at most half of the resident slots of the chip and of every die,
// so every workgroup they wait for can run: the wait ends.  It is bounded all the same (spin_limit polls); a
// workgroup whose wait runs out sets bit 30 of the status word, writes no y and leaves.
// Values that cross workgroups are read with loads that bypass the caches of the reading compute unit and its L2.
#pragma once
#include "ea_decode_kernel.h"
#include "ea_epilogue.h"

namespace ea {

constexpr int kCoherent = 17;              // cache policy sc0 sc1: write through to / read from memory
constexpr int kTailRound = 24;             // k steps of 32 per wave and round of the projection (3072 channels)
constexpr uint32_t kOobTail = 0x7ffffff0u; // an offset beyond every buffer descriptor: reads as zero

__device__ __forceinline__ __amdgpu_buffer_rsrc_t tail_rsrc(const void* p, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}
__device__ __forceinline__ float coherent_load_f32(__amdgpu_buffer_rsrc_t r, uint32_t byte_off) {
  return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, byte_off, 0, kCoherent));
}
__device__ __forceinline__ void coherent_store_f32(__amdgpu_buffer_rsrc_t r, uint32_t byte_off, float v) {
  __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, v), r, byte_off, 0, kCoherent);
}
__device__ __forceinline__ void coherent_store_bf16(__amdgpu_buffer_rsrc_t r, uint32_t byte_off, float v) {
  __builtin_amdgcn_raw_buffer_store_b16((short)f32_to_bf16_rne(v), r, byte_off, 0, kCoherent);
}

// The attention body's results: o (bf16) when the sequence is not split, else the split partials, written through.
struct TailEmit {
  __amdgpu_buffer_rsrc_t o_rsrc, ws_rsrc;
  __device__ __forceinline__ void operator()(const DecodeArgs& a, int b, int n_batch, int split, int head, int c,
                                             int r_v_pad, float mm, float lsum, float val) const {
    const Geo& g = a.g;
    if (a.n_splits == 1) {
      if (c < g.r_v)
        coherent_store_bf16(o_rsrc, (uint32_t)(((b * g.n_heads + head) * g.r_v + c) * 2), lsum > 0.f ? val / lsum : 0.f);
    } else {
      const uint32_t BHS = (uint32_t)(n_batch * g.n_heads * a.n_splits);
      const uint32_t row = (uint32_t)((b * g.n_heads + head) * a.n_splits + split);
      if (c == 0) {
        coherent_store_f32(ws_rsrc, row * 4u, mm);
        coherent_store_f32(ws_rsrc, (BHS + row) * 4u, lsum);
      }
      coherent_store_f32(ws_rsrc, (2u * BHS + row * (uint32_t)r_v_pad + (uint32_t)c) * 4u, val);
    }
  }
};

template <int KS, int NCB, int TBN, int NKK, bool ALIBI = false>
__global__ __launch_bounds__(256, 2) void decode_layer_back_kernel(DecodeArgs a, TailArgs t) {
  __shared__ DecodeSmem<KS, NCB, TBN, NKK> sm;
  __shared__ f32x4 red[4][64];
  __shared__ float mg_m[16 * kTailMaxSplits], mg_l[16 * kTailMaxSplits];   // [head of the group][split]
  __shared__ int flag;
  const Geo& g = a.g;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int col = lane & 15, quad = lane >> 4;
  const int kvh = blockIdx.x, split = blockIdx.y, b = blockIdx.z, n_batch = gridDim.z;
  const __amdgpu_buffer_rsrc_t o_rsrc = tail_rsrc(t.o, (uint32_t)(n_batch * t.K * 2));
  const __amdgpu_buffer_rsrc_t ws_rsrc = tail_rsrc(a.ws, a.n_splits > 1 ? t.ws_bytes : 0u);

  // ---- attention of this (kv head, split, sequence)
  decode_bf16_body<KS, NCB, TBN, 2, NKK, ALIBI, false, false, TailEmit>(a, kvh, split, b, n_batch, sm,
                                                                        TailEmit{o_rsrc, ws_rsrc});
  // every store of the workgroup has been acknowledged before the workgroup is counted anywhere
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();

  // ---- split partials: the last split of a (sequence, kv head) to get here merges them
  if (a.n_splits > 1) {
    if (tid == 0) {
      const uint32_t before = __hip_atomic_fetch_add(t.sync + 1 + b * g.n_kv_heads + kvh, 1u, __ATOMIC_RELAXED,
                                                     __HIP_MEMORY_SCOPE_AGENT);
      flag = before == (uint32_t)a.n_splits - 1u;
    }
    __syncthreads();
    if (flag) {
      const int G = g.group, S = a.n_splits, r_v_pad = NCB * 16;
      const uint32_t BHS = (uint32_t)(n_batch * g.n_heads * S);
      const uint32_t row00 = (uint32_t)((b * g.n_heads + kvh * G) * S);       // rows of the group's heads follow each other
      if (S <= 8) {
        // one round trip to memory: a thread requests its channel of every split together with the splits'
        // exponents and row sums (offsets past the last split lie beyond the descriptor and read as zero)
        for (int idx = tid; idx < G * r_v_pad; idx += 256) {
          const int hd = idx / r_v_pad, c = idx % r_v_pad;
          const uint32_t row0 = row00 + (uint32_t)(hd * S);
          float pm[8], pl[8], v[8];
#pragma unroll
          for (int u = 0; u < 8; ++u) {
            pm[u] = coherent_load_f32(ws_rsrc, u < S ? (row0 + u) * 4u : kOobTail);
            pl[u] = coherent_load_f32(ws_rsrc, u < S ? (BHS + row0 + u) * 4u : kOobTail);
            v[u] = coherent_load_f32(ws_rsrc,
                                     u < S ? (2u * BHS + (row0 + u) * (uint32_t)r_v_pad + (uint32_t)c) * 4u : kOobTail);
          }
          float mm = -INFINITY;
#pragma unroll
          for (int u = 0; u < 8; ++u)
            if (u < S) mm = fmaxf(mm, pm[u]);
          float lsum = 0.f, val = 0.f;
#pragma unroll
          for (int u = 0; u < 8; ++u) {
            if (u < S && mm != -INFINITY) {
              const float wt = __builtin_amdgcn_exp2f(pm[u] - mm);
              lsum += wt * pl[u];
              val += wt * v[u];
            }
          }
          if (c < g.r_v)
            coherent_store_bf16(o_rsrc, (uint32_t)(((b * g.n_heads + kvh * G + hd) * g.r_v + c) * 2),
                                lsum > 0.f ? val / lsum : 0.f);
        }
      } else {
        // two round trips: every (head, split)'s exponent and row sum into LDS, then each thread's channel of
        // eight splits at a time
        for (int i = tid; i < G * S; i += 256) {
          mg_m[i] = coherent_load_f32(ws_rsrc, (row00 + i) * 4u);
          mg_l[i] = coherent_load_f32(ws_rsrc, (BHS + row00 + i) * 4u);
        }
        __syncthreads();
        for (int idx = tid; idx < G * r_v_pad; idx += 256) {
          const int hd = idx / r_v_pad, c = idx % r_v_pad;
          const float* pm = mg_m + hd * S;
          const float* pl = mg_l + hd * S;
          float mm = -INFINITY;
          for (int s = 0; s < S; ++s) mm = fmaxf(mm, pm[s]);
          float lsum = 0.f, val = 0.f;
          for (int s0 = 0; s0 < S; s0 += 8) {
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u)
              v[u] = coherent_load_f32(
                  ws_rsrc,
                  s0 + u < S ? (2u * BHS + (row00 + hd * S + s0 + u) * (uint32_t)r_v_pad + (uint32_t)c) * 4u : kOobTail);
#pragma unroll
            for (int u = 0; u < 8; ++u) {
              if (s0 + u < S && mm != -INFINITY) {
                const float wt = __builtin_amdgcn_exp2f(pm[s0 + u] - mm);
                lsum += wt * pl[s0 + u];
                val += wt * v[u];
              }
            }
          }
          if (c < g.r_v)
            coherent_store_bf16(o_rsrc, (uint32_t)(((b * g.n_heads + kvh * G + hd) * g.r_v + c) * 2),
                                lsum > 0.f ? val / lsum : 0.f);
        }
      }
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
    __syncthreads();
  }

  // ---- arrival: this workgroup writes nothing more that the projection reads
  if (tid == 0) __hip_atomic_fetch_add(t.sync, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  const int n_wgs = gridDim.x * gridDim.y * gridDim.z;
  const int wg = (b * gridDim.y + split) * gridDim.x + kvh;       // dispatch order
  const int wi = wg - (n_wgs - t.n_work);
  if (wi < 0) return;

  // ---- output projection, blocks wi, wi + n_work, ... of 16 channels; the four waves interleave the k steps
  constexpr uint32_t kOob = kOobTail;
  const int steps = t.K / 32, nblks = t.N / 16;
  auto load_w = [&](int blk, int s0, bf16x8 (&bw)[kTailRound]) __attribute__((always_inline)) {
    const __amdgpu_buffer_rsrc_t rsrc = tail_rsrc(t.w_o + (((int64_t)blk * steps) << 9), (uint32_t)(steps * 1024));
#pragma unroll
    for (int u = 0; u < kTailRound; ++u) {
      const int s = s0 + wave + 4 * u;
      bw[u] = __builtin_bit_cast(
          bf16x8, __builtin_amdgcn_raw_buffer_load_b128(rsrc, s < steps ? (uint32_t)((s << 10) + (lane << 4)) : kOob, 0, 2));
    }
  };
  bf16x8 bw[kTailRound];
  int blk = wi, s0 = 0;
  load_w(blk, 0, bw);                      // on their way while the rest of the grid finishes

  if (tid == 0) {
    uint32_t polls = 0;
    int ok;
    while (true) {
      if (__hip_atomic_load(t.sync, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= (uint32_t)n_wgs) {
        ok = 1;
        break;
      }
      if (++polls >= t.spin_limit) {
        ok = 0;
        break;
      }
      __builtin_amdgcn_s_sleep(8);
    }
    if (!ok && t.status) atomicOr(t.status, kStatusWaitExpired);
    flag = ok;
  }
  __syncthreads();
  if (!flag) return;

  while (true) {
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    while (true) {
      // the merged rows, rows past the batch read as zero
      bf16x8 af[kTailRound];
#pragma unroll
      for (int u = 0; u < kTailRound; ++u) {
        const int s = s0 + wave + 4 * u;
        af[u] = __builtin_bit_cast(
            bf16x8, __builtin_amdgcn_raw_buffer_load_b128(
                        o_rsrc, s < steps ? (uint32_t)((col * t.K + s * 32 + quad * 8) * 2) : kOob, 0, kCoherent));
      }
#pragma unroll
      for (int u = 0; u < kTailRound; ++u) acc = mfma16(af[u], bw[u], acc);
      s0 += 4 * kTailRound;
      if (s0 >= steps) break;
      load_w(blk, s0, bw);
    }
    red[wave][lane] = acc;
    __syncthreads();
    if (tid < 64) {
      const f32x4 v = red[0][lane] + red[1][lane] + red[2][lane] + red[3][lane];
      // lane = channel blk * 16 + col, registers = rows 4 * quad .. + 3
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int r = quad * 4 + e;
        if (r < n_batch) t.y[(int64_t)r * t.N + blk * 16 + col] = f32_to_bf16_rne(v[e]);
      }
    }
    blk += t.n_work;
    if (blk >= nblks) break;
    __syncthreads();
    s0 = 0;
    load_w(blk, 0, bw);
  }
}

}  // namespace ea
