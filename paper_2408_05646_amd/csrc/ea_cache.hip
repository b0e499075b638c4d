// Import / export between dense rank-r tensors [B, H_kv, n, r] and the paged pools.
#include "ea_common.h"

namespace ea {

template <typename T, bool IS_K, bool BF16, bool SCATTER>
__global__ void cache_copy_kernel(T* __restrict__ dense, T* __restrict__ pool, const int32_t* __restrict__ page_table,
                                  Geo g, int32_t B, int32_t n, int32_t pos0) {
  const int32_t r = IS_K ? g.r_k : g.r_v;
  const int32_t r_pad = IS_K ? g.r_k_pad : g.r_v_pad;
  const int64_t slab = IS_K ? g.k_slab : g.v_slab;
  const int64_t page_elems = IS_K ? g.k_page : g.v_page;
  const int64_t total = (int64_t)B * g.n_kv_heads * n * r_pad;
  for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
       idx += (int64_t)gridDim.x * blockDim.x) {
    const int32_t c = (int32_t)(idx % r_pad);
    int64_t rest = idx / r_pad;
    const int32_t t = (int32_t)(rest % n);
    rest /= n;
    const int32_t h = (int32_t)(rest % g.n_kv_heads);
    const int32_t b = (int32_t)(rest / g.n_kv_heads);
    const int32_t pos = pos0 + t;
    const int32_t lp = pos / g.page_tokens;
    if (lp >= g.max_pages) continue;
    const int32_t page = page_table[(int64_t)b * g.max_pages + lp];
    if (page < 0 || page >= g.pool_pages) continue;
    const int32_t tp = pos % g.page_tokens;
    const int64_t off = (int64_t)page * page_elems + (int64_t)h * slab +
                        (BF16 ? (IS_K ? bf16_k_slab_off(tp, c, r_pad) : bf16_v_slab_off(tp, c, r_pad))
                              : f32_slab_off(tp, c, r_pad));
    const int64_t didx = (((int64_t)b * g.n_kv_heads + h) * n + t) * r + c;
    if (SCATTER) {
      pool[off] = c < r ? dense[didx] : T(0);
    } else if (c < r) {
      dense[didx] = pool[off];
    }
  }
}

template <typename T, bool BF16>
static void launch_copy(bool scatter, bool is_k, void* dense, void* pool, const int32_t* pt, const Geo& g, int32_t B,
                        int32_t n, int32_t pos0, hipStream_t st) {
  const int64_t total = (int64_t)B * g.n_kv_heads * n * (is_k ? g.r_k_pad : g.r_v_pad);
  int64_t blocks = (total + 255) / 256;
  if (blocks > 65536) blocks = 65536;
  dim3 grid((uint32_t)blocks), block(256);
  T* d = (T*)dense;
  T* p = (T*)pool;
  if (scatter) {
    if (is_k) cache_copy_kernel<T, true, BF16, true><<<grid, block, 0, st>>>(d, p, pt, g, B, n, pos0);
    else cache_copy_kernel<T, false, BF16, true><<<grid, block, 0, st>>>(d, p, pt, g, B, n, pos0);
  } else {
    if (is_k) cache_copy_kernel<T, true, BF16, false><<<grid, block, 0, st>>>(d, p, pt, g, B, n, pos0);
    else cache_copy_kernel<T, false, BF16, false><<<grid, block, 0, st>>>(d, p, pt, g, B, n, pos0);
  }
}

int cache_copy(const ea_layer_desc* d, const Geo& g, bool scatter, void* k_dense, void* v_dense, void* k_pool,
               void* v_pool, const int32_t* page_table, int32_t B, int32_t n, int32_t pos0, hipStream_t st) {
  if (d->dtype == EA_BF16) {
    if (k_dense) launch_copy<uint16_t, true>(scatter, true, k_dense, k_pool, page_table, g, B, n, pos0, st);
    if (v_dense) launch_copy<uint16_t, true>(scatter, false, v_dense, v_pool, page_table, g, B, n, pos0, st);
  } else {
    if (k_dense) launch_copy<float, false>(scatter, true, k_dense, k_pool, page_table, g, B, n, pos0, st);
    if (v_dense) launch_copy<float, false>(scatter, false, v_dense, v_pool, page_table, g, B, n, pos0, st);
  }
  return launch_status();
}

// ---- weights: out-major [N, K] -> matrix-core fragment order [N/16][K/32][4][16][8] (bf16), copy (fp32)
__global__ void pack_weight_bf16_kernel(const uint16_t* __restrict__ src, uint16_t* __restrict__ dst, int32_t N,
                                        int32_t K) {
  const int64_t total = (int64_t)round_up(N, 16) * K / 8;           // 16-byte units
  const u32x4 zero = {0u, 0u, 0u, 0u};
  for (int64_t u = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; u < total; u += (int64_t)gridDim.x * blockDim.x) {
    const int row16 = (int)(u & 15), quad = (int)((u >> 4) & 3);
    const int64_t frag = u >> 6;
    const int steps = K / 32;
    const int64_t nblk = frag / steps;
    const int step = (int)(frag % steps);
    const int64_t n = nblk * 16 + row16;
    const int k = step * 32 + quad * 8;
    reinterpret_cast<u32x4*>(dst)[u] = n < N ? *reinterpret_cast<const u32x4*>(src + n * K + k) : zero;
  }
}

__global__ void copy_f32_kernel(const float* __restrict__ src, float* __restrict__ dst, int64_t n) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
    dst[i] = src[i];
}

int pack_weight(const void* w_t, void* packed, int32_t N, int32_t K, bool bf16, hipStream_t st) {
  if (bf16) {
    const int64_t units = (int64_t)round_up(N, 16) * K / 8;
    int64_t blocks = (units + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    pack_weight_bf16_kernel<<<dim3((uint32_t)blocks), dim3(256), 0, st>>>((const uint16_t*)w_t, (uint16_t*)packed, N, K);
  } else {
    const int64_t n = (int64_t)N * K;
    int64_t blocks = (n + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    copy_f32_kernel<<<dim3((uint32_t)blocks), dim3(256), 0, st>>>((const float*)w_t, (float*)packed, n);
  }
  return launch_status();
}

}  // namespace ea
