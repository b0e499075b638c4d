// Prefill (Eq. 2 in rank space, causal) over a cache whose older tokens are 4- or 3-bit codes (quantisation paragraph
// of the results), by staging: the pages of the 4-bit part are dequantised into stage pools of bfloat16 pages, the
// pages of the bfloat16 part are copied behind them, and the prefill of the 16-bit cache runs on the stage pools,
// which live in the caller's workspace for this call only.  Rotary form (Sec. 4.3, Eq. 9-10; the Llama models of that
// experiment): a rotary prefill brings every cached key back to d_head channels in a 16-bit workspace anyway, so the
// codes are expanded on the way there.  Position-free form (and with the ALiBi bias): the alternative to attending the codes in the attention
// kernel itself -- one layer's sequence exists in 16 bits while the call runs, and the attention runs at the speed of
// the 16-bit kernel.
#include "ea_prefill_q4_staged.h"

namespace ea {

namespace {

int64_t align256(int64_t x) { return (x + 255) / 256 * 256; }

struct StageLists {
  int32_t* src_q;   // [B, max_q4_pages]   4-bit page to expand, or -1
  int32_t* dst_q;   // [B, max_q4_pages]   stage page it goes to, or -1
  int32_t* src_t;   // [B, max_tail_pages] bfloat16 page to copy, or -1
  int32_t* dst_t;   // [B, max_tail_pages] stage page it goes to, or -1
  int32_t* table;   // [B, max_q4_pages + max_tail_pages] page table of the staged sequence (-1: nothing there)
  int32_t* len;     // [B] tokens of the staged sequence
};

constexpr int kCopySlices = 8;   // workgroups per page and pool in the page copy

int64_t list_ints(int32_t B, int32_t mq, int32_t mt) { return (int64_t)B * (3 * (int64_t)(mq + mt) + 1); }

// One thread per (sequence, logical page of the staged sequence).  The 4-bit part counts in whole pages (what
// ea_quantize_pages_q4 produces); the bfloat16 part follows at the next page.
__global__ void stage_lists_kernel(StageLists l, const int32_t* __restrict__ q4_table,
                                   const int32_t* __restrict__ q4_len, const int32_t* __restrict__ tail_table,
                                   const int32_t* __restrict__ tail_len, int32_t B, int32_t mq, int32_t mt,
                                   int32_t page_tokens, int32_t q4_pool_pages, int32_t pool_pages) {
  const int32_t mp = mq + mt;
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (int64_t)B * mp) return;
  const int32_t b = (int32_t)(idx / mp), p = (int32_t)(idx % mp);
  const int32_t nqp = min(max(q4_len[b], 0) / page_tokens, mq);
  const int32_t nt = (int32_t)min((int64_t)max(tail_len[b], 0), (int64_t)mt * page_tokens);
  const int32_t ntp = (nt + page_tokens - 1) / page_tokens;
  const int32_t stage0 = b * mp;
  int32_t entry = -1;
  if (p < mq) {
    const int32_t src = q4_table[(int64_t)b * mq + p];
    const bool ok = p < nqp && src >= 0 && src < q4_pool_pages;
    l.src_q[(int64_t)b * mq + p] = ok ? src : -1;
    l.dst_q[(int64_t)b * mq + p] = ok ? stage0 + p : -1;
  }
  if (p < mt) {
    const int32_t src = tail_table[(int64_t)b * mt + p];
    const bool ok = p < ntp && src >= 0 && src < pool_pages;
    l.src_t[(int64_t)b * mt + p] = ok ? src : -1;
    l.dst_t[(int64_t)b * mt + p] = ok ? stage0 + nqp + p : -1;
  }
  if (p < nqp) {
    const int32_t src = q4_table[(int64_t)b * mq + p];
    if (src >= 0 && src < q4_pool_pages) entry = stage0 + p;
  } else if (p - nqp < ntp) {
    const int32_t src = tail_table[(int64_t)b * mt + (p - nqp)];
    if (src >= 0 && src < pool_pages) entry = stage0 + p;
  }
  l.table[idx] = entry;
  if (p == 0) l.len[b] = nqp * page_tokens + nt;
}

// Whole bfloat16 pages, keys and values, 16 bytes per thread and step: grid (pages in the list, 2, slices of a page).
__global__ __launch_bounds__(256) void copy_pages_kernel(const uint16_t* __restrict__ k_pool,
                                                         const uint16_t* __restrict__ v_pool,
                                                         uint16_t* __restrict__ k_stage, uint16_t* __restrict__ v_stage,
                                                         const int32_t* __restrict__ src_pages,
                                                         const int32_t* __restrict__ dst_pages, int64_t k_page,
                                                         int64_t v_page, int32_t pool_pages, int32_t stage_pages) {
  const int32_t src = src_pages[blockIdx.x], dst = dst_pages[blockIdx.x];
  if (src < 0 || src >= pool_pages || dst < 0 || dst >= stage_pages) return;
  const bool keys = blockIdx.y == 0;
  const int64_t units = (keys ? k_page : v_page) / 8;                       // pages are whole 16-byte units
  const u32x4* from = reinterpret_cast<const u32x4*>((keys ? k_pool : v_pool) + (int64_t)src * (keys ? k_page : v_page));
  u32x4* to = reinterpret_cast<u32x4*>((keys ? k_stage : v_stage) + (int64_t)dst * (keys ? k_page : v_page));
  for (int64_t u = (int64_t)blockIdx.z * 256 + threadIdx.x; u < units; u += (int64_t)gridDim.z * 256) to[u] = from[u];
}

}  // namespace

int64_t prefill_staged_q4_ws_bytes(const ea_layer_desc* d, int32_t B, int32_t n, int32_t mq, int32_t mt, bool rope) {
  const Geo g = make_geo(d, mq + mt, 1);
  const int64_t stage_pages = (int64_t)B * (mq + mt);
  return align256(list_ints(B, mq, mt) * 4) + align256(stage_pages * g.k_page * 2) + align256(stage_pages * g.v_page * 2) +
         (rope ? prefill_rope_ws_bytes(d, B, n, mq + mt) : 0);
}

int prefill_staged_q4(const ea_layer_desc* d, const Q4Geo& qg, const void* q, const void* u_k, double rope_base,
                    const void* kq_pool, const void* vq_pool, const int32_t* q4_table, const int32_t* q4_len, int32_t mq,
                    int32_t q4_pool_pages, const void* k_pool, const void* v_pool, const int32_t* tail_table,
                    const int32_t* tail_len, int32_t mt, int32_t pool_pages, void* out, int32_t B, int32_t n, void* ws,
                    hipStream_t st, const float* slopes) {
  const int64_t stage_pages64 = (int64_t)B * (mq + mt);
  if (stage_pages64 > INT32_MAX || (int64_t)B * mq > INT32_MAX) return EA_ERR_SHAPE;
  const int32_t mp = mq + mt, stage_pages = (int32_t)stage_pages64;
  const Geo gs = make_geo(d, mp, stage_pages);
  char* w = (char*)ws;
  StageLists l;
  l.src_q = (int32_t*)w;
  l.dst_q = l.src_q + (int64_t)B * mq;
  l.src_t = l.dst_q + (int64_t)B * mq;
  l.dst_t = l.src_t + (int64_t)B * mt;
  l.table = l.dst_t + (int64_t)B * mt;
  l.len = l.table + (int64_t)B * mp;
  w += align256(list_ints(B, mq, mt) * 4);
  uint16_t* k_stage = (uint16_t*)w;
  w += align256(stage_pages64 * gs.k_page * 2);
  uint16_t* v_stage = (uint16_t*)w;
  w += align256(stage_pages64 * gs.v_page * 2);
  const int64_t threads = (int64_t)B * mp;
  stage_lists_kernel<<<dim3((uint32_t)((threads + 255) / 256)), 256, 0, st>>>(l, q4_table, q4_len, tail_table, tail_len,
                                                                             B, mq, mt, d->page_tokens, q4_pool_pages,
                                                                             pool_pages);
  int rc = launch_status();
  if (rc != EA_OK) return rc;
  rc = dequantize_pages_q4(gs, qg, kq_pool, vq_pool, l.src_q, k_stage, v_stage, l.dst_q, B * mq, q4_pool_pages, st);
  if (rc != EA_OK) return rc;
  for (int32_t done = 0; done < B * mt; done += 65535) {
    const int32_t now = B * mt - done < 65535 ? B * mt - done : 65535;
    copy_pages_kernel<<<dim3((uint32_t)now, 2, kCopySlices), 256, 0, st>>>((const uint16_t*)k_pool, (const uint16_t*)v_pool, k_stage,
                                                              v_stage, l.src_t + done, l.dst_t + done, gs.k_page,
                                                              gs.v_page, pool_pages, stage_pages);
  }
  rc = launch_status();
  if (rc != EA_OK) return rc;
  if (u_k && slopes) return EA_ERR_ARG;
  if (slopes) return prefill_alibi_bf16(d, gs, q, slopes, k_stage, v_stage, l.table, l.len, out, B, n, st);
  if (!u_k) return prefill_bf16(d, gs, q, k_stage, v_stage, l.table, l.len, out, B, n, st);
  return prefill_rope_bf16(d, gs, q, u_k, rope_base, k_stage, v_stage, l.table, l.len, out, B, n, w, st);
}

}  // namespace ea
