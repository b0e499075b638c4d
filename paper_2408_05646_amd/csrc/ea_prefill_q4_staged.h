// Prefill over a partly quantised cache by staging (codes dequantised into 16-bit stage pools, then the prefill of
// the 16-bit cache; rotary and position-free): internal interface between the C ABI and the launch code.
#pragma once
#include "ea_q4.h"

namespace ea {

// Bytes of: the page lists and the staged table, the bfloat16 stage pools (B * (max_q4_pages + max_tail_pages) pages
// of keys and of values), and (rope) the workspace of the rotary prefill over max_q4_pages + max_tail_pages pages.
int64_t prefill_staged_q4_ws_bytes(const ea_layer_desc* d, int32_t B, int32_t n, int32_t max_q4_pages,
                                   int32_t max_tail_pages, bool rope);
// u_k == nullptr: position-free form (q holds rank-r_k rows; with slopes [H]: plus the ALiBi bias); else the rotary
// form (q holds d_head channels; no slopes).
int prefill_staged_q4(const ea_layer_desc* d, const Q4Geo& qg, const void* q, const void* u_k, double rope_base,
                    const void* kq_pool, const void* vq_pool, const int32_t* q4_table, const int32_t* q4_len,
                    int32_t max_q4_pages, int32_t q4_pool_pages, const void* k_pool, const void* v_pool,
                    const int32_t* tail_table, const int32_t* tail_len, int32_t max_tail_pages, int32_t pool_pages,
                    void* out, int32_t B, int32_t n, void* ws, hipStream_t st, const float* slopes = nullptr);

}  // namespace ea
