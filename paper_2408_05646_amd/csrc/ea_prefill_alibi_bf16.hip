// Launch side of the bf16 prefill-phase attention kernel with the ALiBi position bias.
#include "ea_prefill_kernel.h"

namespace ea {

int prefill_alibi_bf16(const ea_layer_desc* d, const Geo& g, const void* q, const float* slopes, const void* k_pool,
                       const void* v_pool, const int32_t* page_table, const int32_t* seq_len, void* out, int32_t B,
                       int32_t n, hipStream_t st) {
  return prefill_bf16_launch<true>(d, g, q, k_pool, v_pool, page_table, seq_len, out, B, n, st, 0, slopes);
}

}  // namespace ea
