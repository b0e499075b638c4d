// Launch side of the bf16 prefill-phase attention kernel, position-free form.
#include "ea_prefill_kernel.h"

namespace ea {

int prefill_bf16(const ea_layer_desc* d, const Geo& g, const void* q, const void* k_pool, const void* v_pool,
                 const int32_t* page_table, const int32_t* seq_len, void* out, int32_t B, int32_t n, hipStream_t st,
                 int32_t k_compact, float* part_o, float* part_ml) {
  return prefill_bf16_launch<false>(d, g, q, k_pool, v_pool, page_table, seq_len, out, B, n, st, k_compact, nullptr,
                                    part_o, part_ml);
}

}  // namespace ea
