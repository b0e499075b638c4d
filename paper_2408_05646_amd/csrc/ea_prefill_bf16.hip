// placeholder until the MFMA prefill kernel lands
#include "ea_common.h"
namespace ea {
int prefill_bf16(const ea_layer_desc*, const Geo&, const void*, const void*, const void*, const int32_t*,
                 const int32_t*, void*, int32_t, int32_t, hipStream_t) {
  return EA_ERR_SHAPE;
}
}  // namespace ea
