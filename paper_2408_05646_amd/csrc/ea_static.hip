// ea_decode_attn_static: ea_decode_attn for callers that cannot allocate device memory (code under HIP graph
// capture, serving loops with a fixed memory plan, harnesses that forbid hipMalloc).  The split partials, which
// ea_decode_attn takes as a caller-provided workspace, go to a buffer that is part of the library's image.
#include <mutex>
#include "ea_common.h"

namespace ea {

// The split partials (m, l, acc of every (sequence, head, split)) of one call.  Every GPU the library runs on
// holds its own copy of this array, at its own address, until the process ends.
static __device__ __align__(256) float scratch[EA_STATIC_SCRATCH_BYTES / sizeof(float)];

// In host code `scratch` is only a handle for the symbol, not a device address: the address each device gave its
// copy is asked for once per device (with that device current) and kept here.
constexpr int kMaxDevices = 64;
static float* scratch_ptr[kMaxDevices] = {};
static std::mutex scratch_mutex;

static int scratch_for_current_device(float** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return EA_ERR_DEVICE;
  std::lock_guard<std::mutex> lock(scratch_mutex);
  if (!scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
      (void)hipGetLastError();
      return EA_ERR_DEVICE;
    }
    scratch_ptr[dev] = static_cast<float*>(p);
  }
  *out = scratch_ptr[dev];
  return EA_OK;
}

}  // namespace ea

using namespace ea;

extern "C" int ea_decode_attn_static(const ea_layer_desc* desc, const void* dev_q_r, const void* dev_k_pool,
                                     const void* dev_v_pool, const int32_t* dev_page_table,
                                     const int32_t* dev_seq_len, float* dev_out, int32_t B, int32_t max_pages,
                                     int32_t pool_pages, int32_t n_splits, void* stream) {
  int rc = validate_desc(desc);
  if (rc != EA_OK) return rc;
  if (!dev_q_r || !dev_k_pool || !dev_v_pool || !dev_page_table || !dev_seq_len || !dev_out) return EA_ERR_ARG;
  if (B <= 0 || max_pages <= 0 || pool_pages <= 0 || n_splits < 0 || n_splits > 1024) return EA_ERR_ARG;
  if (!aligned16(dev_q_r) || !aligned16(dev_k_pool) || !aligned16(dev_v_pool) || !aligned16(dev_out))
    return EA_ERR_ALIGN;
  if (n_splits == 0) {
    const int64_t cap_tokens = (int64_t)max_pages * desc->page_tokens;
    n_splits = ea_decode_auto_splits(desc, B, cap_tokens > INT32_MAX ? INT32_MAX : (int32_t)cap_tokens);
  }
  // the partials of this call must fit the library's buffer
  if (ea_decode_workspace_bytes(desc, B, n_splits) > (int64_t)EA_STATIC_SCRATCH_BYTES) return EA_ERR_SCRATCH_LIMIT;
  float* ws = nullptr;
  if (n_splits > 1) {
    rc = scratch_for_current_device(&ws);
    if (rc != EA_OK) return rc;
  }
  // Nothing in the buffer has to start at zero: every workgroup of the attention kernel writes the partials of its
  // (sequence, head, split) -- an empty range writes (-inf, 0, 0) -- before the merge kernel, which follows it on the
  // same stream, reads exactly those.
  Geo g = make_geo(desc, max_pages, pool_pages);
  hipStream_t st = (hipStream_t)stream;
  clear_stale_error();
  if (desc->dtype == EA_BF16)
    rc = decode_bf16(desc, g, (const float*)dev_q_r, dev_k_pool, dev_v_pool, dev_page_table, dev_seq_len, dev_out, B,
                     n_splits, ws, st);
  else
    rc = decode_f32(desc, g, (const float*)dev_q_r, (const float*)dev_k_pool, (const float*)dev_v_pool, dev_page_table,
                    dev_seq_len, dev_out, B, n_splits, ws, st);
  if (rc != EA_OK) return rc;
  if (n_splits > 1) rc = merge_splits(g, ws, dev_out, B, n_splits, st);
  return rc;
}
