// Launch side of the generation-phase attention kernel in the form that also stores its scores, for callers that
// accumulate the attention probability each cached token receives (H2O-style eviction on the rank-r cache;
// results, "Eigen Attention with token pruning"): the probabilities follow from the scores and the row's final
// reference exponent and normaliser, so the keys are read once for both the attention output and the statistic.
#include "ea_decode_kernel.h"

namespace ea {

template <int KS, int NCB>
static void launch_decode_scores(const DecodeArgs& a, int32_t B, hipStream_t st) {
  dim3 grid(a.g.n_kv_heads, a.n_splits, B), block(256);
  constexpr int TBN = (KS * 4 + NCB * 2 > 22) ? 2 : 4;
  decode_bf16_kernel<KS, NCB, TBN, 2, 0, false, true><<<grid, block, 0, st>>>(a);
}

template <int KS>
static int dispatch_ncb_scores(int ncb, const DecodeArgs& a, int32_t B, hipStream_t st) {
  switch (ncb) {
    case 1: launch_decode_scores<KS, 1>(a, B, st); break;
    case 2: launch_decode_scores<KS, 2>(a, B, st); break;
    case 3: launch_decode_scores<KS, 3>(a, B, st); break;
    case 4: launch_decode_scores<KS, 4>(a, B, st); break;
    case 5: launch_decode_scores<KS, 5>(a, B, st); break;
    case 6: launch_decode_scores<KS, 6>(a, B, st); break;
    case 7: launch_decode_scores<KS, 7>(a, B, st); break;
    case 8: launch_decode_scores<KS, 8>(a, B, st); break;
    default: return EA_ERR_SHAPE;
  }
  return launch_status();
}

// Always writes split partials (n_splits slots, also for a single split): the merge that follows is what yields
// each row's reference exponent and normaliser.
int decode_scores_bf16(const ea_layer_desc* d, const Geo& g, const float* q, const void* k_pool, const void* v_pool,
                       const int32_t* page_table, const int32_t* seq_len, int32_t B, int32_t n_splits, float* ws,
                       float* scores, int32_t s_row, hipStream_t st) {
  if (B > 65535 || g.n_kv_heads > 65535) return EA_ERR_SHAPE;
  DecodeArgs a;
  a.q = q;
  a.k_pool = (const uint16_t*)k_pool;
  a.v_pool = (const uint16_t*)v_pool;
  a.page_table = page_table;
  a.seq_len = seq_len;
  a.out = nullptr;
  a.ws = ws;
  a.g = g;
  a.n_splits = n_splits;
  a.scale_log2 = 1.4426950408889634f / sqrtf((float)d->d_head);
  a.u_k = nullptr;
  a.d_head = d->d_head;
  a.log2_base = 0.0;
  a.alibi = nullptr;
  a.ws_slots = n_splits;
  a.ws_slot0 = 0;
  a.scores = scores;
  a.s_row = s_row;
  const int ks = (g.r_k_pad + 31) / 32, ncb = g.r_v_pad / 16;
  switch (ks) {
    case 1: return dispatch_ncb_scores<1>(ncb, a, B, st);
    case 2: return dispatch_ncb_scores<2>(ncb, a, B, st);
    case 3: return dispatch_ncb_scores<3>(ncb, a, B, st);
    case 4: return dispatch_ncb_scores<4>(ncb, a, B, st);
    default: return EA_ERR_SHAPE;
  }
}

}  // namespace ea
