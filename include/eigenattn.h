/*
 * eigenattn.h -- C ABI of the Eigen Attention low-rank inference path for MI355X (gfx950).
 *
 * The library computes attention in a rank-r space over a compressed, paged KV
 * cache (arXiv 2408.05646).  The per-head orthonormal bases U^K, U^V are folded
 * into the projection weights offline (Eq. 8), so the cache holds only rank-r
 * keys and values and every call below works on rank-r tensors.
 *
 * Conventions
 *  - Every function returns int: EA_OK (0) or a negative EA_ERR_* code; nothing
 *    aborts, throws, allocates or frees device memory, or synchronises.
 *  - Pointers named dev_* are DEVICE pointers owned by the caller.  `stream` is a
 *    hipStream_t passed as void* (NULL = the default stream).  Kernels are
 *    enqueued on it and the call returns immediately.
 *  - Shapes are row-major with the last index fastest.  B = sequences in the
 *    batch, T = new tokens per sequence in this call, H = query heads,
 *    H_kv = KV heads (H % H_kv == 0; query head i uses KV head i / (H / H_kv)),
 *    d = d_model, d_h = d_head, r_k / r_v = key / value rank per head.
 *  - Host-side argument, shape and alignment checks happen before any launch.
 *    Errors that only the device can see (a page id outside the pool, a position
 *    beyond the page table) never fault: the affected tokens are skipped on
 *    write and masked out on read.  A skipped write is a lost token: the
 *    projection calls count them in a device status word the caller may pass
 *    (dev_status), which the host can read after its next synchronisation.
 *  - dtype EA_F32: x, weights, q_r, o, y and the cache are float.  dtype
 *    EA_BF16: x, weights, y and the cache are bfloat16 with fp32 accumulation;
 *    q_r and o are float or bfloat16 as the q_dtype / o_dtype arguments say.
 *    The cache is written with one round-to-nearest-even of the fp32 accumulator.
 */
#ifndef EIGENATTN_H
#define EIGENATTN_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define EA_API __attribute__((visibility("default")))

enum {
  EA_OK = 0,
  EA_ERR_ARG = -1,         /* null pointer, non-positive size, bad enum          */
  EA_ERR_SHAPE = -2,       /* shape the kernels do not support (see each call)   */
  EA_ERR_ALIGN = -3,       /* pointer not 16-byte aligned                         */
  EA_ERR_WORKSPACE = -4,   /* workspace missing or too small                      */
  EA_ERR_DEVICE = -5,      /* the HIP runtime reported a launch error             */
  EA_ERR_SCRATCH_LIMIT = -6 /* the call needs more than the library's built-in scratch buffer holds */
};

enum { EA_F32 = 0, EA_BF16 = 1 };

/* One attention layer.  The softmax divisor is sqrt(d_head), never sqrt(r):
 * Eq. (7) keeps sqrt(d_h) in rank space. */
typedef struct ea_layer_desc {
  int32_t d_model;
  int32_t n_heads;
  int32_t n_kv_heads;
  int32_t d_head;
  int32_t r_k;           /* 1..128 (EA_BF16) / 1..256 (EA_F32)                    */
  int32_t r_v;
  int32_t dtype;         /* EA_F32 or EA_BF16                                      */
  int32_t page_tokens;   /* tokens per cache page: multiple of 64 (EA_BF16), of 16 (EA_F32) */
  int32_t q4_key_group;  /* 4-bit cache only: tokens that share a key scale, 64 (also meant by 0) or 128;
                            with 128, page_tokens must be a multiple of 128.  Ignored by every other call. */
  int32_t q4_bits;       /* 4-bit cache calls only: width of a code, 4 (also meant by 0) or 3                        */
} ea_layer_desc;

/* Geometry of the two page pools of a layer (K and V are separate pools, page p
 * of a pool starts at element p * page_elems).  Inside a page the kv heads
 * follow each other, slab by slab.  Inside a slab the element order is:
 *  layout_id 0 (EA_F32): token-major rows, [page_tokens][r_pad].
 *  layout_id 1 (EA_BF16): matrix-core fragment order.  Tokens are grouped in tiles
 *    of 64.  K tile: [4 blocks of 16 tokens][r_k_pad/8 chunks][16 tokens][8 channels].
 *    V tile: [2 groups of 32 tokens][r_v_pad/16 blocks][4 quads][16 channels][8 token slots],
 *    token slot j of quad q is token 16*(j/4) + 4*q + j%4 of the group.
 *  Padding channels (r..r_pad-1) are written as zero by ea_project_qkv and
 *  ea_cache_scatter; r_k_pad is a multiple of 8 (4 for EA_F32), r_v_pad of 16 (4).
 *  ea_cache_k_index / ea_cache_v_index give the exact element index. */
typedef struct ea_cache_layout {
  int32_t layout_id;
  int32_t elem_bytes;
  int32_t r_k_pad;
  int32_t r_v_pad;
  int64_t k_slab_elems;   /* page_tokens * r_k_pad                                  */
  int64_t v_slab_elems;
  int64_t k_page_elems;   /* n_kv_heads * k_slab_elems                              */
  int64_t v_page_elems;
} ea_cache_layout;

/* ---- host-only helpers (pure functions, no device access) ---------------- */

EA_API int ea_cache_layout_query(const ea_layer_desc* desc, ea_cache_layout* out);

/* Element index inside the K (V) pool of channel `channel` of the token at
 * offset `token_in_page` of kv head `kv_head` in physical page `page`;
 * -1 on an argument out of range.  This is the reference of the layout. */
EA_API int64_t ea_cache_k_index(const ea_layer_desc* desc, int32_t page, int32_t kv_head, int32_t token_in_page, int32_t channel);
EA_API int64_t ea_cache_v_index(const ea_layer_desc* desc, int32_t page, int32_t kv_head, int32_t token_in_page, int32_t channel);

/* Logical token slot of position `pos` of a sequence whose page-table row is
 * `page_table_row` (host memory, max_pages entries): page * page_tokens +
 * pos % page_tokens, or -1 if pos is beyond the table.  Reference of the paging
 * arithmetic used by every kernel (K <- Concat(K, k) in paged form). */
EA_API int64_t ea_cache_slot(const ea_layer_desc* desc, const int32_t* page_table_row, int32_t max_pages, int32_t pos);

EA_API const char* ea_strerror(int code);
EA_API int ea_version(void);

/* ---- cache import / export (device) -------------------------------------- */

/* Copy dense rank-r tensors into / out of the paged pools.
 * dev_k_dense [B, H_kv, n, r_k], dev_v_dense [B, H_kv, n, r_v] in the cache
 * dtype; token t of sequence b goes to position pos0 + t.  Either dense
 * pointer may be NULL to skip that pool.  Scatter zero-fills padding channels. */
EA_API int ea_cache_scatter(const ea_layer_desc* desc, const void* dev_k_dense, const void* dev_v_dense,
                     void* dev_k_pool, void* dev_v_pool, const int32_t* dev_page_table,
                     int32_t B, int32_t n, int32_t pos0, int32_t max_pages, int32_t pool_pages, void* stream);
EA_API int ea_cache_gather(const ea_layer_desc* desc, void* dev_k_dense, void* dev_v_dense,
                    const void* dev_k_pool, const void* dev_v_pool, const int32_t* dev_page_table,
                    int32_t B, int32_t n, int32_t pos0, int32_t max_pages, int32_t pool_pages, void* stream);

/* ---- weight packing (device, done once, offline like the folding of Eq. 8) - */

/* The projection calls read their folded weights in a packed order.  The source is
 * "out-major": dev_w_t [N, K], one row of K input weights per output channel.
 *   EA_F32 : packed = the same [N, K] array (a plain copy).
 *   EA_BF16: matrix-core fragment order [ceil(N/16)][K/32][4 quads][16 channels][8 k]:
 *            element (n, k) sits at ((n/16 * K/32 + k/32) * 4 + (k%32)/8) * 128 + (n%16)*8 + k%8;
 *            rows N..ceil16(N)-1 are zero.  Requires K % 32 == 0.
 * ea_packed_weight_elems gives the element count of the packed buffer (-1 on bad arguments). */
EA_API int64_t ea_packed_weight_elems(int32_t N, int32_t K, int32_t dtype);
EA_API int ea_pack_weight(const void* dev_w_t, void* dev_packed, int32_t N, int32_t K, int32_t dtype, void* stream);

/* ---- the hot path -------------------------------------------------------- */

/* Fused low-rank QKV projection and cache append: Eq. (1) with the folded
 * weights of Eq. (8), then K <- Concat(K, k), V <- Concat(V, v) (Sec. 2, LLM
 * inference).
 *   dev_x      [B*T, d]  (row b*T + t is token t of sequence b), desc dtype
 *   dev_wqkv   packed by ea_pack_weight from [H*r_k + H_kv*r_k + H_kv*r_v, d]:
 *              one row of d weights per output channel ("out-major"), ordered
 *              q heads, k heads, v heads; row (i*r_k + c) is column c of
 *              W^Q_i U^K_{g(i)}, and so on.
 *   dev_q_r    [B*T, H, r_k] out, float (q_dtype EA_F32) or bfloat16 (EA_BF16)
 *   dev_seq_len[B]: length of each sequence BEFORE this call; token t is
 *              appended at position seq_len[b] + t.  Not modified.
 *   dev_page_table [B, max_pages] int32 physical page ids (< pool_pages).
 *   dev_status NULL, or one int32 in device memory (4-byte aligned) to which the call ADDS the number of
 *              (sequence, token) appends it could not store -- position seq_len[b] + t at or beyond
 *              max_pages * page_tokens (the cache of that sequence is full), or a page id outside
 *              [0, pool_pages).  Such a token's k and v are not written anywhere (its q_r row still is), and
 *              later attention calls see the sequence without it.  The word is never cleared by the library:
 *              zero it once, read it after any synchronisation, nonzero = tokens were lost since.
 * Requires d % 32 == 0 for EA_BF16 (d % 4 == 0 for EA_F32). */
EA_API int ea_project_qkv(const ea_layer_desc* desc, const void* dev_x, const void* dev_wqkv,
                   void* dev_q_r, int32_t q_dtype, void* dev_k_pool, void* dev_v_pool,
                   const int32_t* dev_page_table, const int32_t* dev_seq_len,
                   int32_t B, int32_t T, int32_t max_pages, int32_t pool_pages, int32_t* dev_status, void* stream);

/* The same fused projection for models with rotary position embedding
 * (Sec. 4.3): the query keeps all d_head channels (W^Q is not folded, the
 * rotation has to be applied to the full query), keys are projected with the
 * ONE basis all heads share (W^K' = W^K_g U^K), values as in Eq. (8).
 *   dev_wqkv   packed from [H*d_head + H_kv*r_k + H_kv*r_v, d], same ordering
 *   dev_q      [B*T, H, d_head] out
 * Everything else as ea_project_qkv.  Requires r_k <= d_head. */
EA_API int ea_project_qkv_rope(const ea_layer_desc* desc, const void* dev_x, const void* dev_wqkv,
                   void* dev_q, int32_t q_dtype, void* dev_k_pool, void* dev_v_pool,
                   const int32_t* dev_page_table, const int32_t* dev_seq_len,
                   int32_t B, int32_t T, int32_t max_pages, int32_t pool_pages, int32_t* dev_status, void* stream);

/* Number of splits of the cached sequence ea_decode_attn would pick for
 * n_splits = 0, and the workspace it needs for a given split count. */
EA_API int32_t ea_decode_auto_splits(const ea_layer_desc* desc, int32_t B, int32_t max_seq_len);
EA_API int64_t ea_decode_workspace_bytes(const ea_layer_desc* desc, int32_t B, int32_t n_splits);

/* Generation-phase attention in rank space, Eq. (3) with Eq. (7)'s rank-r
 * operands:  s_t = q_r . K_r[t] / sqrt(d_h) for t < seq_len[b],
 * p = Softmax(s), o = sum_t p_t V_r[t].
 *   dev_q_r [B, H, r_k] float;  dev_out [B, H, r_v] float
 *   dev_seq_len [B]: cached tokens per sequence INCLUDING the one just appended;
 *              a sequence of length 0 yields a zero output row.
 *   n_splits: the cached sequence is cut in this many parts handled by different
 *              workgroups and merged afterwards (0 = choose).  dev_ws must hold
 *              ea_decode_workspace_bytes(desc, B, n_splits) bytes when the
 *              effective split count is > 1. */
EA_API int ea_decode_attn(const ea_layer_desc* desc, const void* dev_q_r, const void* dev_k_pool, const void* dev_v_pool,
                   const int32_t* dev_page_table, const int32_t* dev_seq_len, float* dev_out,
                   int32_t B, int32_t max_pages, int32_t pool_pages, int32_t n_splits,
                   void* dev_ws, int64_t ws_bytes, void* stream);

/* ea_decode_attn for callers that cannot allocate device memory or bring a workspace: code under HIP graph
 * capture, serving loops with a fixed memory plan, harnesses that forbid hipMalloc.  Same arguments and result
 * as ea_decode_attn (same kernels, same n_splits rule) without dev_ws / ws_bytes: the split partials go to a
 * buffer of EA_STATIC_SCRATCH_BYTES that is part of the library's image (every GPU the library is used on holds
 * its own copy until the process ends).  The call allocates and frees nothing.
 *   - A call whose partials need more (ea_decode_workspace_bytes(desc, B, n_splits) > EA_STATIC_SCRATCH_BYTES)
 *     is rejected with EA_ERR_SCRATCH_LIMIT before anything is launched; pass a smaller n_splits or use
 *     ea_decode_attn.
 *   - All calls on one GPU share that GPU's buffer, which keeps the previous call's contents; nothing in it has
 *     to be cleared (the attention kernel writes every partial the merge reads).  Calls that overlap in time on
 *     one GPU (different streams) race on it: serialise them, or use ea_decode_attn with a workspace each.
 *   - The first call on a device looks the buffer's address up (no allocation); make that call before starting
 *     a graph capture. */
#define EA_STATIC_SCRATCH_BYTES (8 * 1024 * 1024)
EA_API int ea_decode_attn_static(const ea_layer_desc* desc, const void* dev_q_r, const void* dev_k_pool,
                   const void* dev_v_pool, const int32_t* dev_page_table, const int32_t* dev_seq_len, float* dev_out,
                   int32_t B, int32_t max_pages, int32_t pool_pages, int32_t n_splits, void* stream);

/* The whole generation step of one attention layer in a single call (Sec. 2, "LLM inference", with the folded
 * weights of Eq. 8): for the newest token of each of B <= 64 sequences
 *   [q_r | k_r | v_r] = x [W^Q' | W^K' | W^V'],  K_r <- Concat(K_r, k_r), V_r <- Concat(V_r, v_r)   (ea_project_qkv, T = 1)
 *   o = Softmax(q_r K_r^T / sqrt(d_h)) V_r over the seq_len[b] + 1 cached tokens                       (ea_decode_attn)
 *   y = [o_1 .. o_H] W^O'                                                                                (ea_out_proj)
 * enqueued back to back on the stream: three launches, four when the sequence is split (ea_decode_layer_fused
 * below does the same step in two).  q_r (float) and o (rounded to bfloat16 once, as after a prefill) never leave
 * the workspace.  EA_BF16 layers only.
 *   dev_x [B, d] bfloat16; dev_wqkv / dev_wo packed as for ea_project_qkv / ea_out_proj; dev_y [B, d] bfloat16
 *   dev_seq_len [B]: lengths BEFORE this step (the token is appended at that position); not modified
 *   n_splits: as ea_decode_attn (0 = choose)
 *   dev_ws: ea_decode_layer_workspace_bytes(desc, B, n_splits, rotary) bytes (n_splits >= 1 there: pass what
 *           ea_decode_auto_splits / ea_decode_rope_auto_splits returns if the call is to choose), 256-byte aligned;
 *           needs no preparation
 *   dev_status: as ea_project_qkv (NULL, or the word that counts appends that could not be stored)
 * ea_decode_layer_rope is the same step for models with rotary position embedding (Sec. 4.3): dev_wqkv as for
 * ea_project_qkv_rope, dev_u_k [d_head, r_k] bfloat16 and rope_base as for ea_decode_attn_rope.
 * ea_decode_layer_alibi is the same step for models with the ALiBi position bias (the MPT family of Sec. 5.1):
 * dev_slopes [H] float as for ea_decode_attn_alibi (NULL: EA_ERR_ARG), workspace as the position-free form
 * (rotary = 0). */
EA_API int64_t ea_decode_layer_workspace_bytes(const ea_layer_desc* desc, int32_t B, int32_t n_splits, int32_t rotary);
EA_API int ea_decode_layer(const ea_layer_desc* desc, const void* dev_x, const void* dev_wqkv, const void* dev_wo,
                   void* dev_k_pool, void* dev_v_pool, const int32_t* dev_page_table, const int32_t* dev_seq_len,
                   void* dev_y, int32_t B, int32_t max_pages, int32_t pool_pages, int32_t n_splits,
                   void* dev_ws, int64_t ws_bytes, int32_t* dev_status, void* stream);
EA_API int ea_decode_layer_rope(const ea_layer_desc* desc, const void* dev_x, const void* dev_wqkv, const void* dev_wo,
                   const void* dev_u_k, double rope_base, void* dev_k_pool, void* dev_v_pool,
                   const int32_t* dev_page_table, const int32_t* dev_seq_len, void* dev_y, int32_t B,
                   int32_t max_pages, int32_t pool_pages, int32_t n_splits, void* dev_ws, int64_t ws_bytes,
                   int32_t* dev_status, void* stream);
EA_API int ea_decode_layer_alibi(const ea_layer_desc* desc, const void* dev_x, const void* dev_wqkv, const void* dev_wo,
                   const float* dev_slopes, void* dev_k_pool, void* dev_v_pool, const int32_t* dev_page_table,
                   const int32_t* dev_seq_len, void* dev_y, int32_t B, int32_t max_pages, int32_t pool_pages,
                   int32_t n_splits, void* dev_ws, int64_t ws_bytes, int32_t* dev_status, void* stream);

/* ea_decode_layer in TWO launches (the same step, Sec. 2 "LLM inference" with the folded weights of Eq. 8; B <= 16):
 *   launch 1: [q_r | k_r | v_r] = x [W^Q' | W^K' | W^V'] and the append, as ea_project_qkv;
 *   launch 2: the attention of ea_decode_attn over seq_len[b] + 1 tokens, the merge of the split partials (by the
 *             workgroup that finishes a (sequence, kv head) last) and y = [o_1 .. o_H] W^O': the last
 *             min(d / 16, compute units, grid size) workgroups of the grid request their share of W^O', wait until
 *             every workgroup of the grid has delivered its part of o, and multiply.
 * Arguments, workspace rules and result as ea_decode_layer, with these differences:
 *   n_splits: at most 64 (EA_ERR_SHAPE above; 0 = choose, which never exceeds it)
 *   dev_ws: ea_decode_layer_fused_workspace_bytes(...) bytes (the counters the second launch uses live there; the
 *           first launch clears them, so the workspace still needs no preparation)
 *   dev_status: NULL, or a word the caller has set to zero: appends that could not be stored are counted in its low
 *           bits as in ea_project_qkv, and bit 30 (EA_STATUS_WAIT_EXPIRED) is set if a workgroup of the second
 *           launch gave up waiting for the rest of its grid -- then dev_y is incomplete.  The wait is bounded
 *           (ea_set_wait_limit polls of the counter, a few seconds by default) so that the launch always ends.
 *   Only workgroups that hold at most half of the chip's resident workgroup slots ever wait, and only for
 *   workgroups dispatched before or with them, so a call that has the GPU to itself, or shares it with kernels
 *   that do not wait for anything, cannot run into the limit.  Two-launch calls that overlap in time with each
 *   other on one GPU (different streams) can: serialise them, or use ea_decode_layer.
 * ea_set_wait_limit(polls >= 1) sets the bound for the calls that follow (process-wide; 1 makes every waiting
 * workgroup give up at once unless the grid has already finished, which is how the expiry path is tested). */
#define EA_STATUS_WAIT_EXPIRED (1 << 30)
/* How many workgroups of the second launch project (and therefore wait): min(d / 16, compute units, grid size),
 * -1 on a bad description.  Host arithmetic only. */
EA_API int32_t ea_decode_layer_fused_workers(const ea_layer_desc* desc, int32_t B, int32_t n_splits);
EA_API int64_t ea_decode_layer_fused_workspace_bytes(const ea_layer_desc* desc, int32_t B, int32_t n_splits,
                   int32_t rotary);
EA_API int ea_decode_layer_fused(const ea_layer_desc* desc, const void* dev_x, const void* dev_wqkv,
                   const void* dev_wo, void* dev_k_pool, void* dev_v_pool, const int32_t* dev_page_table,
                   const int32_t* dev_seq_len, void* dev_y, int32_t B, int32_t max_pages, int32_t pool_pages,
                   int32_t n_splits, void* dev_ws, int64_t ws_bytes, int32_t* dev_status, void* stream);
EA_API int ea_decode_layer_fused_rope(const ea_layer_desc* desc, const void* dev_x, const void* dev_wqkv,
                   const void* dev_wo, const void* dev_u_k, double rope_base, void* dev_k_pool, void* dev_v_pool,
                   const int32_t* dev_page_table, const int32_t* dev_seq_len, void* dev_y, int32_t B,
                   int32_t max_pages, int32_t pool_pages, int32_t n_splits, void* dev_ws, int64_t ws_bytes,
                   int32_t* dev_status, void* stream);
/* (ALiBi form: dev_slopes as ea_decode_layer_alibi, workspace of the position-free form) */
EA_API int ea_decode_layer_fused_alibi(const ea_layer_desc* desc, const void* dev_x, const void* dev_wqkv,
                   const void* dev_wo, const float* dev_slopes, void* dev_k_pool, void* dev_v_pool,
                   const int32_t* dev_page_table, const int32_t* dev_seq_len, void* dev_y, int32_t B,
                   int32_t max_pages, int32_t pool_pages, int32_t n_splits, void* dev_ws, int64_t ws_bytes,
                   int32_t* dev_status, void* stream);
EA_API int ea_set_wait_limit(uint32_t polls);

/* Generation-phase attention for models with rotary position embedding
 * (Sec. 4.3, Eq. 9-10): the query keeps all d_head channels, the cache holds the
 * rank-r_k keys k_r = k U^K of ONE basis U^K shared by all heads, and each cached
 * key is brought back to d_head channels (U^K k_r) before the rotation:
 *   s_t = rot(q, n-1) . rot(U^K K_r[t], t) / sqrt(d_h),  t < n = seq_len[b],
 *   p = Softmax(s), o = sum_t p_t V_r[t],
 * where rot(x, pos) turns the channel pair (2j, 2j+1) by pos * rope_base^(-2j/d_h)
 * (x'[2j] = x[2j] cos - x[2j+1] sin, x'[2j+1] = x[2j] sin + x[2j+1] cos).
 * The query is the token appended last (position seq_len[b] - 1).
 *   dev_q   [B, H, d_head] float, NOT rotated
 *   dev_u_k [d_head, r_k] row-major, desc dtype (EA_F32 float, EA_BF16 bfloat16: the basis enters the
 *           matrix cores in the precision of the cache)
 *   everything else as ea_decode_attn (same workspace size); n_splits = 0 picks
 *   ea_decode_rope_auto_splits(desc, B, max_pages * page_tokens).
 * Requires r_k <= d_head; EA_BF16: d_head 64 or 128; EA_F32: d_head even, <= 256. */
EA_API int32_t ea_decode_rope_auto_splits(const ea_layer_desc* desc, int32_t B, int32_t max_seq_len);
EA_API int ea_decode_attn_rope(const ea_layer_desc* desc, const float* dev_q, const void* dev_u_k, double rope_base,
                    const void* dev_k_pool, const void* dev_v_pool,
                    const int32_t* dev_page_table, const int32_t* dev_seq_len, float* dev_out,
                    int32_t B, int32_t max_pages, int32_t pool_pages, int32_t n_splits,
                    void* dev_ws, int64_t ws_bytes, void* stream);

/* Prefill-phase attention in rank space, Eq. (2) with a causal mask: the n
 * queries of sequence b are its last n cached positions (query j sits at
 * position seq_len[b] - n + j and sees positions <= its own).
 *   dev_q_r [B, n, H, r_k], dev_out [B, n, H, r_v]: desc dtype (EA_F32 float,
 *   EA_BF16 bfloat16).  dev_seq_len [B] includes the n new tokens. */
EA_API int ea_prefill_attn(const ea_layer_desc* desc, const void* dev_q_r, const void* dev_k_pool, const void* dev_v_pool,
                    const int32_t* dev_page_table, const int32_t* dev_seq_len, void* dev_out,
                    int32_t B, int32_t n, int32_t max_pages, int32_t pool_pages, void* stream);

/* Prefill-phase attention for models with rotary position embedding (Sec. 4.3,
 * Eq. 9-10) with a causal mask: query j of sequence b sits at position
 * p_j = seq_len[b] - n + j and sees the cached positions t <= p_j with
 *   s_jt = rot(q_j, p_j) . rot(U^K K_r[t], t) / sqrt(d_h)
 * (rot, U^K, rope_base as in ea_decode_attn_rope).
 *   dev_q   [B, n, H, d_head], NOT rotated; dev_out [B, n, H, r_v]; dev_u_k [d_head, r_k]: desc dtype
 *   dev_ws  EA_BF16: ea_prefill_rope_workspace_bytes(desc, B, n, max_pages) bytes, 16-byte aligned: the
 *           keys, back at d_head channels and rotated, and the rotated queries are kept there for the
 *           duration of the call (B * max_pages * H_kv * page_tokens * d_head + B * n * H * d_head
 *           bfloat16 values).  EA_F32 needs none (0 bytes; dev_ws may be null).
 * dev_seq_len [B] includes the n new tokens. */
EA_API int64_t ea_prefill_rope_workspace_bytes(const ea_layer_desc* desc, int32_t B, int32_t n, int32_t max_pages);
EA_API int ea_prefill_attn_rope(const ea_layer_desc* desc, const void* dev_q, const void* dev_u_k, double rope_base,
                    const void* dev_k_pool, const void* dev_v_pool,
                    const int32_t* dev_page_table, const int32_t* dev_seq_len, void* dev_out,
                    int32_t B, int32_t n, int32_t max_pages, int32_t pool_pages,
                    void* dev_ws, int64_t ws_bytes, void* stream);

/* The two attention calls with the ALiBi position bias (Sec. 5.1 names ALiBi as
 * the position scheme of the MPT models the method is applied to; the bias is
 * the ALiBi paper's): the score of a query at position i against the cached key
 * at position j <= i becomes  q_r . K_r[j] / sqrt(d_h) - slope_h * (i - j).
 * The bias does not involve keys or queries, so it is the same in rank space.
 *   dev_slopes [H] float, slope_h >= 0 (for instance 2^(-8 (h+1) / H))
 * Everything else as ea_decode_attn / ea_prefill_attn (same workspace rule). */
EA_API int ea_decode_attn_alibi(const ea_layer_desc* desc, const void* dev_q_r, const float* dev_slopes,
                    const void* dev_k_pool, const void* dev_v_pool,
                    const int32_t* dev_page_table, const int32_t* dev_seq_len, float* dev_out,
                    int32_t B, int32_t max_pages, int32_t pool_pages, int32_t n_splits,
                    void* dev_ws, int64_t ws_bytes, void* stream);
EA_API int ea_prefill_attn_alibi(const ea_layer_desc* desc, const void* dev_q_r, const float* dev_slopes,
                    const void* dev_k_pool, const void* dev_v_pool,
                    const int32_t* dev_page_table, const int32_t* dev_seq_len, void* dev_out,
                    int32_t B, int32_t n, int32_t max_pages, int32_t pool_pages, void* stream);

/* ---- 4-bit group-quantised cache (results, "Eigen Attention with Quantization") ---- */

/* The paper combines the rank-r cache with integer group quantisation: keys per
 * channel, values per token (as in KIVI and KV-Quant), precisions of 3-4 bits in
 * groups of 16-128.  This library implements two points of that family, EA_BF16
 * layers only: 4 bits; a key scale covers one channel over the 64 tokens of a cache
 * tile or (desc.q4_key_group = 128, the group size of the paper's 4-bit rows) over the
 * 128 tokens of two neighbouring tiles; a value scale covers one token over its r_v
 * channels.  desc.q4_bits = 3 selects 3-bit codes (eight levels: 7 in place of 15 below) in
 * every call of this section.  The paper gives no rounding rule; the one used here is
 *   zero = fp16(lo), scale = fp16((hi - lo) / 15)   (lo / hi = minimum / maximum of
 *          the group, clamped to +-65504; quotient in float),
 *   code = clip(rint((x - zero) / scale), 0, 15) in float (round half to even), code 0
 *          when the scale is 0,
 *   value = scale * code + zero.
 * Only whole pages are quantised (a key group needs all its tokens); the newest tokens
 * of a sequence stay in the bfloat16 pools, and ea_decode_attn_q4 attends both parts.
 *
 * The 4-bit pools mirror the bfloat16 ones: page p of a pool starts at byte
 * p * k_page_bytes (v_page_bytes); inside a page kv head after kv head, tile after
 * tile, one tile block per (kv head, 64 tokens).  A tile block holds the codes in the
 * order the matrix cores consume them, then the fp16 scales and zeros; with key groups
 * of 128 tokens only the first K tile block of every pair carries scales (they are the
 * pair's) and the second one is codes only.
 * ea_q4_k_code_pos and its siblings are the reference of the positions.  The scale
 * and zero slots of padding channels (r_k .. the next multiple of 32) are written as 0
 * by the quantiser; whoever fills the pools by other means must leave finite values there. */
typedef struct ea_q4_layout {
  int32_t r_k_pad;         /* multiple of 8  */
  int32_t r_v_pad;         /* multiple of 16 */
  int64_t k_tile_bytes;    /* of a K tile block WITH scales: 32 * r_k_pad + 128 * ceil(r_k_pad / 32) (3 bits: 24 * r_k_pad + ..) */
  int64_t v_tile_bytes;    /* 32 * r_v_pad + 256 (3 bits: 768 per pair of 16-channel blocks + 512 for an odd one, + 256) */
  int64_t k_page_bytes;    /* n_kv_heads * (page_tokens / 64) * k_tile_bytes with key groups of 64 tokens; with 128,
                              every second tile block is 128 * ceil(r_k_pad / 32) bytes shorter */
  int64_t v_page_bytes;
} ea_q4_layout;

EA_API int ea_q4_layout_query(const ea_layer_desc* desc, ea_q4_layout* out);

/* Position of a code inside its pool: the return value is the BIT offset from the
 * start of the pool of the 4-bit code of channel `channel` of the token at offset
 * `token_in_page` of kv head `kv_head` in page `page` (always a multiple of 4).
 * The *_scale_pos functions return the BYTE offset of the fp16 scale that code is
 * multiplied with; its zero sits 16 bytes (keys) / 128 bytes (values) further.
 * -1 on an argument out of range. */
EA_API int64_t ea_q4_k_code_pos(const ea_layer_desc* desc, int32_t page, int32_t kv_head, int32_t token_in_page, int32_t channel);
EA_API int64_t ea_q4_v_code_pos(const ea_layer_desc* desc, int32_t page, int32_t kv_head, int32_t token_in_page, int32_t channel);
EA_API int64_t ea_q4_k_scale_pos(const ea_layer_desc* desc, int32_t page, int32_t kv_head, int32_t token_in_page, int32_t channel);
EA_API int64_t ea_q4_v_scale_pos(const ea_layer_desc* desc, int32_t page, int32_t kv_head, int32_t token_in_page);

/* The same for 3-bit codes (desc.q4_bits = 3; the *_code_pos functions above return -1 then, these fail
 * otherwise): bit_pos[b] receives the BIT offset from the start of the pool of bit b (b = 0, 1, 2) of the code.
 * A lane's four groups of eight codes share a 12-byte unit: dword k holds group k (k = 0, 1, 2), element 2i + h in
 * bits 3i .. 3i+2 of half word h; group 3 is laid out the same way in a fourth word whose half words are cut into
 * three nibbles each, nibble j kept in bits 12 .. 15 of half word h of dword j -- so the bits of one of its codes
 * can lie in two dwords.  The two groups of an odd last value channel block have a unit of two dwords.  K tile
 * block: 24 * r_k_pad bytes of codes; V tile block: 768 per pair of 16-channel blocks + 512 for an odd last one.
 * The scale positions are given by ea_q4_k_scale_pos / ea_q4_v_scale_pos.  Returns EA_OK or EA_ERR_ARG. */
EA_API int ea_q3_k_code_pos(const ea_layer_desc* desc, int32_t page, int32_t kv_head, int32_t token_in_page,
                            int32_t channel, int64_t* bit_pos);
EA_API int ea_q3_v_code_pos(const ea_layer_desc* desc, int32_t page, int32_t kv_head, int32_t token_in_page,
                            int32_t channel, int64_t* bit_pos);

/* Quantise n_pages full pages: page dev_src_pages[i] of the bfloat16 pools is written
 * as page dev_dst_pages[i] of the 4-bit pools (all kv heads, keys and values).  The
 * source pages are not modified and can be reused by the caller once the call has
 * run.  Page ids outside their pool are skipped.
 *   dev_kq_pool / dev_vq_pool: q4_pool_pages * k_page_bytes / v_page_bytes bytes,
 *   16-byte aligned. */
EA_API int ea_quantize_pages_q4(const ea_layer_desc* desc, const void* dev_k_pool, const void* dev_v_pool,
                    const int32_t* dev_src_pages, void* dev_kq_pool, void* dev_vq_pool,
                    const int32_t* dev_dst_pages, int32_t n_pages, int32_t pool_pages, int32_t q4_pool_pages,
                    void* stream);

/* The way back, for export and inspection: page dev_src_pages[i] of the 4-bit pools is
 * written as page dev_dst_pages[i] of the bfloat16 pools, value = scale * code + zero
 * evaluated in float and rounded once to bfloat16 (padding channels zero).  The
 * attention calls never do this: they work on the codes. */
EA_API int ea_dequantize_pages_q4(const ea_layer_desc* desc, const void* dev_kq_pool, const void* dev_vq_pool,
                    const int32_t* dev_src_pages, void* dev_k_pool, void* dev_v_pool,
                    const int32_t* dev_dst_pages, int32_t n_pages, int32_t q4_pool_pages, int32_t pool_pages,
                    void* stream);

/* Generation-phase attention (Eq. 3 with Eq. 7's rank-r operands, as ea_decode_attn)
 * over a cache whose older part is quantised: sequence b consists of its first
 * q4_len[b] tokens (a multiple of 64; a remainder is ignored) in the 4-bit pools,
 * addressed by dev_q4_page_table [B, max_q4_pages], followed by tail_len[b] tokens in
 * the bfloat16 pools, addressed by dev_tail_page_table [B, max_tail_pages] (entry 0 =
 * the page of the first unquantised token; that token must sit at offset 0 of it,
 * which holds when whole pages are quantised).  The result is attention over the
 * dequantised values of the first part and the bfloat16 values of the second.
 * The codes are expanded inside the matrix-core operands: the scales of a key tile
 * multiply the query (fp16), those of the value tokens the probabilities (fp16).
 *   dev_q_r [B, H, r_k] float; dev_out [B, H, r_v] float
 *   dev_tail_page_table / dev_tail_len may both be NULL (no bfloat16 part)
 *   n_splits: parts the 4-bit range is cut in (0 = ea_decode_auto_splits for
 *             max_q4_pages * page_tokens tokens); the tail is one more part
 *   dev_ws:  ea_decode_q4_workspace_bytes(desc, B, n_splits) bytes, always needed.
 * Position-free form only (no rotary or ALiBi variant). */
EA_API int64_t ea_decode_q4_workspace_bytes(const ea_layer_desc* desc, int32_t B, int32_t n_splits);
EA_API int ea_decode_attn_q4(const ea_layer_desc* desc, const float* dev_q_r,
                    const void* dev_kq_pool, const void* dev_vq_pool,
                    const int32_t* dev_q4_page_table, const int32_t* dev_q4_len,
                    int32_t max_q4_pages, int32_t q4_pool_pages,
                    const void* dev_k_pool, const void* dev_v_pool,
                    const int32_t* dev_tail_page_table, const int32_t* dev_tail_len,
                    int32_t max_tail_pages, int32_t pool_pages,
                    float* dev_out, int32_t B, int32_t n_splits,
                    void* dev_ws, int64_t ws_bytes, void* stream);

/* ea_decode_attn_q4 with the ALiBi position bias (as ea_decode_attn_alibi): the score
 * of the cached token at position j becomes q_r . K_r[j] / sqrt(d_h) - slope_h * (i - j),
 * i = q4_len[b] + tail_len[b] - 1 the position of the newest token; token t of the
 * 4-bit part sits at position t, token t of the tail at q4_len[b] + t (q4_len[b] a
 * multiple of 64).  dev_slopes [H] float, >= 0. */
EA_API int ea_decode_attn_alibi_q4(const ea_layer_desc* desc, const float* dev_q_r, const float* dev_slopes,
                    const void* dev_kq_pool, const void* dev_vq_pool,
                    const int32_t* dev_q4_page_table, const int32_t* dev_q4_len,
                    int32_t max_q4_pages, int32_t q4_pool_pages,
                    const void* dev_k_pool, const void* dev_v_pool,
                    const int32_t* dev_tail_page_table, const int32_t* dev_tail_len,
                    int32_t max_tail_pages, int32_t pool_pages,
                    float* dev_out, int32_t B, int32_t n_splits,
                    void* dev_ws, int64_t ws_bytes, void* stream);

/* Prefill over a partly quantised cache (Eq. (2) in rank space, causal; position-free form): sequence b holds
 * q4_len[b] tokens in the 4-bit pools (whole key groups; a remainder is ignored) followed by tail_len[b] tokens in the
 * bfloat16 pools, and the n queries dev_q_r [B, n, H, r_k] (bfloat16) are its LAST n tokens, all of which must lie in
 * the bfloat16 part (n <= tail_len[b]; the call cannot check this): every query sees the whole 4-bit part and, causally,
 * the bfloat16 part.  This is what lets a long prompt be prefilled chunk by chunk -- ea_project_qkv appends a chunk to
 * bfloat16 pages, this call attends it, ea_quantize_pages_q4 moves its pages to the 4-bit pools, the bfloat16 pages are
 * reused for the next chunk -- so that the prompt never exists in 16 bits as a whole.
 *   dev_out [B, n, H, r_v] bfloat16;  dev_ws: ea_prefill_q4_workspace_bytes(desc, B, n) bytes, 16-byte aligned
 *   (the two parts of every query row's softmax before they are merged).
 * Three launches (bfloat16 part, 4-bit part, merge).  The tiles of the 4-bit part are expanded to half precision in
 * registers; error against attention over the dequantised values as for ea_decode_attn_q4. */
EA_API int64_t ea_prefill_q4_workspace_bytes(const ea_layer_desc* desc, int32_t B, int32_t n);
EA_API int ea_prefill_attn_q4(const ea_layer_desc* desc, const void* dev_q_r,
                    const void* dev_kq_pool, const void* dev_vq_pool,
                    const int32_t* dev_q4_page_table, const int32_t* dev_q4_len,
                    int32_t max_q4_pages, int32_t q4_pool_pages,
                    const void* dev_k_pool, const void* dev_v_pool,
                    const int32_t* dev_tail_page_table, const int32_t* dev_tail_len,
                    int32_t max_tail_pages, int32_t pool_pages,
                    void* dev_out, int32_t B, int32_t n,
                    void* dev_ws, int64_t ws_bytes, void* stream);

/* ea_prefill_attn_q4 by staging: the same result (Eq. (2) in rank space, causal, over q4_len[b] tokens of codes followed
 * by tail_len[b] bfloat16 tokens), computed by dequantising the 4-bit pages (as ea_dequantize_pages_q4) and copying the
 * bfloat16 pages into stage pools inside the workspace and running ea_prefill_attn on those: 4 launches.  While the
 * call runs, this layer's sequence exists in 16 bits in the workspace (the caches of the other layers stay codes);
 * in exchange the attention runs at the speed of the 16-bit kernel (a config-4 prompt in four chunks: about 1.5 ms of
 * attention per layer instead of 2.4-2.5 ms).  q4_len[b] must be a multiple of page_tokens (whole pages; a remainder is ignored).
 * One more rounding than ea_prefill_attn_q4 (dequantised values to bfloat16 instead of half precision).
 *   dev_ws: ea_prefill_q4_staged_workspace_bytes(desc, B, n, max_q4_pages, max_tail_pages) bytes, 256-byte aligned
 *   everything else as ea_prefill_attn_q4 */
EA_API int64_t ea_prefill_q4_staged_workspace_bytes(const ea_layer_desc* desc, int32_t B, int32_t n,
                    int32_t max_q4_pages, int32_t max_tail_pages);
EA_API int ea_prefill_attn_q4_staged(const ea_layer_desc* desc, const void* dev_q_r,
                    const void* dev_kq_pool, const void* dev_vq_pool,
                    const int32_t* dev_q4_page_table, const int32_t* dev_q4_len,
                    int32_t max_q4_pages, int32_t q4_pool_pages,
                    const void* dev_k_pool, const void* dev_v_pool,
                    const int32_t* dev_tail_page_table, const int32_t* dev_tail_len,
                    int32_t max_tail_pages, int32_t pool_pages,
                    void* dev_out, int32_t B, int32_t n,
                    void* dev_ws, int64_t ws_bytes, void* stream);

/* The staged call with the ALiBi position bias (the MPT family of Sec. 5.1): dev_slopes [H] float as for
 * ea_prefill_attn_alibi (NULL: EA_ERR_ARG); token i of the 4-bit part sits at position i, token i of the bfloat16 part
 * at position q4_len[b] + i (q4_len[b] in whole pages).  Workspace as ea_prefill_attn_q4_staged. */
EA_API int ea_prefill_attn_alibi_q4(const ea_layer_desc* desc, const void* dev_q_r, const float* dev_slopes,
                    const void* dev_kq_pool, const void* dev_vq_pool,
                    const int32_t* dev_q4_page_table, const int32_t* dev_q4_len,
                    int32_t max_q4_pages, int32_t q4_pool_pages,
                    const void* dev_k_pool, const void* dev_v_pool,
                    const int32_t* dev_tail_page_table, const int32_t* dev_tail_len,
                    int32_t max_tail_pages, int32_t pool_pages,
                    void* dev_out, int32_t B, int32_t n,
                    void* dev_ws, int64_t ws_bytes, void* stream);

/* ea_prefill_attn_q4 for models with rotary position embedding (Sec. 4.3, Eq. 9-10; the Llama models of the paper's
 * quantisation experiment): token i of the 4-bit part sits at position i, token i of the bfloat16 part at position
 * q4_len[b] + i, the n queries dev_q [B, n, H, d_head] (bfloat16, NOT rotated) are the last n tokens.  Here
 * q4_len[b] must be a multiple of page_tokens (whole pages, as ea_quantize_pages_q4 writes them; a remainder is
 * ignored and the bfloat16 part then counts from the rounded-down length).  A rotary prefill brings every cached key
 * back to d_head channels in a 16-bit workspace anyway (ea_prefill_attn_rope), so this call expands the codes on the
 * way there: staged as in ea_prefill_attn_q4_staged, then ea_prefill_attn_rope runs on the stage pools -- 3 + its
 * own 3 launches.  Page ids outside
 * their pool make that page's tokens vanish, as everywhere.
 *   dev_u_k [d_head, r_k] bfloat16, rope_base, d_head 64 or 128, r_k <= d_head: as ea_prefill_attn_rope
 *   dev_out [B, n, H, r_v] bfloat16
 *   dev_ws: ea_prefill_rope_q4_workspace_bytes(desc, B, n, max_q4_pages, max_tail_pages) bytes, 256-byte aligned
 *           (-1 if B * (max_q4_pages + max_tail_pages) pages cannot be indexed with 32 bits) */
EA_API int64_t ea_prefill_rope_q4_workspace_bytes(const ea_layer_desc* desc, int32_t B, int32_t n, int32_t max_q4_pages,
                    int32_t max_tail_pages);
EA_API int ea_prefill_attn_rope_q4(const ea_layer_desc* desc, const void* dev_q, const void* dev_u_k, double rope_base,
                    const void* dev_kq_pool, const void* dev_vq_pool,
                    const int32_t* dev_q4_page_table, const int32_t* dev_q4_len,
                    int32_t max_q4_pages, int32_t q4_pool_pages,
                    const void* dev_k_pool, const void* dev_v_pool,
                    const int32_t* dev_tail_page_table, const int32_t* dev_tail_len,
                    int32_t max_tail_pages, int32_t pool_pages,
                    void* dev_out, int32_t B, int32_t n,
                    void* dev_ws, int64_t ws_bytes, void* stream);

/* The generation step over such a cache for models with rotary position embedding (Sec. 4.3, Eq. 9-10; the Llama
 * models of the paper's quantisation experiment are of this kind): the 4-bit pools
 * hold the quantised rank-r keys k_r = k U^K of the one shared basis; every key is
 * dequantised, brought back to d_head channels (U^K k_r) and rotated by its position
 * (token i of the 4-bit part sits at position i, token i of the tail at position
 * q4_len[b] + i, the query is the newest token), exactly as ea_decode_attn_rope does
 * for the bfloat16 cache.  q4_len[b] must be a multiple of the key group (64 or 128).
 *   dev_q [B, H, d_head] float, NOT rotated; dev_u_k [d_head, r_k] bfloat16; rope_base as in
 *   ea_decode_attn_rope; n_splits = 0 picks ea_decode_rope_auto_splits; workspace
 *   ea_decode_q4_workspace_bytes(desc, B, n_splits).  d_head 64 or 128, r_k <= d_head. */
EA_API int ea_decode_attn_rope_q4(const ea_layer_desc* desc, const float* dev_q, const void* dev_u_k, double rope_base,
                    const void* dev_kq_pool, const void* dev_vq_pool,
                    const int32_t* dev_q4_page_table, const int32_t* dev_q4_len,
                    int32_t max_q4_pages, int32_t q4_pool_pages,
                    const void* dev_k_pool, const void* dev_v_pool,
                    const int32_t* dev_tail_page_table, const int32_t* dev_tail_len,
                    int32_t max_tail_pages, int32_t pool_pages,
                    float* dev_out, int32_t B, int32_t n_splits,
                    void* dev_ws, int64_t ws_bytes, void* stream);

/* ---- attention statistics for token-eviction policies ----------------------- */

/* The paper combines the rank-r cache with H2O token pruning (results, "Eigen
 * Attention with token pruning"): H2O keeps the tokens that have received the most
 * attention so far plus the most recent ones.  What it accumulates is the softmax
 * probability every cached token receives from each new query; in the rank-r space
 * that is the p of Eq. (3) with Eq. (7)'s operands.  This call adds, for the queries
 * dev_q_r [B, H, r_k] (float) of one generation step,
 *   dev_mass[b, g, t] += sum over the query heads i of kv head g of p_i[t],  t < seq_len[b]
 * (position-free scores, as ea_decode_attn; entries t >= seq_len[b] are not touched).
 * The policy stays with the caller: a dropped token's slot is overwritten by the next
 * append (pass the slot as that sequence's position to ea_project_qkv), because the
 * position-free cache does not care where a token sits.
 *   dev_mass [B, H_kv, max_pages * page_tokens] float
 *   dev_ws   ea_attn_mass_workspace_bytes(desc, B, max_pages) bytes, 16-byte aligned
 * Reads the keys once (the values not at all).  H / H_kv <= 16.
 * The accumulator is updated with plain loads and stores: calls that overlap in time (other streams) must not
 * share dev_mass or dev_ws. */
EA_API int64_t ea_attn_mass_workspace_bytes(const ea_layer_desc* desc, int32_t B, int32_t max_pages);
EA_API int ea_attn_mass(const ea_layer_desc* desc, const float* dev_q_r, const void* dev_k_pool,
                    const int32_t* dev_page_table, const int32_t* dev_seq_len, float* dev_mass,
                    int32_t B, int32_t max_pages, int32_t pool_pages,
                    void* dev_ws, int64_t ws_bytes, void* stream);

/* ea_decode_attn and ea_attn_mass in one pass over the cache (bfloat16 layers; the position-free form): the
 * attention kernel also stores its scaled scores, the split merge each row's maximum and normaliser, and a
 * last kernel turns the scores into probabilities and adds them to dev_mass -- so the keys are read once for
 * the output and the statistic.  Arguments as in ea_decode_attn plus dev_mass as in ea_attn_mass.
 *   n_splits 0 = ea_decode_auto_splits; dev_ws ea_decode_attn_mass_workspace_bytes(desc, B, max_pages, n_splits)
 *   bytes (n_splits >= 1 there), 16-byte aligned, always required.  EA_F32 layers: EA_ERR_SHAPE (call the two
 *   separately).  H / H_kv <= 16.
 * The probabilities are normalised with the attention kernel's own row sum (of probabilities rounded to
 * bfloat16), so they can differ from ea_attn_mass's by one bfloat16 step, relative; each row still sums to
 * H / H_kv within 2e-3.  dev_out is computed as by ea_decode_attn with the same n_splits. */
EA_API int64_t ea_decode_attn_mass_workspace_bytes(const ea_layer_desc* desc, int32_t B, int32_t max_pages,
                                                   int32_t n_splits);
EA_API int ea_decode_attn_mass(const ea_layer_desc* desc, const float* dev_q_r, const void* dev_k_pool,
                           const void* dev_v_pool, const int32_t* dev_page_table, const int32_t* dev_seq_len,
                           float* dev_out, float* dev_mass, int32_t B, int32_t max_pages, int32_t pool_pages,
                           int32_t n_splits, void* dev_ws, int64_t ws_bytes, void* stream);

/* Rotary models after token pruning (results, "Eigen Attention with token pruning": the paper's table is on
 * Llama models, whose attention is the form of Sec. 4.3, Eq. (10)).  A token that stays in the cache keeps the
 * position it had in the text, so once tokens have been dropped the key in cache slot t is no longer at position t:
 *   s_t = rot(q, q_pos[b]) . rot(U^K k_r[t], slot_pos[b][t]) / sqrt(d_h),  o = Softmax(s) V_r
 * ea_decode_attn_rope_pos is ea_decode_attn_rope with those positions given explicitly.  The cache itself is
 * unchanged (rank-r keys, never rotated), so a freed slot is overwritten by ea_project_qkv_rope (pass the slot as
 * that sequence's length) and the caller writes the new token's position into dev_slot_pos.
 *   dev_slot_pos [B, pos_stride] int32: position in the text of the token in logical slot t of sequence b
 *                (slot = index into the sequence's pages, as everywhere); pos_stride >= max_pages * page_tokens;
 *                entries of slots >= seq_len[b] are read (whole 64-token tiles) but not used
 *   dev_q_pos    [B] int32: position of the query
 *   positions must lie in [0, 2^24): the kernel forms angle = position * theta_j exactly from single-precision
 *   parts (EA_F32 layers: in double precision); only position differences enter a score
 *   everything else as in ea_decode_attn_rope (n_splits 0 = ea_decode_rope_auto_splits, dev_ws
 *   ea_decode_workspace_bytes when n_splits > 1).
 * Errors: EA_ERR_ARG also for pos_stride below the page table's capacity; EA_ERR_ALIGN for position arrays that are
 * not 4-byte aligned.
 *
 * ea_decode_attn_mass_rope_pos also adds the attention probability every slot received to dev_mass, as
 * ea_decode_attn_mass does for the position-free form (bfloat16 layers; dev_mass [B, H_kv, max_pages * page_tokens]
 * float; dev_ws ea_decode_attn_mass_workspace_bytes(desc, B, max_pages, n_splits) bytes, always required;
 * H / H_kv <= 16). */
EA_API int ea_decode_attn_rope_pos(const ea_layer_desc* desc, const float* dev_q, const void* dev_u_k, double rope_base,
                               const void* dev_k_pool, const void* dev_v_pool, const int32_t* dev_page_table,
                               const int32_t* dev_seq_len, const int32_t* dev_slot_pos, int32_t pos_stride,
                               const int32_t* dev_q_pos, float* dev_out, int32_t B, int32_t max_pages,
                               int32_t pool_pages, int32_t n_splits, void* dev_ws, int64_t ws_bytes, void* stream);
EA_API int ea_decode_attn_mass_rope_pos(const ea_layer_desc* desc, const float* dev_q, const void* dev_u_k,
                                    double rope_base, const void* dev_k_pool, const void* dev_v_pool,
                                    const int32_t* dev_page_table, const int32_t* dev_seq_len,
                                    const int32_t* dev_slot_pos, int32_t pos_stride, const int32_t* dev_q_pos,
                                    float* dev_out, float* dev_mass, int32_t B, int32_t max_pages, int32_t pool_pages,
                                    int32_t n_splits, void* dev_ws, int64_t ws_bytes, void* stream);

/* Output projection from rank r_v: y = [o_1 .. o_H] W^O' with
 * W^O'_i = U^V_{g(i)}^T W^O_i (Eq. 2, second line, and Eq. 8).
 *   dev_o    [M, H*r_v] float (o_dtype EA_F32) or bfloat16 (EA_BF16), M = B*T
 *   dev_wo   packed by ea_pack_weight from [d, H*r_v] out-major: row a holds
 *            column a of the stacked W^O'
 *   dev_y    [M, d] desc dtype.
 * Requires (H*r_v) % 32 == 0 for EA_BF16 (% 4 for EA_F32). */
EA_API int ea_out_proj(const ea_layer_desc* desc, const void* dev_o, int32_t o_dtype, const void* dev_wo,
                void* dev_y, int32_t M, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* EIGENATTN_H */
