"""Plain CPU oracle of the integer group quantisation of the rank-r KV cache and of attention over it.

TEST INFRASTRUCTURE ONLY -- never imported by the product package, shares no code with the HIP kernels.

What the paper fixes ("Eigen Attention with Quantization" paragraph of the results, and the quantisation table
of the appendix): the rank-r cache is quantised to integers of a few bits in groups; keys are quantised per
CHANNEL (the values that share a scale are one channel's values over a group of tokens), values per TOKEN (one
token's values over a group of channels); precisions 3-4 bits and group sizes 16-128 for the compressed cache.
The paper prints no rounding rule, no zero-point convention and no storage type for the scales, so everything
below that goes beyond "uniform integer grid per group" is this build's reading, and the functions that depend
on that reading are PARITY UNPINNED with respect to the paper; they are pinned only to what the mathematics
fixes for any such quantiser (see tests/test_oracle_quant.py): codes in range, the round-trip error bound of
half a step, exactness on constant groups and on values that lie on the grid, extremes mapping to the end
codes, invariance of the codes under the affine map that the scale and zero absorb, and attention over the
quantised cache being plain attention over the dequantised values.

One thing here IS pinned to the paper: quantized_cache_bytes, the size accounting (bits + 16 / group per scalar), reproduces
all 15 KV-cache sizes of the appendix's quantisation table.

The reading:
  * 4 bits (or 3: `bits`, the two precisions of the paper's Eigen Attention rows; 15 and 7 below are 2^bits - 1),
    asymmetric: a group with minimum lo and maximum hi gets  zero = fp16(lo),
    scale = fp16((hi - lo) / 15), both first clamped to the finite fp16 range; the quotient is taken in
    float32.  A group whose scale rounds to 0 (all values equal, or a spread below fp16's smallest step)
    gets code 0 everywhere.
  * code = clip(rint((x - zero) / scale), 0, 15) with x, zero, scale as float32, IEEE division, round half
    to even: the integer decision is taken in float32 on both sides of the parity tests.
  * value = scale * code + zero (evaluated in float64 here).
  * keys: groups of 64 consecutive tokens per channel (token 64 g .. 64 g + 63 of a sequence), or -- the
    group size of the appendix table's 4-bit Eigen Attention rows -- of 128 (group_tokens = 128);
    values: one group per token over all r_v channels.
  * only whole key groups are quantised; the newest tokens of a sequence stay in the 16-bit cache
    until their group is complete (the key groups need all their tokens before a scale exists).
"""
from __future__ import annotations

import numpy as np

from . import eigen_attention as ea_oracle

GROUP_TOKENS = 64
LEVELS = 15          # 4 bits: codes 0 .. 15
F16_MAX = 65504.0


def _levels(bits: int) -> int:
    assert bits in (3, 4)
    return LEVELS if bits == 4 else 7


def _scale_zero(lo, hi, levels: int = LEVELS):
    """fp16 scale and zero of groups with minima lo and maxima hi (float32 arrays)."""
    lo = np.clip(lo.astype(np.float32), -F16_MAX, F16_MAX)
    hi = np.clip(hi.astype(np.float32), -F16_MAX, F16_MAX)
    step = np.minimum((hi - lo) / np.float32(levels), np.float32(F16_MAX))
    return step.astype(np.float16), lo.astype(np.float16)


def _codes(x, scale, zero, levels: int = LEVELS):
    """clip(rint((x - zero) / scale), 0, levels) in float32; scale == 0 gives code 0."""
    x32 = x.astype(np.float32)
    s32 = scale.astype(np.float32)
    z32 = zero.astype(np.float32)
    safe = np.where(s32 > 0, s32, np.float32(1.0))
    q = np.rint((x32 - z32) / safe)
    q = np.where(s32 > 0, q, np.float32(0.0))
    return np.clip(q, 0, levels).astype(np.uint8)


def quantize_keys(K, group_tokens: int = GROUP_TOKENS, bits: int = 4):
    """K [n, r] (n a multiple of the group) -> codes uint8 [n, r], scale fp16 [n/group, r], zero fp16 [n/group, r]:
    one scale per channel and group of `group_tokens` consecutive tokens; codes 0 .. 2^bits - 1."""
    n, r = K.shape
    assert n % group_tokens == 0
    Kg = K.astype(np.float32).reshape(n // group_tokens, group_tokens, r)
    scale, zero = _scale_zero(Kg.min(axis=1), Kg.max(axis=1), _levels(bits))
    codes = _codes(Kg, scale[:, None, :], zero[:, None, :], _levels(bits)).reshape(n, r)
    return codes, scale, zero


def quantize_values(V, bits: int = 4):
    """V [n, r] -> codes uint8 [n, r], scale fp16 [n], zero fp16 [n]: one scale per token."""
    V32 = V.astype(np.float32)
    scale, zero = _scale_zero(V32.min(axis=1), V32.max(axis=1), _levels(bits))
    return _codes(V32, scale[:, None], zero[:, None], _levels(bits)), scale, zero


def dequantize_keys(codes, scale, zero):
    n, r = codes.shape
    group_tokens = n // scale.shape[0]                     # the scales say how long a group is
    c = codes.astype(np.float64).reshape(n // group_tokens, group_tokens, r)
    return (scale.astype(np.float64)[:, None, :] * c + zero.astype(np.float64)[:, None, :]).reshape(n, r)


def dequantize_values(codes, scale, zero):
    return scale.astype(np.float64)[:, None] * codes.astype(np.float64) + zero.astype(np.float64)[:, None]


def quantized_view(K, V, n_quant: int, group_tokens: int = GROUP_TOKENS, bits: int = 4):
    """The cache as attention sees it when its first n_quant tokens (a multiple of the key group) are held in 4
    bits: K [H_kv, n, r_k], V [H_kv, n, r_v] -> arrays of the same shapes, the prefix replaced by its
    quantise-dequantise round trip, the rest untouched."""
    assert n_quant % group_tokens == 0 and n_quant <= K.shape[1]
    Kq, Vq = np.array(K, dtype=np.float64), np.array(V, dtype=np.float64)
    for h in range(K.shape[0]):
        if n_quant:
            Kq[h, :n_quant] = dequantize_keys(*quantize_keys(K[h, :n_quant], group_tokens, bits))
            Vq[h, :n_quant] = dequantize_values(*quantize_values(V[h, :n_quant], bits))
    return Kq, Vq


def quantized_cache_bytes(n_elements, bits: int, group: int, meta_bits_per_group: int = 16) -> float:
    """Bytes of n_elements cached scalars held as `bits`-bit codes in groups of `group`, every group carrying
    meta_bits_per_group bits of metadata: n * (bits + meta / group) / 8.
    The KV-cache sizes the appendix's quantisation table prints (15 rows: Llama-2-7b and -13b, standard and Eigen
    Attention at 0.6x, 2-4 bits, groups of 16-512, sequence length 2048, GB = 2^30 bytes) are reproduced by this
    count with 16 bits of metadata per group -- one 16-bit scale -- and by neither 0 nor 32 (a pin).  The paper does
    not say whether a zero point exists or where it is kept; this build's format stores a 16-bit scale AND a 16-bit
    zero per group (32 bits), so its pools are larger than the paper's accounting: see bits_per_element_q4."""
    return n_elements * (bits + meta_bits_per_group / group) / 8.0


def bits_per_element_q4(r_k: int, r_v: int, group_tokens: int = GROUP_TOKENS, bits: int = 4):
    """Bits per cached scalar of this build's 4-bit (3-bit) format, without layout padding: keys in groups of 64 (or
    128) tokens, values in groups of r_v channels, 32 bits of metadata (fp16 scale, fp16 zero) per group."""
    return bits + 32 / group_tokens, bits + 32 / r_v


def decode_attention_quantized(q_r, K_list, V_list, n_quant, d_head: int, alibi_slopes=None,
                               group_tokens: int = GROUP_TOKENS, bits: int = 4):
    """Generation-phase attention (Eq. 3 in the rank-r space) of one new token per sequence over a cache whose
    first n_quant[b] tokens are quantised: plain attention over the dequantised values (with the ALiBi bias of the
    MPT models when slopes are given: it involves positions only, so quantisation does not touch it).
    q_r [B, H, r_k]; K_list[b] [H_kv, n_b, r_k]; V_list[b] [H_kv, n_b, r_v]."""
    views = [quantized_view(K_list[b], V_list[b], int(n_quant[b]), group_tokens, bits) for b in range(len(K_list))]
    cache = ea_oracle.RankCache.from_arrays([v[0] for v in views], [v[1] for v in views])
    return ea_oracle.decode_attention(q_r, cache, d_head, alibi_slopes=alibi_slopes)


def decode_attention_rope_quantized(q, K_list, V_list, n_quant, Uk, d_head: int, base: float = 10000.0,
                                    group_tokens: int = GROUP_TOKENS, bits: int = 4):
    """The same for models with rotary position embedding (Sec. 4.3, Eq. 9-10): the cached rank-r keys (of the one
    shared basis Uk) are quantised BEFORE they are brought back to d_head channels and rotated, so this is the
    rotary generation-phase attention over the dequantised rank-r keys and values.
    q [B, H, d_head] (not rotated); the rest as decode_attention_quantized."""
    rope_views = [quantized_view(K_list[b], V_list[b], int(n_quant[b]), group_tokens, bits) for b in range(len(K_list))]
    cache = ea_oracle.RankCache.from_arrays([v[0] for v in rope_views], [v[1] for v in rope_views])
    return ea_oracle.decode_attention_rope(q, cache, Uk, d_head, base)


def prefill_attention_quantized(q_r, K_list, V_list, n_quant, d_head: int, group_tokens: int = GROUP_TOKENS,
                                bits: int = 4, alibi_slopes=None):
    """Prefill-phase attention (Eq. 2 in the rank-r space, causal) of the LAST n tokens of every sequence over a
    cache whose first n_quant[b] tokens are quantised: plain causal attention over the dequantised values.
    q_r [B, n, H, r_k]; K_list[b] [H_kv, len_b, r_k]; V_list[b] [H_kv, len_b, r_v]; n <= len_b - n_quant[b] (the
    queries belong to tokens that are still held in 16 bits).  With alibi_slopes [H] the ALiBi bias of the MPT models
    is added to the scores (positions only: quantisation does not touch it)."""
    n = np.asarray(q_r).shape[1]
    for b in range(len(K_list)):
        assert n <= K_list[b].shape[1] - int(n_quant[b])
    prefill_views = [quantized_view(K_list[b], V_list[b], int(n_quant[b]), group_tokens, bits)
                     for b in range(len(K_list))]
    cache = ea_oracle.RankCache.from_arrays([v[0] for v in prefill_views], [v[1] for v in prefill_views])
    return ea_oracle.prefill_attention(q_r, cache, d_head, alibi_slopes=alibi_slopes)


def prefill_attention_rope_quantized(q, K_list, V_list, n_quant, Uk, d_head: int, base: float = 10000.0,
                                     group_tokens: int = GROUP_TOKENS, bits: int = 4):
    """prefill_attention_quantized for models with rotary position embedding (Sec. 4.3, Eq. 9-10; the Llama models of
    the quantisation experiment): causal rotary attention of the LAST n tokens over the dequantised rank-r keys and
    values, token t of a sequence at position t whether it is held in codes or in 16 bits.
    q [B, n, H, d_head] (not rotated); the rest as prefill_attention_quantized."""
    n = np.asarray(q).shape[1]
    for b in range(len(K_list)):
        assert n <= K_list[b].shape[1] - int(n_quant[b])
    rope_prefill_views = [quantized_view(K_list[b], V_list[b], int(n_quant[b]), group_tokens, bits)
                          for b in range(len(K_list))]
    cache = ea_oracle.RankCache.from_arrays([v[0] for v in rope_prefill_views], [v[1] for v in rope_prefill_views])
    return ea_oracle.prefill_attention_rope(q, cache, Uk, d_head, base)


def chunked_prefill_quantized(q_r, K, V, chunk: int, d_head: int, group_tokens: int = GROUP_TOKENS, bits: int = 4):
    """A prompt of n tokens prefilled chunk by chunk, every chunk's keys and values quantised as soon as the chunk
    has been attended -- so that at no time more than one chunk exists in 16 bits (what the quantisation paragraph
    of the results amounts to for a long prompt): the queries of chunk c see the tokens of chunks < c as their
    quantise-dequantise round trip and those of chunk c itself, causally, as they are.
    q_r [n, H, r_k], K [H_kv, n, r_k], V [H_kv, n, r_v] of ONE sequence; chunk a multiple of the key group;
    returns o [n, H, r_v]."""
    q_r = np.asarray(q_r, np.float64)
    n = q_r.shape[0]
    assert chunk % group_tokens == 0
    out = np.zeros((n, q_r.shape[1], V.shape[2]))
    for c0 in range(0, n, chunk):
        c1 = min(n, c0 + chunk)
        out[c0:c1] = prefill_attention_quantized(q_r[None, c0:c1], [K[:, :c1]], [V[:, :c1]], [c0], d_head,
                                                 group_tokens, bits)[0]
    return out
