"""Plain fp64 CPU oracle: attention in a low-rank space over a rank-r KV cache.

TEST INFRASTRUCTURE ONLY -- never imported by the product package, shares no
code with the HIP kernels.  Everything is float64 numpy, one (batch, head) at a
time, in the order and notation of the paper:

  Eq. (1)  Q_i = X W_i^Q,  K_i = X W_i^K,  V_i = X W_i^V          (Background)
  Eq. (2)  h_i = Softmax(Q_i K_i^T / sqrt(d_h)) V_i ; MHA = [h_1..h_h] W^O
  LLM-Inference paragraph: K_i <- Concat(K_i, k_i), V_i <- Concat(V_i, v_i)
  Eq. (3)  h_i = Softmax(q_i K_i^T / sqrt(d_h)) V_i                (generation)
  Eq. (6)  Q' = Q U^K U^K^T, K' = K U^K U^K^T, V' = V U^V U^V^T    (Sec. 4.2)
  Eq. (7)  A' = Softmax(Q' K'^T / sqrt(d_h)) V'
  Eq. (8)  W^Q' = W^Q U^K, W^K' = W^K U^K, W^V' = W^V U^V, W^O' = U^V^T W^O
  Table 1  KV-cache size, parameter and generation-FLOP closed forms
  Eq. (9)-(10), Sec. 4.3: the variant for RoPE models (full-rank query, rank-r keys of ONE shared
           basis brought back to d_h channels before the rotation), generation and prefill
  ALiBi bias (the MPT family's position scheme, named in Sec. 5.1; definition of the ALiBi paper)

Row-vector convention (x W) throughout, as in Eq. (1).  With grouped-query
attention query head i uses the bases of its KV head g(i) = i // (H / H_kv).

Pins (tests/test_oracle_pins.py): r = d_h equals standard attention; the
rank-space form equals the project-back form of Eq. (6)-(7); softmax rows sum
to one; brute force on tiny inputs; closed-form special cases; basis-rotation
invariance; Table 1 and the Introduction's 256 GB worked example; for the RoPE variant the rotation's
definition and relative-position invariance, equality with standard RoPE attention at r = d_h and
whenever the keys lie in the basis' span, prefill rows = decode results of their prefixes; for ALiBi
the bias definition, its limits and the softmax shift invariance.
No function here is "parity unpinned" with respect to its stated definition; the ALiBi definition itself
comes from the ALiBi paper (this paper prints no formula for it).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

F64 = np.float64


@dataclass
class OpCounter:
    """Counts multiply-accumulates and cache elements as the oracle runs (Table 1)."""
    macs: int = 0

    def add(self, n: int) -> None:
        self.macs += int(n)


def _kv_head_of(i: int, n_heads: int, n_kv_heads: int) -> int:
    assert n_heads % n_kv_heads == 0
    return i // (n_heads // n_kv_heads)


# --------------------------------------------------------------------------
# Eq. (8): fold the bases into the projection weights (done once, offline)
# --------------------------------------------------------------------------
def fold_weights(Wq, Wk, Wv, Wo, Uk, Uv, n_heads: int, n_kv_heads: int):
    """Eq. (8).

    Wq: [d, H*d_h]; Wk, Wv: [d, H_kv*d_h]; Wo: [H*d_h, d] (Eq. 2: heads are
    concatenated, so W^O_i is the i-th block of d_h rows).
    Uk: [H_kv, d_h, r_k], Uv: [H_kv, d_h, r_v], orthonormal columns.
    Returns Wq_f [H, d, r_k], Wk_f [H_kv, d, r_k], Wv_f [H_kv, d, r_v], Wo_f [H, r_v, d].
    """
    Wq, Wk, Wv, Wo = (np.asarray(a, F64) for a in (Wq, Wk, Wv, Wo))
    Uk, Uv = np.asarray(Uk, F64), np.asarray(Uv, F64)
    d = Wq.shape[0]
    d_h = Uk.shape[1]
    assert Wq.shape == (d, n_heads * d_h) and Wo.shape == (n_heads * d_h, d)
    assert Wk.shape == (d, n_kv_heads * d_h) and Wv.shape == (d, n_kv_heads * d_h)
    Wq_f, Wo_f, Wk_f, Wv_f = [], [], [], []
    for i in range(n_heads):
        g = _kv_head_of(i, n_heads, n_kv_heads)
        Wq_i = Wq[:, i * d_h:(i + 1) * d_h]
        Wo_i = Wo[i * d_h:(i + 1) * d_h, :]
        Wq_f.append(Wq_i @ Uk[g])            # W^Q' = W^Q U^K
        Wo_f.append(Uv[g].T @ Wo_i)          # W^O' = U^V^T W^O
    for g in range(n_kv_heads):
        Wk_g = Wk[:, g * d_h:(g + 1) * d_h]
        Wv_g = Wv[:, g * d_h:(g + 1) * d_h]
        Wk_f.append(Wk_g @ Uk[g])            # W^K' = W^K U^K
        Wv_f.append(Wv_g @ Uv[g])            # W^V' = W^V U^V
    return np.stack(Wq_f), np.stack(Wk_f), np.stack(Wv_f), np.stack(Wo_f)


# --------------------------------------------------------------------------
# Eq. (1) with the folded weights
# --------------------------------------------------------------------------
def project_qkv(x, Wq_f, Wk_f, Wv_f, counter: Optional[OpCounter] = None):
    """x [M, d] -> q_r [M, H, r_k], k_r [M, H_kv, r_k], v_r [M, H_kv, r_v]."""
    x = np.asarray(x, F64)
    M, d = x.shape
    q = np.stack([x @ np.asarray(W, F64) for W in Wq_f], axis=1)
    k = np.stack([x @ np.asarray(W, F64) for W in Wk_f], axis=1)
    v = np.stack([x @ np.asarray(W, F64) for W in Wv_f], axis=1)
    if counter is not None:
        counter.add(M * d * (q.shape[1] * q.shape[2] + k.shape[1] * k.shape[2] + v.shape[1] * v.shape[2]))
    return q, k, v


# --------------------------------------------------------------------------
# The rank-r KV cache: K <- Concat(K, k), V <- Concat(V, v)
# --------------------------------------------------------------------------
@dataclass
class RankCache:
    """Per sequence b: K[b] is [H_kv, len_b, r_k] and V[b] is [H_kv, len_b, r_v]."""
    n_kv_heads: int
    r_k: int
    r_v: int
    K: List[np.ndarray] = field(default_factory=list)
    V: List[np.ndarray] = field(default_factory=list)

    @classmethod
    def empty(cls, batch: int, n_kv_heads: int, r_k: int, r_v: int) -> "RankCache":
        c = cls(n_kv_heads, r_k, r_v)
        c.K = [np.zeros((n_kv_heads, 0, r_k), F64) for _ in range(batch)]
        c.V = [np.zeros((n_kv_heads, 0, r_v), F64) for _ in range(batch)]
        return c

    @classmethod
    def from_arrays(cls, K_list, V_list) -> "RankCache":
        K_list = [np.asarray(a, F64) for a in K_list]
        V_list = [np.asarray(a, F64) for a in V_list]
        c = cls(K_list[0].shape[0], K_list[0].shape[2], V_list[0].shape[2])
        c.K, c.V = K_list, V_list
        return c

    @property
    def batch(self) -> int:
        return len(self.K)

    def seq_len(self, b: int) -> int:
        return self.K[b].shape[1]

    def append(self, b: int, k_new, v_new) -> None:
        """k_new [T, H_kv, r_k], v_new [T, H_kv, r_v] go to positions len_b .. len_b+T-1."""
        k_new = np.asarray(k_new, F64).transpose(1, 0, 2)
        v_new = np.asarray(v_new, F64).transpose(1, 0, 2)
        self.K[b] = np.concatenate([self.K[b], k_new], axis=1)
        self.V[b] = np.concatenate([self.V[b], v_new], axis=1)

    def elements(self) -> int:
        """Number of cached scalars actually held (Table 1, first row)."""
        return int(sum(a.size for a in self.K) + sum(a.size for a in self.V))


def softmax(s):
    """Softmax of a score vector; the max is subtracted first (same value, no overflow)."""
    s = np.asarray(s, F64)
    e = np.exp(s - np.max(s))
    return e / np.sum(e)


# --------------------------------------------------------------------------
# Eq. (3) in rank space: one new query per sequence over the whole cache
# --------------------------------------------------------------------------
def alibi_bias(slope: float, pos_q: int, n_keys: int):
    """ALiBi (Sec. 5.1 names it as the MPT models' position scheme; the definition is that of the ALiBi paper):
    the score of query position i against key position j <= i gets -slope * (i - j), slope > 0 per head."""
    return -float(slope) * (pos_q - np.arange(n_keys, dtype=F64))


def decode_attention(q_r, cache: RankCache, d_head: int, counter: Optional[OpCounter] = None,
                     return_probs: bool = False, alibi_slopes=None):
    """q_r [B, H, r_k] -> o [B, H, r_v].

    s_t = q_r . K_r[t] / sqrt(d_h) for every cached token t (the one just
    appended included), p = Softmax(s), o = sum_t p_t V_r[t].  The divisor is
    sqrt(d_h), not sqrt(r): Eq. (7) keeps it because the rank-space product
    equals Q' K'^T of the d_h-dimensional projected vectors.
    With alibi_slopes [H] the ALiBi bias of the query's distance to each key is added to s.
    """
    q_r = np.asarray(q_r, F64)
    B, H, _ = q_r.shape
    out = np.zeros((B, H, cache.r_v), F64)
    probs = []
    for b in range(B):
        n = cache.seq_len(b)
        if n == 0:
            raise ValueError("decode over an empty sequence")
        for i in range(H):
            g = _kv_head_of(i, H, cache.n_kv_heads)
            K, V = cache.K[b][g], cache.V[b][g]
            s = (K @ q_r[b, i]) / math.sqrt(d_head)
            if alibi_slopes is not None:
                s = s + alibi_bias(alibi_slopes[i], n - 1, n)
            p = softmax(s)
            out[b, i] = p @ V
            if return_probs:
                probs.append(p)
            if counter is not None:
                counter.add(K.size + V.size)
    return (out, probs) if return_probs else out


# --------------------------------------------------------------------------
# Eq. (2) in rank space with a causal mask: the prefill phase
# --------------------------------------------------------------------------
def prefill_attention(q_r, cache: RankCache, d_head: int, alibi_slopes=None):
    """q_r [B, n, H, r_k] -> o [B, n, H, r_v].

    The n queries of sequence b are its LAST n cached positions: query j sits
    at absolute position len_b - n + j and attends to positions <= its own
    (decoder-only models are causal; the diagonal is included).
    """
    q_r = np.asarray(q_r, F64)
    B, n, H, _ = q_r.shape
    out = np.zeros((B, n, H, cache.r_v), F64)
    for b in range(B):
        L = cache.seq_len(b)
        assert L >= n
        for i in range(H):
            g = _kv_head_of(i, H, cache.n_kv_heads)
            K, V = cache.K[b][g], cache.V[b][g]
            for j in range(n):
                pos = L - n + j
                s = (K[:pos + 1] @ q_r[b, j, i]) / math.sqrt(d_head)
                if alibi_slopes is not None:
                    s = s + alibi_bias(alibi_slopes[i], pos, pos + 1)
                out[b, j, i] = softmax(s) @ V[:pos + 1]
    return out


# --------------------------------------------------------------------------
# Eq. (2) second line with W^O' of Eq. (8)
# --------------------------------------------------------------------------
def out_proj(o, Wo_f, counter: Optional[OpCounter] = None):
    """o [M, H, r_v], Wo_f [H, r_v, d] -> y [M, d] = sum_i o_i W^O'_i."""
    o = np.asarray(o, F64)
    Wo_f = np.asarray(Wo_f, F64)
    M, H, r_v = o.shape
    y = np.zeros((M, Wo_f.shape[2]), F64)
    for i in range(H):
        y += o[:, i, :] @ Wo_f[i]
    if counter is not None:
        counter.add(M * H * r_v * Wo_f.shape[2])
    return y


# --------------------------------------------------------------------------
# One generation step of the low-rank attention block (all rows of the path)
# --------------------------------------------------------------------------
def decode_step(x, folded, cache: RankCache, d_head: int, counter: Optional[OpCounter] = None, alibi_slopes=None):
    """x [B, d]: project, append one token per sequence, attend, project out -> y [B, d].  With alibi_slopes [H]
    (the MPT family of Sec. 5.1) the attention adds each head's distance bias to its scores."""
    Wq_f, Wk_f, Wv_f, Wo_f = folded
    q, k, v = project_qkv(x, Wq_f, Wk_f, Wv_f, counter)
    for b in range(x.shape[0]):
        cache.append(b, k[b:b + 1], v[b:b + 1])
    o = decode_attention(q, cache, d_head, counter, alibi_slopes=alibi_slopes)
    return out_proj(o, Wo_f, counter)


def prefill_step(x, folded, cache: RankCache, d_head: int):
    """x [B, n, d]: project, append n tokens per sequence, causal attention, project out."""
    Wq_f, Wk_f, Wv_f, Wo_f = folded
    x = np.asarray(x, F64)
    B, n, d = x.shape
    q, k, v = project_qkv(x.reshape(B * n, d), Wq_f, Wk_f, Wv_f)
    q = q.reshape(B, n, *q.shape[1:])
    k = k.reshape(B, n, *k.shape[1:])
    v = v.reshape(B, n, *v.shape[1:])
    for b in range(B):
        cache.append(b, k[b], v[b])
    o = prefill_attention(q, cache, d_head)
    y = out_proj(o.reshape(B * n, *o.shape[2:]), Wo_f)
    return y.reshape(B, n, -1)


# --------------------------------------------------------------------------
# Standard (full-rank) attention, Eq. (1)-(3): the comparison baseline
# --------------------------------------------------------------------------
def standard_attention_block(x_hist, Wq, Wk, Wv, Wo, n_heads: int, n_kv_heads: int, causal_all: bool = False):
    """x_hist [n, d] (one sequence).  Returns the block output for the LAST
    token (generation, Eq. 3) or for every token with a causal mask (prefill)."""
    x_hist = np.asarray(x_hist, F64)
    Wq, Wk, Wv, Wo = (np.asarray(a, F64) for a in (Wq, Wk, Wv, Wo))
    n, d = x_hist.shape
    d_h = Wq.shape[1] // n_heads
    rows = range(n) if causal_all else [n - 1]
    heads_out = np.zeros((len(rows), n_heads * d_h), F64)
    for i in range(n_heads):
        g = _kv_head_of(i, n_heads, n_kv_heads)
        Q = x_hist @ Wq[:, i * d_h:(i + 1) * d_h]
        K = x_hist @ Wk[:, g * d_h:(g + 1) * d_h]
        V = x_hist @ Wv[:, g * d_h:(g + 1) * d_h]
        for ri, j in enumerate(rows):
            s = (K[:j + 1] @ Q[j]) / math.sqrt(d_h)
            heads_out[ri, i * d_h:(i + 1) * d_h] = softmax(s) @ V[:j + 1]
    return heads_out @ Wo


# --------------------------------------------------------------------------
# Eq. (6)-(7): the same quantity computed in d_h space (project-back form)
# --------------------------------------------------------------------------
def eigen_attention_block_projected_back(x_hist, Wq, Wk, Wv, Wo, Uk, Uv, n_heads: int, n_kv_heads: int,
                                         causal_all: bool = False):
    """Q' = Q U^K U^K^T, K' = K U^K U^K^T, V' = V U^V U^V^T, then Eq. (2) with the ORIGINAL W^O."""
    x_hist = np.asarray(x_hist, F64)
    Wq, Wk, Wv, Wo = (np.asarray(a, F64) for a in (Wq, Wk, Wv, Wo))
    n, d = x_hist.shape
    d_h = Wq.shape[1] // n_heads
    rows = range(n) if causal_all else [n - 1]
    heads_out = np.zeros((len(rows), n_heads * d_h), F64)
    for i in range(n_heads):
        g = _kv_head_of(i, n_heads, n_kv_heads)
        Pk = np.asarray(Uk[g], F64) @ np.asarray(Uk[g], F64).T
        Pv = np.asarray(Uv[g], F64) @ np.asarray(Uv[g], F64).T
        Qp = (x_hist @ Wq[:, i * d_h:(i + 1) * d_h]) @ Pk
        Kp = (x_hist @ Wk[:, g * d_h:(g + 1) * d_h]) @ Pk
        Vp = (x_hist @ Wv[:, g * d_h:(g + 1) * d_h]) @ Pv
        for ri, j in enumerate(rows):
            s = (Kp[:j + 1] @ Qp[j]) / math.sqrt(d_h)
            heads_out[ri, i * d_h:(i + 1) * d_h] = softmax(s) @ Vp[:j + 1]
    return heads_out @ Wo


# --------------------------------------------------------------------------
# Sec. 4.3 (Rotational Position Embedding): the variant for models with RoPE
# --------------------------------------------------------------------------
def rope_rotate(x, pos, base: float = 10000.0):
    """Rotary position embedding of d-dimensional rows x [.., d] at integer positions pos [..]:
    the pairs (x[2j], x[2j+1]) are rotated by the angle pos * base**(-2j/d)  (Eq. 9: Q R, K R).

    Reading (the paper cites the RoFormer definition and prints only "Q R"): adjacent channels form a
    pair; x'[2j] = x[2j] cos - x[2j+1] sin, x'[2j+1] = x[2j] sin + x[2j+1] cos."""
    x = np.asarray(x, F64)
    d = x.shape[-1]
    assert d % 2 == 0
    theta = np.asarray(base, F64) ** (-np.arange(0, d, 2, dtype=F64) / d)
    ang = np.asarray(pos, F64)[..., None] * theta
    c, sn = np.cos(ang), np.sin(ang)
    out = np.empty_like(x)
    out[..., 0::2] = x[..., 0::2] * c - x[..., 1::2] * sn
    out[..., 1::2] = x[..., 0::2] * sn + x[..., 1::2] * c
    return out


def decode_attention_rope(q, cache: RankCache, Uk, d_head: int, base: float = 10000.0):
    """Generation-phase Eigen Attention for a RoPE model (Sec. 4.3, Eq. 10).

    q [B, H, d_h]: the FULL-rank query of the new token (not projected, not yet rotated).
    cache.K[b][g]: rank-r_k keys k_r = k U^K; Uk [d_h, r_k] is ONE basis shared by all heads.
    Each cached key is brought back to d_h dimensions, k' = U^K k_r, then rotated to its position t;
    the query is rotated to its position len_b - 1 (the token just appended).  Values are untouched.
    """
    q = np.asarray(q, F64)
    Uk = np.asarray(Uk, F64)
    B, H, d_h = q.shape
    assert d_h == d_head and Uk.shape[0] == d_h
    out = np.zeros((B, H, cache.r_v), F64)
    for b in range(B):
        n = cache.seq_len(b)
        if n == 0:
            raise ValueError("decode over an empty sequence")
        for i in range(H):
            g = _kv_head_of(i, H, cache.n_kv_heads)
            K_up = cache.K[b][g] @ Uk.T                               # [n, d_h]: (U^K)^T applied back
            K_pos = rope_rotate(K_up, np.arange(n), base)
            q_pos = rope_rotate(q[b, i], n - 1, base)
            s = (K_pos @ q_pos) / math.sqrt(d_head)
            out[b, i] = softmax(s) @ cache.V[b][g]
    return out


def prefill_attention_rope(q, cache: RankCache, Uk, d_head: int, base: float = 10000.0):
    """Prefill-phase Eigen Attention for a RoPE model (Sec. 4.3, Eq. 10 with the causal mask of the prefill):
    q [B, n, H, d_h] full-rank and not rotated -> o [B, n, H, r_v].  Query j of sequence b sits at position
    len_b - n + j, is rotated to it, and attends to the cached keys at positions <= its own, each brought back
    to d_h channels with the shared basis and rotated to its position."""
    q = np.asarray(q, F64)
    Uk = np.asarray(Uk, F64)
    B, n, H, _ = q.shape
    out = np.zeros((B, n, H, cache.r_v), F64)
    for b in range(B):
        L = cache.seq_len(b)
        assert L >= n
        for i in range(H):
            g = _kv_head_of(i, H, cache.n_kv_heads)
            K_pos = rope_rotate(cache.K[b][g] @ Uk.T, np.arange(L), base)
            V = cache.V[b][g]
            for j in range(n):
                pos = L - n + j
                s = (K_pos[:pos + 1] @ rope_rotate(q[b, j, i], pos, base)) / math.sqrt(d_head)
                out[b, j, i] = softmax(s) @ V[:pos + 1]
    return out


def standard_rope_decode(q, K_full, V, d_head: int, base: float = 10000.0):
    """Standard attention with RoPE for one head: q [d_h] at position n-1, K_full [n, d_h], V [n, r_v]."""
    K_full = np.asarray(K_full, F64)
    n = K_full.shape[0]
    s = (rope_rotate(K_full, np.arange(n), base) @ rope_rotate(np.asarray(q, F64), n - 1, base)) / math.sqrt(d_head)
    return softmax(s) @ np.asarray(V, F64)


def fold_weights_rope(Wq, Wk, Wv, Wo, Uk_shared, Uv, n_heads: int, n_kv_heads: int):
    """Weight folding for a RoPE model (Sec. 4.3): W^Q stays as it is (the rotation acts on the full query),
    W^K'_g = W^K_g U^K with ONE basis U^K [d_h, r_k] for all heads; values and output as in Eq. (8).
    Returns Wq_h [H, d, d_h], Wk_f [H_kv, d, r_k], Wv_f [H_kv, d, r_v], Wo_f [H, r_v, d]."""
    Wq, Wk, Wv, Wo = (np.asarray(a, F64) for a in (Wq, Wk, Wv, Wo))
    Uk_shared, Uv = np.asarray(Uk_shared, F64), np.asarray(Uv, F64)
    d_h = Uk_shared.shape[0]
    Wq_h = [Wq[:, i * d_h:(i + 1) * d_h] for i in range(n_heads)]
    Wk_f = [Wk[:, g * d_h:(g + 1) * d_h] @ Uk_shared for g in range(n_kv_heads)]
    Wv_f = [Wv[:, g * d_h:(g + 1) * d_h] @ Uv[g] for g in range(n_kv_heads)]
    Wo_f = [Uv[_kv_head_of(i, n_heads, n_kv_heads)].T @ Wo[i * d_h:(i + 1) * d_h, :] for i in range(n_heads)]
    return np.stack(Wq_h), np.stack(Wk_f), np.stack(Wv_f), np.stack(Wo_f)


def decode_step_rope(x, folded, Uk_shared, cache: RankCache, d_head: int, base: float = 10000.0):
    """One generation step of a RoPE model: x [B, d] -> project (full q, rank-r k and v), append one token per
    sequence, attend with Eq. (10), project out -> y [B, d]."""
    Wq_h, Wk_f, Wv_f, Wo_f = folded
    q, k, v = project_qkv(x, Wq_h, Wk_f, Wv_f)
    for b in range(x.shape[0]):
        cache.append(b, k[b:b + 1], v[b:b + 1])
    return out_proj(decode_attention_rope(q, cache, Uk_shared, d_head, base), Wo_f)


def prefill_step_rope(x, folded, Uk_shared, cache: RankCache, d_head: int, base: float = 10000.0):
    """Prefill of a RoPE model: x [B, n, d] -> project, append n tokens per sequence, causal attention with
    Eq. (10), project out -> y [B, n, d]."""
    Wq_h, Wk_f, Wv_f, Wo_f = folded
    x = np.asarray(x, F64)
    B, n, d = x.shape
    q, k, v = project_qkv(x.reshape(B * n, d), Wq_h, Wk_f, Wv_f)
    q, k, v = (a.reshape(B, n, *a.shape[1:]) for a in (q, k, v))
    for b in range(B):
        cache.append(b, k[b], v[b])
    o = prefill_attention_rope(q, cache, Uk_shared, d_head, base)
    return out_proj(o.reshape(B * n, *o.shape[2:]), Wo_f).reshape(B, n, -1)


def standard_rope_attention_block(x_hist, Wq, Wk, Wv, Wo, n_heads: int, n_kv_heads: int, base: float = 10000.0):
    """Standard attention with RoPE (Eq. 9) for the LAST token of one sequence x_hist [n, d]: full-rank q and k,
    both rotated to their positions."""
    x_hist = np.asarray(x_hist, F64)
    Wq, Wk, Wv, Wo = (np.asarray(a, F64) for a in (Wq, Wk, Wv, Wo))
    n = x_hist.shape[0]
    d_h = Wq.shape[1] // n_heads
    heads_out = np.zeros((1, n_heads * d_h), F64)
    for i in range(n_heads):
        g = _kv_head_of(i, n_heads, n_kv_heads)
        q = x_hist[n - 1] @ Wq[:, i * d_h:(i + 1) * d_h]
        K = x_hist @ Wk[:, g * d_h:(g + 1) * d_h]
        V = x_hist @ Wv[:, g * d_h:(g + 1) * d_h]
        heads_out[0, i * d_h:(i + 1) * d_h] = standard_rope_decode(q, K, V, d_h, base)
    return heads_out @ Wo


def project_to_basis(A, U):
    """Rank-space coordinates of d_h-dimensional rows: A [.., d_h] U [d_h, r] (what Eq. 8 caches)."""
    return np.asarray(A, F64) @ np.asarray(U, F64)


# --------------------------------------------------------------------------
# Table 1 and the KV-size formula of the LLM-Inference paragraph
# --------------------------------------------------------------------------
def kv_cache_bytes(batch: int, n: int, n_kv_heads: int, r_k: int, r_v: int, n_layers: int, bytes_per_el: int) -> int:
    """b * n * H_kv * (r_k + r_v) * L * p.  With r_k = r_v = d_h and H_kv = H this
    is the paper's 2*b*n*d*L*p (its printed formula carries a stray factor h;
    the Introduction's 256 GB example fixes the reading d = h * d_h)."""
    return batch * n * n_kv_heads * (r_k + r_v) * n_layers * bytes_per_el


def rel_l2(a, b) -> float:
    a = np.asarray(a, F64).ravel()
    b = np.asarray(b, F64).ravel()
    den = float(np.linalg.norm(b))
    return float(np.linalg.norm(a - b)) / (den if den > 0 else 1.0)
