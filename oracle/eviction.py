"""Plain fp64 CPU oracle of the attention statistics a token-eviction policy needs, and of the H2O selection rule.

TEST INFRASTRUCTURE ONLY -- never imported by the product package, shares no code with the HIP kernels.

The paper combines Eigen Attention with H2O token pruning (results, "Eigen Attention with token pruning", and its
table of zero-shot accuracies at 0.6x / 0.4x / 0.24x cache): H2O keeps, per sequence, the tokens that have received
the most attention so far ("heavy hitters") plus the most recent ones, and drops the rest from the KV cache.  The
paper gives no formula of its own; what H2O accumulates is the softmax probability each cached token receives from
every new query.  In the rank-r space those probabilities are the p_t of Eq. (3)/(7) -- nothing changes.

  attention_mass   mass[b][g, t] = sum over the query heads i of kv head g of p_i[t],
                   p_i = Softmax(q_r,i . K_r[g]^T / sqrt(d_h))      (Eq. 3 with Eq. 7's operands)
  h2o_victim       the cached token to drop: smallest accumulated mass among all but the n_recent newest

Rotary models (the paper's token-pruning table is on Llama models, whose attention is the form of Sec. 4.3): a token
that survives an eviction keeps the position it had in the text, so once tokens have been dropped the position of the
key in cache slot t is no longer t.  The two functions below are Eq. 10 with the position of every cached key, and of
the query, given explicitly:

  decode_attention_rope_positions   s_t = rot(q, pos_q) . rot(U^K k_r[t], pos_k[t]) / sqrt(d_h), o = Softmax(s) V_r
  attention_mass_rope_positions     the same probabilities summed over the query heads of a kv head

Pins (tests/test_oracle_eviction.py): every (sequence, kv head) row of the mass sums to the number of query heads
in the group; brute force; closed-form cases (zero query: uniform; one dominant key); permutation equivariance;
heads of different kv heads do not mix; the selection rule on hand-made accumulators.
"""
from __future__ import annotations

import numpy as np

from . import eigen_attention as ea_oracle


def attention_mass(q_r, cache: "ea_oracle.RankCache", d_head: int):
    """q_r [B, H, r_k] -> list over b of arrays [H_kv, len_b]."""
    q_r = np.asarray(q_r, np.float64)
    B, H, _ = q_r.shape
    _, probs = ea_oracle.decode_attention(q_r, cache, d_head, return_probs=True)
    G = H // cache.n_kv_heads
    out = []
    for b in range(B):
        m = np.zeros((cache.n_kv_heads, cache.seq_len(b)))
        for i in range(H):
            m[i // G] += probs[b * H + i]
        out.append(m)
    return out


def h2o_victim(acc, n_recent: int) -> int:
    """acc [n]: accumulated mass of the n cached tokens (oldest first).  Returns the index of the token H2O evicts:
    the smallest accumulated mass among the tokens that are not among the n_recent newest (first index on ties)."""
    acc = np.asarray(acc, np.float64)
    n = acc.shape[0]
    assert 0 <= n_recent < n
    return int(np.argmin(acc[:n - n_recent]))


def decode_attention_rope_positions(q, pos_q, cache: "ea_oracle.RankCache", pos_k, Uk, d_head: int,
                                    base: float = 10000.0, return_probs: bool = False):
    """Generation-phase Eigen Attention of a rotary model (Sec. 4.3, Eq. 10) over a cache whose slots hold tokens
    of arbitrary original positions (what is left after token pruning).

    q [B, H, d_h]: full-rank query, not rotated; pos_q [B]: its position in the text.
    cache.K[b][g] [n_b, r_k]: rank-r keys k_r = k U^K (never rotated); pos_k[b] [n_b]: the position of the token in
    each slot; Uk [d_h, r_k]: the basis shared by all heads.
    Each key is brought back to d_h channels, k' = U^K k_r, rotated to ITS position; the query to its own.
    Returns o [B, H, r_v] (and, with return_probs, the list over b*H + i of the probabilities p[n_b])."""
    q = np.asarray(q, np.float64)
    Uk = np.asarray(Uk, np.float64)
    B, H, d_h = q.shape
    assert d_h == d_head and Uk.shape[0] == d_h
    out = np.zeros((B, H, cache.r_v))
    probs = []
    for b in range(B):
        n = cache.seq_len(b)
        if n == 0:
            raise ValueError("decode over an empty sequence")
        pk = np.asarray(pos_k[b])
        assert pk.shape == (n,)
        for i in range(H):
            g = i // (H // cache.n_kv_heads)
            K_up = cache.K[b][g] @ Uk.T                                            # [n, d_h]
            K_rot = ea_oracle.rope_rotate(K_up, pk, base)
            q_rot = ea_oracle.rope_rotate(q[b, i], int(pos_q[b]), base)
            p = ea_oracle.softmax((K_rot @ q_rot) / np.sqrt(d_head))
            probs.append(p)
            out[b, i] = p @ cache.V[b][g]
    return (out, probs) if return_probs else out


def attention_mass_rope_positions(q, pos_q, cache: "ea_oracle.RankCache", pos_k, Uk, d_head: int,
                                  base: float = 10000.0):
    """mass[b][g, t] = sum over the query heads i of kv head g of p_i[t], p from decode_attention_rope_positions."""
    q = np.asarray(q, np.float64)
    B, H, _ = q.shape
    _, probs = decode_attention_rope_positions(q, pos_q, cache, pos_k, Uk, d_head, base, return_probs=True)
    G = H // cache.n_kv_heads
    out = []
    for b in range(B):
        per_kv_head = np.zeros((cache.n_kv_heads, cache.seq_len(b)))
        for i in range(H):
            per_kv_head[i // G] += probs[b * H + i]
        out.append(per_kv_head)
    return out
