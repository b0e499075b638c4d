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
