"""Pins of oracle/eviction.py: the attention mass per cached token (what H2O-style eviction accumulates; results,
"Eigen Attention with token pruning") and the selection rule."""
import numpy as np

from oracle import eigen_attention as ora
from oracle import eviction as oe
from paper_2408_05646_amd import synth


def test_mass_rows_sum_to_the_group_size_and_match_brute_force():
    g = synth.rng(201)
    H, Hkv, r, d_h = 6, 2, 8, 16
    lens = [37, 5]
    K = [synth.gaussian(g, (Hkv, n, r)) for n in lens]
    V = [synth.gaussian(g, (Hkv, n, 4)) for n in lens]
    q = synth.gaussian(g, (2, H, r))
    mass = oe.attention_mass(q, ora.RankCache.from_arrays(K, V), d_h)
    for b, n in enumerate(lens):
        assert mass[b].shape == (Hkv, n)
        assert np.allclose(mass[b].sum(axis=1), H // Hkv, rtol=0, atol=1e-12)
        for kv in range(Hkv):
            ref = np.zeros(n)
            for h in range(kv * 3, kv * 3 + 3):
                s = [sum(q[b, h, c] * K[b][kv, t, c] for c in range(r)) / np.sqrt(d_h) for t in range(n)]
                e = np.exp(np.array(s) - max(s))
                ref += e / e.sum()
            assert np.allclose(mass[b][kv], ref, rtol=0, atol=1e-12)


def test_mass_closed_forms_and_equivariance():
    g = synth.rng(202)
    Hkv, r, d_h, n = 1, 8, 16, 20
    K = [synth.gaussian(g, (Hkv, n, r))]
    V = [np.zeros((Hkv, n, 2))]
    cache = ora.RankCache.from_arrays(K, V)
    assert np.allclose(oe.attention_mass(np.zeros((1, 2, r)), cache, d_h)[0], 2.0 / n)        # zero query: uniform
    q = synth.gaussian(g, (1, 2, r))
    Kd = [K[0].copy()]
    Kd[0][0, 7] = 200.0 * q[0, 0] / np.linalg.norm(q[0, 0])                                   # head 0 sees only token 7
    m = oe.attention_mass(q, ora.RankCache.from_arrays(Kd, V), d_h)[0][0]
    p1 = ora.decode_attention(q, ora.RankCache.from_arrays(Kd, V), d_h, return_probs=True)[1][1]
    assert abs(m[7] - (1.0 + p1[7])) < 1e-9
    perm = g.permutation(n)
    mp = oe.attention_mass(q, ora.RankCache.from_arrays([K[0][:, perm]], V), d_h)[0]
    assert np.allclose(mp, oe.attention_mass(q, cache, d_h)[0][:, perm], rtol=0, atol=1e-12)


def test_heads_of_different_kv_heads_do_not_mix():
    g = synth.rng(203)
    H, Hkv, r, d_h, n = 4, 2, 4, 8, 9
    K = [synth.gaussian(g, (Hkv, n, r))]
    V = [np.zeros((Hkv, n, 2))]
    q = synth.gaussian(g, (1, H, r))
    base = oe.attention_mass(q, ora.RankCache.from_arrays(K, V), d_h)[0]
    q2 = q.copy()
    q2[0, 2:] = synth.gaussian(g, (2, r))                      # change the heads of kv head 1 only
    other = oe.attention_mass(q2, ora.RankCache.from_arrays(K, V), d_h)[0]
    assert np.array_equal(base[0], other[0]) and not np.allclose(base[1], other[1])


def test_h2o_selection_rule():
    acc = np.array([5.0, 0.2, 3.0, 0.1, 0.05, 9.0])
    assert oe.h2o_victim(acc, 0) == 4
    assert oe.h2o_victim(acc, 2) == 3              # the two newest are protected
    assert oe.h2o_victim(acc, 3) == 1
    assert oe.h2o_victim(np.array([1.0, 1.0, 1.0]), 1) == 0     # ties: the oldest


def test_combined_cache_size_is_the_product_the_paper_prints():
    """Rank compression and token pruning shrink the cache along different axes: 0.6x ranks and 40 % of the tokens
    give the 0.24x of the paper's H2O table."""
    import json, os
    v = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_values.json")))["h2o_combination"]
    n, H, d_h, L = 2000, 32, 100, 4
    r = round(d_h * v["eigen_attention_cache"])
    kept = round(n * v["tokens_kept"])
    full = ora.kv_cache_bytes(1, n, H, d_h, d_h, L, 2)
    assert abs(ora.kv_cache_bytes(1, kept, H, r, r, L, 2) / full - v["combined_cache"]) < 1e-12
    # ... and that is what a fixed-budget cache of `kept` slots holds, whatever the policy evicts
    cache = ora.RankCache.empty(1, H, r, r)
    cache.append(0, np.zeros((kept, H, r)), np.zeros((kept, H, r)))
    assert cache.elements() * 2 * L == ora.kv_cache_bytes(1, kept, H, r, r, L, 2)
