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


# ---------------------------------------------------------------------------
# Rotary models after token pruning (Sec. 4.3, Eq. 10 with explicit positions)
# ---------------------------------------------------------------------------
def _rope_case(seed, H=4, Hkv=2, r=6, r_v=3, d_h=8, lens=(23, 9)):
    g = synth.rng(seed)
    K = [synth.gaussian(g, (Hkv, n, r)) for n in lens]
    V = [synth.gaussian(g, (Hkv, n, r_v)) for n in lens]
    q = synth.gaussian(g, (len(lens), H, d_h))
    Uk = np.linalg.qr(synth.gaussian(g, (d_h, d_h)))[0][:, :r]
    return g, K, V, q, Uk


def test_rope_positions_reduce_to_the_plain_rotary_form_when_nothing_was_dropped():
    """Slot t holds position t, the query sits at the last position: Eq. 10 as oracle.decode_attention_rope has it."""
    g, K, V, q, Uk = _rope_case(211)
    cache = ora.RankCache.from_arrays(K, V)
    lens = [cache.seq_len(b) for b in range(2)]
    got = oe.decode_attention_rope_positions(q, [n - 1 for n in lens], cache, [np.arange(n) for n in lens], Uk, 8, 500.0)
    assert np.allclose(got, ora.decode_attention_rope(q, cache, Uk, 8, 500.0), rtol=0, atol=1e-13)


def test_a_kept_token_scores_as_in_the_sequence_it_was_kept_from():
    """Drop tokens from a sequence: every kept token's probability, renormalised over the kept ones, is what it was
    in the full sequence (its score has not changed: it still sits at its original position), the output is the
    kept tokens' weighted values, and the mass statistic follows."""
    g, K, V, q, Uk = _rope_case(212, lens=(40,))
    n = 40
    full = ora.RankCache.from_arrays(K, V)
    _, p_full = oe.decode_attention_rope_positions(q[:1], [n - 1], full, [np.arange(n)], Uk, 8, return_probs=True)
    kept = np.sort(g.permutation(n - 1)[:17])
    kept = np.r_[kept, n - 1]                                   # the newest token is always there
    sub = ora.RankCache.from_arrays([K[0][:, kept]], [V[0][:, kept]])
    o_sub, p_sub = oe.decode_attention_rope_positions(q[:1], [n - 1], sub, [kept], Uk, 8, return_probs=True)
    for i in range(4):
        want = p_full[i][kept] / p_full[i][kept].sum()
        assert np.allclose(p_sub[i], want, rtol=0, atol=1e-13)
        assert np.allclose(o_sub[0, i], want @ V[0][i // 2][kept], rtol=0, atol=1e-13)
    # the same slots numbered 0..17 (what the position-free indexing would do) give something else
    o_wrong = oe.decode_attention_rope_positions(q[:1], [len(kept) - 1], sub, [np.arange(len(kept))], Uk, 8)
    assert not np.allclose(o_wrong, o_sub, atol=1e-3)
    mass = oe.attention_mass_rope_positions(q[:1], [n - 1], sub, [kept], Uk, 8)[0]
    assert np.allclose(mass[0], p_sub[0] + p_sub[1]) and np.allclose(mass[1], p_sub[2] + p_sub[3])
    assert np.allclose(mass.sum(axis=1), 2.0)


def test_rope_positions_against_the_complex_form_slot_order_and_a_common_shift():
    """(1) Brute force in another formulation: channel pairs as complex numbers, s = Re sum_j q_j conj(k'_j)
    e^{i (pos_q - pos_k) theta_j} / sqrt(d_h) -- only the position difference enters.  (2) The order of the slots
    does not matter.  (3) Neither does a shift of all positions."""
    g, K, V, q, Uk = _rope_case(213, lens=(12, 30))
    base, d_h = 10000.0, 8
    pos_k = [np.sort(g.permutation(200)[:12]), np.sort(g.permutation(5000)[:30])]
    pos_q = [int(pos_k[0][-1]) + 3, int(pos_k[1][-1])]
    cache = ora.RankCache.from_arrays(K, V)
    out, probs = oe.decode_attention_rope_positions(q, pos_q, cache, pos_k, Uk, d_h, base, return_probs=True)
    theta = base ** (-2.0 * np.arange(d_h // 2) / d_h)
    for b in range(2):
        for i in range(4):
            kv = i // 2
            qc = q[b, i, 0::2] + 1j * q[b, i, 1::2]
            s = []
            for t in range(len(pos_k[b])):
                k_up = Uk @ K[b][kv, t]
                kc = k_up[0::2] + 1j * k_up[1::2]
                s.append(np.real(np.sum(qc * np.conj(kc) * np.exp(1j * (pos_q[b] - pos_k[b][t]) * theta))) / np.sqrt(d_h))
            e = np.exp(np.array(s) - max(s))
            assert np.allclose(probs[b * 4 + i], e / e.sum(), rtol=0, atol=1e-12)
            assert np.allclose(out[b, i], (e / e.sum()) @ V[b][kv], rtol=0, atol=1e-12)
    perm = [g.permutation(12), g.permutation(30)]
    shuffled = ora.RankCache.from_arrays([K[b][:, perm[b]] for b in range(2)], [V[b][:, perm[b]] for b in range(2)])
    out_p = oe.decode_attention_rope_positions(q, pos_q, shuffled, [pos_k[b][perm[b]] for b in range(2)], Uk, d_h, base)
    assert np.allclose(out_p, out, rtol=0, atol=1e-12)
    m0 = oe.attention_mass_rope_positions(q, pos_q, cache, pos_k, Uk, d_h, base)
    mp = oe.attention_mass_rope_positions(q, pos_q, shuffled, [pos_k[b][perm[b]] for b in range(2)], Uk, d_h, base)
    for b in range(2):
        assert np.allclose(mp[b], m0[b][:, perm[b]], rtol=0, atol=1e-12)
    out_s = oe.decode_attention_rope_positions(q, [p + 77 for p in pos_q], cache, [p + 77 for p in pos_k], Uk, d_h, base)
    assert np.allclose(out_s, out, rtol=0, atol=1e-10)
