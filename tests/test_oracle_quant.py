"""Pins of oracle/quant_cache.py (4-bit group quantisation of the rank-r cache: keys per channel over 64 tokens,
values per token; results paragraph on quantisation and the appendix's quantisation table).  The paper fixes
the grouping axes and "integer quantisation"; rounding and zero-point are this build's reading, so these pins
are the properties any such quantiser must have, chosen so that a swapped axis, a wrong group size, a wrong
level count, truncation instead of rounding or a sign slip fails one of them."""
import numpy as np
import pytest

from oracle import eigen_attention as ora
from oracle import quant_cache as oq
from paper_2408_05646_amd import synth


def grid_keys(g, n, r):
    """Keys that lie exactly on a 16-level grid per (64-token group, channel), every group using both end
    codes; scale a power of two, zero a small multiple of the scale: all exactly representable."""
    G = n // 64
    codes = g.integers(0, 16, size=(G, 64, r)).astype(np.uint8)
    codes[:, 0, :] = 0
    codes[:, 1, :] = 15
    scale = 2.0 ** g.integers(-6, 3, size=(G, 1, r))
    zero = scale * g.integers(-40, 40, size=(G, 1, r))
    return (scale * codes + zero).reshape(n, r), codes.reshape(n, r), scale[:, 0, :], zero[:, 0, :]


def grid_values(g, n, r):
    codes = g.integers(0, 16, size=(n, r)).astype(np.uint8)
    codes[:, 0] = 0
    codes[:, 1] = 15
    scale = 2.0 ** g.integers(-6, 3, size=(n, 1))
    zero = scale * g.integers(-40, 40, size=(n, 1))
    return scale * codes + zero, codes, scale[:, 0], zero[:, 0]


def test_values_on_the_grid_round_trip_exactly():
    g = synth.rng(101)
    K, codes, scale, zero = grid_keys(g, 192, 24)
    c, s, z = oq.quantize_keys(K)
    assert np.array_equal(c, codes) and np.array_equal(s.astype(np.float64), scale)
    assert np.array_equal(z.astype(np.float64), zero)
    assert np.array_equal(oq.dequantize_keys(c, s, z), K)
    V, codes, scale, zero = grid_values(g, 100, 40)
    c, s, z = oq.quantize_values(V)
    assert np.array_equal(c, codes) and np.array_equal(s.astype(np.float64), scale)
    assert np.array_equal(z.astype(np.float64), zero)
    assert np.array_equal(oq.dequantize_values(c, s, z), V)


@pytest.mark.parametrize("std", [0.01, 1.0, 300.0])
def test_round_trip_error_is_at_most_half_a_step(std):
    """|x - value(code(x))| <= scale/2, plus what rounding scale and zero to fp16 can add: 15 steps of the
    scale's rounding error and the zero's own."""
    g = synth.rng(102)
    K = np.float32(synth.gaussian(g, (256, 48), std)).astype(np.float64)
    c, s, z = oq.quantize_keys(K)
    assert c.dtype == np.uint8 and c.max() <= 15
    Kg = K.reshape(4, 64, 48)
    lo, hi = Kg.min(axis=1), Kg.max(axis=1)
    s64, z64 = s.astype(np.float64), z.astype(np.float64)
    slack = 15 * np.abs(s64 - (hi - lo) / 15) + np.abs(z64 - lo) + 1e-6 * std
    err = np.abs(oq.dequantize_keys(c, s, z) - K).reshape(4, 64, 48)
    assert np.all(err <= s64[:, None, :] / 2 + slack[:, None, :])
    assert err.max() > s64.min() / 8            # ... and it is a 16-level grid, not a finer one
    V = np.float32(synth.gaussian(g, (77, 80), std)).astype(np.float64)
    c, s, z = oq.quantize_values(V)
    lo, hi = V.min(axis=1), V.max(axis=1)
    s64, z64 = s.astype(np.float64), z.astype(np.float64)
    slack = 15 * np.abs(s64 - (hi - lo) / 15) + np.abs(z64 - lo) + 1e-6 * std
    err = np.abs(oq.dequantize_values(c, s, z) - V)
    assert np.all(err <= (s64 / 2 + slack)[:, None])


def test_group_extremes_take_the_end_codes_and_codes_are_monotone():
    g = synth.rng(103)
    K = np.float32(synth.gaussian(g, (128, 16))).astype(np.float64)
    c, s, z = oq.quantize_keys(K)
    for grp in range(2):
        rows = slice(64 * grp, 64 * grp + 64)
        for ch in range(16):
            col, cc = K[rows, ch], c[rows, ch]
            assert cc[np.argmin(col)] == 0 and cc[np.argmax(col)] == 15
            order = np.argsort(col, kind="stable")
            assert np.all(np.diff(cc[order].astype(int)) >= 0)


def test_rounding_is_to_nearest_not_truncation():
    """zero 0, scale 1: 3.4 -> 3, 3.6 -> 4, halves go to the even code."""
    row = np.array([[0.0, 15.0, 3.4, 3.6, 2.5, 3.5, 14.49, 0.51]])
    c, s, z = oq.quantize_values(row)
    assert float(s[0]) == 1.0 and float(z[0]) == 0.0
    assert c[0].tolist() == [0, 15, 3, 4, 2, 4, 14, 1]


def test_constant_group_is_exact_and_has_code_zero():
    K = np.full((64, 3), 0.375)
    c, s, z = oq.quantize_keys(K)
    assert not c.any() and not s.astype(np.float64).any()
    assert np.array_equal(oq.dequantize_keys(c, s, z), K)
    V = np.full((5, 7), -2.5)
    c, s, z = oq.quantize_values(V)
    assert not c.any() and np.array_equal(oq.dequantize_values(c, s, z), V)


def test_codes_do_not_change_under_a_power_of_two_rescaling():
    g = synth.rng(104)
    K = np.float32(synth.gaussian(g, (64, 32))).astype(np.float64)
    V = np.float32(synth.gaussian(g, (40, 32))).astype(np.float64)
    for a in (0.25, 8.0):
        assert np.array_equal(oq.quantize_keys(a * K)[0], oq.quantize_keys(K)[0])
        assert np.array_equal(oq.quantize_values(a * V)[0], oq.quantize_values(V)[0])


def test_keys_are_grouped_per_channel_and_values_per_token():
    """Channels (tokens) with very different offsets: a quantiser that shared one scale across the wrong axis
    would have an error of the order of the offsets, the right one of the order of the unit spread."""
    g = synth.rng(105)
    K = np.float32(g.random((64, 20)) + 50.0 * np.arange(20)[None, :]).astype(np.float64)
    err = np.abs(oq.dequantize_keys(*oq.quantize_keys(K)) - K)
    assert err.max() < 0.3                       # spread 1, 15 steps, plus fp16 rounding of offsets up to 950
    V = np.float32(g.random((30, 64)) + 50.0 * np.arange(30)[:, None]).astype(np.float64)
    err = np.abs(oq.dequantize_values(*oq.quantize_values(V)) - V)
    assert err.max() < 0.6
    # and the transposed use is indeed that bad
    bad = np.abs(oq.dequantize_values(*oq.quantize_values(K)) - K)
    assert bad.max() > 10.0


def test_key_groups_are_64_tokens_long():
    g = synth.rng(106)
    K = np.float32(synth.gaussian(g, (192, 8))).astype(np.float64)
    K[64:128] *= 1000.0
    c, s, z = oq.quantize_keys(K)
    assert s.shape == (3, 8)
    s64 = s.astype(np.float64)
    assert np.all(s64[1] > 100 * s64[0]) and np.all(s64[1] > 100 * s64[2])
    err = np.abs(oq.dequantize_keys(c, s, z) - K)
    assert err[:64].max() < 0.3 and err[128:].max() < 0.3       # the loud group does not leak into its neighbours


def test_attention_over_a_quantised_cache():
    """(a) nothing quantised = plain attention; (b) a cache on the grid is attended exactly; (c) brute force
    over hand-dequantised values; (d) on ordinary data quantisation changes the result a little, not a lot."""
    g = synth.rng(107)
    H, Hkv, r_k, r_v, d_h = 4, 2, 16, 24, 64
    q = synth.gaussian(g, (2, H, r_k))
    lens = [130, 200]
    K = [synth.gaussian(g, (Hkv, n, r_k)) for n in lens]
    V = [synth.gaussian(g, (Hkv, n, r_v)) for n in lens]
    plain = ora.decode_attention(q, ora.RankCache.from_arrays(K, V), d_h)
    assert np.array_equal(oq.decode_attention_quantized(q, K, V, [0, 0], d_h), plain)
    # (b)
    Kg = [np.stack([grid_keys(g, 128, r_k)[0] for _ in range(Hkv)])]
    Vg = [np.stack([grid_values(g, 128, r_v)[0] for _ in range(Hkv)])]
    exact = ora.decode_attention(q[:1], ora.RankCache.from_arrays(Kg, Vg), d_h)
    assert np.allclose(oq.decode_attention_quantized(q[:1], Kg, Vg, [128], d_h), exact, rtol=0, atol=1e-13)
    # (c) sequence 1: 128 quantised tokens, 72 as they are
    got = oq.decode_attention_quantized(q, K, V, [64, 128], d_h)
    for h in range(H):
        kv = h // 2
        ck, sk, zk = oq.quantize_keys(K[1][kv, :128])
        cv, sv, zv = oq.quantize_values(V[1][kv, :128])
        scores = []
        vals = []
        for t in range(200):
            if t < 128:
                key = [float(sk[t // 64, c]) * int(ck[t, c]) + float(zk[t // 64, c]) for c in range(r_k)]
                val = [float(sv[t]) * int(cv[t, c]) + float(zv[t]) for c in range(r_v)]
            else:
                key, val = K[1][kv, t], V[1][kv, t]
            scores.append(sum(a * b for a, b in zip(q[1, h], key)) / np.sqrt(d_h))
            vals.append(val)
        w = np.exp(np.array(scores) - max(scores))
        ref = (w[:, None] * np.array(vals)).sum(axis=0) / w.sum()
        assert np.allclose(got[1, h], ref, rtol=0, atol=1e-12)
    # (d)
    diff = ora.rel_l2(got, plain)
    assert 1e-3 < diff < 0.2


def test_rotary_attention_over_a_quantised_cache():
    """(a) nothing quantised = the rotary oracle; (b) a cache on the grid is attended exactly; (c) brute force: keys
    dequantised by hand, brought back to d_head channels, rotated pair by pair at their positions."""
    g = synth.rng(108)
    H, Hkv, r_k, r_v, d_h, n = 2, 1, 8, 8, 16, 130
    Uk = synth.orthonormal_basis(g, d_h, r_k)
    q = synth.gaussian(g, (1, H, d_h))
    K = [synth.gaussian(g, (Hkv, n, r_k))]
    V = [synth.gaussian(g, (Hkv, n, r_v))]
    plain = ora.decode_attention_rope(q, ora.RankCache.from_arrays(K, V), Uk, d_h, 100.0)
    assert np.array_equal(oq.decode_attention_rope_quantized(q, K, V, [0], Uk, d_h, 100.0), plain)
    Kg = [np.stack([grid_keys(g, 128, r_k)[0]])]
    Vg = [np.stack([grid_values(g, 128, r_v)[0]])]
    exact = ora.decode_attention_rope(q, ora.RankCache.from_arrays(Kg, Vg), Uk, d_h, 100.0)
    assert np.allclose(oq.decode_attention_rope_quantized(q, Kg, Vg, [128], Uk, d_h, 100.0), exact, rtol=0, atol=1e-13)
    got = oq.decode_attention_rope_quantized(q, K, V, [128], Uk, d_h, 100.0)
    ck, sk, zk = oq.quantize_keys(K[0][0, :128])
    cv, sv, zv = oq.quantize_values(V[0][0, :128])

    def rot(x, pos):
        y = np.array(x, dtype=np.float64)
        for j in range(d_h // 2):
            th = pos * 100.0 ** (-2.0 * j / d_h)
            y[2 * j] = x[2 * j] * np.cos(th) - x[2 * j + 1] * np.sin(th)
            y[2 * j + 1] = x[2 * j] * np.sin(th) + x[2 * j + 1] * np.cos(th)
        return y
    for h in range(H):
        scores, vals = [], []
        qr = rot(q[0, h], n - 1)
        for t in range(n):
            if t < 128:
                key = np.array([float(sk[t // 64, c]) * int(ck[t, c]) + float(zk[t // 64, c]) for c in range(r_k)])
                val = np.array([float(sv[t]) * int(cv[t, c]) + float(zv[t]) for c in range(r_v)])
            else:
                key, val = K[0][0, t], V[0][0, t]
            scores.append(float(rot(Uk @ key, t) @ qr) / np.sqrt(d_h))
            vals.append(val)
        w = np.exp(np.array(scores) - max(scores))
        ref = (w[:, None] * np.array(vals)).sum(axis=0) / w.sum()
        assert np.allclose(got[0, h], ref, rtol=0, atol=1e-12)
    assert 1e-3 < ora.rel_l2(got, plain) < 0.3


def test_alibi_attention_over_a_quantised_cache():
    """The bias is added to the scores of the dequantised keys, by distance to the newest token: brute force."""
    g = synth.rng(109)
    H, r, d_h, n = 2, 8, 16, 70
    q = synth.gaussian(g, (1, H, r))
    K = [synth.gaussian(g, (1, n, r))]
    V = [synth.gaussian(g, (1, n, r))]
    slopes = np.array([0.5, 0.0625])
    got = oq.decode_attention_quantized(q, K, V, [64], d_h, alibi_slopes=slopes)
    Kq, Vq = oq.quantized_view(K[0], V[0], 64)
    for h in range(H):
        sc = np.array([Kq[0, t] @ q[0, h] / np.sqrt(d_h) - slopes[h] * (n - 1 - t) for t in range(n)])
        w = np.exp(sc - sc.max())
        assert np.allclose(got[0, h], (w[:, None] * Vq[0]).sum(axis=0) / w.sum(), rtol=0, atol=1e-12)
    assert ora.rel_l2(got, oq.decode_attention_quantized(q, K, V, [64], d_h)) > 0.05


def test_cache_size_accounting_reproduces_the_papers_quantisation_table():
    """Appendix, Quantization Results: every printed KV-cache size equals elements * (bits + 16 / group) / 8 in GiB,
    rounded to two decimals -- 16 bits of metadata per group; 0 or 32 bits do not reproduce the table."""
    import json, os
    t = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_values.json")))
    t = t["appendix_quantization_kv_sizes_GB"]
    rows = []
    for model in ("llama2_13b", "llama2_7b"):
        m = t[model]
        full = 2 * t["sequence_length"] * m["d_model"] * m["n_layers"]          # K and V scalars of one sequence
        for bits, group, printed in m["standard"]:
            rows.append((full, bits, group, printed))
        for bits, group, printed in m["eigen"]:
            rows.append((full * t["eigen_attention_compression"], bits, group, printed))
    assert len(rows) == 15

    def misses(meta):
        return sum(abs(oq.quantized_cache_bytes(n, b, g, meta) / 2 ** 30 - printed) > 0.005 + 1e-12
                   for n, b, g, printed in rows)
    assert misses(16) == 0
    assert misses(0) >= 5 and misses(32) >= 5
    # the 16-bit baseline of the same accounting: 2 * 2048 * 4096 * 32 scalars at 16 bits and no groups = 1 GiB
    assert oq.quantized_cache_bytes(2 * 2048 * 4096 * 32, 16, 1, 0) == 2 ** 30
    # this build's format carries a scale and a zero: 4.5 bits per key scalar, 4.4 per value scalar at r_v = 80
    assert oq.bits_per_element_q4(80, 80) == (4.5, 4.4)


def test_key_groups_of_128_tokens():
    """The group size of the appendix table's 4-bit Eigen Attention rows: one scale per channel and 128 tokens.
    A loud stretch of 64 tokens now sets the step of the whole group it lies in (and of no other); values on a
    128-token grid round-trip exactly; the error stays within half a step of the group's own scale."""
    g = synth.rng(120)
    K = np.float32(synth.gaussian(g, (384, 8))).astype(np.float64)
    K[128:192] *= 1000.0
    c, s, z = oq.quantize_keys(K, 128)
    assert c.shape == (384, 8) and s.shape == (3, 8) and z.shape == (3, 8)
    s64 = s.astype(np.float64)
    assert np.all(s64[1] > 100 * s64[0]) and np.all(s64[1] > 100 * s64[2])
    back = oq.dequantize_keys(c, s, z)
    err = np.abs(back - K)
    assert err[:128].max() < 0.3 and err[256:].max() < 0.3
    assert err[192:256].max() > 10.0                  # the quiet half of the loud group pays for its neighbour
    for grp in range(3):
        assert np.all(err[128 * grp:128 * (grp + 1)] <= 0.5 * s64[grp] * (1 + 1e-3) + 1e-30)
    # with 64-token groups the same quiet stretch is fine: the two group sizes really differ
    assert np.abs(oq.dequantize_keys(*oq.quantize_keys(K, 64)) - K)[192:256].max() < 0.3
    # a cache on a 128-token grid is reproduced exactly
    lo, step = g.standard_normal(8), 2.0 ** g.integers(-6, 2, size=8)
    grid = lo + step * g.integers(0, 16, size=(128, 8))
    grid[0], grid[1] = lo, lo + 15 * step               # both ends present: the grid is the group's own
    grid = np.float16(grid).astype(np.float64)
    if np.all(np.float16(lo).astype(np.float64) == lo):
        cg, sg, zg = oq.quantize_keys(grid, 128)
        assert np.array_equal(oq.dequantize_keys(cg, sg, zg), grid)
    # attention over the view with 128-token groups = attention over its dequantised keys (brute force on one head)
    H, Hkv, r_k, r_v, d_h, n = 2, 1, 8, 4, 16, 300
    Kc = [synth.gaussian(g, (Hkv, n, r_k))]
    Vc = [synth.gaussian(g, (Hkv, n, r_v))]
    q = synth.gaussian(g, (1, H, r_k))
    got = oq.decode_attention_quantized(q, Kc, Vc, [256], d_h, group_tokens=128)
    ck, sk, zk = oq.quantize_keys(Kc[0][0, :256], 128)
    cv, sv, zv = oq.quantize_values(Vc[0][0, :256])
    for h in range(H):
        keys = np.concatenate([sk.astype(np.float64)[np.arange(256) // 128] * ck + zk.astype(np.float64)[np.arange(256) // 128],
                               Kc[0][0, 256:]])
        vals = np.concatenate([sv.astype(np.float64)[:, None] * cv + zv.astype(np.float64)[:, None], Vc[0][0, 256:]])
        sc = keys @ q[0, h] / np.sqrt(d_h)
        w = np.exp(sc - sc.max())
        assert np.allclose(got[0, h], (w / w.sum()) @ vals, rtol=0, atol=1e-12)


def test_group_128_against_the_tables_rows():
    """The appendix table's 4-bit Eigen Attention rows at group 128 (Llama-2-7b: 0.15 GB, Llama-2-13b: 0.24 GB) are
    4 + 16/128 = 4.125 bits per scalar in the paper's accounting.  This build's format at key group 128 stores a
    scale AND a zero per group, and groups values per token over r_v channels: 4.25 bits per key scalar and
    4 + 32/r_v per value scalar -- for the 7b model at 0.6x (r = 77 of 128 channels per head on average; r_v = 80
    here) 0.158 GiB against the printed 0.15: 5 % above the row it corresponds to, all of it metadata."""
    import json, os
    t = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_values.json")))
    t = t["appendix_quantization_kv_sizes_GB"]
    for model, printed in (("llama2_7b", 0.15), ("llama2_13b", 0.24)):
        m = t[model]
        assert [4, 128, printed] in m["eigen"]
        scalars = 2 * t["sequence_length"] * m["d_model"] * m["n_layers"] * t["eigen_attention_compression"]
        assert abs(oq.quantized_cache_bytes(scalars, 4, 128) / 2 ** 30 - printed) <= 0.005
        bk, bv = oq.bits_per_element_q4(80, 80, 128)
        assert (bk, bv) == (4.25, 4.4)
        ours = scalars / 2 * (bk + bv) / 8 / 2 ** 30
        assert 1.04 < ours / (oq.quantized_cache_bytes(scalars, 4, 128) / 2 ** 30) < 1.06
    assert oq.bits_per_element_q4(80, 80, 64)[0] == 4.5


def test_prefill_attention_over_a_partly_quantised_cache():
    """(a) nothing quantised = plain causal attention; (b) the last query row = the generation-phase function on the
    same cache; (c) brute force for one (query, head); (d) a prompt prefilled in chunks: the first chunk is plain
    attention, later chunks see the earlier ones quantised, and each chunk equals the one-shot function at its cut."""
    g = synth.rng(121)
    H, Hkv, r_k, r_v, d_h, L, n = 4, 2, 8, 6, 16, 200, 70
    K = [synth.gaussian(g, (Hkv, L, r_k))]
    V = [synth.gaussian(g, (Hkv, L, r_v))]
    q = synth.gaussian(g, (1, n, H, r_k))
    plain = ora.prefill_attention(q, ora.RankCache.from_arrays(K, V), d_h)
    assert np.array_equal(oq.prefill_attention_quantized(q, K, V, [0], d_h), plain)
    got = oq.prefill_attention_quantized(q, K, V, [128], d_h)
    assert not np.allclose(got, plain, atol=1e-3)
    assert np.allclose(got[:, -1], oq.decode_attention_quantized(q[:, -1], K, V, [128], d_h), rtol=0, atol=1e-13)
    # with ALiBi slopes: zero slopes change nothing, and every row is the generation-phase function (whose bias is
    # pinned by brute force elsewhere) on the prefix that ends with it
    slopes = np.array([0.5, 0.25, 0.125, 0.0625])
    assert np.array_equal(oq.prefill_attention_quantized(q, K, V, [128], d_h, alibi_slopes=np.zeros(H)), got)
    biased = oq.prefill_attention_quantized(q, K, V, [128], d_h, alibi_slopes=slopes)
    assert not np.allclose(biased, got, atol=1e-3)
    for jj in (0, 33, n - 1):
        pp = L - n + jj
        row = oq.decode_attention_quantized(q[:, jj], [K[0][:, :pp + 1]], [V[0][:, :pp + 1]], [128], d_h, alibi_slopes=slopes)
        assert np.allclose(biased[:, jj], row, rtol=0, atol=1e-12)
    # (c) query j = 10 (position 140), head 3 (kv head 1): keys 0..127 dequantised, 128..140 as they are
    j, h, kv = 10, 3, 1
    pos = L - n + j
    ck, sk, zk = oq.quantize_keys(K[0][kv, :128])
    cv, sv, zv = oq.quantize_values(V[0][kv, :128])
    sc, vals = [], []
    for t in range(pos + 1):
        if t < 128:
            key = [float(sk[t // 64, c]) * int(ck[t, c]) + float(zk[t // 64, c]) for c in range(r_k)]
            val = [float(sv[t]) * int(cv[t, c]) + float(zv[t]) for c in range(r_v)]
        else:
            key, val = K[0][kv, t], V[0][kv, t]
        sc.append(sum(a * b for a, b in zip(q[0, j, h], key)) / np.sqrt(d_h))
        vals.append(val)
    w = np.exp(np.array(sc) - max(sc))
    assert np.allclose(got[0, j, h], (w[:, None] * np.array(vals)).sum(axis=0) / w.sum(), rtol=0, atol=1e-12)
    # (d)
    n_all = 192
    qa = synth.gaussian(g, (n_all, H, r_k))
    Ka, Va = K[0][:, :n_all], V[0][:, :n_all]
    ch = oq.chunked_prefill_quantized(qa, Ka, Va, 64, d_h)
    one = ora.prefill_attention(qa[None], ora.RankCache.from_arrays([Ka], [Va]), d_h)[0]
    assert np.allclose(ch[:64], one[:64], rtol=0, atol=1e-13) and not np.allclose(ch[64:], one[64:], atol=1e-3)
    assert np.allclose(ch[128:], oq.prefill_attention_quantized(qa[None, 128:], [Ka], [Va], [128], d_h)[0], rtol=0, atol=1e-13)
    # with 128-token key groups the third chunk sees one group, not two
    ch128 = oq.chunked_prefill_quantized(qa[:256], Ka, Va, 128, d_h, group_tokens=128)
    assert np.allclose(ch128[128:], oq.prefill_attention_quantized(qa[None, 128:], [Ka], [Va], [128], d_h, 128)[0], atol=1e-13)


def test_rotary_prefill_over_a_partly_quantised_cache():
    """(a) nothing quantised = the rotary prefill oracle; (b) every query row = the rotary generation-phase function
    (pinned by brute force above) on the prefix that ends with it, the quantised part unchanged; (c) brute force
    for one (query, head) with the rotation written in complex numbers; (d) 3-bit
    codes give something else than 4-bit ones."""
    g = synth.rng(131)
    H, Hkv, r_k, r_v, d_h, L, n = 4, 2, 8, 6, 16, 200, 40
    Uk = synth.orthonormal_basis(g, d_h, r_k)
    K = [synth.gaussian(g, (Hkv, L, r_k))]
    V = [synth.gaussian(g, (Hkv, L, r_v))]
    q = synth.gaussian(g, (1, n, H, d_h))
    plain = ora.prefill_attention_rope(q, ora.RankCache.from_arrays(K, V), Uk, d_h, 100.0)
    assert np.array_equal(oq.prefill_attention_rope_quantized(q, K, V, [0], Uk, d_h, 100.0), plain)
    got = oq.prefill_attention_rope_quantized(q, K, V, [128], Uk, d_h, 100.0)
    assert not np.allclose(got, plain, atol=1e-3)
    for j in (0, 17, n - 1):
        pos = L - n + j
        row = oq.decode_attention_rope_quantized(q[:, j], [K[0][:, :pos + 1]], [V[0][:, :pos + 1]], [128], Uk, d_h, 100.0)
        assert np.allclose(got[:, j], row, rtol=0, atol=1e-12)
    # (c) brute force for one (query, head): keys dequantised by hand, brought back to d_head channels, pairs turned
    # as complex numbers; the score depends on the two positions only through their difference
    j, h, kv = 23, 2, 1
    pos = L - n + j
    ck, sk, zk = oq.quantize_keys(K[0][kv, :128])
    cv, sv, zv = oq.quantize_values(V[0][kv, :128])
    theta = 100.0 ** (-np.arange(0, d_h, 2) / d_h)
    qc = q[0, j, h, 0::2] + 1j * q[0, j, h, 1::2]
    sc, vals = [], []
    for t in range(pos + 1):
        if t < 128:
            key = np.array([float(sk[t // 64, c]) * int(ck[t, c]) + float(zk[t // 64, c]) for c in range(r_k)])
            val = np.array([float(sv[t]) * int(cv[t, c]) + float(zv[t]) for c in range(r_v)])
        else:
            key, val = K[0][kv, t], V[0][kv, t]
        full = Uk @ key
        kc = full[0::2] + 1j * full[1::2]
        sc.append(float(np.real(np.sum(qc * np.conj(kc) * np.exp(1j * theta * (pos - t))))) / np.sqrt(d_h))
        vals.append(val)
    w = np.exp(np.array(sc) - max(sc))
    assert np.allclose(got[0, j, h], (w[:, None] * np.array(vals)).sum(axis=0) / w.sum(), rtol=0, atol=1e-12)
    three = oq.prefill_attention_rope_quantized(q, K, V, [128], Uk, d_h, 100.0, bits=3)
    assert not np.allclose(three, got, atol=1e-3)


def test_three_bit_codes():
    """bits = 3 (the other precision of the paper's Eigen Attention rows): eight levels per group.  Codes 0..7 with
    both ends taken, error within half a step of the group's own scale (seven steps between minimum and maximum),
    values on an eight-level grid reproduced exactly, coarser than four bits by the ratio of the steps, and attention
    over the view is attention over the dequantised values."""
    g = synth.rng(122)
    K = np.float32(synth.gaussian(g, (128, 12))).astype(np.float64)
    c, s, z = oq.quantize_keys(K, 64, bits=3)
    assert c.max() == 7 and c.min() == 0 and s.shape == (2, 12)
    Kg = K.reshape(2, 64, 12)
    span = (Kg.max(axis=1) - Kg.min(axis=1))
    assert np.allclose(s.astype(np.float64), span / 7, rtol=2 ** -10)
    for grp in range(2):
        sel = slice(64 * grp, 64 * grp + 64)
        assert np.all(c[sel][Kg[grp].argmax(axis=0), np.arange(12)] == 7) and np.all(c[sel][Kg[grp].argmin(axis=0), np.arange(12)] == 0)
    err = np.abs(oq.dequantize_keys(c, s, z) - K).reshape(2, 64, 12)
    assert np.all(err <= 0.5 * s.astype(np.float64)[:, None, :] * (1 + 2e-3) + np.abs(z.astype(np.float64) - Kg.min(axis=1))[:, None, :])
    e4 = np.abs(oq.dequantize_keys(*oq.quantize_keys(K, 64)) - K)
    assert 1.7 < err.mean() / e4.mean() < 2.6                     # steps 15/7 times as long
    V = np.float32(synth.gaussian(g, (40, 24))).astype(np.float64)
    cv, sv, zv = oq.quantize_values(V, bits=3)
    assert cv.max() == 7 and np.all(cv.max(axis=1) == 7) and np.all(cv.min(axis=1) == 0)
    assert np.all(np.abs(oq.dequantize_values(cv, sv, zv) - V) <= 0.5 * sv.astype(np.float64)[:, None] * (1 + 2e-3) + 2e-3)
    # an eight-level grid round-trips; a sixteen-level one does not fit
    lo, step = np.float16(g.standard_normal(12)).astype(np.float64), 2.0 ** g.integers(-5, 1, size=12)
    grid = lo + step * g.integers(0, 8, size=(64, 12))
    grid[0], grid[1] = lo, lo + 7 * step
    assert np.array_equal(oq.dequantize_keys(*oq.quantize_keys(grid, 64, bits=3)), grid)
    grid16 = lo + step * g.integers(0, 16, size=(64, 12))
    grid16[0], grid16[1] = lo, lo + 15 * step
    assert not np.array_equal(oq.dequantize_keys(*oq.quantize_keys(grid16, 64, bits=3)), grid16)
    # attention: brute force over hand-dequantised 3-bit values
    H, r_k, r_v, d_h, n = 2, 12, 6, 16, 150
    Kc, Vc = [synth.gaussian(g, (1, n, r_k))], [synth.gaussian(g, (1, n, r_v))]
    q = synth.gaussian(g, (1, H, r_k))
    got = oq.decode_attention_quantized(q, Kc, Vc, [128], d_h, bits=3)
    ck, sk, zk = oq.quantize_keys(Kc[0][0, :128], 64, bits=3)
    cv, sv, zv = oq.quantize_values(Vc[0][0, :128], bits=3)
    keys = np.concatenate([sk.astype(np.float64)[np.arange(128) // 64] * ck + zk.astype(np.float64)[np.arange(128) // 64], Kc[0][0, 128:]])
    vals = np.concatenate([sv.astype(np.float64)[:, None] * cv + zv.astype(np.float64)[:, None], Vc[0][0, 128:]])
    for h in range(H):
        sc = keys @ q[0, h] / np.sqrt(d_h)
        w = np.exp(sc - sc.max())
        assert np.allclose(got[0, h], (w / w.sum()) @ vals, rtol=0, atol=1e-12)
    assert not np.allclose(got, oq.decode_attention_quantized(q, Kc, Vc, [128], d_h), atol=1e-3)
    # the table's 3-bit rows in its own accounting; this build's format at 3 bits
    assert oq.bits_per_element_q4(80, 80, 128, bits=3) == (3.25, 3.4)


def test_three_bit_codes_in_the_rotary_and_the_prefill_form():
    """bits = 3 reaches the other two attention functions: each equals its plain form over the 3-bit view built by
    hand from the quantiser (which test_three_bit_codes pins), differs from the 4-bit result, and the last row of
    the prefill is the generation-phase function; a prompt prefilled in chunks sees its earlier chunks at 3 bits."""
    g = synth.rng(123)
    H, Hkv, r_k, r_v, d_h, L, n = 2, 1, 8, 6, 16, 200, 70

    def view3(X, quantize, dequantize, *a):
        out = np.array(X, np.float64)
        out[:128] = dequantize(*quantize(X[:128], *a, bits=3))
        return out
    K, V = [synth.gaussian(g, (Hkv, L, r_k))], [synth.gaussian(g, (Hkv, L, r_v))]
    K3 = [np.stack([view3(K[0][0], oq.quantize_keys, oq.dequantize_keys, 64)])]
    V3 = [np.stack([view3(V[0][0], oq.quantize_values, oq.dequantize_values)])]
    Uk = synth.orthonormal_basis(g, d_h, r_k)
    qd = synth.gaussian(g, (1, H, d_h))
    rope3 = oq.decode_attention_rope_quantized(qd, K, V, [128], Uk, d_h, 100.0, bits=3)
    assert np.allclose(rope3, ora.decode_attention_rope(qd, ora.RankCache.from_arrays(K3, V3), Uk, d_h, 100.0), rtol=0, atol=1e-13)
    assert not np.allclose(rope3, oq.decode_attention_rope_quantized(qd, K, V, [128], Uk, d_h, 100.0), atol=1e-3)
    q = synth.gaussian(g, (1, n, H, r_k))
    pre3 = oq.prefill_attention_quantized(q, K, V, [128], d_h, bits=3)
    assert np.allclose(pre3, ora.prefill_attention(q, ora.RankCache.from_arrays(K3, V3), d_h), rtol=0, atol=1e-13)
    assert not np.allclose(pre3, oq.prefill_attention_quantized(q, K, V, [128], d_h), atol=1e-3)
    assert np.allclose(pre3[:, -1], oq.decode_attention_quantized(q[:, -1], K, V, [128], d_h, bits=3), rtol=0, atol=1e-13)
    qa = synth.gaussian(g, (192, H, r_k))
    Ka, Va = K[0][:, :192], V[0][:, :192]
    ch3 = oq.chunked_prefill_quantized(qa, Ka, Va, 64, d_h, bits=3)
    assert np.allclose(ch3[128:], oq.prefill_attention_quantized(qa[None, 128:], [Ka], [Va], [128], d_h, bits=3)[0], rtol=0, atol=1e-13)
    assert np.array_equal(ch3[:64], oq.chunked_prefill_quantized(qa, Ka, Va, 64, d_h)[:64])
    assert not np.allclose(ch3[64:], oq.chunked_prefill_quantized(qa, Ka, Va, 64, d_h)[64:], atol=1e-3)

