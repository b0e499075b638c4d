"""Seeded random shapes through the C ABI against the fp64 oracle: group sizes, head counts, ranks 8..128 (mostly off
every chunk size), page sizes, ragged / empty / tile-edge lengths and split counts drawn at random, for the
generation-phase attention in its five forms (plain, with the attention mass, over the 4-bit cache, ALiBi, rotary)
and the causal prefill attention, the quantised cache in its four formats (4 or 3 bits, key groups of 64 or 128 tokens:
position-free and rotary decode, prefill over codes), the projection GEMMs, and the fp32 form of every call."""
import numpy as np
import pytest
import torch

import paper_2408_05646_amd as ea
from oracle import eigen_attention as ora
from oracle import eviction as oe
from paper_2408_05646_amd import synth
from helpers import DeviceCache, TOL_BF16, assert_close, quantize, random_cache, to_dev
import test_gpu_decode as dec
import test_gpu_q4 as q4

pytestmark = pytest.mark.gpu


def draw(rs, max_len, with_empty):
    G = int(rs.choice([1, 1, 2, 4, 8, 16]))
    Hkv = int(rs.choice([1, 2, 3, 4]))
    r_k, r_v = int(rs.integers(8, 129)), int(rs.integers(8, 129))
    P = int(rs.choice([64, 128, 192, 256]))
    B = int(rs.integers(1, 5))
    edge = [1, 63, 64, 65, 128] + ([0] if with_empty else [])
    lens = [int(rs.choice(edge + [int(rs.integers(1, max_len))])) for _ in range(B)]
    if max(lens) == 0:
        lens[0] = 17
    S = int(rs.choice([0, 1, 2, 3, 5, 8]))
    return G * Hkv, Hkv, r_k, r_v, P, lens, S


@pytest.mark.parametrize("seed", [101, 102])
def test_decode_and_attention_mass_random_shapes(seed):
    rs = np.random.default_rng(seed)
    for case in range(40):
        H, Hkv, r_k, r_v, P, lens, S = draw(rs, 2500, with_empty=True)
        print(f"seed {seed} case {case}: H={H}/{Hkv} r=({r_k},{r_v}) P={P} lens={lens} S={S}", flush=True)
        desc = ea.LayerDesc(H * 128, H, Hkv, 128, r_k, r_v, ea.EA_BF16, P)
        g = synth.rng(seed, case)
        K, V = random_cache(desc, lens, g, k_std=float(rs.choice([0.5, 1.0, 2.0])))
        B = len(lens)
        q = np.float32(synth.gaussian(g, (B, H, r_k), 1.5)).astype(np.float64)
        assert_close(dec.run_decode(desc, K, V, q, g, S), dec.oracle_decode(desc, K, V, q), TOL_BF16, "decode")
        dc = DeviceCache(desc, K, V, g)
        n_cap = dc.max_pages * P
        S_eff = S or ea.decode_auto_splits(desc, B, n_cap)
        ws = torch.full((ea.decode_attn_mass_workspace_bytes(desc, B, dc.max_pages, S_eff) // 4,), float("nan"),
                        device="cuda")
        mass = torch.zeros((B, Hkv, n_cap), device="cuda")
        out = torch.full((B, H, r_v), float("nan"), device="cuda")
        ea.decode_attn_mass(desc, torch.from_numpy(q.astype(np.float32)).cuda(), dc.k_pool, dc.v_pool, dc.page_table,
                            dc.seq_len, out, mass, S, ws)
        torch.cuda.synchronize()
        keep = [b for b in range(B) if lens[b] > 0]
        cache = ora.RankCache.from_arrays([K[b] for b in keep], [V[b] for b in keep])
        assert_close(out.cpu().numpy()[keep], ora.decode_attention(q[keep], cache, 128), TOL_BF16, "fused output")
        ref_m = oe.attention_mass(q[keep], cache, 128)
        got_m = mass.cpu().numpy()
        for i, b in enumerate(keep):
            assert_close(got_m[b, :, :lens[b]], ref_m[i], TOL_BF16, f"mass b={b}")
        for b in range(B):
            assert not got_m[b, :, lens[b]:].any()


@pytest.mark.parametrize("seed", [201, 202])
def test_q4_prefill_alibi_and_rotary_random_shapes(seed):
    rs = np.random.default_rng(seed)
    for case in range(30):
        H, Hkv, r_k, r_v, P, lens, S = draw(rs, 2000, with_empty=False)
        P = min(P, 192)
        print(f"seed {seed} case {case}: H={H}/{Hkv} r=({r_k},{r_v}) P={P} lens={lens} S={S}", flush=True)
        desc = ea.LayerDesc(H * 128, H, Hkv, 128, r_k, r_v, ea.EA_BF16, P)
        g = synth.rng(seed, case)
        B = len(lens)
        # ---- 4-bit cache: a random number of whole pages quantised, the rest bf16
        K, V = q4.offset_cache(desc, lens, g, k_std=1.5)
        n_quant = [int(rs.integers(0, n // P + 1)) * P for n in lens]
        q = np.float32(synth.gaussian(g, (B, H, r_k), 1.5)).astype(np.float64)
        qc = q4.Q4Cache(desc, K, V, n_quant, g)
        assert_close(q4.run_q4(desc, qc, q, S), q4.oracle_q4(desc, K, V, q, n_quant), TOL_BF16, "q4 decode")
        # ---- causal prefill of the last n tokens
        Kp, Vp = random_cache(desc, lens, g)
        cache = ora.RankCache.from_arrays(Kp, Vp)
        n = min(int(rs.integers(1, min(lens) + 1)), 300)
        qp = quantize(desc, synth.gaussian(g, (B, n, H, r_k)))
        dc = DeviceCache(desc, Kp, Vp, g)
        out = torch.full((B, n, H, r_v), float("nan"), dtype=torch.bfloat16, device="cuda")
        ea.prefill_attn(desc, to_dev(desc, qp), dc.k_pool, dc.v_pool, dc.page_table, dc.seq_len, out)
        torch.cuda.synchronize()
        assert_close(out.float().cpu().numpy(), ora.prefill_attention(qp, cache, 128), TOL_BF16, "prefill")
        # ---- the same prefill with the ALiBi bias: the MPT slopes, steep ones (1 or 3 per token) or none, per case
        slopes = [2.0 ** (-8.0 * (np.arange(H) + 1) / H), np.where(np.arange(H) % 2 == 0, 1.0, 3.0),
                  np.zeros(H)][case % 3].astype(np.float32).astype(np.float64)
        out.fill_(float("nan"))
        ea.prefill_attn_alibi(desc, to_dev(desc, qp), torch.from_numpy(slopes.astype(np.float32)).cuda(), dc.k_pool,
                              dc.v_pool, dc.page_table, dc.seq_len, out)
        torch.cuda.synchronize()
        assert_close(out.float().cpu().numpy(), ora.prefill_attention(qp, cache, 128, alibi_slopes=slopes), TOL_BF16,
                     "alibi prefill")
        # ---- ALiBi decode
        slopes = 2.0 ** (-8.0 * (np.arange(H) + 1) / H)
        qa = np.float32(synth.gaussian(g, (B, H, r_k))).astype(np.float64)
        oa = torch.full((B, H, r_v), float("nan"), device="cuda")
        S_eff = S or ea.decode_auto_splits(desc, B, dc.max_pages * P)
        ws = torch.empty(max(ea.decode_workspace_bytes(desc, B, S_eff) // 4, 4), device="cuda")
        ea.decode_attn_alibi(desc, torch.from_numpy(qa.astype(np.float32)).cuda(),
                             torch.from_numpy(slopes.astype(np.float32)).cuda(), dc.k_pool, dc.v_pool, dc.page_table,
                             dc.seq_len, oa, n_splits=S_eff, ws=ws)
        torch.cuda.synchronize()
        assert_close(oa.cpu().numpy(), ora.decode_attention(qa, cache, 128, alibi_slopes=slopes), TOL_BF16, "alibi decode")
        # ---- rotary decode (one shared key basis, r_k <= d_h)
        U = quantize(desc, synth.orthonormal_basis(g, 128, r_k))
        qr = np.float32(synth.gaussian(g, (B, H, 128), 1.5)).astype(np.float64)
        orr = torch.full((B, H, r_v), float("nan"), device="cuda")
        S_r = S or ea.decode_rope_auto_splits(desc, B, dc.max_pages * P)
        ws = torch.empty(max(ea.decode_workspace_bytes(desc, B, S_r) // 4, 4), device="cuda")
        ea.decode_attn_rope(desc, torch.from_numpy(qr.astype(np.float32)).cuda(), to_dev(desc, U), 10000.0, dc.k_pool,
                            dc.v_pool, dc.page_table, dc.seq_len, orr, n_splits=S_r, ws=ws)
        torch.cuda.synchronize()
        assert_close(orr.cpu().numpy(), ora.decode_attention_rope(qr, cache, U, 128), TOL_BF16, "rotary decode")


@pytest.mark.parametrize("seed", [251, 252])
def test_quantised_cache_random_formats(seed):
    """Code width (4 or 3 bits) and key group (64 or 128 tokens) drawn with the shape: the position-free and the rotary
    generation-phase attention and the prefill over codes, each against the oracle that quantises the same way."""
    from oracle import quant_cache as oq
    import test_gpu_q4_prefill as q4p
    rs = np.random.default_rng(seed)
    for case in range(24):
        H, Hkv, r_k, r_v, P, lens, S = draw(rs, 1800, with_empty=False)
        bits, group = int(rs.choice([3, 4])), int(rs.choice([64, 128]))
        if group == 128 and P % 128:
            P = 128
        print(f"seed {seed} case {case}: H={H}/{Hkv} r=({r_k},{r_v}) P={P} bits={bits} group={group} lens={lens} S={S}",
              flush=True)
        desc = ea.LayerDesc(H * 128, H, Hkv, 128, r_k, r_v, ea.EA_BF16, P, group, bits)
        g = synth.rng(seed, case)
        B = len(lens)
        K, V = q4.offset_cache(desc, lens, g, k_std=1.5)
        n_quant = [int(rs.integers(0, (n - 1) // P + 1)) * P for n in lens]        # at least one token stays in 16 bits
        qc = q4.Q4Cache(desc, K, V, n_quant, g)
        q = np.float32(synth.gaussian(g, (B, H, r_k), 1.5)).astype(np.float64)
        ref = oq.decode_attention_quantized(q, K, V, n_quant, 128, group_tokens=group, bits=bits)
        assert_close(q4.run_q4(desc, qc, q, S), ref, TOL_BF16, "quantised decode")
        U = quantize(desc, synth.orthonormal_basis(g, 128, r_k))
        qr = np.float32(synth.gaussian(g, (B, H, 128), 1.5)).astype(np.float64)
        ref = oq.decode_attention_rope_quantized(qr, K, V, n_quant, U, 128, 10000.0, group_tokens=group, bits=bits)
        assert_close(q4.run_rope_q4(desc, qc, qr, U, 10000.0, S), ref, TOL_BF16, "quantised rotary decode")
        n = min(min(lens[b] - n_quant[b] for b in range(B)), 200)
        qp = quantize(desc, synth.gaussian(g, (B, n, H, r_k)))
        ref = oq.prefill_attention_quantized(qp, K, V, n_quant, 128, group_tokens=group, bits=bits)
        assert_close(q4p.run_prefill_q4(desc, qc, qp), ref, TOL_BF16, "prefill over codes")


@pytest.mark.parametrize("seed", [301])
def test_projection_gemms_random_shapes(seed):
    """ea_project_qkv (q, and the cache contents it appends) and ea_out_proj over random widths, ranks, row counts from
    one to a few thousand (the generation-phase kernel, the 128- and 256-row tiled kernels, the asynchronous one) and
    sequences that already hold a few tokens."""
    import contextlib
    import io
    import test_gpu_layer as layer
    rs = np.random.default_rng(seed)
    for case in range(40):
        H, Hkv = 4, int(rs.choice([1, 2, 4]))
        r_k, r_v = int(rs.integers(8, 129)), int(rs.integers(1, 17)) * 8          # (H r_v) % 32 == 0 for the packing
        P, d = int(rs.choice([64, 128, 192])), int(rs.integers(3, 21)) * 32
        B = int(rs.integers(1, 4))
        T = int(rs.choice([1, 5, 16, 21, 64, 100, 333, 700, 2048 // B + 1, 2500 // B]))
        lens = [int(rs.choice([0, 5, 63, 64, 100])) for _ in range(B)]
        M = int(rs.choice([1, 16, 37, 64, 65, 127, 300, 2047, 2048, 2100, 2600, 3000]))
        print(f"seed {seed} case {case}: d={d} H={H}/{Hkv} r=({r_k},{r_v}) P={P} B={B} T={T} lens={lens} M={M}", flush=True)
        with contextlib.redirect_stdout(io.StringIO()):
            layer.test_project_qkv(ea.EA_BF16, d, H, Hkv, r_k, r_v, B, T, P, lens)
            layer.test_out_proj(ea.EA_BF16, d, H, r_v, M)


@pytest.mark.parametrize("seed", [401])
def test_f32_path_random_shapes(seed):
    """The fp32 (reference-precision) form of every call: any rank from 1, any page size that is a multiple of 16,
    group sizes 1..4, empty and tile-edge lengths, through the parametrised tests of the other files."""
    import contextlib
    import io
    import test_gpu_alibi as alibi
    import test_gpu_eviction as evict
    import test_gpu_layer as layer
    import test_gpu_rope as rope
    rs = np.random.default_rng(seed)
    for case in range(40):
        G, Hkv = int(rs.choice([1, 2, 3, 4])), int(rs.choice([1, 2, 3]))
        H = G * Hkv
        r_k, r_v = int(rs.integers(1, 129)), int(rs.integers(1, 129))
        P, B = int(rs.choice([16, 32, 48, 64, 80])), int(rs.integers(1, 4))
        lens = [int(rs.choice([0, 1, 15, 16, 17, int(rs.integers(1, 1500))])) for _ in range(B)]
        if max(lens) == 0:
            lens[0] = 9
        S = int(rs.choice([0, 1, 2, 3]))
        d_h = int(rs.choice([32, 48, 64, 128]))
        rk_rot = int(rs.integers(1, d_h + 1))
        full = [max(1, n) for n in lens]
        n = int(rs.integers(1, min(full) + 1))
        print(f"seed {seed} case {case}: H={H}/{Hkv} r=({r_k},{r_v}) d_h={d_h} r_k(rotary)={rk_rot} P={P} lens={lens} "
              f"S={S} n={n}", flush=True)
        with contextlib.redirect_stdout(io.StringIO()):
            dec.test_f32_shapes(H, Hkv, r_k, r_v, lens, P, S)
            rope.test_f32_shapes(H, Hkv, d_h, rk_rot, r_v, lens, P, S, 10000.0)
            layer.test_prefill_attn(ea.EA_F32, H, Hkv, r_k, r_v, full, n, P)
            alibi.test_prefill_alibi(ea.EA_F32, H, Hkv, r_k, r_v, full, n, P)
            rope.test_prefill_rope(ea.EA_F32, H, Hkv, d_h, rk_rot, r_v, full, n, P)
            evict.test_attn_mass_matches_oracle(ea.EA_F32, H, Hkv, r_k, lens, P)
