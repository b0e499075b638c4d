"""Parity at the full sizes of the workload configurations, in the launch configuration
bench.py times, on sampled outputs the oracle computes one by one.

Oracle inputs never pass through the library: cache contents are read from raw device
memory with torch and un-laid-out here, with index arithmetic written from the header's
description of the layout."""
import numpy as np
import pytest
import torch

import paper_2408_05646_amd as ea
from oracle import eigen_attention as ora
from oracle import eviction as oe
from paper_2408_05646_amd import synth
from helpers import TOL_BF16, assert_close

pytestmark = pytest.mark.gpu


def k_slabs_to_rows(slabs: np.ndarray, r_pad: int) -> np.ndarray:
    """[n_tiles, 64*r_pad] K tiles -> [n_tiles*64, r_pad]: tile = [4 blocks][r_pad/8 chunks][16 tokens][8 channels]."""
    t = slabs.reshape(-1, 4, r_pad // 8, 16, 8)
    return t.transpose(0, 1, 3, 2, 4).reshape(-1, r_pad)


def v_slabs_to_rows(slabs: np.ndarray, r_pad: int) -> np.ndarray:
    """V tile = [2 groups][r_pad/16 blocks][4 quads][16 channels][8 slots], slot j of quad q = token 16*(j/4)+4*q+j%4."""
    t = slabs.reshape(-1, 2, r_pad // 16, 4, 16, 2, 4)           # tile, grp, cb, quad, c, j/4, j%4
    return t.transpose(0, 1, 5, 3, 6, 2, 4).reshape(-1, r_pad)   # token = grp*32 + (j/4)*16 + quad*4 + j%4


def stream_from_pool(pool, page_table_row, head, n_kv_heads, r_pad, rows_fn, page_tokens):
    """Rows [n, r_pad] (float64) of one (sequence, kv head) stream, read from raw pool memory."""
    slab = page_tokens * r_pad
    view = pool.view(pool.shape[0], n_kv_heads, slab)
    got = view[page_table_row.long(), head].float().cpu().numpy()          # [pages, slab]
    return rows_fn(got.reshape(-1, 64 * r_pad), r_pad).astype(np.float64)


def shape_stream(desc, k_pool, pt, q, b, kvh, kind, n):
    """Rewrites the keys of one (sequence, kv head) stream in place so that its scores against the stream's first
    query head follow a pattern: "peak" = one token (two thirds into the sequence) scores 40 above the rest,
    "ramp" = the scores climb by 30 over the sequence (the softmax reference moves many times on the way)."""
    Hkv, G = desc.n_kv_heads, desc.n_heads // desc.n_kv_heads
    row = pt[b:b + 1].contiguous()
    kd = torch.empty((1, Hkv, n, desc.r_k), dtype=torch.bfloat16, device="cuda")
    ea.cache_gather(desc, kd, None, k_pool, None, row)
    qv = q[b, kvh * G].double()
    t = torch.arange(n, device="cuda", dtype=torch.float64)
    alpha = torch.zeros(n, dtype=torch.float64, device="cuda")
    if kind == "peak":
        alpha[(2 * n) // 3] = 40.0
    else:
        alpha = 30.0 * t / n
    along = alpha[:, None] * (desc.d_head ** 0.5 / float(qv.norm()) ** 2) * qv[None, :]     # q . along[t] / sqrt(d_h) = alpha[t]
    kd[0, kvh] = (0.1 * kd[0, kvh].double() + along).to(torch.bfloat16)
    ea.cache_scatter(desc, kd, None, k_pool, None, row)
    torch.cuda.synchronize()


def run_sampled_decode(desc, B, n, samples, seed, n_splits=0, with_mass=False, shaped=None):
    P = desc.page_tokens
    max_pages = n // P
    pool_pages = B * max_pages
    gen = torch.Generator(device="cuda"); gen.manual_seed(seed)
    k_pool, v_pool = ea.alloc_pools(desc, pool_pages, zero=False)
    k_pool.normal_(0.0, 1.00125, generator=gen); v_pool.normal_(0.0, 1.00125, generator=gen)
    pt = torch.randperm(pool_pages, generator=gen, device="cuda").to(torch.int32).reshape(B, max_pages).contiguous()
    seq = torch.full((B,), n, dtype=torch.int32, device="cuda")
    q = torch.randn((B, desc.n_heads, desc.r_k), generator=gen, device="cuda")
    out = torch.full((B, desc.n_heads, desc.r_v), float("nan"), device="cuda")
    for (b, kvh), kind in (shaped or {}).items():
        shape_stream(desc, k_pool, pt, q, b, kvh, kind, n)
    S = n_splits or ea.decode_auto_splits(desc, B, n)
    mass = None
    if with_mass:      # the fused call: the same output, and the attention mass of every cached token
        mass = torch.zeros((B, desc.n_kv_heads, n), device="cuda")
        ws = torch.empty(ea.decode_attn_mass_workspace_bytes(desc, B, max_pages, S) // 4, device="cuda")
        ea.decode_attn_mass(desc, q, k_pool, v_pool, pt, seq, out, mass, S, ws)
    else:
        ws = torch.empty(max(ea.decode_workspace_bytes(desc, B, S) // 4, 4), device="cuda")
        ea.decode_attn(desc, q, k_pool, v_pool, pt, seq, out, n_splits=S, ws=ws)
    torch.cuda.synchronize()
    got_all = out.cpu().numpy()
    assert np.isfinite(got_all).all()
    lay = ea.cache_layout_query(desc)
    G = desc.n_heads // desc.n_kv_heads
    qh = q.cpu().numpy().astype(np.float64)
    for (b, kvh) in samples:
        K = stream_from_pool(k_pool, pt[b], kvh, desc.n_kv_heads, lay.r_k_pad, k_slabs_to_rows, P)[:, :desc.r_k]
        V = stream_from_pool(v_pool, pt[b], kvh, desc.n_kv_heads, lay.r_v_pad, v_slabs_to_rows, P)[:, :desc.r_v]
        cache = ora.RankCache.from_arrays([K[None]], [V[None]])
        heads = list(range(kvh * G, (kvh + 1) * G))
        ref = ora.decode_attention(qh[b:b + 1, heads], cache, desc.d_head)
        assert_close(got_all[b:b + 1, heads], ref, TOL_BF16, f"stream b={b} kvh={kvh}")
        if with_mass:
            ref_m = oe.attention_mass(qh[b:b + 1, heads], cache, desc.d_head)[0]
            assert_close(mass[b, kvh].cpu().numpy()[None], ref_m, TOL_BF16, f"mass b={b} kvh={kvh}")
    if with_mass:      # any size: every row of the statistic sums to the group's number of query heads
        sums = mass.sum(dim=2).cpu().numpy()
        assert np.allclose(sums, G, rtol=0, atol=2e-3), (sums.min(), sums.max())
    # any size: the output is a convex combination of value rows
    assert np.abs(got_all).max() <= float(v_pool.abs().max()) * 1.001
    return S


def test_cfg3_one_layer_sampled():
    """B=16, n=32768, H=32, r=80 (one of the 32 resident layers), split count as bench.py uses."""
    s = synth.CFG3
    desc = ea.LayerDesc(s.d_model, s.n_heads, s.n_kv_heads, s.d_head, s.r_k, s.r_v, ea.EA_BF16, 64)
    g = synth.rng(3, 1)
    samples = [(0, 0), (15, 31)] + [(int(g.integers(16)), int(g.integers(32))) for _ in range(10)]
    print("cfg3 samples", samples, flush=True)
    S = run_sampled_decode(desc, s.batch, s.n_ctx, samples, seed=33)
    assert S == ea.decode_auto_splits(desc, s.batch, s.n_ctx) == 1


def test_cfg3_full_length_peaked_and_ramped_streams():
    """The same launch with two streams whose softmax is far from flat over all 32768 tokens: one token that takes
    (almost) all of the probability, and scores that climb steadily to the end of the sequence."""
    s = synth.CFG3
    desc = ea.LayerDesc(s.d_model, s.n_heads, s.n_kv_heads, s.d_head, s.r_k, s.r_v, ea.EA_BF16, 64)
    shaped = {(3, 5): "peak", (12, 30): "ramp", (0, 0): "ramp", (15, 31): "peak"}
    print("cfg3 shaped streams", shaped, flush=True)
    run_sampled_decode(desc, s.batch, s.n_ctx, list(shaped) + [(3, 6), (12, 29)], seed=36, shaped=shaped)


def test_cfg3_one_layer_with_attention_mass_sampled():
    """The same shape through ea_decode_attn_mass, as `bench.py --workload cfg3-h2o` runs it."""
    s = synth.CFG3
    desc = ea.LayerDesc(s.d_model, s.n_heads, s.n_kv_heads, s.d_head, s.r_k, s.r_v, ea.EA_BF16, 64)
    g = synth.rng(3, 2)
    samples = [(0, 0), (15, 31)] + [(int(g.integers(16)), int(g.integers(32))) for _ in range(6)]
    print("cfg3 mass samples", samples, flush=True)
    run_sampled_decode(desc, s.batch, s.n_ctx, samples, seed=35, with_mass=True)


def test_cfg3_fullrank_baseline_sampled():
    """The d_h = 128 comparison kernel at the same B and n."""
    s = synth.CFG3_FULLRANK
    desc = ea.LayerDesc(s.d_model, s.n_heads, s.n_kv_heads, s.d_head, 128, 128, ea.EA_BF16, 64)
    print("cfg3 full rank", flush=True)
    run_sampled_decode(desc, s.batch, s.n_ctx, [(0, 0), (7, 13), (15, 31)], seed=34)


def test_cfg5_gqa_heterogeneous_ranks_sampled():
    """B=8, n=16384, 32 query heads on 8 kv heads; every distinct rank from {48,..,112} as r_k and as r_v."""
    s = synth.CFG5
    ranks = synth.cfg5_layer_ranks(32)
    assert set(r for pair in ranks for r in pair) <= set(synth.CFG5_RANKS)
    seen, picked = set(), []
    for rk, rv in ranks:                      # layers in order until every rank was used on both sides
        if ("k", rk) not in seen or ("v", rv) not in seen:
            picked.append((rk, rv)); seen.add(("k", rk)); seen.add(("v", rv))
    print("cfg5 layers checked", picked, flush=True)
    for li, (rk, rv) in enumerate(picked):
        desc = ea.LayerDesc(s.d_model, s.n_heads, s.n_kv_heads, s.d_head, rk, rv, ea.EA_BF16, 64)
        run_sampled_decode(desc, s.batch, s.n_ctx, [(0, 0), (7, 7), (3, li % 8)], seed=50 + li)


def test_cfg4_prefill_chain_sampled():
    """B=4, n=8192, d=4096, H=32, r=64, bf16: project_qkv + cache write + causal attention + out_proj,
    checked end to end (fp64, no rounding in the oracle) on sampled rows of one sequence."""
    s = synth.CFG4
    d, H, r, B, n = s.d_model, s.n_heads, s.r_k, s.batch, s.n_ctx
    desc = ea.LayerDesc(d, H, H, s.d_head, r, r, ea.EA_BF16, 64)
    g = synth.rng(4, 0)
    print("cfg4 generating inputs", flush=True)
    # folded weights = N(0, 1/d) weights times a 128 x 64 orthonormal basis per head, rounded to bf16
    U = np.stack([synth.orthonormal_basis(g, 128, r) for _ in range(H)])
    def folded(shape_heads):
        W = synth.gaussian(g, (shape_heads, d, 128), d ** -0.5)
        return np.einsum("hdk,hkr->hdr", W, U)
    Wq_f, Wk_f, Wv_f = folded(H), folded(H), folded(H)
    Wo_f = np.einsum("hkr,hkd->hrd", U, synth.gaussian(g, (H, 128, d), d ** -0.5))
    wqkv_t = synth.round_to_bf16(np.concatenate([w.T for w in Wq_f] + [w.T for w in Wk_f] + [w.T for w in Wv_f])
                                 .astype(np.float32))                       # [3*H*r, d]
    wo_t = synth.round_to_bf16(np.concatenate(list(Wo_f)).T.astype(np.float32))   # [d, H*r]
    x = synth.round_to_bf16(g.standard_normal((B, n, d), dtype=np.float32))
    dev = lambda a: torch.from_numpy(a).to(torch.bfloat16).cuda()
    max_pages = n // 64
    pool_pages = B * max_pages
    k_pool, v_pool = ea.alloc_pools(desc, pool_pages)
    pt = torch.from_numpy(synth.random_page_table(g, B, max_pages, pool_pages)).cuda()
    seq0 = torch.zeros((B,), dtype=torch.int32, device="cuda")
    q_r = torch.empty((B * n, H, r), dtype=torch.bfloat16, device="cuda")
    o = torch.empty((B, n, H, r), dtype=torch.bfloat16, device="cuda")
    y = torch.empty((B * n, d), dtype=torch.bfloat16, device="cuda")
    print("cfg4 running the HIP path", flush=True)
    ea.project_qkv(desc, dev(x.reshape(B * n, d)), ea.pack_weight(dev(wqkv_t)), q_r, k_pool, v_pool, pt, seq0, n)
    ea.prefill_attn(desc, q_r.view(B, n, H, r), k_pool, v_pool, pt, seq0 + n, o)
    ea.out_proj(desc, o.view(B * n, H * r), ea.pack_weight(dev(wo_t)), y)
    torch.cuda.synchronize()
    y_gpu = y.float().view(B, n, d).cpu().numpy()
    assert np.isfinite(y_gpu).all()
    print("cfg4 oracle on sampled rows", flush=True)
    b = 3
    rows = [0, 1, 63, 64, 255, 256, 257, 4095, 4096, 8000, 8190, 8191]
    w64 = wqkv_t.astype(np.float64)
    xb = x[b].astype(np.float64)
    proj = xb @ w64.T                                                      # [n, 3*H*r] in fp64
    q_all, k_all, v_all = proj[:, :H * r], proj[:, H * r:2 * H * r], proj[:, 2 * H * r:]
    Wo_q = np.stack([wo_t.T[i * r:(i + 1) * r] for i in range(H)]).astype(np.float64)
    ref = np.zeros((len(rows), d))
    for ri, j in enumerate(rows):
        K = [k_all[:j + 1].reshape(j + 1, H, r).transpose(1, 0, 2)]
        V = [v_all[:j + 1].reshape(j + 1, H, r).transpose(1, 0, 2)]
        o_j = ora.decode_attention(q_all[j].reshape(1, H, r), ora.RankCache.from_arrays(K, V), s.d_head)
        ref[ri] = ora.out_proj(o_j, Wo_q)[0]
    err = assert_close(y_gpu[b, rows], ref, TOL_BF16, "cfg4 y rows")
    print(f"  cfg4 end-to-end rel-L2 {err:.2e}", flush=True)


def test_one_million_cached_tokens():
    """One sequence of 2^20 tokens (16384 pages in random order), one kv head, r = 16: index arithmetic at the large
    end, 64 splits, checked against the oracle in full (the oracle's cost is one 2^20 x 16 product)."""
    desc = ea.LayerDesc(128, 2, 1, 128, 16, 16, ea.EA_BF16, 64)
    n = 1 << 20
    print("2^20 tokens", flush=True)
    S = run_sampled_decode(desc, 1, n, [(0, 0)], seed=71, n_splits=64)
    assert S == 64
