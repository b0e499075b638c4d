"""ea_decode_attn_rope (Sec. 4.3, Eq. 10: full-rank query, rank-r keys brought back to d_head channels and
rotated) against the fp64 oracle on identical inputs."""
import numpy as np
import pytest
import torch

import paper_2408_05646_amd as ea
from oracle import eigen_attention as ora
from paper_2408_05646_amd import synth
from helpers import DeviceCache, TOL_BF16, TOL_F32, assert_close, quantize, random_cache, to_dev
from test_gpu_fullsize import k_slabs_to_rows, stream_from_pool, v_slabs_to_rows

pytestmark = pytest.mark.gpu


def run_rope(desc, K, V, q, U, base, g, n_splits, page_table_edit=None):
    dc = DeviceCache(desc, K, V, g)
    B = len(K)
    pt = dc.page_table if page_table_edit is None else page_table_edit(dc)
    out = torch.full((B, desc.n_heads, desc.r_v), float("nan"), dtype=torch.float32, device="cuda")
    S = n_splits if n_splits else ea.decode_rope_auto_splits(desc, B, dc.max_pages * desc.page_tokens)
    ws = None
    nbytes = ea.decode_workspace_bytes(desc, B, S)
    if nbytes:
        ws = torch.full((nbytes // 4,), float("nan"), dtype=torch.float32, device="cuda")
    ea.decode_attn_rope(desc, torch.from_numpy(q.astype(np.float32)).cuda(),
                        to_dev(desc, U), base, dc.k_pool, dc.v_pool, pt,
                        dc.seq_len, out, n_splits=S, ws=ws)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def oracle_rope(desc, K, V, q, U, base):
    keep = [b for b in range(len(K)) if K[b].shape[1] > 0]
    ref = np.zeros((len(K), desc.n_heads, desc.r_v))
    if keep:
        cache = ora.RankCache.from_arrays([K[b] for b in keep], [V[b] for b in keep])
        ref[keep] = ora.decode_attention_rope(q[keep], cache, U, desc.d_head, base)
    return ref


def inputs(desc, lens, g, std=1.0):
    U = quantize(desc, synth.orthonormal_basis(g, desc.d_head, desc.r_k))   # one basis for all heads, layer dtype
    K, V = random_cache(desc, lens, g, k_std=std)
    q = np.float32(synth.gaussian(g, (len(lens), desc.n_heads, desc.d_head), std)).astype(np.float64)
    return U, K, V, q


@pytest.mark.parametrize("H,Hkv,d_h,r_k,r_v,lens,P,n_splits,base", [
    (4, 4, 64, 32, 32, [1, 15, 16, 17], 16, 1, 10000.0),
    (4, 2, 64, 30, 33, [255, 256, 257, 700], 32, 3, 10000.0),
    (6, 2, 128, 80, 16, [1000, 3, 511], 64, 0, 500000.0),     # the larger base of the Llama-3 family
    (2, 1, 48, 48, 64, [300], 16, 2, 10000.0),                # r_k = d_h: plain rotary attention
    (4, 4, 64, 32, 32, [0, 40], 16, 1, 10000.0),              # an empty sequence gives a zero row
])
def test_f32_shapes(H, Hkv, d_h, r_k, r_v, lens, P, n_splits, base):
    print(f"rope f32 H={H}/{Hkv} d_h={d_h} r=({r_k},{r_v}) lens={lens} P={P} S={n_splits}", flush=True)
    desc = ea.LayerDesc(H * d_h, H, Hkv, d_h, r_k, r_v, ea.EA_F32, P)
    g = synth.rng(21, H, r_k, len(lens))
    U, K, V, q = inputs(desc, lens, g)
    got = run_rope(desc, K, V, q, U, base, g, n_splits)
    assert_close(got, oracle_rope(desc, K, V, q, U, base), TOL_F32, "rope f32")


def test_f32_far_positions_keep_their_angle():
    """70 000 cached tokens: the fastest pair has turned 70 000 radians, which single precision alone
    would resolve to 4e-3 only."""
    desc = ea.LayerDesc(128, 1, 1, 128, 40, 24, ea.EA_F32, 64)
    g = synth.rng(22)
    U, K, V, q = inputs(desc, [70000], g, std=1.5)
    got = run_rope(desc, K, V, q, U, 10000.0, g, 8)
    assert_close(got, oracle_rope(desc, K, V, q, U, 10000.0), TOL_F32, "rope f32 far")


@pytest.mark.parametrize("H,Hkv,d_h,r_k,r_v,lens,P,n_splits", [
    (2, 2, 128, 80, 80, [1, 63, 64, 65], 64, 1),
    (2, 2, 128, 80, 80, [200, 1000, 129], 64, 3),
    (8, 2, 128, 48, 112, [777, 64, 1500], 128, 0),          # GQA 4:1, r_k != r_v
    (8, 2, 128, 112, 48, [2048, 31], 64, 5),
    (16, 1, 128, 96, 64, [300], 64, 2),                     # 16 query heads on one kv head
    (4, 4, 128, 128, 128, [513, 100], 64, 2),               # r_k = d_h: plain rotary attention
    (4, 2, 128, 72, 40, [150, 70], 64, 2),                  # ranks that need padding channels
    (4, 2, 64, 40, 48, [900, 64], 64, 2),                   # d_h = 64
    (2, 2, 64, 64, 16, [333], 192, 1),
    (2, 2, 128, 80, 80, [0, 100], 64, 1),                   # an empty sequence gives a zero row
    (2, 2, 128, 80, 80, [90], 64, 4),                       # more splits than tiles: empty workgroups
    (2, 1, 128, 80, 80, [20000], 64, 1),                    # one workgroup walks 313 tiles: the stepped rotation
                                                            # of the query is re-computed exactly on the way
    (2, 2, 128, 128, 96, [9000], 64, 1),                    # same with half-tile iterations
    (4, 2, 128, 30, 33, [150, 70], 64, 2),                  # basis rows that are no whole 16-byte units
])
def test_bf16_shapes(H, Hkv, d_h, r_k, r_v, lens, P, n_splits):
    print(f"rope bf16 H={H}/{Hkv} d_h={d_h} r=({r_k},{r_v}) lens={lens} P={P} S={n_splits}", flush=True)
    desc = ea.LayerDesc(H * d_h, H, Hkv, d_h, r_k, r_v, ea.EA_BF16, P)
    g = synth.rng(23, H, r_k, len(lens), n_splits)
    U, K, V, q = inputs(desc, lens, g, std=2.0)
    got = run_rope(desc, K, V, q, U, 10000.0, g, n_splits)
    err = assert_close(got, oracle_rope(desc, K, V, q, U, 10000.0), TOL_BF16, "rope bf16")
    print(f"  rel-L2 {err:.2e}", flush=True)


def test_bf16_position_matters():
    """Same cache, same query: moving the keys one page further (a different position for every key) must change
    the result the way the oracle says -- a kernel that ignored positions would pass every test whose scores
    happen to be position independent, so make sure this one is not."""
    desc = ea.LayerDesc(256, 2, 2, 128, 80, 80, ea.EA_BF16, 64)
    g = synth.rng(24)
    U, K, V, q = inputs(desc, [640], g, std=2.0)
    ref = oracle_rope(desc, K, V, q, U, 10000.0)
    plain = ora.decode_attention(np.einsum("bhc,cr->bhr", q, U), ora.RankCache.from_arrays(K, V), 128)
    assert ora.rel_l2(plain, ref) > 0.2                     # rotary and position-free attention differ a lot here
    got = run_rope(desc, K, V, q, U, 10000.0, g, 2)
    assert_close(got, ref, TOL_BF16, "rope position")


def test_bf16_out_of_range_pages_are_masked_not_read():
    desc = ea.LayerDesc(256, 2, 2, 128, 80, 80, ea.EA_BF16, 64)
    g = synth.rng(25)
    U, K, V, q = inputs(desc, [256], g)

    def edit(dc):
        pt = dc.page_table.clone()
        pt[0, 1] = dc.pool_pages + 1000      # tokens 64..127 vanish (the others keep their positions)
        pt[0, 2] = -5                        # tokens 128..191 vanish
        return pt
    got = run_rope(desc, K, V, q, U, 10000.0, g, 1, page_table_edit=edit)
    # oracle: the same attention with those tokens' scores removed = keys kept at their own positions
    keep = np.r_[0:64, 192:256]
    Uq = U
    refs = []
    for i in range(2):
        K_up = K[0][i] @ Uq.T
        s = (ora.rope_rotate(K_up, np.arange(256)) @ ora.rope_rotate(q[0, i], 255)) / np.sqrt(128.0)
        refs.append(ora.softmax(s[keep]) @ V[0][i][keep])
    assert_close(got, np.stack(refs)[None], TOL_BF16, "rope masked pages")


def test_cfg3_rope_one_layer_sampled():
    """Llama-2-7B-shaped layer at B=16, n=32768, r=80 with rotary positions, split count as bench.py uses; sampled
    (sequence, head) outputs against the oracle, cache contents read back from raw pool memory."""
    s = synth.CFG3
    desc = ea.LayerDesc(s.d_model, s.n_heads, s.n_kv_heads, s.d_head, s.r_k, s.r_v, ea.EA_BF16, 64)
    B, n, P = s.batch, s.n_ctx, 64
    g = synth.rng(26)
    samples = [(0, 0), (15, 31)] + [(int(g.integers(16)), int(g.integers(32))) for _ in range(6)]
    print("cfg3 rope samples", samples, flush=True)
    max_pages = n // P
    pool_pages = B * max_pages
    gen = torch.Generator(device="cuda"); gen.manual_seed(66)
    k_pool, v_pool = ea.alloc_pools(desc, pool_pages, zero=False)
    k_pool.normal_(0.0, 1.00125, generator=gen); v_pool.normal_(0.0, 1.00125, generator=gen)
    pt = torch.randperm(pool_pages, generator=gen, device="cuda").to(torch.int32).reshape(B, max_pages).contiguous()
    seq = torch.full((B,), n, dtype=torch.int32, device="cuda")
    q = torch.randn((B, desc.n_heads, desc.d_head), generator=gen, device="cuda")
    U = quantize(desc, synth.orthonormal_basis(g, desc.d_head, desc.r_k))
    out = torch.full((B, desc.n_heads, desc.r_v), float("nan"), device="cuda")
    S = ea.decode_rope_auto_splits(desc, B, n)
    assert S == 4
    ws = torch.empty(max(ea.decode_workspace_bytes(desc, B, S) // 4, 4), device="cuda")
    ea.decode_attn_rope(desc, q, to_dev(desc, U), 10000.0, k_pool, v_pool, pt, seq, out, n_splits=S, ws=ws)
    torch.cuda.synchronize()
    got_all = out.cpu().numpy()
    assert np.isfinite(got_all).all()
    lay = ea.cache_layout_query(desc)
    qh = q.cpu().numpy().astype(np.float64)
    for (b, h) in samples:
        K = stream_from_pool(k_pool, pt[b], h, desc.n_kv_heads, lay.r_k_pad, k_slabs_to_rows, P)[:, :desc.r_k]
        V = stream_from_pool(v_pool, pt[b], h, desc.n_kv_heads, lay.r_v_pad, v_slabs_to_rows, P)[:, :desc.r_v]
        cache = ora.RankCache.from_arrays([K[None]], [V[None]])
        ref = ora.decode_attention_rope(qh[b:b + 1, h:h + 1], cache, U, desc.d_head)
        assert_close(got_all[b:b + 1, h:h + 1], ref, TOL_BF16, f"rope stream b={b} h={h}")


# ---------------------------------------------------------------------------
# whole generation steps of a rotary model: ea_project_qkv_rope -> ea_decode_attn_rope -> ea_out_proj
# ---------------------------------------------------------------------------
def rope_weights(desc, g):
    """Unfolded weights ~ N(0, 1/d), ONE key basis for all heads, one value basis per kv head; folded
    (Sec. 4.3), rounded to the layer dtype, in the library's out-major layout.  Returns the packed device
    weights, the basis on the device, and the same rounded values as oracle operands."""
    d, H, Hkv, d_h, r_k, r_v = desc.d_model, desc.n_heads, desc.n_kv_heads, desc.d_head, desc.r_k, desc.r_v
    Wq = synth.gaussian(g, (d, H * d_h), d ** -0.5)
    Wk = synth.gaussian(g, (d, Hkv * d_h), d ** -0.5)
    Wv = synth.gaussian(g, (d, Hkv * d_h), d ** -0.5)
    Wo = synth.gaussian(g, (H * d_h, d), d ** -0.5)
    Uk = quantize(desc, synth.orthonormal_basis(g, d_h, r_k))
    Uv = np.stack([synth.orthonormal_basis(g, d_h, r_v) for _ in range(Hkv)])
    Wq_h, Wk_f, Wv_f, Wo_f = ora.fold_weights_rope(Wq, Wk, Wv, Wo, Uk, Uv, H, Hkv)
    rows = [w.T for w in Wq_h] + [w.T for w in Wk_f] + [w.T for w in Wv_f]
    wqkv_t = quantize(desc, np.concatenate(rows, axis=0))                       # [H*d_h + Hkv*(r_k + r_v), d]
    wo_t = quantize(desc, np.concatenate(list(Wo_f), axis=0).T)                 # [d, H*r_v]
    nq, nk = H * d_h, Hkv * r_k
    folded_q = (np.stack([wqkv_t[i * d_h:(i + 1) * d_h].T for i in range(H)]),
                np.stack([wqkv_t[nq + i * r_k:nq + (i + 1) * r_k].T for i in range(Hkv)]),
                np.stack([wqkv_t[nq + nk + i * r_v:nq + nk + (i + 1) * r_v].T for i in range(Hkv)]),
                np.stack([wo_t.T[i * r_v:(i + 1) * r_v] for i in range(H)]))
    return (ea.pack_weight(to_dev(desc, wqkv_t)), ea.pack_weight(to_dev(desc, wo_t)), to_dev(desc, Uk), Uk, folded_q,
            (Wq, Wk, Wv, Wo))


@pytest.mark.parametrize("r", [32, 64])
def test_f32_rope_decode_step(r):
    """Tiny fp32 layer (d=256, H=4, d_h=64, n=256): cache of n-1 tokens, one generation step on the last."""
    print(f"rope step f32 r={r}", flush=True)
    s = synth.CFG1
    desc = ea.LayerDesc(s.d_model, s.n_heads, s.n_kv_heads, s.d_head, r, r, ea.EA_F32, 16)
    g = synth.rng(27, r)
    wqkv, wo, U_dev, Uk, folded_q, unfolded = rope_weights(desc, g)
    x_hist = np.float32(synth.gaussian(g, (s.n_ctx, s.d_model))).astype(np.float64)
    _, k_hist, v_hist = ora.project_qkv(x_hist[:-1], *folded_q[:3])
    K0 = [quantize(desc, k_hist.transpose(1, 0, 2))]
    V0 = [quantize(desc, v_hist.transpose(1, 0, 2))]
    dc = DeviceCache(desc, K0, V0, g, extra_len=1)
    q = torch.empty((1, s.n_heads, s.d_head), dtype=torch.float32, device="cuda")
    o = torch.empty((1, s.n_heads, r), dtype=torch.float32, device="cuda")
    y = torch.empty((1, s.d_model), dtype=torch.float32, device="cuda")
    ea.project_qkv_rope(desc, to_dev(desc, x_hist[-1:]), wqkv, q, dc.k_pool, dc.v_pool, dc.page_table, dc.seq_len, 1)
    ea.decode_attn_rope(desc, q, U_dev, 10000.0, dc.k_pool, dc.v_pool, dc.page_table, dc.seq_len + 1, o, n_splits=1)
    ea.out_proj(desc, o.view(1, -1), wo, y)
    torch.cuda.synchronize()
    y_ref = ora.decode_step_rope(x_hist[-1:], folded_q, Uk, ora.RankCache.from_arrays(K0, V0), s.d_head)
    assert_close(y.cpu().numpy(), y_ref, TOL_F32, "rope step y")
    if r == s.d_head:   # full rank: the variant IS standard rotary attention (up to float32 weights)
        y_std = ora.standard_rope_attention_block(x_hist, *unfolded, s.n_heads, s.n_kv_heads)
        assert ora.rel_l2(y.cpu().numpy(), y_std) <= 2e-5


def test_bf16_project_qkv_rope_many_rows():
    """2100 prompt tokens of one sequence at once (the tall-tile GEMM with the rotary layout of its output: full-rank
    query, rank-r keys of the shared basis, rank-r values): q and the cache contents against the oracle."""
    desc = ea.LayerDesc(256, 4, 2, 64, 40, 32, ea.EA_BF16, 64)
    g = synth.rng(30)
    wqkv, _, _, _, folded_q, _ = rope_weights(desc, g)
    T = 2100
    x = quantize(desc, synth.gaussian(g, (T, 256)))
    dc = DeviceCache(desc, [np.zeros((2, 0, 40))], [np.zeros((2, 0, 32))], g, extra_len=T)
    q = torch.full((T, 4, 64), float("nan"), dtype=torch.bfloat16, device="cuda")
    ea.project_qkv_rope(desc, to_dev(desc, x), wqkv, q, dc.k_pool, dc.v_pool, dc.page_table, dc.seq_len, T)
    kd = torch.zeros((1, 2, T, 40), dtype=torch.bfloat16, device="cuda")
    vd = torch.zeros((1, 2, T, 32), dtype=torch.bfloat16, device="cuda")
    ea.cache_gather(desc, kd, vd, dc.k_pool, dc.v_pool, dc.page_table, pos0=0)
    torch.cuda.synchronize()
    q_ref, k_ref, v_ref = ora.project_qkv(x, *folded_q[:3])             # [T, H, d_h], [T, Hkv, r_k], [T, Hkv, r_v]
    assert_close(q.float().cpu().numpy(), q_ref, TOL_BF16, "q")
    assert_close(kd.float().cpu().numpy()[0], k_ref.transpose(1, 0, 2), TOL_BF16, "cached keys")
    assert_close(vd.float().cpu().numpy()[0], v_ref.transpose(1, 0, 2), TOL_BF16, "cached values")


def test_bf16_rope_decode_steps_end_to_end():
    """GQA layer (d=512, 8 query heads on 2 kv heads, d_h=128, r=(80,48)), bf16: the cache is filled through
    ea_project_qkv_rope (T = 333 tokens at once) and the prompt attended with ea_prefill_attn_rope, then three
    generation steps; against the un-rounded fp64 oracle, so the cache quantisation is part of what is compared."""
    desc = ea.LayerDesc(512, 8, 2, 128, 80, 48, ea.EA_BF16, 64)
    g = synth.rng(28)
    wqkv, wo, U_dev, Uk, folded_q, _ = rope_weights(desc, g)
    B, n0, steps = 4, 333, 3
    x_hist = quantize(desc, synth.gaussian(g, (B, n0 + steps, 512)))
    dc = DeviceCache(desc, [np.zeros((2, 0, 80))] * B, [np.zeros((2, 0, 48))] * B, g, extra_len=n0 + steps)
    q_pre = torch.empty((B * n0, 8, 128), dtype=torch.bfloat16, device="cuda")
    ea.project_qkv_rope(desc, to_dev(desc, x_hist[:, :n0].reshape(B * n0, 512)), wqkv, q_pre, dc.k_pool, dc.v_pool,
                        dc.page_table, dc.seq_len, n0)
    o_pre = torch.empty((B, n0, 8, 48), dtype=torch.bfloat16, device="cuda")
    ws = torch.empty((ea.prefill_rope_workspace_bytes(desc, B, n0, dc.max_pages) // 2,), dtype=torch.bfloat16,
                     device="cuda")
    ea.prefill_attn_rope(desc, q_pre.view(B, n0, 8, 128), U_dev, 10000.0, dc.k_pool, dc.v_pool, dc.page_table,
                         dc.seq_len + n0, o_pre, ws=ws)
    y_pre = torch.empty((B * n0, 512), dtype=torch.bfloat16, device="cuda")
    ea.out_proj(desc, o_pre.view(B * n0, -1), wo, y_pre)
    torch.cuda.synchronize()
    cache = ora.RankCache.empty(B, 2, 80, 48)
    y_pre_ref = ora.prefill_step_rope(x_hist[:, :n0], folded_q, Uk, cache, 128)
    err = assert_close(y_pre.float().cpu().numpy().reshape(B, n0, 512), y_pre_ref, TOL_BF16, "rope bf16 prefill y")
    print(f"  prefill: rel-L2 {err:.2e}", flush=True)
    q = torch.empty((B, 8, 128), dtype=torch.float32, device="cuda")
    o = torch.empty((B, 8, 48), dtype=torch.float32, device="cuda")
    y = torch.empty((B, 512), dtype=torch.bfloat16, device="cuda")
    for t in range(steps):
        ea.project_qkv_rope(desc, to_dev(desc, x_hist[:, n0 + t]), wqkv, q, dc.k_pool, dc.v_pool, dc.page_table,
                            dc.seq_len + n0 + t, 1)
        ea.decode_attn_rope(desc, q, U_dev, 10000.0, dc.k_pool, dc.v_pool, dc.page_table, dc.seq_len + n0 + t + 1, o,
                            n_splits=1)
        ea.out_proj(desc, o.view(B, -1), wo, y)
        torch.cuda.synchronize()
        y_ref = ora.decode_step_rope(x_hist[:, n0 + t], folded_q, Uk, cache, 128)
        err = assert_close(y.float().cpu().numpy(), y_ref, TOL_BF16, f"rope bf16 step {t}")
        print(f"  step {t}: rel-L2 {err:.2e}", flush=True)


def test_rope_decode_step_is_graph_capturable():
    """A rotary generation step (ea_project_qkv_rope -> ea_decode_attn_rope with splits -> ea_out_proj) captured in
    a HIP graph: every replay, with eager work in between, reproduces the eager result bit for bit."""
    desc = ea.LayerDesc(512, 8, 2, 128, 80, 48, ea.EA_BF16, 64)
    g = synth.rng(29)
    wqkv, wo, U_dev, _, _, _ = rope_weights(desc, g)
    B, n0, S = 4, 700, 3
    K0, V0 = random_cache(desc, [n0] * B, g)
    dc = DeviceCache(desc, K0, V0, g, extra_len=1)
    x = to_dev(desc, quantize(desc, synth.gaussian(g, (B, 512))))
    q = torch.empty((B, 8, 128), dtype=torch.float32, device="cuda")
    o = torch.empty((B, 8, 48), dtype=torch.float32, device="cuda")
    y = torch.empty((B, 512), dtype=torch.bfloat16, device="cuda")
    ws = torch.empty(ea.decode_workspace_bytes(desc, B, S) // 4, dtype=torch.float32, device="cuda")
    seq_after = dc.seq_len + 1

    def step():
        ea.project_qkv_rope(desc, x, wqkv, q, dc.k_pool, dc.v_pool, dc.page_table, dc.seq_len, 1)
        ea.decode_attn_rope(desc, q, U_dev, 10000.0, dc.k_pool, dc.v_pool, dc.page_table, seq_after, o, n_splits=S,
                            ws=ws)
        ea.out_proj(desc, o.view(B, -1), wo, y)

    step()
    torch.cuda.synchronize()
    y_eager = y.clone()
    assert float(y_eager.float().abs().sum()) > 0
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                   # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(4):
        y.zero_(); o.zero_(); q.zero_()          # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, y_eager), f"replay {rep} differs from the eager result"


# ---------------------------------------------------------------------------
# ea_prefill_attn_rope
# ---------------------------------------------------------------------------
def run_prefill_rope(desc, K, V, q, U, base, g):
    dc = DeviceCache(desc, K, V, g)
    B, n = q.shape[0], q.shape[1]
    out = torch.full((B, n, desc.n_heads, desc.r_v), float("nan"), dtype=torch.float32, device="cuda").to(
        torch.bfloat16 if desc.dtype == ea.EA_BF16 else torch.float32)
    nbytes = ea.prefill_rope_workspace_bytes(desc, B, n, dc.max_pages)
    ws = torch.full((max(nbytes // 2, 8),), float("nan"), dtype=torch.bfloat16, device="cuda") if nbytes else None
    ea.prefill_attn_rope(desc, to_dev(desc, q), to_dev(desc, U), base, dc.k_pool, dc.v_pool, dc.page_table, dc.seq_len,
                         out, ws=ws)
    torch.cuda.synchronize()
    return out.float().cpu().numpy()


@pytest.mark.parametrize("dtype,H,Hkv,d_h,r_k,r_v,lens,n,P", [
    (ea.EA_F32, 4, 2, 64, 32, 24, [40, 17, 64], 17, 16),
    (ea.EA_F32, 2, 2, 48, 48, 16, [130], 130, 32),
    (ea.EA_BF16, 4, 2, 128, 80, 48, [300, 257, 512], 200, 64),        # queries = the last 200 positions
    (ea.EA_BF16, 2, 2, 128, 80, 80, [333], 333, 64),                  # whole prompt
    (ea.EA_BF16, 8, 2, 64, 40, 32, [129, 64], 64, 128),
    (ea.EA_BF16, 2, 1, 128, 128, 64, [700], 100, 64),                 # r_k = d_h: plain rotary attention
    (ea.EA_BF16, 2, 2, 128, 72, 40, [1500], 70, 192),                 # padded ranks, three tiles per page
])
def test_prefill_rope(dtype, H, Hkv, d_h, r_k, r_v, lens, n, P):
    print(f"rope prefill dtype={dtype} H={H}/{Hkv} d_h={d_h} r=({r_k},{r_v}) lens={lens} n={n} P={P}", flush=True)
    desc = ea.LayerDesc(H * d_h, H, Hkv, d_h, r_k, r_v, dtype, P)
    g = synth.rng(29, H, r_k, n)
    U = quantize(desc, synth.orthonormal_basis(g, d_h, r_k))
    K, V = random_cache(desc, lens, g, k_std=1.5)
    q = quantize(desc, synth.gaussian(g, (len(lens), n, H, d_h), 1.5))
    got = run_prefill_rope(desc, K, V, q, U, 10000.0, g)
    ref = ora.prefill_attention_rope(q, ora.RankCache.from_arrays(K, V), U, d_h)
    err = assert_close(got, ref, TOL_BF16 if dtype == ea.EA_BF16 else TOL_F32, "rope prefill")
    print(f"  rel-L2 {err:.2e}", flush=True)


def test_bf16_rope_half_a_million_tokens():
    """One sequence of 2^19 tokens, GQA 2:1, r = (32, 16): the query has turned 524 287 radians in its fastest pair;
    the stepped rotation is re-seeded exactly 256 times per wave on the way."""
    desc = ea.LayerDesc(256, 2, 1, 128, 32, 16, ea.EA_BF16, 64)
    g = synth.rng(30)
    n = 1 << 19
    print("rope 2^19 tokens", flush=True)
    U = quantize(desc, synth.orthonormal_basis(g, 128, 32))
    K = [quantize(desc, g.standard_normal((1, n, 32), dtype=np.float32))]
    V = [quantize(desc, g.standard_normal((1, n, 16), dtype=np.float32))]
    q = np.float32(synth.gaussian(g, (1, 2, 128), 1.5)).astype(np.float64)
    got = run_rope(desc, K, V, q, U, 10000.0, g, 2)
    err = assert_close(got, oracle_rope(desc, K, V, q, U, 10000.0), TOL_BF16, "rope 2^19")
    print(f"  rel-L2 {err:.2e}", flush=True)
