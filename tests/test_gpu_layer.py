"""ea_project_qkv, ea_out_proj, ea_prefill_attn and whole layer steps against the fp64 oracle."""
import numpy as np
import pytest
import torch

import paper_2408_05646_amd as ea
from oracle import eigen_attention as ora
from paper_2408_05646_amd import synth
from helpers import DeviceCache, TOL_BF16, TOL_F32, assert_close, quantize, random_cache, tdtype, to_dev

pytestmark = pytest.mark.gpu


def make_weights(desc, g):
    """Unfolded weights ~ N(0, 1/d) and per-kv-head orthonormal bases (QR of a Gaussian)."""
    d, H, Hkv, d_h = desc.d_model, desc.n_heads, desc.n_kv_heads, desc.d_head
    Wq = synth.gaussian(g, (d, H * d_h), d ** -0.5)
    Wk = synth.gaussian(g, (d, Hkv * d_h), d ** -0.5)
    Wv = synth.gaussian(g, (d, Hkv * d_h), d ** -0.5)
    Wo = synth.gaussian(g, (H * d_h, d), d ** -0.5)
    Uk = np.stack([synth.orthonormal_basis(g, d_h, desc.r_k) for _ in range(Hkv)])
    Uv = np.stack([synth.orthonormal_basis(g, d_h, desc.r_v) for _ in range(Hkv)])
    return Wq, Wk, Wv, Wo, Uk, Uv


def device_weights(desc, folded):
    """Folded weights in the library's out-major layout, rounded to the layer dtype.
    Returns (wqkv_t, wo_t) on the GPU and the same rounded values as oracle operands."""
    Wq_f, Wk_f, Wv_f, Wo_f = folded
    rows = [Wq_f[i].T for i in range(Wq_f.shape[0])] + [Wk_f[i].T for i in range(Wk_f.shape[0])] + \
           [Wv_f[i].T for i in range(Wv_f.shape[0])]
    wqkv_t = quantize(desc, np.concatenate(rows, axis=0))                       # [N_qkv, d]
    wo_t = quantize(desc, np.concatenate(list(Wo_f), axis=0).T)                 # [d, H*r_v]
    H, Hkv, r_k, r_v = desc.n_heads, desc.n_kv_heads, desc.r_k, desc.r_v
    q_rows, k_rows = H * r_k, Hkv * r_k
    Wq_q = np.stack([wqkv_t[i * r_k:(i + 1) * r_k].T for i in range(H)])
    Wk_q = np.stack([wqkv_t[q_rows + i * r_k:q_rows + (i + 1) * r_k].T for i in range(Hkv)])
    Wv_q = np.stack([wqkv_t[q_rows + k_rows + i * r_v:q_rows + k_rows + (i + 1) * r_v].T for i in range(Hkv)])
    Wo_q = np.stack([wo_t.T[i * r_v:(i + 1) * r_v] for i in range(H)])
    return ea.pack_weight(to_dev(desc, wqkv_t)), ea.pack_weight(to_dev(desc, wo_t)), (Wq_q, Wk_q, Wv_q, Wo_q)


def assert_one_bf16_rounding(got: np.ndarray, ref: np.ndarray):
    """`got` must be ONE round-to-nearest-even of an fp32 accumulation of `ref` (fp64): at most one bf16 step
    away from the rounded reference, plus the fp32 accumulation slack that matters only for values near zero
    (there a bf16 step is smaller than the accumulation error)."""
    ref32 = ref.astype(np.float32)
    step = np.exp2(np.floor(np.log2(np.maximum(np.abs(ref32), 1e-30))) - 7)      # bf16 spacing at |ref|
    slack = 1e-5 * np.abs(ref32).max()
    err = np.abs(got - synth.round_to_bf16(ref32))
    assert (err <= step + slack).all(), float((err - step).max())


# ---------------------------------------------------------------------------
# ea_project_qkv: values and cache placement
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("dtype,d,H,Hkv,r_k,r_v,B,T,P,lens", [
    (ea.EA_F32, 256, 4, 4, 32, 32, 1, 1, 16, [255]),
    (ea.EA_F32, 128, 4, 2, 30, 33, 3, 5, 16, [0, 14, 40]),
    (ea.EA_BF16, 256, 4, 4, 80, 80, 16, 1, 64, list(range(50, 66))),            # generation step, skinny GEMM
    (ea.EA_BF16, 512, 8, 2, 48, 112, 5, 3, 64, [0, 62, 63, 64, 200]),           # 15 rows, appends cross page ends
    (ea.EA_BF16, 256, 4, 2, 72, 40, 2, 100, 128, [0, 60]),                      # 200 rows: tiled GEMM, padded ranks
    (ea.EA_BF16, 4096, 32, 32, 80, 80, 2, 1, 64, [100, 4095]),                  # Llama-2-7B width
    # fragment-wise cache stores of the tiled GEMM: 16-token aligned appends, and sequences that are not aligned
    (ea.EA_BF16, 256, 4, 4, 64, 48, 3, 48, 64, [0, 16, 40]),
    (ea.EA_BF16, 256, 8, 2, 32, 96, 2, 80, 128, [48, 7]),
    (ea.EA_BF16, 512, 4, 4, 80, 80, 1, 300, 64, [64]),                          # rows not a multiple of the tile
    (ea.EA_BF16, 256, 32, 2, 30, 33, 3, 5, 64, [0, 14, 60]),                    # ranks off the 8-channel chunk
    (ea.EA_BF16, 256, 32, 2, 30, 33, 2, 40, 64, [0, 50]),                       # same through the tiled GEMM
    (ea.EA_BF16, 256, 4, 2, 80, 48, 1, 2100, 64, [37]),                         # 2100 rows: the tall (256-row) tiles, ragged
    (ea.EA_BF16, 96, 4, 4, 32, 32, 2, 1100, 64, [0, 5]),                        # ... with three k steps only
    (ea.EA_BF16, 2048, 32, 32, 64, 64, 2, 130, 64, [0, 70]),                    # 260 rows x 6144 columns: 64-row tiles
])
def test_project_qkv(dtype, d, H, Hkv, r_k, r_v, B, T, P, lens):
    print(f"project dtype={dtype} d={d} H={H}/{Hkv} r=({r_k},{r_v}) B={B} T={T} lens={lens}", flush=True)
    desc = ea.LayerDesc(d, H, Hkv, d // H if dtype == ea.EA_F32 else 128, r_k, r_v, dtype, P)
    g = synth.rng(20, d, r_k, T)
    folded = (synth.gaussian(g, (H, d, r_k), d ** -0.5), synth.gaussian(g, (Hkv, d, r_k), d ** -0.5),
              synth.gaussian(g, (Hkv, d, r_v), d ** -0.5), synth.gaussian(g, (H, r_v, d), d ** -0.5))
    wqkv_t, _, (Wq_q, Wk_q, Wv_q, _) = device_weights(desc, folded)
    x = quantize(desc, synth.gaussian(g, (B * T, d)))
    K0, V0 = random_cache(desc, lens, g)
    dc = DeviceCache(desc, K0, V0, g, extra_len=T)
    q_ref, k_ref, v_ref = ora.project_qkv(x, Wq_q, Wk_q, Wv_q)
    for q_dt in ([torch.float32] if dtype == ea.EA_F32 else [torch.float32, torch.bfloat16]):
        q_r = torch.full((B * T, H, r_k), float("nan"), dtype=q_dt, device="cuda")
        ea.project_qkv(desc, to_dev(desc, x), wqkv_t, q_r, dc.k_pool, dc.v_pool, dc.page_table, dc.seq_len, T)
        torch.cuda.synchronize()
        assert_close(q_r.float().cpu().numpy(), q_ref, TOL_F32 if q_dt == torch.float32 else TOL_BF16, "q_r")
    # the appended tokens, read back from their pages
    for b in range(B):
        kd = torch.zeros((1, Hkv, T, r_k), dtype=tdtype(desc), device="cuda")
        vd = torch.zeros((1, Hkv, T, r_v), dtype=tdtype(desc), device="cuda")
        ea.cache_gather(desc, kd, vd, dc.k_pool, dc.v_pool, dc.page_table[b:b + 1].contiguous(), pos0=lens[b])
        torch.cuda.synchronize()
        k_got = kd.float().cpu().numpy()[0].transpose(1, 0, 2)          # [T, Hkv, r_k]
        v_got = vd.float().cpu().numpy()[0].transpose(1, 0, 2)
        kr, vr = k_ref[b * T:(b + 1) * T], v_ref[b * T:(b + 1) * T]
        if dtype == ea.EA_F32:
            assert_close(k_got, kr, TOL_F32, "k append"); assert_close(v_got, vr, TOL_F32, "v append")
        else:   # one RNE rounding of an fp32 accumulator: at most one bf16 step from the rounded fp64 value
            assert_one_bf16_rounding(k_got, kr)
            assert_one_bf16_rounding(v_got, vr)
            assert_close(k_got, kr, TOL_BF16, "k append"); assert_close(v_got, vr, TOL_BF16, "v append")
        # the tokens that were there before are untouched, bit for bit
        if lens[b]:
            kd0 = torch.zeros((1, Hkv, lens[b], r_k), dtype=tdtype(desc), device="cuda")
            ea.cache_gather(desc, kd0, None, dc.k_pool, None, dc.page_table[b:b + 1].contiguous(), pos0=0)
            torch.cuda.synchronize()
            assert np.array_equal(kd0.float().cpu().numpy()[0], K0[b].astype(np.float32))


# ---------------------------------------------------------------------------
# ea_out_proj
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("dtype,d,H,r_v,M", [
    (ea.EA_F32, 256, 4, 32, 1), (ea.EA_F32, 128, 4, 33, 70),
    (ea.EA_BF16, 256, 4, 80, 16), (ea.EA_BF16, 512, 8, 48, 37), (ea.EA_BF16, 256, 4, 40, 300),
    (ea.EA_BF16, 4096, 32, 80, 16),
    (ea.EA_BF16, 256, 4, 40, 2100), (ea.EA_BF16, 200, 2, 16, 2048), (ea.EA_BF16, 640, 4, 16, 2305),   # tall tiles; 5, 1, 2 k steps
    (ea.EA_BF16, 128, 4, 16, 2100),                                # tall tiles, a single 128-wide column tile
    (ea.EA_BF16, 4096, 32, 16, 512), (ea.EA_BF16, 4096, 32, 16, 130),   # 64-row and 32-row tiles over 32 column tiles
])
def test_out_proj(dtype, d, H, r_v, M):
    print(f"out_proj dtype={dtype} d={d} H={H} r_v={r_v} M={M}", flush=True)
    if dtype == ea.EA_F32 and (H * r_v) % 4:
        H = 4; r_v = 36
    desc = ea.LayerDesc(d, H, H, 128, 16, r_v, dtype, 64)
    g = synth.rng(21, d, r_v, M)
    Wo_f = synth.gaussian(g, (H, r_v, d), d ** -0.5)
    wo_t = quantize(desc, np.concatenate(list(Wo_f), axis=0).T)
    Wo_q = np.stack([wo_t.T[i * r_v:(i + 1) * r_v] for i in range(H)])
    o = np.float32(synth.gaussian(g, (M, H, r_v))).astype(np.float64)
    for o_dt in ([torch.float32] if dtype == ea.EA_F32 else [torch.float32, torch.bfloat16]):
        o_in = o if o_dt == torch.float32 else quantize(desc, o)
        y = torch.full((M, d), float("nan"), dtype=tdtype(desc), device="cuda")
        ea.out_proj(desc, torch.from_numpy(o_in.astype(np.float32)).to(o_dt).cuda(), ea.pack_weight(to_dev(desc, wo_t)), y)
        torch.cuda.synchronize()
        assert_close(y.float().cpu().numpy(), ora.out_proj(o_in, Wo_q), TOL_F32 if dtype == ea.EA_F32 else TOL_BF16, "y")


# ---------------------------------------------------------------------------
# ea_prefill_attn (causal)
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("dtype,H,Hkv,r_k,r_v,lens,n,P", [
    (ea.EA_F32, 4, 4, 32, 32, [256], 256, 16),
    (ea.EA_F32, 4, 2, 30, 33, [100, 70], 60, 16),                 # earlier tokens already cached (chunked prefill)
    (ea.EA_BF16, 4, 4, 64, 64, [300], 300, 64),                   # ragged tail, several query tiles
    (ea.EA_BF16, 4, 2, 80, 48, [513, 400], 350, 64),              # GQA, r_k != r_v, cache longer than the chunk
    (ea.EA_BF16, 2, 2, 128, 128, [200], 200, 128),                # full rank
    (ea.EA_BF16, 2, 1, 16, 112, [129], 129, 64),
    (ea.EA_BF16, 2, 2, 64, 64, [64, 1], 1, 64),                   # a single query row
    (ea.EA_BF16, 4, 2, 30, 33, [150, 70], 70, 64),                # ranks off the 8-channel chunk and the 4-channel store
    (ea.EA_BF16, 2, 2, 83, 50, [300], 300, 128),
])
def test_prefill_attn(dtype, H, Hkv, r_k, r_v, lens, n, P):
    print(f"prefill dtype={dtype} H={H}/{Hkv} r=({r_k},{r_v}) lens={lens} n={n}", flush=True)
    d_h = 64 if dtype == ea.EA_F32 else 128
    desc = ea.LayerDesc(H * d_h, H, Hkv, d_h, r_k, r_v, dtype, P)
    g = synth.rng(22, H, r_k, n)
    lens_eff = [max(L, n) for L in lens]
    K, V = random_cache(desc, lens_eff, g, k_std=1.5)
    B = len(lens)
    q = quantize(desc, synth.gaussian(g, (B, n, H, r_k), 1.5))
    dc = DeviceCache(desc, K, V, g)
    out = torch.full((B, n, H, r_v), float("nan"), dtype=tdtype(desc), device="cuda")
    ea.prefill_attn(desc, to_dev(desc, q), dc.k_pool, dc.v_pool, dc.page_table, dc.seq_len, out)
    torch.cuda.synchronize()
    ref = ora.prefill_attention(q, ora.RankCache.from_arrays(K, V), d_h)
    err = assert_close(out.float().cpu().numpy(), ref, TOL_F32 if dtype == ea.EA_F32 else TOL_BF16, "prefill")
    print(f"  rel-L2 {err:.2e}", flush=True)


@pytest.mark.parametrize("shape", ["slow rise", "steep rise", "one giant key"])
@pytest.mark.parametrize("r_k,r_v", [(64, 64), (128, 128), (80, 48)])
def test_prefill_attn_scores_far_above_the_first_tile(shape, r_k, r_v):
    """The bf16 kernel takes unmasked tiles without searching for their maximum and looks at the row sums every few
    tiles.  Scores that climb along the sequence make it move its reference exponent (slow rise: 48 binary orders
    over the sequence), or give the walk up and redo it with the exact maximum (steep rise: 200 orders within eight
    tiles; one key whose score overflows fp32 when exponentiated against the old reference)."""
    print(f"prefill {shape} r=({r_k},{r_v})", flush=True)
    H, d_h, n, P = 2, 128, 1536, 64
    desc = ea.LayerDesc(H * d_h, H, H, d_h, r_k, r_v, ea.EA_BF16, P)
    g = synth.rng(23, r_k, len(shape))
    u = synth.gaussian(g, (H, r_k))
    u /= np.linalg.norm(u, axis=1, keepdims=True)
    rise = {"slow rise": 48.0, "steep rise": 600.0, "one giant key": 0.0}[shape]       # in binary orders over n tokens
    c = rise * np.sqrt(d_h) / (np.log2(np.e) * 4.0)
    ramp = (np.arange(n) / n)[None, :, None]
    K = c * ramp * u[:, None, :] + 0.3 * synth.gaussian(g, (H, n, r_k))
    if shape == "one giant key":
        K[:, 700] = 1000.0 * u
    V = synth.gaussian(g, (H, n, r_v))
    q = 4.0 * u[None, None] + 0.3 * synth.gaussian(g, (1, n, H, r_k))
    K, V, q = quantize(desc, K), quantize(desc, V), quantize(desc, q)
    dc = DeviceCache(desc, [K], [V], g)
    out = torch.full((1, n, H, r_v), float("nan"), dtype=torch.bfloat16, device="cuda")
    ea.prefill_attn(desc, to_dev(desc, q), dc.k_pool, dc.v_pool, dc.page_table, dc.seq_len, out)
    torch.cuda.synchronize()
    ref = ora.prefill_attention(q, ora.RankCache.from_arrays([K], [V]), d_h)
    err = assert_close(out.float().cpu().numpy(), ref, TOL_BF16, "prefill")
    print(f"  rel-L2 {err:.2e}", flush=True)


# ---------------------------------------------------------------------------
# config 1 end to end: project -> append -> decode -> out_proj, r = 32 and the full-rank rerun r = 64
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("r", [32, 64])
def test_cfg1_decode_step(r):
    print(f"cfg1 step r={r}", flush=True)
    s = synth.CFG1
    desc = ea.LayerDesc(s.d_model, s.n_heads, s.n_kv_heads, s.d_head, r, r, ea.EA_F32, 16)
    g = synth.rng(1, 20, r)
    Wq, Wk, Wv, Wo, Uk, Uv = make_weights(desc, g)
    x_hist = np.float32(synth.gaussian(g, (s.n_ctx, s.d_model))).astype(np.float64)
    folded = ora.fold_weights(Wq, Wk, Wv, Wo, Uk, Uv, s.n_heads, s.n_kv_heads)
    wqkv_t, wo_t, folded_q = device_weights(desc, folded)
    # cache of the first n-1 tokens (values as float32 will hold them), then one generation step on the last
    _, k_hist, v_hist = ora.project_qkv(x_hist[:-1], *folded_q[:3])
    K0 = [quantize(desc, k_hist.transpose(1, 0, 2))]
    V0 = [quantize(desc, v_hist.transpose(1, 0, 2))]
    dc = DeviceCache(desc, K0, V0, g, extra_len=1)
    q_r = torch.empty((1, s.n_heads, r), dtype=torch.float32, device="cuda")
    o = torch.empty((1, s.n_heads, r), dtype=torch.float32, device="cuda")
    y = torch.empty((1, s.d_model), dtype=torch.float32, device="cuda")
    ea.project_qkv(desc, to_dev(desc, x_hist[-1:]), wqkv_t, q_r, dc.k_pool, dc.v_pool, dc.page_table, dc.seq_len, 1)
    ea.decode_attn(desc, q_r, dc.k_pool, dc.v_pool, dc.page_table, dc.seq_len + 1, o, n_splits=1)
    ea.out_proj(desc, o.view(1, -1), wo_t, y)
    torch.cuda.synchronize()
    cache = ora.RankCache.from_arrays(K0, V0)
    y_ref = ora.decode_step(x_hist[-1:], folded_q, cache, s.d_head)
    assert_close(y.cpu().numpy(), y_ref, TOL_F32, "cfg1 y")
    if r == s.d_head:   # full rank: the low-rank path IS standard attention (up to float32 weights)
        y_std = ora.standard_attention_block(x_hist, Wq, Wk, Wv, Wo, s.n_heads, s.n_kv_heads)
        assert ora.rel_l2(y.cpu().numpy(), y_std) <= 1e-5


def test_cfg1_prefill_step():
    s = synth.CFG1
    desc = ea.LayerDesc(s.d_model, s.n_heads, s.n_kv_heads, s.d_head, 32, 32, ea.EA_F32, 16)
    g = synth.rng(1, 21)
    Wq, Wk, Wv, Wo, Uk, Uv = make_weights(desc, g)
    x = np.float32(synth.gaussian(g, (1, s.n_ctx, s.d_model))).astype(np.float64)
    folded = ora.fold_weights(Wq, Wk, Wv, Wo, Uk, Uv, s.n_heads, s.n_kv_heads)
    wqkv_t, wo_t, folded_q = device_weights(desc, folded)
    dc = DeviceCache(desc, [np.zeros((4, 0, 32))], [np.zeros((4, 0, 32))], g, extra_len=s.n_ctx)
    n = s.n_ctx
    q_r = torch.empty((n, 4, 32), dtype=torch.float32, device="cuda")
    o = torch.empty((1, n, 4, 32), dtype=torch.float32, device="cuda")
    y = torch.empty((n, s.d_model), dtype=torch.float32, device="cuda")
    ea.project_qkv(desc, to_dev(desc, x[0]), wqkv_t, q_r, dc.k_pool, dc.v_pool, dc.page_table, dc.seq_len, n)
    ea.prefill_attn(desc, q_r.view(1, n, 4, 32), dc.k_pool, dc.v_pool, dc.page_table, dc.seq_len + n, o)
    ea.out_proj(desc, o.view(n, -1), wo_t, y)
    torch.cuda.synchronize()
    y_ref = ora.prefill_step(x, folded_q, ora.RankCache.empty(1, 4, 32, 32), s.d_head)[0]
    assert_close(y.cpu().numpy(), y_ref, TOL_F32, "cfg1 prefill y")


# ---------------------------------------------------------------------------
# bf16 layer steps, end to end against the un-rounded fp64 oracle (includes cache quantisation)
# ---------------------------------------------------------------------------
def test_bf16_decode_step_end_to_end():
    desc = ea.LayerDesc(512, 8, 2, 128, 80, 48, ea.EA_BF16, 64)
    g = synth.rng(23)
    Wq, Wk, Wv, Wo, Uk, Uv = make_weights(desc, g)
    folded = ora.fold_weights(Wq, Wk, Wv, Wo, Uk, Uv, 8, 2)
    wqkv_t, wo_t, folded_q = device_weights(desc, folded)
    B, n0 = 4, 333
    x_hist = quantize(desc, synth.gaussian(g, (B, n0 + 1, 512)))
    dc = DeviceCache(desc, [np.zeros((2, 0, 80))] * B, [np.zeros((2, 0, 48))] * B, g, extra_len=n0 + 1)
    # prefill n0 tokens through the library, then one generation step
    q_pre = torch.empty((B * n0, 8, 80), dtype=torch.bfloat16, device="cuda")
    ea.project_qkv(desc, to_dev(desc, x_hist[:, :n0].reshape(B * n0, 512)), wqkv_t, q_pre, dc.k_pool, dc.v_pool,
                   dc.page_table, dc.seq_len, n0)
    o_pre = torch.empty((B, n0, 8, 48), dtype=torch.bfloat16, device="cuda")
    ea.prefill_attn(desc, q_pre.view(B, n0, 8, 80), dc.k_pool, dc.v_pool, dc.page_table, dc.seq_len + n0, o_pre)
    y_pre = torch.empty((B * n0, 512), dtype=torch.bfloat16, device="cuda")
    ea.out_proj(desc, o_pre.view(B * n0, -1), wo_t, y_pre)
    q_r = torch.empty((B, 8, 80), dtype=torch.float32, device="cuda")
    o = torch.empty((B, 8, 48), dtype=torch.float32, device="cuda")
    y = torch.empty((B, 512), dtype=torch.bfloat16, device="cuda")
    ea.project_qkv(desc, to_dev(desc, x_hist[:, n0]), wqkv_t, q_r, dc.k_pool, dc.v_pool, dc.page_table,
                   dc.seq_len + n0, 1)
    ea.decode_attn(desc, q_r, dc.k_pool, dc.v_pool, dc.page_table, dc.seq_len + n0 + 1, o, n_splits=1)
    ea.out_proj(desc, o.view(B, -1), wo_t, y)
    torch.cuda.synchronize()
    cache = ora.RankCache.empty(B, 2, 80, 48)
    y_pre_ref = ora.prefill_step(x_hist[:, :n0], folded_q, cache, 128)
    y_ref = ora.decode_step(x_hist[:, n0], folded_q, cache, 128)
    assert_close(y_pre.float().cpu().numpy().reshape(B, n0, 512), y_pre_ref, TOL_BF16, "prefill y")
    assert_close(y.float().cpu().numpy(), y_ref, TOL_BF16, "decode y")


def test_decode_step_is_graph_capturable():
    """The library only enqueues kernels on the caller's stream (no allocation, no sync, no memset), so a whole
    decode step can be captured in a HIP graph; every replay must reproduce the eager result."""
    desc = ea.LayerDesc(512, 8, 2, 128, 80, 48, ea.EA_BF16, 64)
    g = synth.rng(24)
    Wq, Wk, Wv, Wo, Uk, Uv = make_weights(desc, g)
    wqkv, wo, _ = device_weights(desc, ora.fold_weights(Wq, Wk, Wv, Wo, Uk, Uv, 8, 2))
    B, n0, S = 4, 700, 3
    K0, V0 = random_cache(desc, [n0] * B, g)
    dc = DeviceCache(desc, K0, V0, g, extra_len=1)
    x = to_dev(desc, quantize(desc, synth.gaussian(g, (B, 512))))
    q_r = torch.empty((B, 8, 80), dtype=torch.float32, device="cuda")
    o = torch.empty((B, 8, 48), dtype=torch.float32, device="cuda")
    y = torch.empty((B, 512), dtype=torch.bfloat16, device="cuda")
    ws = torch.empty(ea.decode_workspace_bytes(desc, B, S) // 4, dtype=torch.float32, device="cuda")
    seq_after = dc.seq_len + 1

    def step():
        ea.project_qkv(desc, x, wqkv, q_r, dc.k_pool, dc.v_pool, dc.page_table, dc.seq_len, 1)
        ea.decode_attn(desc, q_r, dc.k_pool, dc.v_pool, dc.page_table, seq_after, o, n_splits=S, ws=ws)
        ea.out_proj(desc, o.view(B, -1), wo, y)

    step()
    torch.cuda.synchronize()
    y_eager = y.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                   # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(4):
        y.zero_(); o.zero_(); q_r.zero_()        # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, y_eager), f"replay {rep} differs from the eager result"
