"""ea_decode_attn against the fp64 oracle on identical inputs."""
import numpy as np
import pytest
import torch

import paper_2408_05646_amd as ea
from oracle import eigen_attention as ora
from paper_2408_05646_amd import synth
from helpers import DeviceCache, TOL_BF16, TOL_F32, assert_close, random_cache

pytestmark = pytest.mark.gpu


def run_decode(desc, K, V, q, g, n_splits, **kw):
    dc = DeviceCache(desc, K, V, g, **kw)
    B = len(K)
    out = torch.full((B, desc.n_heads, desc.r_v), float("nan"), dtype=torch.float32, device="cuda")
    S = n_splits if n_splits else ea.decode_auto_splits(desc, B, dc.max_pages * desc.page_tokens)
    ws = None
    nbytes = ea.decode_workspace_bytes(desc, B, S)
    if nbytes:
        ws = torch.full((nbytes // 4,), float("nan"), dtype=torch.float32, device="cuda")
    ea.decode_attn(desc, torch.from_numpy(q.astype(np.float32)).cuda(), dc.k_pool, dc.v_pool, dc.page_table,
                   dc.seq_len, out, n_splits=S, ws=ws)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def oracle_decode(desc, K, V, q):
    keep = [b for b in range(len(K)) if K[b].shape[1] > 0]
    ref = np.zeros((len(K), desc.n_heads, desc.r_v))
    if keep:
        cache = ora.RankCache.from_arrays([K[b] for b in keep], [V[b] for b in keep])
        ref[keep] = ora.decode_attention(q[keep], cache, desc.d_head)
    return ref


# ---- config 1: tiny fp32 layer (d=256, H=4, d_h=64, B=1, n=256), r=32 and the full-rank rerun r=64
@pytest.mark.parametrize("r", [32, 64])
@pytest.mark.parametrize("n_splits", [1, 2])
def test_cfg1_f32(r, n_splits):
    print(f"cfg1 r={r} splits={n_splits}", flush=True)
    desc = ea.LayerDesc(256, 4, 4, 64, r, r, ea.EA_F32, 16)
    g = synth.rng(1, 10, r)
    U = np.stack([synth.orthonormal_basis(g, 64, r) for _ in range(4)])
    Kfull, Vfull = synth.gaussian(g, (4, 256, 64)), synth.gaussian(g, (4, 256, 64))
    K = [np.float32(ora.project_to_basis(Kfull, U)).astype(np.float64)]
    V = [np.float32(ora.project_to_basis(Vfull, U)).astype(np.float64)]
    q = np.float32(ora.project_to_basis(synth.gaussian(g, (1, 4, 1, 64)), U)[:, :, 0]).astype(np.float64)
    got = run_decode(desc, K, V, q, g, n_splits)
    assert_close(got, oracle_decode(desc, K, V, q), TOL_F32, "cfg1 decode")


@pytest.mark.parametrize("H,Hkv,r_k,r_v,lens,P,n_splits", [
    (4, 4, 32, 32, [1, 15, 16, 17], 16, 1),
    (4, 2, 30, 33, [255, 256, 257, 700], 32, 3),
    (6, 2, 64, 16, [1000, 3, 511], 64, 0),
    (2, 1, 200, 256, [300], 16, 2),
    (4, 4, 32, 32, [0, 40], 16, 1),           # an empty sequence gives a zero row
])
def test_f32_shapes(H, Hkv, r_k, r_v, lens, P, n_splits):
    print(f"f32 H={H}/{Hkv} r=({r_k},{r_v}) lens={lens} P={P} S={n_splits}", flush=True)
    desc = ea.LayerDesc(H * 64, H, Hkv, 64, r_k, r_v, ea.EA_F32, P)
    g = synth.rng(2, H, r_k, len(lens))
    K, V = random_cache(desc, lens, g)
    q = np.float32(synth.gaussian(g, (len(lens), H, r_k))).astype(np.float64)
    got = run_decode(desc, K, V, q, g, n_splits)
    assert_close(got, oracle_decode(desc, K, V, q), TOL_F32, "f32 decode")


# ---- bf16 cache: sizes that span several 64-token tiles, ragged tails, several splits, GQA, mixed ranks
@pytest.mark.parametrize("H,Hkv,r_k,r_v,lens,P,n_splits", [
    (2, 2, 80, 80, [1, 63, 64, 65], 64, 1),
    (2, 2, 80, 80, [200, 1000, 129], 64, 3),
    (8, 2, 48, 112, [777, 64, 1500], 128, 0),          # GQA 4:1, r_k != r_v
    (8, 2, 112, 48, [2048, 31], 64, 5),
    (16, 1, 96, 64, [300], 64, 2),                     # 16 query heads on one kv head
    (4, 4, 128, 128, [513, 100], 64, 2),               # full rank d_h = 128: the standard-attention baseline
    (4, 2, 72, 40, [150, 70], 64, 2),                  # ranks that need padding channels
    (2, 2, 16, 16, [5000], 192, 7),
    (2, 2, 80, 80, [0, 100], 64, 1),                   # an empty sequence gives a zero row
    (2, 2, 80, 80, [90], 64, 4),                       # more splits than tiles: empty workgroups
    (4, 2, 30, 33, [150, 70, 1], 64, 2),               # ranks that are no multiple of the 8-channel chunk
])
def test_bf16_shapes(H, Hkv, r_k, r_v, lens, P, n_splits):
    print(f"bf16 H={H}/{Hkv} r=({r_k},{r_v}) lens={lens} P={P} S={n_splits}", flush=True)
    desc = ea.LayerDesc(H * 128, H, Hkv, 128, r_k, r_v, ea.EA_BF16, P)
    g = synth.rng(3, H, r_k, len(lens), n_splits)
    K, V = random_cache(desc, lens, g, k_std=2.0)
    q = np.float32(synth.gaussian(g, (len(lens), H, r_k), 2.0)).astype(np.float64)
    got = run_decode(desc, K, V, q, g, n_splits)
    err = assert_close(got, oracle_decode(desc, K, V, q), TOL_BF16, "bf16 decode")
    print(f"  rel-L2 {err:.2e}", flush=True)


def test_bf16_peaked_softmax_and_large_scores():
    """Scores far apart (one dominant key) and large magnitudes: the running max must carry them."""
    desc = ea.LayerDesc(256, 2, 2, 128, 80, 80, ea.EA_BF16, 64)
    g = synth.rng(4)
    K, V = random_cache(desc, [900], g)
    K[0][:, 777, :] *= 40.0
    K[0][:, 5, :] *= -40.0
    q = np.float32(synth.gaussian(g, (1, 2, 80), 4.0)).astype(np.float64)
    got = run_decode(desc, K, V, q, g, 3)
    assert_close(got, oracle_decode(desc, K, V, q), TOL_BF16, "peaked")


def test_split_count_does_not_change_the_result():
    desc = ea.LayerDesc(512, 4, 4, 128, 80, 80, ea.EA_BF16, 64)
    g = synth.rng(5)
    K, V = random_cache(desc, [3000, 2500], g)
    q = np.float32(synth.gaussian(g, (2, 4, 80))).astype(np.float64)
    ref = oracle_decode(desc, K, V, q)
    outs = [run_decode(desc, K, V, q, synth.rng(5, 1), s) for s in (1, 2, 7, 16)]
    for o in outs:
        assert_close(o, ref, TOL_BF16, "split sweep")
        # P is rounded to bf16 relative to a running max that depends on the split, so results
        # agree to bf16-rounding level, not to fp32 bits
        dev = float(np.abs(o - outs[0]).max() / np.abs(outs[0]).max())
        assert dev <= 5e-3, dev


def test_out_of_range_pages_are_masked_not_read():
    """A page id outside the pool must never be dereferenced: its tokens simply drop out."""
    desc = ea.LayerDesc(256, 2, 2, 128, 80, 80, ea.EA_BF16, 64)
    g = synth.rng(6)
    K, V = random_cache(desc, [256], g)
    dc = DeviceCache(desc, K, V, g)
    pt = dc.page_table.clone()
    pt[0, 1] = dc.pool_pages + 1000      # tokens 64..127 vanish
    pt[0, 3] = -5                        # tokens 192..255 vanish
    q = np.float32(synth.gaussian(g, (1, 2, 80))).astype(np.float64)
    out = torch.zeros((1, 2, 80), dtype=torch.float32, device="cuda")
    ea.decode_attn(desc, torch.from_numpy(q.astype(np.float32)).cuda(), dc.k_pool, dc.v_pool, pt, dc.seq_len, out,
                   n_splits=1)
    torch.cuda.synchronize()
    keep = np.r_[0:64, 128:192]
    ref = oracle_decode(desc, [K[0][:, keep]], [V[0][:, keep]], q)
    assert_close(out.cpu().numpy(), ref, TOL_BF16, "masked pages")


# ---- config 2 at full size: Llama-2-7B-shaped layer, B=16, n=4096, r=80, low-rank-plus-noise data
def test_cfg2_full_size():
    print("cfg2 full size", flush=True)
    s = synth.CFG2
    desc = ea.LayerDesc(s.d_model, s.n_heads, s.n_kv_heads, s.d_head, s.r_k, s.r_v, ea.EA_BF16, 64)
    g = synth.rng(2, 0)
    K, V, qs = [], [], []
    Uk, Uv = [], []
    for h in range(s.n_kv_heads):           # per head: 80 dominant directions + sigma = 0.05 noise, basis from 2048 samples
        Ak, Av = synth.orthonormal_basis(g, 128, 80).T, synth.orthonormal_basis(g, 128, 80).T
        Uk.append(synth.top_singular_basis(synth.lowrank_plus_noise(g, 2048, Ak, 0.05), 80))
        Uv.append(synth.top_singular_basis(synth.lowrank_plus_noise(g, 2048, Av, 0.05), 80))
        K.append(ora.project_to_basis(synth.lowrank_plus_noise(g, s.batch * s.n_ctx, Ak, 0.05), Uk[-1]))
        V.append(ora.project_to_basis(synth.lowrank_plus_noise(g, s.batch * s.n_ctx, Av, 0.05), Uv[-1]))
        qs.append(ora.project_to_basis(synth.lowrank_plus_noise(g, s.batch, Ak, 0.05), Uk[-1]))
    from helpers import quantize
    Kb = [quantize(desc, np.stack([K[h][b * s.n_ctx:(b + 1) * s.n_ctx] for h in range(32)])) for b in range(s.batch)]
    Vb = [quantize(desc, np.stack([V[h][b * s.n_ctx:(b + 1) * s.n_ctx] for h in range(32)])) for b in range(s.batch)]
    q = np.float32(np.stack(qs, axis=1)).astype(np.float64)            # [B, H, r_k]
    got = run_decode(desc, Kb, Vb, q, g, 0)
    err = assert_close(got, oracle_decode(desc, Kb, Vb, q), TOL_BF16, "cfg2 decode")
    print(f"  cfg2 rel-L2 {err:.2e}", flush=True)
