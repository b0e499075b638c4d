"""ea_attn_mass and its fused form ea_decode_attn_mass (the attention statistic H2O-style eviction accumulates;
results, "Eigen Attention with token pruning") against the fp64 oracle, and a generation loop over a fixed-budget cache whose dropped tokens' slots are
overwritten by the new ones."""
import numpy as np
import pytest
import torch

import paper_2408_05646_amd as ea
from oracle import eigen_attention as ora
from oracle import eviction as oe
from paper_2408_05646_amd import synth
from helpers import DeviceCache, TOL_BF16, TOL_F32, assert_close, quantize, random_cache, to_dev

pytestmark = pytest.mark.gpu


def run_mass(desc, dc, q, mass=None):
    B = q.shape[0]
    n_cap = dc.max_pages * desc.page_tokens
    if mass is None:
        mass = torch.zeros((B, desc.n_kv_heads, n_cap), dtype=torch.float32, device="cuda")
    ws = torch.full((ea.attn_mass_workspace_bytes(desc, B, dc.max_pages) // 4,), float("nan"), dtype=torch.float32,
                    device="cuda")
    ea.attn_mass(desc, torch.from_numpy(q.astype(np.float32)).cuda(), dc.k_pool, dc.page_table, dc.seq_len, mass, ws)
    torch.cuda.synchronize()
    return mass


@pytest.mark.parametrize("dtype,H,Hkv,r_k,lens,P", [
    (ea.EA_F32, 4, 2, 30, [255, 256, 700, 1], 16),
    (ea.EA_F32, 8, 8, 32, [40, 0], 48),                       # 64-token tiles that straddle pages of 48
    (ea.EA_BF16, 2, 2, 80, [1, 63, 64, 65], 64),
    (ea.EA_BF16, 8, 2, 48, [777, 64, 1500], 128),             # GQA 4:1
    (ea.EA_BF16, 16, 1, 96, [300], 64),                       # 16 query heads on one kv head
    (ea.EA_BF16, 4, 4, 128, [513, 100, 0], 64),
    (ea.EA_BF16, 4, 2, 30, [150, 70], 64),
    (ea.EA_BF16, 2, 1, 80, [20000], 64),                      # 313 tiles to normalise across
])
def test_attn_mass_matches_oracle(dtype, H, Hkv, r_k, lens, P):
    print(f"mass dtype={dtype} H={H}/{Hkv} r_k={r_k} lens={lens} P={P}", flush=True)
    d_h = 128 if dtype == ea.EA_BF16 else 64
    desc = ea.LayerDesc(H * d_h, H, Hkv, d_h, r_k, 16, dtype, P)
    g = synth.rng(61, H, r_k, len(lens))
    K, V = random_cache(desc, lens, g, k_std=1.5)
    B = len(lens)
    q = np.float32(synth.gaussian(g, (B, H, r_k), 1.5)).astype(np.float64)
    dc = DeviceCache(desc, K, V, g)
    mass = run_mass(desc, dc, q)
    got = mass.cpu().numpy()
    keep = [b for b in range(B) if lens[b] > 0]
    ref = oe.attention_mass(q[keep], ora.RankCache.from_arrays([K[b] for b in keep], [V[b] for b in keep]), d_h)
    tol = TOL_F32 if dtype == ea.EA_F32 else TOL_BF16
    for b in range(B):
        assert not got[b, :, lens[b]:].any(), "entries past the sequence end must stay untouched"
    for i, b in enumerate(keep):
        assert_close(got[b, :, :lens[b]], ref[i], tol, f"mass b={b}")
        assert np.allclose(got[b, :, :lens[b]].sum(axis=1), H // Hkv, rtol=0, atol=1e-3)
    # a second call accumulates
    mass2 = run_mass(desc, dc, q, mass.clone())
    assert torch.allclose(mass2, 2 * mass, rtol=1e-6, atol=1e-7)


@pytest.mark.parametrize("H,Hkv,r_k,r_v,lens,P,S", [
    (2, 2, 80, 80, [1, 63, 64, 65], 64, 1),                   # a single split still goes through the merge
    (8, 2, 48, 64, [777, 64, 1500], 128, 3),                  # GQA 4:1, splits that some sequences leave empty
    (16, 1, 96, 112, [300, 2000], 64, 2),                     # half-tile iterations (large ranks)
    (4, 4, 128, 128, [513, 100, 0], 64, 4),                   # an empty sequence
    (4, 2, 30, 20, [150, 70], 64, 0),                         # odd ranks, automatic split count
    (2, 1, 80, 80, [20000], 64, 8),
])
def test_decode_attn_mass_matches_oracle_and_the_two_separate_calls(H, Hkv, r_k, r_v, lens, P, S):
    """One pass over the cache: the attention output of ea_decode_attn and the statistic of ea_attn_mass."""
    print(f"fused mass H={H}/{Hkv} r=({r_k},{r_v}) lens={lens} P={P} S={S}", flush=True)
    desc = ea.LayerDesc(H * 128, H, Hkv, 128, r_k, r_v, ea.EA_BF16, P)
    g = synth.rng(64, H, r_k, len(lens))
    K, V = random_cache(desc, lens, g, k_std=1.5)
    B = len(lens)
    q = np.float32(synth.gaussian(g, (B, H, r_k), 1.5)).astype(np.float64)
    dc = DeviceCache(desc, K, V, g)
    q_t = torch.from_numpy(q.astype(np.float32)).cuda()
    n_cap = dc.max_pages * P
    S_eff = S or ea.decode_auto_splits(desc, B, n_cap)
    ws = torch.full((ea.decode_attn_mass_workspace_bytes(desc, B, dc.max_pages, S_eff) // 4,), float("nan"),
                    dtype=torch.float32, device="cuda")
    prior = torch.rand((B, Hkv, n_cap), dtype=torch.float32, device="cuda")      # the call adds to what is there
    mass = prior.clone()
    out = torch.full((B, H, r_v), float("nan"), dtype=torch.float32, device="cuda")
    ea.decode_attn_mass(desc, q_t, dc.k_pool, dc.v_pool, dc.page_table, dc.seq_len, out, mass, S, ws)
    torch.cuda.synchronize()
    got = (mass - prior).cpu().numpy()
    keep = [b for b in range(B) if lens[b] > 0]
    cache = ora.RankCache.from_arrays([K[b] for b in keep], [V[b] for b in keep])
    ref_m = oe.attention_mass(q[keep], cache, 128)
    ref_o = ora.decode_attention(q[keep], cache, 128)
    assert_close(out.cpu().numpy()[keep], ref_o, TOL_BF16, "fused output")
    for b in range(B):
        assert torch.equal(mass[b, :, lens[b]:], prior[b, :, lens[b]:]), "entries past the sequence end were touched"
    for i, b in enumerate(keep):
        assert_close(got[b, :, :lens[b]], ref_m[i], TOL_BF16, f"fused mass b={b}")
        assert np.allclose(got[b, :, :lens[b]].sum(axis=1), H // Hkv, rtol=0, atol=2e-3)
    # against the two calls it replaces: the same output, and the same statistic up to the normaliser, which here is
    # the attention kernel's own row sum (of probabilities rounded to bfloat16: within one bf16 step, 2^-8, relative)
    out2 = torch.empty_like(out)
    ws2 = torch.empty(max(ea.decode_workspace_bytes(desc, B, S_eff) // 4, 4), dtype=torch.float32, device="cuda")
    ea.decode_attn(desc, q_t, dc.k_pool, dc.v_pool, dc.page_table, dc.seq_len, out2, n_splits=S_eff, ws=ws2)
    sep = run_mass(desc, dc, q).cpu().numpy()
    assert torch.allclose(out, out2, rtol=1e-5, atol=1e-6)
    assert np.allclose(got, sep, rtol=4e-3, atol=1e-6)


def test_attn_mass_skips_pages_that_are_not_there():
    desc = ea.LayerDesc(256, 2, 2, 128, 80, 16, ea.EA_BF16, 64)
    g = synth.rng(62)
    K, V = random_cache(desc, [256], g)
    q = np.float32(synth.gaussian(g, (1, 2, 80))).astype(np.float64)
    dc = DeviceCache(desc, K, V, g)
    pt = dc.page_table.clone()
    pt[0, 1] = dc.pool_pages + 5
    dc.page_table = pt
    got = run_mass(desc, dc, q).cpu().numpy()[0]
    keep = np.r_[0:64, 128:256]
    ref = oe.attention_mass(q, ora.RankCache.from_arrays([K[0][:, keep]], [V[0][:, keep]]), 128)[0]
    assert not got[:, 64:128].any()
    assert_close(got[:, keep], ref, TOL_BF16, "mass with a missing page")


@pytest.mark.parametrize("fused", [False, True])
def test_h2o_generation_loop_over_a_fixed_budget(fused):
    """A cache of `budget` slots per sequence.  Every step: project the new token into the slot the policy freed
    (the oldest-first H2O rule on the accumulated mass, the newest n_recent tokens protected; the decision is the
    oracle's, so that a near-tie cannot send the two sides down different paths), attend over the budget, add the
    step's attention mass.  Outputs and accumulated masses must follow the oracle, which keeps its kept tokens
    in a plain list."""
    from test_gpu_layer import make_weights, device_weights
    desc = ea.LayerDesc(512, 8, 2, 128, 80, 48, ea.EA_BF16, 64)
    B, budget, n_recent, steps = 2, 128, 16, 60
    g = synth.rng(63)
    Wq, Wk, Wv, Wo, Uk, Uv = make_weights(desc, g)
    wqkv_t, wo_t, folded_q = device_weights(desc, ora.fold_weights(Wq, Wk, Wv, Wo, Uk, Uv, 8, 2))
    Wq_q, Wk_q, Wv_q, Wo_q = folded_q
    x_hist = quantize(desc, synth.gaussian(g, (B, budget + steps, 512)))
    _, k_all, v_all = ora.project_qkv(x_hist.reshape(B * (budget + steps), 512), Wq_q, Wk_q, Wv_q)
    k_all = quantize(desc, k_all).reshape(B, budget + steps, 2, 80).transpose(0, 2, 1, 3)
    v_all = quantize(desc, v_all).reshape(B, budget + steps, 2, 48).transpose(0, 2, 1, 3)

    # the first `budget` tokens fill the cache through the library; slot s holds token s
    dc = DeviceCache(desc, [np.zeros((2, 0, 80))] * B, [np.zeros((2, 0, 48))] * B, g, extra_len=budget)
    q_pre = torch.empty((B * budget, 8, 80), dtype=torch.bfloat16, device="cuda")
    ea.project_qkv(desc, to_dev(desc, x_hist[:, :budget].reshape(B * budget, 512)), wqkv_t, q_pre, dc.k_pool, dc.v_pool,
                   dc.page_table, dc.seq_len, budget)
    full = torch.full((B,), budget, dtype=torch.int32, device="cuda")
    slot_token = [list(range(budget)) for _ in range(B)]          # which token sits in which slot
    acc_ref = [np.zeros((2, budget)) for _ in range(B)]           # accumulated mass per slot, oracle
    mass = torch.zeros((B, 2, budget), dtype=torch.float32, device="cuda")
    ws_m = torch.empty(ea.attn_mass_workspace_bytes(desc, B, dc.max_pages) // 4, dtype=torch.float32, device="cuda")
    ws_f = torch.empty(ea.decode_attn_mass_workspace_bytes(desc, B, dc.max_pages, 2) // 4, dtype=torch.float32,
                       device="cuda")
    q_r = torch.empty((B, 8, 80), dtype=torch.float32, device="cuda")
    o = torch.empty((B, 8, 48), dtype=torch.float32, device="cuda")
    y = torch.empty((B, 512), dtype=torch.bfloat16, device="cuda")
    worst = 0.0
    for t in range(steps):
        tok = budget + t
        # the policy (oracle side): drop the slot with the least mass (summed over kv heads) that is not recent
        slots = []
        for b in range(B):
            age_order = np.argsort(slot_token[b])                 # slots from oldest to newest token
            victim_rank = oe.h2o_victim(acc_ref[b].sum(axis=0)[age_order], n_recent)
            slots.append(int(age_order[victim_rank]))
        slot_t = torch.tensor(slots, dtype=torch.int32).cuda()
        for b in range(B):
            slot_token[b][slots[b]] = tok
            acc_ref[b][:, slots[b]] = 0.0
        mass[torch.arange(B), :, slot_t.long()] = 0.0
        # the step: the new token goes to the freed slot (its "position"), attention runs over all slots
        ea.project_qkv(desc, to_dev(desc, x_hist[:, tok]), wqkv_t, q_r, dc.k_pool, dc.v_pool, dc.page_table, slot_t, 1)
        if fused:
            ea.decode_attn_mass(desc, q_r, dc.k_pool, dc.v_pool, dc.page_table, full, o, mass, 2, ws_f)
        else:
            ea.decode_attn(desc, q_r, dc.k_pool, dc.v_pool, dc.page_table, full, o, n_splits=1)
            ea.attn_mass(desc, q_r, dc.k_pool, dc.page_table, full, mass, ws_m)
        ea.out_proj(desc, o.view(B, -1), wo_t, y)
        torch.cuda.synchronize()
        # oracle: the kept tokens, in slot order
        q_ref, _, _ = ora.project_qkv(x_hist[:, tok], Wq_q, Wk_q, Wv_q)
        cache = ora.RankCache.from_arrays([k_all[b][:, slot_token[b]] for b in range(B)],
                                          [v_all[b][:, slot_token[b]] for b in range(B)])
        y_ref = ora.out_proj(ora.decode_attention(q_ref, cache, 128), Wo_q)
        step_mass = oe.attention_mass(q_ref, cache, 128)
        for b in range(B):
            acc_ref[b] += step_mass[b]
        worst = max(worst, assert_close(y.float().cpu().numpy(), y_ref, TOL_BF16, f"h2o step {t}"))
    got = mass.cpu().numpy()
    for b in range(B):
        assert_close(got[b], acc_ref[b], TOL_BF16, f"accumulated mass b={b}")
        assert len(set(slot_token[b])) == budget and max(slot_token[b]) == budget + steps - 1
    print(f"  worst step rel-L2 {worst:.2e}", flush=True)


def test_decode_attn_mass_step_is_graph_capturable():
    """project_qkv -> ea_decode_attn_mass (three launches) -> out_proj captured in a HIP graph; every replay, with
    eager work in between, reproduces the eager output bit for bit and adds the eager step's statistic once more."""
    desc = ea.LayerDesc(512, 8, 2, 128, 80, 48, ea.EA_BF16, 64)
    g = synth.rng(65)
    B, n, S = 3, 700, 3
    K, V = random_cache(desc, [n] * B, g)
    dc = DeviceCache(desc, K, V, g, extra_len=1)
    n_qkv = 8 * 80 + 2 * (80 + 48)
    wqkv = ea.pack_weight(torch.from_numpy(synth.gaussian(g, (n_qkv, 512), 512 ** -0.5)).float().to(torch.bfloat16).cuda())
    wo = ea.pack_weight(torch.from_numpy(synth.gaussian(g, (512, 8 * 48), 512 ** -0.5)).float().to(torch.bfloat16).cuda())
    x = torch.from_numpy(synth.gaussian(g, (B, 512))).float().to(torch.bfloat16).cuda()
    q_r = torch.empty((B, 8, 80), dtype=torch.float32, device="cuda")
    o = torch.empty((B, 8, 48), dtype=torch.float32, device="cuda")
    y = torch.empty((B, 512), dtype=torch.bfloat16, device="cuda")
    mass = torch.zeros((B, 2, dc.max_pages * 64), dtype=torch.float32, device="cuda")
    ws = torch.empty(ea.decode_attn_mass_workspace_bytes(desc, B, dc.max_pages, S) // 4, dtype=torch.float32, device="cuda")
    before = dc.seq_len.clone()
    after = before + 1

    def step():
        ea.project_qkv(desc, x, wqkv, q_r, dc.k_pool, dc.v_pool, dc.page_table, before, 1)
        ea.decode_attn_mass(desc, q_r, dc.k_pool, dc.v_pool, dc.page_table, after, o, mass, S, ws)
        ea.out_proj(desc, o.view(B, -1), wo, y)

    step()
    torch.cuda.synchronize()
    y_eager, mass_eager = y.clone(), mass.clone()
    assert float(y_eager.float().abs().sum()) > 0
    assert np.allclose(mass_eager.sum(dim=2).cpu().numpy(), 4, rtol=0, atol=2e-3)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(4):
        y.zero_(); o.zero_(); q_r.zero_(); ws.zero_(); mass.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, y_eager), f"replay {rep}: output differs from the eager result"
        assert torch.equal(mass, mass_eager), f"replay {rep}: statistic differs from the eager result"
