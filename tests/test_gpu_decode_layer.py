"""The generation step of a layer in one call: ea_decode_layer / ea_decode_layer_rope (projection + append,
attention, output projection) against the fp64 oracle and against the separate calls they replace."""
import numpy as np
import pytest
import torch

import paper_2408_05646_amd as ea
from oracle import eigen_attention as ora
from paper_2408_05646_amd import synth
from helpers import DeviceCache, TOL_BF16, assert_close, quantize, random_cache, to_dev
from test_gpu_layer import device_weights, make_weights
from test_gpu_rope import rope_weights

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("rope", [False, True])
@pytest.mark.parametrize("H,Hkv,r_k,r_v,B,n0,S", [
    (8, 2, 80, 48, 4, 700, 3),          # GQA, splits > 1
    (8, 8, 80, 80, 16, 130, 1),         # one split
    (4, 2, 72, 40, 3, 333, 2),          # padded ranks
    (8, 2, 112, 96, 5, 1000, 0),        # the split count the library picks itself
])
def test_decode_layer_matches_oracle_decode_step(rope, H, Hkv, r_k, r_v, B, n0, S):
    print(f"decode layer rope={rope} H={H}/{Hkv} r=({r_k},{r_v}) B={B} n0={n0} S={S}", flush=True)
    d, d_h, P = 512, 128, 64
    desc = ea.LayerDesc(d, H, Hkv, d_h, r_k, r_v, ea.EA_BF16, P)
    g = synth.rng(82, H, r_k, int(rope))
    x = quantize(desc, synth.gaussian(g, (B, d)))
    lens = [n0 - 7 * b for b in range(B)]
    K0, V0 = random_cache(desc, lens, g)
    dc = DeviceCache(desc, K0, V0, g, extra_len=1)
    if rope:
        wqkv, wo, u_dev, Uk1, folded_q, _ = rope_weights(desc, g)     # one key basis for all heads (Sec. 4.3)
    else:
        Wq, Wk, Wv, Wo, Uk, Uv = make_weights(desc, g)
        wqkv, wo, folded_q = device_weights(desc, ora.fold_weights(Wq, Wk, Wv, Wo, Uk, Uv, H, Hkv))
        u_dev = None
    S_eff = S or (ea.decode_rope_auto_splits if rope else ea.decode_auto_splits)(desc, B, dc.max_pages * P)
    ws = torch.full((ea.decode_layer_workspace_bytes(desc, B, S_eff, rope) // 4,), float("nan"), device="cuda")
    y = torch.full((B, d), float("nan"), dtype=torch.bfloat16, device="cuda")
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    xd = to_dev(desc, x)
    k_before, v_before = dc.k_pool.clone(), dc.v_pool.clone()
    ea.decode_layer(desc, xd, wqkv, wo, dc.k_pool, dc.v_pool, dc.page_table, dc.seq_len, y, S, ws, u_k=u_dev,
                    status=status)
    torch.cuda.synchronize()
    cache = ora.RankCache.from_arrays(K0, V0)
    if rope:
        y_ref = ora.decode_step_rope(x, folded_q, Uk1, cache, d_h, 10000.0)
    else:
        y_ref = ora.decode_step(x, folded_q, cache, d_h)
    assert_close(y.float().cpu().numpy(), y_ref, TOL_BF16, "decode layer y")
    assert int(status.item()) == 0
    # the same step through the separate calls (same kernels; the layer call keeps its intermediate o in bfloat16,
    # the separate calls here pass it in float: one rounding of o apart)
    dc.k_pool.copy_(k_before); dc.v_pool.copy_(v_before)
    q_dim = d_h if rope else r_k
    q_r = torch.empty((B, H, q_dim), dtype=torch.float32, device="cuda")
    o = torch.empty((B, H, r_v), dtype=torch.float32, device="cuda")
    y2 = torch.empty_like(y)
    ws2 = torch.empty(max(ea.decode_workspace_bytes(desc, B, S_eff) // 4, 4), device="cuda")
    if rope:
        ea.project_qkv_rope(desc, xd, wqkv, q_r, dc.k_pool, dc.v_pool, dc.page_table, dc.seq_len, 1)
        ea.decode_attn_rope(desc, q_r, u_dev, 10000.0, dc.k_pool, dc.v_pool, dc.page_table, dc.seq_len + 1, o,
                            n_splits=S_eff, ws=ws2)
    else:
        ea.project_qkv(desc, xd, wqkv, q_r, dc.k_pool, dc.v_pool, dc.page_table, dc.seq_len, 1)
        ea.decode_attn(desc, q_r, dc.k_pool, dc.v_pool, dc.page_table, dc.seq_len + 1, o, n_splits=S_eff, ws=ws2)
    ea.out_proj(desc, o.view(B, -1), wo, y2)
    torch.cuda.synchronize()
    assert ora.rel_l2(y.float().cpu().numpy(), y2.float().cpu().numpy()) < 6e-3
    assert_close(y2.float().cpu().numpy(), y_ref, TOL_BF16, "separate calls y")


def test_decode_layer_reports_a_full_cache():
    desc = ea.LayerDesc(256, 4, 2, 64, 48, 32, ea.EA_BF16, 64)
    g = synth.rng(83)
    B = 3
    K0, V0 = random_cache(desc, [64, 128, 100], g)
    dc = DeviceCache(desc, K0, V0, g)                     # two pages per sequence: sequence 1 is full
    assert dc.max_pages == 2
    w = ea.pack_weight(to_dev(desc, synth.gaussian(g, (4 * 48 + 2 * 80, 256), 0.06)))
    wo = ea.pack_weight(to_dev(desc, synth.gaussian(g, (256, 4 * 32), 0.06)))
    x = to_dev(desc, synth.gaussian(g, (B, 256)))
    y = torch.empty((B, 256), dtype=torch.bfloat16, device="cuda")
    ws = torch.zeros(ea.decode_layer_workspace_bytes(desc, B, 2) // 4, device="cuda")
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    ea.decode_layer(desc, x, w, wo, dc.k_pool, dc.v_pool, dc.page_table, dc.seq_len, y, 2, ws, status=status)
    torch.cuda.synchronize()
    assert int(status.item()) == 1 and torch.isfinite(y.float()).all()


def test_decode_layers_are_graph_capturable():
    """Several layer steps captured in one HIP graph and replayed with eager work in between: every replay must give
    the eager result, whatever the workspace held before."""
    desc = ea.LayerDesc(512, 8, 2, 128, 80, 48, ea.EA_BF16, 64)
    g = synth.rng(84)
    B, n0, S, L = 4, 700, 3, 3
    layers = []
    for _ in range(L):
        Wq, Wk, Wv, Wo, Uk, Uv = make_weights(desc, g)
        wqkv, wo, _ = device_weights(desc, ora.fold_weights(Wq, Wk, Wv, Wo, Uk, Uv, 8, 2))
        K0, V0 = random_cache(desc, [n0] * B, g)
        layers.append((wqkv, wo, DeviceCache(desc, K0, V0, g, extra_len=1)))
    x = to_dev(desc, quantize(desc, synth.gaussian(g, (B, 512))))
    ys = [torch.empty((B, 512), dtype=torch.bfloat16, device="cuda") for _ in range(L)]
    ws = torch.full((ea.decode_layer_workspace_bytes(desc, B, S) // 4,), float("nan"), device="cuda")

    def step():
        for (wqkv, wo, dc), y in zip(layers, ys):
            ea.decode_layer(desc, x, wqkv, wo, dc.k_pool, dc.v_pool, dc.page_table, dc.seq_len, y, S, ws)

    step()
    torch.cuda.synchronize()
    eager = [y.clone() for y in ys]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(4):
        for y in ys:
            y.zero_()
        ws.fill_(float("nan"))                      # whatever the workspace holds, the step prepares what it needs
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for y, e in zip(ys, eager):
            assert torch.equal(y, e), f"replay {rep} differs from the eager result"
