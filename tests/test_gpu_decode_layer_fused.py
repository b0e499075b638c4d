"""The generation step of a layer in two launches: ea_decode_layer_fused / ea_decode_layer_fused_rope (projection +
append; then attention, split merge and output projection in one launch) against the fp64 oracle, against the
three-launch call, over steps in a row that share one workspace, under HIP-graph replay, and with the bounded wait
of the second launch forced to expire from the host."""
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


def same_bits(a, b):
    """Bit for bit (the never-written slots of a test cache hold NaNs, which compare unequal as numbers)."""
    return torch.equal(a.view(torch.int16), b.view(torch.int16))


def layer_weights(desc, g, rope):
    if rope:
        wqkv, wo, u_dev, Uk1, folded, _ = rope_weights(desc, g)
        return wqkv, wo, u_dev, Uk1, folded
    Wq, Wk, Wv, Wo, Uk, Uv = make_weights(desc, g)
    wqkv, wo, folded = device_weights(desc, ora.fold_weights(Wq, Wk, Wv, Wo, Uk, Uv, desc.n_heads, desc.n_kv_heads))
    return wqkv, wo, None, None, folded


@pytest.mark.parametrize("rope", [False, True])
@pytest.mark.parametrize("d,H,Hkv,r_k,r_v,B,n0,S", [
    (512, 8, 2, 80, 48, 4, 700, 3),          # GQA, splits > 1: more channel blocks than workgroups
    (512, 8, 8, 80, 80, 16, 130, 1),         # one split, a full batch
    (512, 4, 2, 72, 40, 3, 333, 2),          # padded ranks
    (512, 8, 2, 112, 96, 5, 1000, 0),        # the split count the library picks itself
    (1024, 32, 8, 64, 64, 8, 2100, 8),       # 512 workgroups: one per resident slot, a quarter of them project
    (256, 2, 1, 32, 16, 1, 70, 1),           # a single workgroup does everything
    (512, 8, 2, 80, 48, 2, 1700, 12),        # more than eight splits: the merge goes through LDS
    (4096, 32, 32, 128, 128, 2, 300, 2),     # full rank: 4096 channels, two rounds of weights per wave
    (8192, 8, 2, 80, 48, 2, 200, 2),         # d = 8192: the projection launch takes its general form; 512 channel blocks
])
def test_fused_decode_layer_matches_oracle_decode_step(rope, d, H, Hkv, r_k, r_v, B, n0, S):
    print(f"fused decode layer rope={rope} d={d} H={H}/{Hkv} r=({r_k},{r_v}) B={B} n0={n0} S={S}", flush=True)
    d_h, P = 128, 64
    desc = ea.LayerDesc(d, H, Hkv, d_h, r_k, r_v, ea.EA_BF16, P)
    g = synth.rng(91, H, r_k, int(rope), d)
    x = quantize(desc, synth.gaussian(g, (B, d)))
    lens = [n0 - 7 * b for b in range(B)]
    K0, V0 = random_cache(desc, lens, g)
    dc = DeviceCache(desc, K0, V0, g, extra_len=1)
    wqkv, wo, u_dev, Uk1, folded = layer_weights(desc, g, rope)
    S_eff = S or (ea.decode_rope_auto_splits if rope else ea.decode_auto_splits)(desc, B, dc.max_pages * P)
    ws = torch.full((ea.decode_layer_fused_workspace_bytes(desc, B, S_eff, rope) // 4,), float("nan"), device="cuda")
    y = torch.full((B, d), float("nan"), dtype=torch.bfloat16, device="cuda")
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    xd = to_dev(desc, x)
    k_before, v_before = dc.k_pool.clone(), dc.v_pool.clone()
    ea.decode_layer(desc, xd, wqkv, wo, dc.k_pool, dc.v_pool, dc.page_table, dc.seq_len, y, S, ws, u_k=u_dev,
                    status=status, fused=True)
    torch.cuda.synchronize()
    assert int(status.item()) == 0
    cache = ora.RankCache.from_arrays(K0, V0)
    if rope:
        y_ref = ora.decode_step_rope(x, folded, Uk1, cache, d_h, 10000.0)
    else:
        y_ref = ora.decode_step(x, folded, cache, d_h)
    assert_close(y.float().cpu().numpy(), y_ref, TOL_BF16, "fused decode layer y")
    # the appended token is in the cache exactly as the three-launch call leaves it
    k_after, v_after = dc.k_pool.clone(), dc.v_pool.clone()
    dc.k_pool.copy_(k_before); dc.v_pool.copy_(v_before)
    y3 = torch.empty_like(y)
    ws3 = torch.empty(ea.decode_layer_workspace_bytes(desc, B, S_eff, rope) // 4, device="cuda")
    ea.decode_layer(desc, xd, wqkv, wo, dc.k_pool, dc.v_pool, dc.page_table, dc.seq_len, y3, S, ws3, u_k=u_dev)
    torch.cuda.synchronize()
    assert same_bits(k_after, dc.k_pool) and same_bits(v_after, dc.v_pool)
    # and y differs from that call's only by the one rounding of o to bfloat16
    assert ora.rel_l2(y.float().cpu().numpy(), y3.float().cpu().numpy()) < 6e-3


@pytest.mark.parametrize("rope", [False, True])
def test_fused_steps_in_a_row_share_one_workspace(rope):
    """Twelve generation steps through one workspace, every step with new activations and a longer cache: a value
    read from a stale cache line (the previous step's o or partials) would show as a mismatch with the three-launch
    call on the same inputs."""
    d, H, Hkv, r_k, r_v, B, S = 1024, 16, 4, 80, 64, 8, 4
    desc = ea.LayerDesc(d, H, Hkv, 128, r_k, r_v, ea.EA_BF16, 64)
    g = synth.rng(92, int(rope))
    K0, V0 = random_cache(desc, [900 - 11 * b for b in range(B)], g)
    dcf = DeviceCache(desc, K0, V0, synth.rng(5), extra_len=16)
    dc3 = DeviceCache(desc, K0, V0, synth.rng(5), extra_len=16)
    wqkv, wo, u_dev, _, _ = layer_weights(desc, g, rope)
    wsf = torch.full((ea.decode_layer_fused_workspace_bytes(desc, B, S, rope) // 4,), float("nan"), device="cuda")
    ws3 = torch.empty(ea.decode_layer_workspace_bytes(desc, B, S, rope) // 4, device="cuda")
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    yf = torch.empty((B, d), dtype=torch.bfloat16, device="cuda")
    y3 = torch.empty_like(yf)
    for step in range(12):
        x = to_dev(desc, quantize(desc, synth.gaussian(g, (B, d), 1.0 + 0.25 * step)))
        ea.decode_layer(desc, x, wqkv, wo, dcf.k_pool, dcf.v_pool, dcf.page_table, dcf.seq_len, yf, S, wsf, u_k=u_dev,
                        status=status, fused=True)
        ea.decode_layer(desc, x, wqkv, wo, dc3.k_pool, dc3.v_pool, dc3.page_table, dc3.seq_len, y3, S, ws3, u_k=u_dev)
        dcf.seq_len += 1
        dc3.seq_len += 1
        torch.cuda.synchronize()
        err = ora.rel_l2(yf.float().cpu().numpy(), y3.float().cpu().numpy())
        assert err < 6e-3, f"step {step}: {err}"
    assert int(status.item()) == 0
    assert same_bits(dcf.k_pool, dc3.k_pool) and same_bits(dcf.v_pool, dc3.v_pool)


def test_fused_decode_layer_wait_expires_and_the_next_call_recovers():
    """A wait limit of one poll set from the host: the projecting workgroups (the last of the grid, here the short
    sequences) look at the arrival counter once while sequence 0 is still streaming, give up, flag the status word
    and leave -- the launch ends normally.  With the limit restored the next call on the same workspace is right."""
    d, H, Hkv, r_k, r_v, B = 512, 8, 8, 80, 80, 8
    desc = ea.LayerDesc(d, H, Hkv, 128, r_k, r_v, ea.EA_BF16, 64)
    g = synth.rng(93)
    lens = [60000] + [70] * (B - 1)
    K0, V0 = random_cache(desc, lens, g)
    dc = DeviceCache(desc, K0, V0, g, extra_len=2)
    wqkv, wo, _, _, folded = layer_weights(desc, g, False)
    x = quantize(desc, synth.gaussian(g, (B, d)))
    xd = to_dev(desc, x)
    ws = torch.full((ea.decode_layer_fused_workspace_bytes(desc, B, 1) // 4,), float("nan"), device="cuda")
    y = torch.zeros((B, d), dtype=torch.bfloat16, device="cuda")
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    k_before, v_before = dc.k_pool.clone(), dc.v_pool.clone()
    ea.set_wait_limit(1)
    try:
        ea.decode_layer(desc, xd, wqkv, wo, dc.k_pool, dc.v_pool, dc.page_table, dc.seq_len, y, 1, ws, status=status,
                        fused=True)
        torch.cuda.synchronize()
    finally:
        ea.set_wait_limit(1 << 20)
    assert int(status.item()) == ea.STATUS_WAIT_EXPIRED          # flagged, and no append was dropped
    assert torch.isfinite(y.float()).all()
    dc.k_pool.copy_(k_before); dc.v_pool.copy_(v_before)
    status.zero_()
    ea.decode_layer(desc, xd, wqkv, wo, dc.k_pool, dc.v_pool, dc.page_table, dc.seq_len, y, 1, ws, status=status,
                    fused=True)
    torch.cuda.synchronize()
    assert int(status.item()) == 0
    y_ref = ora.decode_step(x, folded, ora.RankCache.from_arrays(K0, V0), 128)
    assert_close(y.float().cpu().numpy(), y_ref, TOL_BF16, "fused decode layer after an expired wait")


def test_fused_decode_layer_reports_a_full_cache():
    desc = ea.LayerDesc(256, 4, 2, 64, 48, 32, ea.EA_BF16, 64)
    g = synth.rng(94)
    B = 3
    K0, V0 = random_cache(desc, [64, 128, 100], g)
    dc = DeviceCache(desc, K0, V0, g)                     # two pages per sequence: sequence 1 is full
    assert dc.max_pages == 2
    w = ea.pack_weight(to_dev(desc, synth.gaussian(g, (4 * 48 + 2 * 80, 256), 0.06)))
    wo = ea.pack_weight(to_dev(desc, synth.gaussian(g, (256, 4 * 32), 0.06)))
    x = to_dev(desc, synth.gaussian(g, (B, 256)))
    y = torch.empty((B, 256), dtype=torch.bfloat16, device="cuda")
    ws = torch.zeros(ea.decode_layer_fused_workspace_bytes(desc, B, 2) // 4, device="cuda")
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    ea.decode_layer(desc, x, w, wo, dc.k_pool, dc.v_pool, dc.page_table, dc.seq_len, y, 2, ws, status=status, fused=True)
    torch.cuda.synchronize()
    assert int(status.item()) == 1 and torch.isfinite(y.float()).all()


def test_fused_decode_layers_are_graph_capturable():
    """Several two-launch layer steps captured in one HIP graph and replayed with eager work in between: every replay
    must give the eager result, whatever the workspace (its counters included) held before."""
    desc = ea.LayerDesc(512, 8, 2, 128, 80, 48, ea.EA_BF16, 64)
    g = synth.rng(95)
    B, n0, S, L = 4, 700, 3, 3
    layers = []
    for _ in range(L):
        wqkv, wo, _, _, _ = layer_weights(desc, g, False)
        K0, V0 = random_cache(desc, [n0] * B, g)
        layers.append((wqkv, wo, DeviceCache(desc, K0, V0, g, extra_len=1)))
    x = to_dev(desc, quantize(desc, synth.gaussian(g, (B, 512))))
    ys = [torch.empty((B, 512), dtype=torch.bfloat16, device="cuda") for _ in range(L)]
    ws = torch.full((ea.decode_layer_fused_workspace_bytes(desc, B, S) // 4,), float("nan"), device="cuda")
    status = torch.zeros(1, dtype=torch.int32, device="cuda")

    def step():
        for (wqkv, wo, dc), y in zip(layers, ys):
            ea.decode_layer(desc, x, wqkv, wo, dc.k_pool, dc.v_pool, dc.page_table, dc.seq_len, y, S, ws, status=status,
                            fused=True)

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
    assert int(status.item()) == 0


def test_fused_decode_layer_beside_other_work_on_the_gpu():
    """The two-launch step while another stream keeps the compute units busy with kernels that wait for nothing
    (large matrix products): the projecting workgroups may have to wait longer for the rest of their grid, which is
    dispatched as slots come free, but the wait ends, nothing expires and the result is the one of a quiet GPU."""
    d, H, Hkv, r_k, r_v, B, S = 1024, 32, 8, 64, 64, 8, 8              # 512 workgroups: every resident slot
    desc = ea.LayerDesc(d, H, Hkv, 128, r_k, r_v, ea.EA_BF16, 64)
    g = synth.rng(101)
    K0, V0 = random_cache(desc, [2100 - 7 * b for b in range(B)], g)
    dc = DeviceCache(desc, K0, V0, g, extra_len=1)
    wqkv, wo, _, _, _ = layer_weights(desc, g, False)
    xd = to_dev(desc, quantize(desc, synth.gaussian(g, (B, d))))
    ws = torch.empty(ea.decode_layer_fused_workspace_bytes(desc, B, S) // 4, device="cuda")
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    y_quiet = torch.empty((B, d), dtype=torch.bfloat16, device="cuda")
    k_before, v_before = dc.k_pool.clone(), dc.v_pool.clone()
    ea.decode_layer(desc, xd, wqkv, wo, dc.k_pool, dc.v_pool, dc.page_table, dc.seq_len, y_quiet, S, ws, status=status,
                    fused=True)
    torch.cuda.synchronize()
    a = torch.randn(4096, 4096, device="cuda", dtype=torch.bfloat16)
    side = torch.cuda.Stream()
    y = torch.empty_like(y_quiet)
    for rep in range(3):
        dc.k_pool.copy_(k_before); dc.v_pool.copy_(v_before)
        torch.cuda.synchronize()
        with torch.cuda.stream(side):
            for _ in range(40):
                a @ a                                            # a few milliseconds of other kernels
        for _ in range(10):
            ea.decode_layer(desc, xd, wqkv, wo, dc.k_pool, dc.v_pool, dc.page_table, dc.seq_len, y, S, ws,
                            status=status, fused=True)
        torch.cuda.synchronize()
        assert int(status.item()) == 0
        assert torch.equal(y, y_quiet), f"round {rep}"


@pytest.mark.parametrize("seed", [201, 202])
def test_fused_decode_layer_random_shapes(seed):
    """Drawn shapes through the two-launch step (group sizes, head counts, ranks off every chunk size, page sizes,
    ragged lengths down to an empty cache, split counts 1..16, model widths from fewer channel blocks than
    workgroups to many more) against the oracle's generation step; the appended token against the three-launch call."""
    rs = np.random.default_rng(seed)
    for case in range(16):
        G = int(rs.choice([1, 1, 2, 4, 8, 16]))
        Hkv = int(rs.choice([1, 2, 3, 4, 8]))
        H = G * Hkv
        r_k = int(rs.integers(1, 17)) * 8
        r_v = 0
        while r_v == 0 or (H * r_v) % 32 != 0:                   # the output projection contracts H * r_v in steps of 32
            r_v = int(rs.integers(1, 17)) * 8
        P = int(rs.choice([64, 128, 256]))
        B = int(rs.integers(1, 17))
        d = int(rs.choice([128, 256, 512, 1024, 2048]))
        rope = bool(rs.integers(2))
        lens = [int(rs.choice([0, 1, 63, 64, 65, 128, int(rs.integers(1, 1500))])) for _ in range(B)]
        S = int(rs.choice([0, 1, 2, 3, 5, 8, 9, 16]))
        print(f"seed {seed} case {case}: d={d} H={H}/{Hkv} r=({r_k},{r_v}) P={P} B={B} lens={lens} S={S} rope={rope}", flush=True)
        desc = ea.LayerDesc(d, H, Hkv, 128, r_k, r_v, ea.EA_BF16, P)
        g = synth.rng(seed, case)
        x = quantize(desc, synth.gaussian(g, (B, d)))
        K0, V0 = random_cache(desc, lens, g)
        dc = DeviceCache(desc, K0, V0, g, extra_len=1)
        wqkv, wo, u_dev, Uk1, folded = layer_weights(desc, g, rope)
        S_eff = S or (ea.decode_rope_auto_splits if rope else ea.decode_auto_splits)(desc, B, dc.max_pages * P)
        ws = torch.full((ea.decode_layer_fused_workspace_bytes(desc, B, S_eff, rope) // 4,), float("nan"), device="cuda")
        y = torch.full((B, d), float("nan"), dtype=torch.bfloat16, device="cuda")
        status = torch.zeros(1, dtype=torch.int32, device="cuda")
        xd = to_dev(desc, x)
        k_before, v_before = dc.k_pool.clone(), dc.v_pool.clone()
        ea.decode_layer(desc, xd, wqkv, wo, dc.k_pool, dc.v_pool, dc.page_table, dc.seq_len, y, S, ws, u_k=u_dev,
                        status=status, fused=True)
        torch.cuda.synchronize()
        assert int(status.item()) == 0
        cache = ora.RankCache.from_arrays(K0, V0)
        y_ref = (ora.decode_step_rope(x, folded, Uk1, cache, 128, 10000.0) if rope
                 else ora.decode_step(x, folded, cache, 128))
        assert_close(y.float().cpu().numpy(), y_ref, TOL_BF16, f"seed {seed} case {case}")
        k_after, v_after = dc.k_pool.clone(), dc.v_pool.clone()
        dc.k_pool.copy_(k_before); dc.v_pool.copy_(v_before)
        y3 = torch.empty_like(y)
        ws3 = torch.empty(max(ea.decode_layer_workspace_bytes(desc, B, S_eff, rope) // 4, 4), device="cuda")
        ea.decode_layer(desc, xd, wqkv, wo, dc.k_pool, dc.v_pool, dc.page_table, dc.seq_len, y3, S, ws3, u_k=u_dev)
        torch.cuda.synchronize()
        assert same_bits(k_after, dc.k_pool) and same_bits(v_after, dc.v_pool)
