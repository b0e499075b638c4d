"""The generation step of a layer with the ALiBi position bias (the MPT family of Sec. 5.1): ea_decode_layer_alibi
(projection + append, attention, merge, output projection as separate launches) and ea_decode_layer_fused_alibi (the
two-launch form) against the fp64 oracle's decode_step with slopes, against each other, and against the separate
calls (ea_project_qkv, ea_decode_attn_alibi, ea_out_proj)."""
import numpy as np
import pytest
import torch

import paper_2408_05646_amd as ea
from oracle import eigen_attention as ora
from paper_2408_05646_amd import synth
from helpers import DeviceCache, TOL_BF16, assert_close, quantize, random_cache, to_dev
from test_gpu_decode_layer_fused import layer_weights, same_bits

pytestmark = pytest.mark.gpu


def mpt_slopes(H):
    """Slopes of the geometric sequence the ALiBi paper gives for a power-of-two head count: 2^(-8 (h + 1) / H)."""
    return np.array([2.0 ** (-8.0 * (h + 1) / H) for h in range(H)])


@pytest.mark.parametrize("fused", [False, True])
@pytest.mark.parametrize("d,H,Hkv,r_k,r_v,B,n0,S", [
    (512, 8, 8, 80, 80, 4, 700, 3),          # MHA as the MPT models, splits > 1
    (512, 8, 2, 80, 48, 16, 130, 1),         # GQA, one split, a full batch of the two-launch form
    (512, 4, 2, 72, 40, 3, 333, 2),          # padded ranks
    (1024, 32, 32, 96, 64, 5, 1000, 0),      # the split count the library picks itself
    (512, 8, 8, 128, 128, 2, 1700, 12),      # full rank, more than eight splits
    (256, 2, 1, 32, 16, 1, 70, 1),           # a single workgroup
])
def test_alibi_decode_layer_matches_oracle_decode_step(fused, d, H, Hkv, r_k, r_v, B, n0, S):
    print(f"alibi decode layer fused={fused} d={d} H={H}/{Hkv} r=({r_k},{r_v}) B={B} n0={n0} S={S}", flush=True)
    d_h, P = 128, 64
    desc = ea.LayerDesc(d, H, Hkv, d_h, r_k, r_v, ea.EA_BF16, P)
    g = synth.rng(95, H, r_k, d)
    x = quantize(desc, synth.gaussian(g, (B, d)))
    lens = [n0 - 7 * b for b in range(B)]
    K0, V0 = random_cache(desc, lens, g)
    dc = DeviceCache(desc, K0, V0, g, extra_len=1)
    wqkv, wo, _, _, folded = layer_weights(desc, g, False)
    slopes = mpt_slopes(H)
    sl = torch.tensor(slopes, dtype=torch.float32, device="cuda")
    S_eff = S or ea.decode_auto_splits(desc, B, dc.max_pages * P)
    nbytes = (ea.decode_layer_fused_workspace_bytes if fused else ea.decode_layer_workspace_bytes)(desc, B, S_eff)
    ws = torch.full((nbytes // 4,), float("nan"), device="cuda")
    y = torch.full((B, d), float("nan"), dtype=torch.bfloat16, device="cuda")
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    xd = to_dev(desc, x)
    k_before, v_before = dc.k_pool.clone(), dc.v_pool.clone()
    ea.decode_layer_alibi(desc, xd, wqkv, wo, sl, dc.k_pool, dc.v_pool, dc.page_table, dc.seq_len, y, S, ws,
                          status=status, fused=fused)
    torch.cuda.synchronize()
    assert int(status.item()) == 0
    cache = ora.RankCache.from_arrays(K0, V0)
    y_ref = ora.decode_step(x, folded, cache, d_h, alibi_slopes=slopes.astype(np.float32).astype(np.float64))
    assert_close(y.float().cpu().numpy(), y_ref, TOL_BF16, "alibi decode layer y")
    # the bias is in there: the plain step's result is further away than the tolerance
    y_plain = ora.decode_step(x, folded, ora.RankCache.from_arrays(K0, V0), d_h)
    assert ora.rel_l2(y_plain, y_ref) > 0.05
    # the same step through the separate calls: identical cache, y up to the one rounding of o
    k_after, v_after = dc.k_pool.clone(), dc.v_pool.clone()
    dc.k_pool.copy_(k_before); dc.v_pool.copy_(v_before)
    q = torch.empty((B, H, r_k), dtype=torch.float32, device="cuda")
    ea.project_qkv(desc, xd, wqkv, q, dc.k_pool, dc.v_pool, dc.page_table, dc.seq_len, 1)
    lens1 = dc.seq_len + 1
    o = torch.empty((B, H, r_v), dtype=torch.float32, device="cuda")
    wsa = torch.empty(max(ea.decode_workspace_bytes(desc, B, S_eff), 4) // 4, device="cuda")
    ea.decode_attn_alibi(desc, q, sl, dc.k_pool, dc.v_pool, dc.page_table, lens1, o, S_eff, wsa)
    y_sep = torch.empty_like(y)
    ea.out_proj(desc, o, wo, y_sep)
    torch.cuda.synchronize()
    assert same_bits(k_after, dc.k_pool) and same_bits(v_after, dc.v_pool)
    assert ora.rel_l2(y.float().cpu().numpy(), y_sep.float().cpu().numpy()) < 6e-3


def test_alibi_two_launch_form_equals_the_separate_launches_over_steps_in_a_row():
    """Eight steps through one workspace each; both forms read the same bf16 o, so they may differ only in the
    summation order of the output projection."""
    d, H, Hkv, r_k, r_v, B, S = 1024, 16, 16, 80, 64, 8, 4
    desc = ea.LayerDesc(d, H, Hkv, 128, r_k, r_v, ea.EA_BF16, 64)
    g = synth.rng(96)
    K0, V0 = random_cache(desc, [900 - 11 * b for b in range(B)], g)
    dcf = DeviceCache(desc, K0, V0, synth.rng(5), extra_len=16)
    dc3 = DeviceCache(desc, K0, V0, synth.rng(5), extra_len=16)
    wqkv, wo, _, _, _ = layer_weights(desc, g, False)
    sl = torch.tensor(mpt_slopes(H), dtype=torch.float32, device="cuda")
    wsf = torch.full((ea.decode_layer_fused_workspace_bytes(desc, B, S) // 4,), float("nan"), device="cuda")
    ws3 = torch.empty(ea.decode_layer_workspace_bytes(desc, B, S) // 4, device="cuda")
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    yf = torch.empty((B, d), dtype=torch.bfloat16, device="cuda")
    y3 = torch.empty_like(yf)
    for step in range(8):
        x = to_dev(desc, quantize(desc, synth.gaussian(g, (B, d), 1.0 + 0.25 * step)))
        ea.decode_layer_fused_alibi(desc, x, wqkv, wo, sl, dcf.k_pool, dcf.v_pool, dcf.page_table, dcf.seq_len, yf, S,
                                    wsf, status=status)
        ea.decode_layer_alibi(desc, x, wqkv, wo, sl, dc3.k_pool, dc3.v_pool, dc3.page_table, dc3.seq_len, y3, S, ws3)
        dcf.seq_len += 1
        dc3.seq_len += 1
        torch.cuda.synchronize()
        err = ora.rel_l2(yf.float().cpu().numpy(), y3.float().cpu().numpy())
        assert err < 6e-3, f"step {step}: {err}"
    assert int(status.item()) == 0
    assert same_bits(dcf.k_pool, dc3.k_pool) and same_bits(dcf.v_pool, dc3.v_pool)


def test_alibi_layer_calls_reject_missing_slopes_and_slopes_with_a_rotary_basis():
    desc = ea.LayerDesc(512, 8, 8, 128, 80, 80, ea.EA_BF16, 64)
    g = synth.rng(97)
    K0, V0 = random_cache(desc, [100], g)
    dc = DeviceCache(desc, K0, V0, g, extra_len=1)
    wqkv, wo, _, _, _ = layer_weights(desc, g, False)
    x = to_dev(desc, quantize(desc, synth.gaussian(g, (1, 512))))
    y = torch.empty((1, 512), dtype=torch.bfloat16, device="cuda")
    ws = torch.empty(ea.decode_layer_fused_workspace_bytes(desc, 1, 1) // 4, device="cuda")
    sl = torch.zeros(8, dtype=torch.float32, device="cuda")
    with pytest.raises(ValueError):
        ea.decode_layer(desc, x, wqkv, wo, dc.k_pool, dc.v_pool, dc.page_table, dc.seq_len, y, 1, ws,
                        u_k=torch.empty((128, 80), dtype=torch.bfloat16, device="cuda"), alibi_slopes=sl)
    with pytest.raises(ValueError):
        ea.decode_layer_alibi(desc, x, wqkv, wo, sl[:4], dc.k_pool, dc.v_pool, dc.page_table, dc.seq_len, y, 1, ws)
    lib = ea.load_library()
    import ctypes
    for fn in (lib.ea_decode_layer_alibi, lib.ea_decode_layer_fused_alibi):
        rc = fn(ctypes.byref(desc), x.data_ptr(), wqkv.data_ptr(), wo.data_ptr(), None, dc.k_pool.data_ptr(),
                dc.v_pool.data_ptr(), dc.page_table.data_ptr(), dc.seq_len.data_ptr(), y.data_ptr(), 1,
                dc.page_table.shape[1], dc.k_pool.shape[0], 1, ws.data_ptr(), ws.numel() * 4, None, None)
        assert rc == -1                      # EA_ERR_ARG
    # zero slopes: the plain step (the bias term is an exact zero)
    k0, v0 = dc.k_pool.clone(), dc.v_pool.clone()
    ea.decode_layer_alibi(desc, x, wqkv, wo, sl, dc.k_pool, dc.v_pool, dc.page_table, dc.seq_len, y, 1, ws)
    y0 = y.clone()
    dc.k_pool.copy_(k0); dc.v_pool.copy_(v0)
    ea.decode_layer(desc, x, wqkv, wo, dc.k_pool, dc.v_pool, dc.page_table, dc.seq_len, y, 1, ws)
    torch.cuda.synchronize()
    assert ora.rel_l2(y0.float().cpu().numpy(), y.float().cpu().numpy()) < 1e-3


@pytest.mark.parametrize("seed", [4101, 4102])
def test_alibi_decode_layer_random_shapes(seed):
    """Drawn shapes (group sizes, head counts that are no power of two, ranks off every chunk size, page sizes, ragged
    lengths down to an empty cache, split counts, model widths, slopes from zero to steep) through both forms against
    the oracle's generation step with slopes."""
    rs = np.random.default_rng(seed)
    for case in range(12):
        G = int(rs.choice([1, 1, 2, 4, 8, 16]))
        Hkv = int(rs.choice([1, 2, 3, 4, 8]))
        H = G * Hkv
        r_k = int(rs.integers(1, 17)) * 8
        r_v = 0
        while r_v == 0 or (H * r_v) % 32 != 0:
            r_v = int(rs.integers(1, 17)) * 8
        P = int(rs.choice([64, 128, 256]))
        B = int(rs.integers(1, 17))
        d = int(rs.choice([128, 256, 512, 1024, 2048]))
        lens = [int(rs.choice([0, 1, 63, 64, 65, 128, int(rs.integers(1, 1500))])) for _ in range(B)]
        S = int(rs.choice([0, 1, 2, 3, 5, 8, 9, 16]))
        slopes = (rs.choice([0.0, 1.0, 4.0], size=H) * rs.random(H) * 0.1 + 2.0 ** -rs.integers(1, 10, size=H) *
                  rs.integers(0, 2, size=H)).astype(np.float32)
        print(f"seed {seed} case {case}: d={d} H={H}/{Hkv} r=({r_k},{r_v}) P={P} B={B} lens={lens} S={S}", flush=True)
        desc = ea.LayerDesc(d, H, Hkv, 128, r_k, r_v, ea.EA_BF16, P)
        g = synth.rng(seed, case)
        x = quantize(desc, synth.gaussian(g, (B, d)))
        K0, V0 = random_cache(desc, lens, g)
        wqkv, wo, _, _, folded = layer_weights(desc, g, False)
        sl = torch.tensor(slopes, device="cuda")
        xd = to_dev(desc, x)
        y_ref = ora.decode_step(x, folded, ora.RankCache.from_arrays(K0, V0), 128, alibi_slopes=slopes.astype(np.float64))
        pools = []
        for fused in (False, True):
            dc = DeviceCache(desc, K0, V0, synth.rng(seed, case, 1), extra_len=1)
            S_eff = S or ea.decode_auto_splits(desc, B, dc.max_pages * P)
            nbytes = (ea.decode_layer_fused_workspace_bytes if fused else ea.decode_layer_workspace_bytes)(desc, B, S_eff)
            ws = torch.full((max(nbytes // 4, 4),), float("nan"), device="cuda")
            y = torch.full((B, d), float("nan"), dtype=torch.bfloat16, device="cuda")
            status = torch.zeros(1, dtype=torch.int32, device="cuda")
            ea.decode_layer_alibi(desc, xd, wqkv, wo, sl, dc.k_pool, dc.v_pool, dc.page_table, dc.seq_len, y, S, ws,
                                  status=status, fused=fused)
            torch.cuda.synchronize()
            assert int(status.item()) == 0
            assert_close(y.float().cpu().numpy(), y_ref, TOL_BF16, f"seed {seed} case {case} fused={fused}")
            pools.append((dc.k_pool, dc.v_pool))
        assert same_bits(pools[0][0], pools[1][0]) and same_bits(pools[0][1], pools[1][1])
