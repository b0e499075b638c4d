"""ea_decode_attn_static (the entry point that allocates nothing: split partials in the library's built-in buffer)
against ea_decode_attn on the same inputs, and against the fp64 oracle, on calls that follow each other and so
share the buffer -- the second smaller than the first."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2408_05646_amd as ea
from oracle import eigen_attention as ora
from paper_2408_05646_amd import synth
from helpers import DeviceCache, TOL_BF16, TOL_F32, assert_close, random_cache

pytestmark = pytest.mark.gpu


def _case(desc, lens, seed):
    g = synth.rng(77, seed, len(lens))
    K, V = random_cache(desc, lens, g)
    q = np.float32(synth.gaussian(g, (len(lens), desc.n_heads, desc.r_k))).astype(np.float64)
    dc = DeviceCache(desc, K, V, g)
    cache = ora.RankCache.from_arrays(K, V)
    return dc, torch.from_numpy(q.astype(np.float32)).cuda(), ora.decode_attention(q, cache, desc.d_head)


def _both(desc, dc, q, S):
    """(static entry point's output, ea_decode_attn's output with a caller workspace) for the same split count."""
    B = q.shape[0]
    ref = torch.full((B, desc.n_heads, desc.r_v), float("nan"), dtype=torch.float32, device="cuda")
    got = torch.full_like(ref, float("nan"))
    nbytes = ea.decode_workspace_bytes(desc, B, S)
    ws = torch.full((max(nbytes // 4, 4),), float("nan"), dtype=torch.float32, device="cuda")
    ea.decode_attn(desc, q, dc.k_pool, dc.v_pool, dc.page_table, dc.seq_len, ref, n_splits=S, ws=ws)
    ea.decode_attn_static(desc, q, dc.k_pool, dc.v_pool, dc.page_table, dc.seq_len, got, n_splits=S)
    torch.cuda.synchronize()
    return got.cpu().numpy(), ref.cpu().numpy()


@pytest.mark.parametrize("dtype,tol", [(ea.EA_BF16, TOL_BF16), (ea.EA_F32, TOL_F32)])
def test_static_entry_point_matches_decode_attn_on_two_calls_in_a_row(dtype, tol):
    print(f"static decode dtype={dtype}", flush=True)
    P = 64 if dtype == ea.EA_BF16 else 16
    big = ea.LayerDesc(1024, 8, 2, 128, 80, 112, dtype, P)        # GQA 4:1, ragged lengths, 6 splits
    small = ea.LayerDesc(256, 4, 4, 64, 48, 32, dtype, P)         # fewer heads, lower ranks, 3 splits
    dc1, q1, o1 = _case(big, [1500, 700, 2047], 1)
    dc2, q2, o2 = _case(small, [300, 129], 2)
    # first call, then a smaller one that finds the first call's partials in the buffer, then the first again
    for desc, dc, q, ora_out, S in ((big, dc1, q1, o1, 6), (small, dc2, q2, o2, 3), (big, dc1, q1, o1, 6)):
        got, ref = _both(desc, dc, q, S)
        assert np.array_equal(got, ref), "same kernels, same split count: the two entry points must agree bit for bit"
        assert_close(got, ora_out, tol, "ea_decode_attn_static vs oracle")


def test_static_entry_point_auto_splits_and_single_split():
    print("static decode auto / single split", flush=True)
    desc = ea.LayerDesc(512, 8, 1, 64, 64, 64, ea.EA_BF16, 64)
    dc, q, ora_out = _case(desc, [4096, 100], 3)
    for S in (0, 1):
        out = torch.full((2, 8, 64), float("nan"), dtype=torch.float32, device="cuda")
        ea.decode_attn_static(desc, q, dc.k_pool, dc.v_pool, dc.page_table, dc.seq_len, out, n_splits=S)
        torch.cuda.synchronize()
        assert_close(out.cpu().numpy(), ora_out, TOL_BF16, f"static, n_splits={S}")


def test_static_entry_point_rejects_what_does_not_fit():
    print("static decode limit", flush=True)
    desc = ea.LayerDesc(4096, 32, 32, 128, 128, 128, ea.EA_BF16, 64)
    B, S = 16, 64                                                 # 16 * 32 * 64 * 130 floats = 17 MB of partials
    assert ea.decode_workspace_bytes(desc, B, S) > ea.STATIC_SCRATCH_BYTES
    dummy = torch.zeros(64, dtype=torch.float32, device="cuda")
    pools = torch.zeros(64, dtype=torch.bfloat16, device="cuda")
    ints = torch.zeros(64, dtype=torch.int32, device="cuda")
    rc = ea.load_library().ea_decode_attn_static(ctypes.byref(desc), dummy.data_ptr(), pools.data_ptr(), pools.data_ptr(),
                                                 ints.data_ptr(), ints.data_ptr(), dummy.data_ptr(), B, 1, 1, S, None)
    assert rc == -6 and "scratch" in ea.strerror(rc)
