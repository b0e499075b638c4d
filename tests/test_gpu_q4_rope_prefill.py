"""ea_prefill_attn_rope_q4: causal rotary prefill (Sec. 4.3, Eq. 9-10) over a cache whose older tokens are 4- or 3-bit
codes (quantisation paragraph of the results; the Llama models of that experiment are rotary) against the oracle's
rotary prefill over the dequantised values, and a prompt prefilled chunk by chunk with every chunk quantised at once."""
import numpy as np
import pytest
import torch

import paper_2408_05646_amd as ea
from oracle import eigen_attention as ora
from oracle import quant_cache as oq
from paper_2408_05646_amd import synth
from helpers import TOL_BF16, assert_close, quantize, to_dev
from test_gpu_q4 import Q4Cache

pytestmark = pytest.mark.gpu


def offset_cache(desc, lens, g, k_std=1.0):
    """Keys with a different mean per channel and values with a different mean per token, as in the position-free
    tests of the quantised cache but with smaller means (1.0 and 0.5 instead of 2.0 and 1.5): the rotary path rounds
    the staged keys, the rotated keys and the rotated queries to bfloat16, and with the larger means single query
    rows of the d_head = 64 case sit at 4 % against the fp64 oracle in a CPU emulation of just these roundings."""
    K, V = [], []
    for n in lens:
        k = synth.gaussian(g, (desc.n_kv_heads, n, desc.r_k), k_std) + 1.0 * synth.gaussian(g, (desc.n_kv_heads, 1, desc.r_k))
        v = synth.gaussian(g, (desc.n_kv_heads, n, desc.r_v)) + 0.5 * synth.gaussian(g, (desc.n_kv_heads, n, 1))
        K.append(quantize(desc, k))
        V.append(quantize(desc, v))
    return K, V


def run_prefill_rope_q4(desc, qc, q, U, base):
    B, n = q.shape[0], q.shape[1]
    out = torch.full((B, n, desc.n_heads, desc.r_v), float("nan"), dtype=torch.bfloat16, device="cuda")
    nbytes = ea.prefill_rope_q4_workspace_bytes(desc, B, n, qc.q4_table.shape[1], qc.tail_table.shape[1])
    ws = torch.full((nbytes // 4,), float("nan"), dtype=torch.float32, device="cuda")
    ea.prefill_attn_rope_q4(desc, to_dev(desc, q), to_dev(desc, U), base, qc.kq, qc.vq, qc.q4_table, qc.q4_len,
                            qc.dc.k_pool, qc.dc.v_pool, qc.tail_table, qc.tail_len, out, ws)
    torch.cuda.synchronize()
    return out.float().cpu().numpy()


@pytest.mark.parametrize("H,Hkv,d_h,r_k,r_v,P,group,bits,lens,n_quant,n", [
    (2, 2, 128, 80, 80, 64, 64, 4, [200, 130], [128, 64], 60),          # two pages / one page quantised, ragged query count
    (2, 2, 128, 80, 80, 64, 64, 4, [300, 300], [0, 128], 150),          # a sequence with nothing quantised yet
    (8, 2, 128, 48, 112, 128, 64, 4, [777, 1500], [512, 1280], 200),    # GQA 4:1, r_k != r_v, two key groups per page
    (4, 4, 64, 64, 64, 64, 64, 4, [513, 400], [256, 192], 129),         # d_head = 64 at full rank
    (4, 2, 128, 30, 33, 64, 64, 4, [150, 270], [64, 192], 70),          # ranks off the chunk sizes
    (2, 2, 128, 80, 80, 128, 128, 4, [600, 300], [384, 128], 170),      # key groups of 128 tokens
    (4, 2, 128, 64, 64, 256, 128, 3, [2100], [1792], 300),              # 3-bit codes, pages of 256 tokens
    (2, 1, 128, 96, 64, 64, 64, 3, [900, 64], [832, 0], 64),            # 3-bit codes; a sequence of one page, all of it queries
])
def test_prefill_attn_rope_q4_matches_oracle(H, Hkv, d_h, r_k, r_v, P, group, bits, lens, n_quant, n):
    print(f"q{bits} rope prefill H={H}/{Hkv} d_h={d_h} r=({r_k},{r_v}) P={P} group={group} lens={lens} "
          f"quantised={n_quant} n={n}", flush=True)
    desc = ea.LayerDesc(H * d_h, H, Hkv, d_h, r_k, r_v, ea.EA_BF16, P, group, bits)
    g = synth.rng(171, H, r_k, len(lens), n)
    U = quantize(desc, synth.orthonormal_basis(g, d_h, r_k))
    K, V = offset_cache(desc, lens, g, k_std=1.5)
    q = quantize(desc, synth.gaussian(g, (len(lens), n, H, d_h), 1.0))
    qc = Q4Cache(desc, K, V, n_quant, g)
    got = run_prefill_rope_q4(desc, qc, q, U, 10000.0)
    ref = oq.prefill_attention_rope_quantized(q, K, V, n_quant, U, d_h, 10000.0, group_tokens=group, bits=bits)
    err = assert_close(got, ref, TOL_BF16, "q4 rope prefill")
    print(f"  rel-L2 {err:.2e}", flush=True)
    # positions are in there: the position-free prefill of the projected queries gives something else
    flat = oq.prefill_attention_quantized(np.einsum("bnhc,cr->bnhr", q, U), K, V, n_quant, d_h, group_tokens=group, bits=bits)
    assert ora.rel_l2(flat, ref) > 10 * err
    if max(n_quant) >= 256:
        # and so is the quantisation
        plain = ora.prefill_attention_rope(q, ora.RankCache.from_arrays(K, V), U, d_h, 10000.0)
        assert ora.rel_l2(plain, ref) > 3 * err


def test_prefill_rope_q4_skips_pages_that_are_not_there_and_leaves_the_pools_alone():
    """A 4-bit page-table entry outside its pool makes that page's tokens vanish (the positions of the others stay);
    neither the 4-bit pools nor the bfloat16 pools are written."""
    desc = ea.LayerDesc(512, 4, 2, 128, 80, 48, ea.EA_BF16, 64)
    g = synth.rng(172)
    lens, n_quant, n = [384], [256], 100
    U = quantize(desc, synth.orthonormal_basis(g, 128, 80))
    K, V = offset_cache(desc, lens, g)
    q = quantize(desc, synth.gaussian(g, (1, n, 4, 128)))
    qc = Q4Cache(desc, K, V, n_quant, g)
    table = qc.q4_table.clone()
    table[0, 1] = qc.q4_pool_pages + 9
    qc.q4_table = table
    before = [t.clone() for t in (qc.kq, qc.vq, qc.dc.k_pool, qc.dc.v_pool)]
    got = run_prefill_rope_q4(desc, qc, q, U, 10000.0)
    for a, b in zip(before, (qc.kq, qc.vq, qc.dc.k_pool, qc.dc.v_pool)):
        assert torch.equal(a.view(torch.uint8), b.view(torch.uint8))
    # oracle: scores of every (query, key) pair at their true positions, the missing page's keys left out
    Kq, Vq = oq.quantized_view(K[0], V[0], 256)
    keep = np.r_[0:64, 128:384]
    ref = np.zeros((1, n, 4, 48))
    for j in range(n):
        pos = 384 - n + j
        for h in range(4):
            kv = h // 2
            ts = keep[keep <= pos]
            k_rot = ora.rope_rotate(Kq[kv, ts] @ U.T, ts, 10000.0)
            q_rot = ora.rope_rotate(q[0, j, h], pos, 10000.0)
            ref[0, j, h] = ora.softmax(k_rot @ q_rot / np.sqrt(128)) @ Vq[kv, ts]
    assert_close(got, ref, TOL_BF16, "q4 rope prefill with a missing page")


def test_a_rotary_prompt_prefilled_in_chunks_with_every_chunk_quantised_at_once():
    """Four chunks of one sequence: each is written to the same few bfloat16 pages, attended with the rotary call
    (earlier chunks as codes), quantised, and its bfloat16 pages reused.  Every chunk follows the oracle at its cut."""
    H, Hkv, d_h, r_k, r_v, P, chunk = 4, 2, 128, 80, 48, 64, 192
    desc = ea.LayerDesc(H * d_h, H, Hkv, d_h, r_k, r_v, ea.EA_BF16, P)
    g = synth.rng(173)
    n_chunks = 4
    n_all = n_chunks * chunk
    U = quantize(desc, synth.orthonormal_basis(g, d_h, r_k))
    K, V = offset_cache(desc, [n_all], g, k_std=1.5)
    q = quantize(desc, synth.gaussian(g, (1, n_all, H, d_h)))
    stage_pages = chunk // P
    k_pool, v_pool = ea.alloc_pools(desc, stage_pages)
    stage_table = torch.arange(stage_pages, dtype=torch.int32, device="cuda").reshape(1, stage_pages).contiguous()
    q4_pages = n_all // P
    kq, vq = ea.alloc_q4_pools(desc, q4_pages + 2)
    ids = g.permutation(q4_pages + 2).astype(np.int32)[:q4_pages]
    q4_table = torch.from_numpy(ids.reshape(1, q4_pages)).cuda()
    out = torch.empty((1, chunk, H, r_v), dtype=torch.bfloat16, device="cuda")
    ws = torch.empty(ea.prefill_rope_q4_workspace_bytes(desc, 1, chunk, q4_pages, stage_pages) // 4, device="cuda")
    for c in range(n_chunks):
        c0 = c * chunk
        k_pool.fill_(float("nan")); v_pool.fill_(float("nan"))
        ea.cache_scatter(desc, to_dev(desc, K[0][None, :, c0:c0 + chunk]), to_dev(desc, V[0][None, :, c0:c0 + chunk]),
                         k_pool, v_pool, stage_table)
        ea.prefill_attn_rope_q4(desc, to_dev(desc, q[:, c0:c0 + chunk]), to_dev(desc, U), 10000.0, kq, vq, q4_table,
                                torch.tensor([c0], dtype=torch.int32).cuda(), k_pool, v_pool, stage_table,
                                torch.tensor([chunk], dtype=torch.int32).cuda(), out, ws)
        ea.quantize_pages_q4(desc, k_pool, v_pool, stage_table[0].contiguous(), kq, vq,
                             q4_table[0, c0 // P:(c0 + chunk) // P].contiguous())
        torch.cuda.synchronize()
        ref = oq.prefill_attention_rope_quantized(q[:, c0:c0 + chunk], [K[0][:, :c0 + chunk]], [V[0][:, :c0 + chunk]],
                                                  [c0], U, d_h, 10000.0)
        err = assert_close(out.float().cpu().numpy(), ref, TOL_BF16, f"chunk {c}")
        print(f"  chunk {c}: rel-L2 {err:.2e}", flush=True)


@pytest.mark.parametrize("seed", [5201])
def test_prefill_attn_rope_q4_random_shapes(seed):
    """Drawn shapes: group sizes, ranks off every chunk size, both head sizes, page sizes, key groups and code widths,
    ragged lengths, sequences with nothing quantised and with nothing but one page in 16 bits."""
    rs = np.random.default_rng(seed)
    for case in range(10):
        G = int(rs.choice([1, 2, 4, 8]))
        Hkv = int(rs.choice([1, 2, 3]))
        H = G * Hkv
        d_h = int(rs.choice([64, 128]))
        r_k = int(rs.integers(1, d_h // 8 + 1)) * 8
        r_v = int(rs.integers(1, 17)) * 8
        group = int(rs.choice([64, 128]))
        P = int(rs.choice([64, 128, 256] if group == 64 else [128, 256]))
        bits = int(rs.choice([4, 3]))
        B = int(rs.integers(1, 4))
        n = int(rs.integers(1, 150))
        n_quant = [int(rs.integers(0, 6)) * P for _ in range(B)]
        lens = [nq + n + int(rs.integers(0, 200)) for nq in n_quant]
        print(f"seed {seed} case {case}: H={H}/{Hkv} d_h={d_h} r=({r_k},{r_v}) P={P} group={group} bits={bits} "
              f"lens={lens} quantised={n_quant} n={n}", flush=True)
        desc = ea.LayerDesc(H * d_h, H, Hkv, d_h, r_k, r_v, ea.EA_BF16, P, group, bits)
        g = synth.rng(seed, case)
        U = quantize(desc, synth.orthonormal_basis(g, d_h, r_k))
        K, V = offset_cache(desc, lens, g)
        q = quantize(desc, synth.gaussian(g, (B, n, H, d_h)))
        qc = Q4Cache(desc, K, V, n_quant, g)
        got = run_prefill_rope_q4(desc, qc, q, U, 10000.0)
        ref = oq.prefill_attention_rope_quantized(q, K, V, n_quant, U, d_h, 10000.0, group_tokens=group, bits=bits)
        assert_close(got, ref, TOL_BF16, f"seed {seed} case {case}")


@pytest.mark.parametrize("rope", [False, True])
def test_staged_quantised_prefill_is_graph_capturable(rope):
    """The staged calls only enqueue kernels on the caller's stream (the stage lives in the caller's workspace; no
    allocation, no memset), so they can be captured in a HIP graph; every replay, with the workspace and the output
    overwritten in between, reproduces the eager result."""
    H, Hkv, d_h, r_k, r_v, P = 4, 2, 128, 80, 48, 64
    desc = ea.LayerDesc(H * d_h, H, Hkv, d_h, r_k, r_v, ea.EA_BF16, P)
    g = synth.rng(174, int(rope))
    lens, n_quant, n = [700, 400], [512, 192], 150
    U = quantize(desc, synth.orthonormal_basis(g, d_h, r_k))
    K, V = offset_cache(desc, lens, g)
    q = to_dev(desc, quantize(desc, synth.gaussian(g, (2, n, H, d_h if rope else r_k))))
    qc = Q4Cache(desc, K, V, n_quant, g)
    Ud = to_dev(desc, U)
    out = torch.empty((2, n, H, r_v), dtype=torch.bfloat16, device="cuda")
    mq, mt = qc.q4_table.shape[1], qc.tail_table.shape[1]
    nbytes = (ea.prefill_rope_q4_workspace_bytes if rope else ea.prefill_q4_staged_workspace_bytes)(desc, 2, n, mq, mt)
    ws = torch.empty(nbytes // 4, dtype=torch.float32, device="cuda")

    def call():
        if rope:
            ea.prefill_attn_rope_q4(desc, q, Ud, 10000.0, qc.kq, qc.vq, qc.q4_table, qc.q4_len, qc.dc.k_pool,
                                    qc.dc.v_pool, qc.tail_table, qc.tail_len, out, ws)
        else:
            ea.prefill_attn_q4(desc, q, qc.kq, qc.vq, qc.q4_table, qc.q4_len, qc.dc.k_pool, qc.dc.v_pool,
                               qc.tail_table, qc.tail_len, out, ws, staged=True)

    call()
    torch.cuda.synchronize()
    eager = out.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        call()
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        call()
    for rep in range(3):
        out.zero_(); ws.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), eager.view(torch.int16)), f"replay {rep} differs from the eager result"
