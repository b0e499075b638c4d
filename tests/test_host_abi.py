"""CPU-only checks of the C-ABI library: it loads, exports every declared symbol,
and its host-side layout / paging reference functions behave as documented."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2408_05646_amd as ea

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def desc(dtype=ea.EA_BF16, H=8, Hkv=2, r_k=80, r_v=48, P=128, d=1024, d_h=128):
    return ea.LayerDesc(d, H, Hkv, d_h, r_k, r_v, dtype, P)


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "eigenattn.h")).read()
    declared = set(re.findall(r"EA_API\s+[\w\s\*]+?\b(ea_\w+)\s*\(", header))
    assert declared == set(ea.EXPORTED_SYMBOLS) and len(declared) == 60
    lib = ctypes.CDLL(ea.library_path())
    for name in declared:
        assert getattr(lib, name) is not None
    assert ea.version() >= 100
    assert ea.strerror(0) == "ok" and "aligned" in ea.strerror(-3)


def test_layout_query_and_padding():
    lay = ea.cache_layout_query(desc(r_k=80, r_v=40))
    assert (lay.layout_id, lay.elem_bytes, lay.r_k_pad, lay.r_v_pad) == (1, 2, 80, 48)
    assert lay.k_slab_elems == 128 * 80 and lay.k_page_elems == 2 * 128 * 80
    assert lay.v_slab_elems == 128 * 48
    lay = ea.cache_layout_query(desc(ea.EA_F32, r_k=30, r_v=33, P=16))
    assert (lay.layout_id, lay.elem_bytes, lay.r_k_pad, lay.r_v_pad) == (0, 4, 32, 36)


@pytest.mark.parametrize("dtype,P,r_k,r_v", [(ea.EA_BF16, 64, 80, 80), (ea.EA_BF16, 192, 48, 112),
                                             (ea.EA_BF16, 128, 128, 16), (ea.EA_F32, 16, 32, 64)])
def test_cache_index_is_a_bijection_per_slab(dtype, P, r_k, r_v):
    d = desc(dtype, Hkv=2, r_k=r_k, r_v=r_v, P=P)
    lay = ea.cache_layout_query(d)
    for fn, r, slab, page_elems in ((ea.cache_k_index, r_k, lay.k_slab_elems, lay.k_page_elems),
                                    (ea.cache_v_index, r_v, lay.v_slab_elems, lay.v_page_elems)):
        for page, head in ((0, 0), (3, 1)):
            idx = np.array([[fn(d, page, head, t, c) for c in range(r)] for t in range(P)])
            base = page * page_elems + head * slab
            assert idx.min() == base and idx.max() == base + slab - 1      # ranks here need no padding
            assert np.unique(idx).size == P * r


def k_index_from_description(t, c, r_pad):
    """Written from the header's words: tiles of 64 tokens; [4 blocks of 16 tokens][r_pad/8 chunks][16 tokens][8 channels]."""
    tile, tt = divmod(t, 64)
    tb, row = divmod(tt, 16)
    chunk, e = divmod(c, 8)
    return tile * 64 * r_pad + ((tb * (r_pad // 8) + chunk) * 16 + row) * 8 + e


def v_index_from_description(t, c, r_pad):
    """[2 groups of 32 tokens][r_pad/16 blocks][4 quads][16 channels][8 slots]; slot j of quad q is token 16*(j/4)+4*q+j%4."""
    tile, tt = divmod(t, 64)
    grp, t32 = divmod(tt, 32)
    cb, c16 = divmod(c, 16)
    for quad in range(4):
        for j in range(8):
            if 16 * (j // 4) + 4 * quad + j % 4 == t32:
                return tile * 64 * r_pad + ((((grp * (r_pad // 16) + cb) * 4 + quad) * 16 + c16) * 8 + j)
    raise AssertionError


def test_bf16_fragment_order_matches_its_description():
    d = desc(ea.EA_BF16, Hkv=2, r_k=72, r_v=40, P=128)
    lay = ea.cache_layout_query(d)
    assert (lay.r_k_pad, lay.r_v_pad) == (72, 48)
    rng = np.random.default_rng(0)
    for _ in range(300):
        page, head, t = int(rng.integers(0, 5)), int(rng.integers(0, 2)), int(rng.integers(0, 128))
        ck, cv = int(rng.integers(0, 72)), int(rng.integers(0, 40))
        assert ea.cache_k_index(d, page, head, t, ck) == page * lay.k_page_elems + head * lay.k_slab_elems + \
            k_index_from_description(t, ck, 72)
        assert ea.cache_v_index(d, page, head, t, cv) == page * lay.v_page_elems + head * lay.v_slab_elems + \
            v_index_from_description(t, cv, 48)
    # one wave-wide load of a K block is contiguous: 16 tokens x 8 channels of one chunk = 128 consecutive elements
    base = ea.cache_k_index(d, 0, 0, 16, 8)
    got = sorted(ea.cache_k_index(d, 0, 0, 16 + row, 8 + e) - base for row in range(16) for e in range(8))
    assert got == list(range(128))
    assert ea.cache_k_index(d, 0, 0, 0, 72) == -1 and ea.cache_k_index(d, 0, 2, 0, 0) == -1
    assert ea.cache_v_index(d, 0, 0, 128, 0) == -1 and ea.cache_v_index(d, -1, 0, 0, 0) == -1


def test_f32_rows_are_token_major():
    d = desc(ea.EA_F32, Hkv=2, r_k=30, r_v=64, P=16)
    assert ea.cache_k_index(d, 2, 1, 5, 7) == 2 * (2 * 16 * 32) + 1 * 16 * 32 + 5 * 32 + 7
    assert ea.cache_v_index(d, 1, 0, 15, 63) == 1 * (2 * 16 * 64) + 15 * 64 + 63


def test_cache_slot_paging_arithmetic():
    d = desc(P=128)
    row = np.array([7, 3, 11, 0], np.int32)
    for pos in (0, 1, 127, 128, 129, 383, 384, 511):
        assert ea.cache_slot(d, row, pos) == int(row[pos // 128]) * 128 + pos % 128
    assert ea.cache_slot(d, row, 512) == -1 and ea.cache_slot(d, row, -1) == -1
    assert ea.cache_slot(d, np.array([-1], np.int32), 0) == -1


def test_argument_errors_are_reported_before_any_launch():
    lib = ea.load_library()
    good = desc()
    bad_group = desc(H=8, Hkv=3)
    bad_rank = desc(r_k=136)
    bad_page = desc(P=48)
    out = ea.CacheLayout()
    assert lib.ea_cache_layout_query(ctypes.byref(bad_group), ctypes.byref(out)) == -2
    assert lib.ea_cache_layout_query(ctypes.byref(bad_rank), ctypes.byref(out)) == -2
    assert lib.ea_cache_layout_query(ctypes.byref(bad_page), ctypes.byref(out)) == -2
    assert lib.ea_cache_layout_query(None, ctypes.byref(out)) == -1
    # null pointers / bad sizes: rejected on the host, nothing is launched
    assert lib.ea_decode_attn(ctypes.byref(good), None, None, None, None, None, None, 1, 1, 1, 0, None, 0, None) == -1
    assert lib.ea_project_qkv(ctypes.byref(good), None, None, None, 0, None, None, None, None, 1, 1, 1, 1, None, None) == -1
    assert lib.ea_out_proj(ctypes.byref(good), None, 0, None, None, 4, None) == -1
    assert lib.ea_prefill_attn(ctypes.byref(good), None, None, None, None, None, None, 1, 1, 1, 1, None) == -1
    # misaligned pointer (fake, never dereferenced: the check comes first)
    p = 0x1000
    assert lib.ea_decode_attn(ctypes.byref(good), p + 4, p, p, p, p, p, 1, 1, 1, 1, None, 0, None) == -3
    # splits > 1 without a workspace
    assert lib.ea_decode_attn(ctypes.byref(good), p, p, p, p, p, p, 1, 1, 1, 4, None, 0, None) == -4
    assert ea.decode_workspace_bytes(good, 2, 4) == 2 * 8 * 4 * (2 + 48) * 4
    assert ea.decode_workspace_bytes(good, 2, 1) == 0
    assert 1 <= ea.decode_auto_splits(good, 16, 32768) <= 64


def test_packed_weight_size():
    assert ea.packed_weight_elems(7680, 4096, ea.EA_BF16) == 7680 * 4096
    assert ea.packed_weight_elems(100, 64, ea.EA_BF16) == 112 * 64        # channel rows padded to 16
    assert ea.packed_weight_elems(100, 48, ea.EA_BF16) == -1              # K must be a multiple of 32
    assert ea.packed_weight_elems(100, 50, ea.EA_F32) == 5000
    assert ea.packed_weight_elems(0, 64, ea.EA_BF16) == -1


def test_auto_splits_fill_the_chip():
    d = ea.LayerDesc(4096, 32, 32, 128, 80, 80, ea.EA_BF16, 64)
    assert ea.decode_auto_splits(d, 16, 32768) == 1          # 512 streams: one workgroup per resident slot
    assert ea.decode_auto_splits(d, 16, 64) == 1
    g = ea.LayerDesc(4096, 32, 8, 128, 80, 80, ea.EA_BF16, 64)
    assert ea.decode_auto_splits(g, 8, 16384) == 8            # 64 streams x 8 = 512 workgroups
    assert ea.decode_auto_splits(g, 1, 16384) == 32           # 8 streams: capped at 8 tiles per workgroup


# ---------------------------------------------------------------------------
# Error behaviour of the hot-path entry points: every check below fails BEFORE anything is launched or
# dereferenced, so made-up addresses are enough and no GPU is needed.
# ---------------------------------------------------------------------------
OK_PTR, ODD_PTR = 0x10000, 0x10008          # 16-byte aligned / not aligned; never dereferenced


def raw():
    lib = ea.load_library()
    return lib


def call_decode(lib, d, q=OK_PTR, k=OK_PTR, v=OK_PTR, pt=OK_PTR, sl=OK_PTR, out=OK_PTR, B=2, max_pages=4,
                pool_pages=8, n_splits=1, ws=None, ws_bytes=0):
    return lib.ea_decode_attn(ctypes.byref(d), q, k, v, pt, sl, out, B, max_pages, pool_pages, n_splits, ws, ws_bytes,
                              None)


def call_decode_rope(lib, d, q=OK_PTR, u=OK_PTR, base=10000.0, k=OK_PTR, n_splits=1, ws=None, ws_bytes=0):
    return lib.ea_decode_attn_rope(ctypes.byref(d), q, u, base, k, OK_PTR, OK_PTR, OK_PTR, OK_PTR, 2, 4, 8, n_splits,
                                   ws, ws_bytes, None)


def test_decode_attn_rejects_bad_arguments_before_launching():
    lib, d = raw(), desc()
    assert call_decode(lib, d, q=None) == -1                              # EA_ERR_ARG: null pointer
    assert call_decode(lib, d, B=0) == -1
    assert call_decode(lib, d, n_splits=1025) == -1
    assert call_decode(lib, d, k=ODD_PTR) == -3                           # EA_ERR_ALIGN
    assert call_decode(lib, d, n_splits=4) == -4                          # EA_ERR_WORKSPACE: splits need a workspace
    need = ea.decode_workspace_bytes(d, 2, 4)
    assert need == 2 * 8 * 4 * (2 + 48) * 4
    assert call_decode(lib, d, n_splits=4, ws=OK_PTR, ws_bytes=need - 1) == -4
    assert call_decode(lib, desc(H=8, Hkv=3)) == -2                       # EA_ERR_SHAPE: heads do not group evenly
    assert call_decode(lib, desc(r_k=136)) == -2                          # bf16 ranks stop at 128
    assert call_decode(lib, desc(P=96)) == -2                             # bf16 pages hold whole 64-token tiles
    bad = desc(); bad.dtype = 7
    assert call_decode(lib, bad) == -1


def test_static_decode_entry_point_rejects_bad_arguments_and_oversized_calls_before_launching():
    lib, d = raw(), desc()

    def call(dd=d, q=OK_PTR, k=OK_PTR, B=2, n_splits=1):
        return lib.ea_decode_attn_static(ctypes.byref(dd), q, k, OK_PTR, OK_PTR, OK_PTR, OK_PTR, B, 4, 8, n_splits, None)

    assert call(q=None) == -1 and call(B=0) == -1 and call(n_splits=1025) == -1
    assert call(k=ODD_PTR) == -3
    assert call(desc(r_k=136)) == -2
    # the partials of a call must fit the library's built-in buffer: checked on the host, nothing is launched
    big = ea.LayerDesc(4096, 32, 32, 128, 128, 128, ea.EA_BF16, 64)
    assert ea.decode_workspace_bytes(big, 16, 31) <= ea.STATIC_SCRATCH_BYTES < ea.decode_workspace_bytes(big, 16, 32)
    assert call(big, B=16, n_splits=32) == -6                             # EA_ERR_SCRATCH_LIMIT
    assert "scratch" in ea.strerror(-6)
    header = open(os.path.join(ROOT, "include", "eigenattn.h")).read()
    assert re.search(r"#define\s+EA_STATIC_SCRATCH_BYTES\s+\(8 \* 1024 \* 1024\)", header)
    assert ea.STATIC_SCRATCH_BYTES == 8 * 1024 * 1024


def test_rotary_entry_points_reject_bad_arguments_before_launching():
    lib = raw()
    d = desc()
    assert call_decode_rope(lib, d, u=None) == -1
    assert call_decode_rope(lib, d, base=1.0) == -1                       # the base must exceed 1
    assert call_decode_rope(lib, d, base=float("nan")) == -1
    assert call_decode_rope(lib, d, q=ODD_PTR) == -3
    assert call_decode_rope(lib, d, n_splits=2) == -4
    assert call_decode_rope(lib, desc(d_h=96, r_k=80)) == -2              # bf16 rotary kernels exist for d_head 64 and 128
    assert call_decode_rope(lib, desc(d_h=64, r_k=80)) == -2              # a basis cannot have more columns than rows
    assert call_decode_rope(lib, desc(ea.EA_F32, d_h=63, r_k=32, P=16)) == -2   # rotary pairs need an even d_head
    need = ea.prefill_rope_workspace_bytes(d, 2, 100, 4)
    assert need >= 2 * 4 * 2 * 128 * 128 * 2 + 2 * 100 * 8 * 128 * 2
    rc = lib.ea_prefill_attn_rope(ctypes.byref(d), OK_PTR, OK_PTR, 10000.0, OK_PTR, OK_PTR, OK_PTR, OK_PTR, OK_PTR, 2, 100,
                                  4, 8, OK_PTR, need - 1, None)
    assert rc == -4
    rc = lib.ea_project_qkv_rope(ctypes.byref(desc(d_h=64, r_k=80)), OK_PTR, OK_PTR, OK_PTR, ea.EA_BF16, OK_PTR, OK_PTR,
                                 OK_PTR, OK_PTR, 2, 1, 4, 8, None, None)
    assert rc == -2


def test_projection_and_prefill_reject_bad_arguments_before_launching():
    lib, d = raw(), desc()
    f = lib.ea_project_qkv
    assert f(ctypes.byref(d), None, OK_PTR, OK_PTR, ea.EA_BF16, OK_PTR, OK_PTR, OK_PTR, OK_PTR, 2, 1, 4, 8, None, None) == -1
    assert f(ctypes.byref(d), OK_PTR, OK_PTR, OK_PTR, 5, OK_PTR, OK_PTR, OK_PTR, OK_PTR, 2, 1, 4, 8, None, None) == -1
    assert f(ctypes.byref(d), OK_PTR, ODD_PTR, OK_PTR, ea.EA_BF16, OK_PTR, OK_PTR, OK_PTR, OK_PTR, 2, 1, 4, 8, None, None) == -3
    # the status word is optional, but when given it must be a 4-byte aligned address
    assert f(ctypes.byref(d), OK_PTR, OK_PTR, OK_PTR, ea.EA_BF16, OK_PTR, OK_PTR, OK_PTR, OK_PTR, 2, 1, 4, 8, OK_PTR + 2, None) == -3
    assert f(ctypes.byref(desc(d=1000)), OK_PTR, OK_PTR, OK_PTR, ea.EA_BF16, OK_PTR, OK_PTR, OK_PTR, OK_PTR, 2, 1, 4, 8,
             None, None) == -2                                             # bf16 needs d % 32 == 0
    f32 = desc(ea.EA_F32, P=16)
    assert f(ctypes.byref(f32), OK_PTR, OK_PTR, OK_PTR, ea.EA_BF16, OK_PTR, OK_PTR, OK_PTR, OK_PTR, 2, 1, 4, 8, None, None) == -1
    g = lib.ea_prefill_attn
    assert g(ctypes.byref(d), OK_PTR, OK_PTR, OK_PTR, OK_PTR, OK_PTR, None, 2, 5, 4, 8, None) == -1
    assert g(ctypes.byref(d), OK_PTR, OK_PTR, OK_PTR, OK_PTR, OK_PTR, OK_PTR, 2, 0, 4, 8, None) == -1
    assert g(ctypes.byref(d), OK_PTR, OK_PTR, ODD_PTR, OK_PTR, OK_PTR, OK_PTR, 2, 5, 4, 8, None) == -3
    h = lib.ea_out_proj
    assert h(ctypes.byref(d), OK_PTR, ea.EA_F32, OK_PTR, None, 4, None) == -1
    assert h(ctypes.byref(desc(H=3, Hkv=3, r_v=40)), OK_PTR, ea.EA_F32, OK_PTR, OK_PTR, 4, None) == -2   # (H r_v) % 32
    assert ea.strerror(-4).startswith("workspace") and ea.strerror(-2) == "unsupported shape"


# ---------------------------------------------------------------------------
# 4-bit group-quantised cache: layout reference functions and argument checks
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("P,r_k,r_v,Hkv", [(64, 80, 80, 2), (128, 30, 33, 1), (192, 128, 16, 3), (64, 8, 128, 1)])
def test_q4_positions_tile_the_page_exactly(P, r_k, r_v, Hkv):
    """Every code has its own nibble, every scale and zero its own two bytes, nothing overlaps, and all of it
    lies inside the page; the sizes are the documented ones."""
    d = desc(Hkv=Hkv, H=Hkv, r_k=r_k, r_v=r_v, P=P)
    lay = ea.q4_layout_query(d)
    assert lay.r_k_pad == -(-r_k // 8) * 8 and lay.r_v_pad == -(-r_v // 16) * 16
    assert lay.k_tile_bytes == 32 * lay.r_k_pad + 128 * (-(-lay.r_k_pad // 32))
    assert lay.v_tile_bytes == 32 * lay.r_v_pad + 256
    assert lay.k_page_bytes == Hkv * (P // 64) * lay.k_tile_bytes
    assert lay.v_page_bytes == Hkv * (P // 64) * lay.v_tile_bytes
    page = 2
    used_k = np.zeros(lay.k_page_bytes * 2, np.int32)          # per nibble
    used_v = np.zeros(lay.v_page_bytes * 2, np.int32)
    for h in range(Hkv):
        for t in range(P):
            for c in range(r_k):
                pos = ea.q4_k_code_pos(d, page, h, t, c)
                assert pos % 4 == 0
                used_k[pos // 4 - page * lay.k_page_bytes * 2] += 1
            for c in range(r_v):
                pos = ea.q4_v_code_pos(d, page, h, t, c)
                assert pos % 4 == 0
                used_v[pos // 4 - page * lay.v_page_bytes * 2] += 1
            sp = ea.q4_v_scale_pos(d, page, h, t) - page * lay.v_page_bytes
            for off in (sp, sp + 128):                          # scale, zero
                used_v[2 * off:2 * off + 4] += 1
        for tile in range(P // 64):
            for c in range(r_k):
                sp = ea.q4_k_scale_pos(d, page, h, tile * 64 + 5, c) - page * lay.k_page_bytes
                assert sp == ea.q4_k_scale_pos(d, page, h, tile * 64, c) - page * lay.k_page_bytes
                for off in (sp, sp + 16):
                    used_k[2 * off:2 * off + 4] += 1
    assert used_k.max() == 1 and used_v.max() == 1
    # what is left over are the padding channels only
    assert used_k.sum() == Hkv * P * r_k + Hkv * (P // 64) * r_k * 8
    assert used_v.sum() == Hkv * P * r_v + Hkv * P * 8
    assert ea.q4_k_code_pos(d, 0, Hkv, 0, 0) == -1 and ea.q4_k_code_pos(d, 0, 0, P, 0) == -1
    assert ea.q4_v_code_pos(d, 0, 0, 0, r_v) == -1 and ea.q4_v_scale_pos(d, -1, 0, 0) == -1
    assert ea.q4_k_scale_pos(d, 0, 0, 0, r_k) == -1


def test_q4_code_order_matches_its_description():
    """Keys: the dword of (token 16*tb + t, channels 32*kk + 8*quad ..) is dword tb of the 16-byte unit of lane
    16*quad + t in the run of k-step kk; element e of the eight sits in nibble e/2 (even) or 4 + e/2 (odd)."""
    d = desc(Hkv=1, H=1, r_k=80, r_v=80, P=64)
    for (t, c) in [(0, 0), (17, 9), (63, 79), (35, 44)]:
        tb, tt, kk, quad, e = t // 16, t % 16, c // 32, (c // 8) % 4, c % 8
        byte = kk * 1024 + (quad * 16 + tt) * 16 + tb * 4
        nib = e // 2 if e % 2 == 0 else 4 + e // 2
        assert ea.q4_k_code_pos(d, 0, 0, t, c) == byte * 8 + 4 * nib
        assert ea.q4_k_scale_pos(d, 0, 0, t, c) == 10 * 256 + (kk * 4 + quad) * 32 + 2 * e
    # values: dword (cb, u) of lane 16*quad + ch, token slot j <-> token 32*u + 16*(j/4) + 4*quad + j%4; the odd
    # last channel block (cb = 4 of 5) has 8-byte units
    for (t, c) in [(0, 0), (21, 37), (63, 79), (40, 64)]:
        u, t32 = t // 32, t % 32
        half, quad, j = t32 // 16, (t32 % 16) // 4, (t32 // 16) * 4 + t32 % 4
        cb, ch = c // 16, c % 16
        lane = quad * 16 + ch
        byte = (cb // 2) * 1024 + (lane * 8 + u * 4 if cb == 4 else lane * 16 + ((cb % 2) * 2 + u) * 4)
        nib = j // 2 if j % 2 == 0 else 4 + j // 2
        assert ea.q4_v_code_pos(d, 0, 0, t, c) == byte * 8 + 4 * nib
        assert ea.q4_v_scale_pos(d, 0, 0, t) == 5 * 512 + ((u * 4 + quad) * 8 + j) * 2


def test_q4_entry_points_reject_bad_arguments_before_launching():
    lib, d = raw(), desc()

    def quant(dd=d, k=OK_PTR, kq=OK_PTR, src=OK_PTR, n=3, pool=8, qpool=8):
        return lib.ea_quantize_pages_q4(ctypes.byref(dd), k, OK_PTR, src, kq, OK_PTR, OK_PTR, n, pool, qpool, None)

    assert quant(src=None) == -1 and quant(n=-1) == -1 and quant(qpool=0) == -1
    assert quant(kq=ODD_PTR) == -3
    assert quant(dd=desc(dtype=ea.EA_F32, P=64)) == -2                     # bf16 layers only
    assert quant(n=0) == 0                                                 # nothing to do, nothing launched

    def dequant(dd=d, kq=OK_PTR, src=OK_PTR, n=3, qpool=8, pool=8):
        return lib.ea_dequantize_pages_q4(ctypes.byref(dd), kq, OK_PTR, src, OK_PTR, OK_PTR, OK_PTR, n, qpool, pool, None)

    assert dequant(src=None) == -1 and dequant(pool=0) == -1 and dequant(kq=ODD_PTR) == -3 and dequant(n=0) == 0
    assert dequant(dd=desc(dtype=ea.EA_F32, P=64)) == -2

    def dec(dd=d, q=OK_PTR, kq=OK_PTR, tail_pt=OK_PTR, tail_len=OK_PTR, k=OK_PTR, max_tail=2, pool=8, n_splits=2,
            ws=OK_PTR, ws_bytes=1 << 30, max_q=4):
        return lib.ea_decode_attn_q4(ctypes.byref(dd), q, kq, OK_PTR, OK_PTR, OK_PTR, max_q, 8, k, OK_PTR, tail_pt,
                                     tail_len, max_tail, pool, OK_PTR, 2, n_splits, ws, ws_bytes, None)

    assert dec(q=None) == -1 and dec(max_q=0) == -1 and dec(n_splits=1025) == -1
    assert dec(tail_len=None) == -1                                        # half a tail
    assert dec(k=None) == -1 and dec(max_tail=0) == -1
    assert dec(kq=ODD_PTR) == -3 and dec(k=ODD_PTR) == -3
    assert dec(ws=None) == -4                                              # the workspace is always needed
    need = ea.decode_q4_workspace_bytes(d, 2, 2)
    assert need == 2 * 8 * 3 * (2 + 48) * 4                                # n_splits + 1 slots
    assert dec(ws_bytes=need - 1) == -4
    assert dec(dd=desc(dtype=ea.EA_F32, P=64)) == -2
    assert ea.decode_q4_workspace_bytes(d, 0, 2) == -1
    assert lib.ea_decode_attn_alibi_q4(ctypes.byref(d), OK_PTR, None, OK_PTR, OK_PTR, OK_PTR, OK_PTR, 4, 8, OK_PTR, OK_PTR,
                                       OK_PTR, OK_PTR, 2, 8, OK_PTR, 2, 2, OK_PTR, 1 << 30, None) == -1      # no slopes


def test_rotary_q4_entry_point_rejects_bad_arguments_before_launching():
    lib, d = raw(), desc()

    def dec(dd=d, q=OK_PTR, u=OK_PTR, base=10000.0, tail_pt=OK_PTR, tail_len=OK_PTR, n_splits=2, ws=OK_PTR,
            ws_bytes=1 << 30):
        return lib.ea_decode_attn_rope_q4(ctypes.byref(dd), q, u, base, OK_PTR, OK_PTR, OK_PTR, OK_PTR, 4, 8, OK_PTR,
                                          OK_PTR, tail_pt, tail_len, 2, 8, OK_PTR, 2, n_splits, ws, ws_bytes, None)

    assert dec(u=None) == -1 and dec(base=1.0) == -1 and dec(tail_pt=None) == -1
    assert dec(u=ODD_PTR) == -3
    assert dec(ws=None) == -4 and dec(ws_bytes=16) == -4
    assert dec(dd=desc(d_h=96)) == -2                                      # d_head 64 or 128
    assert dec(dd=desc(d_h=64, r_k=80)) == -2                              # r_k <= d_head
    assert dec(dd=desc(dtype=ea.EA_F32, P=64)) == -2


def test_attn_mass_rejects_bad_arguments_before_launching():
    lib, d = raw(), desc()

    def mass(dd=d, q=OK_PTR, k=OK_PTR, pt=OK_PTR, out=OK_PTR, B=2, max_pages=4, pool=8, ws=OK_PTR, ws_bytes=1 << 30):
        return lib.ea_attn_mass(ctypes.byref(dd), q, k, pt, OK_PTR, out, B, max_pages, pool, ws, ws_bytes, None)

    assert mass(q=None) == -1 and mass(pt=None) == -1 and mass(out=None) == -1
    assert mass(B=0) == -1 and mass(max_pages=0) == -1 and mass(pool=0) == -1
    assert mass(k=ODD_PTR) == -3 and mass(out=ODD_PTR) == -3
    assert mass(ws=None) == -4 and mass(ws=ODD_PTR) == -4
    need = ea.attn_mass_workspace_bytes(d, 2, 4)
    tiles = 4 * 128 // 64
    assert need == 2 * 8 * (tiles * 64 + 1088 + tiles * 2) * 4             # e rows (whole tiles + pad) + (m, l) per tile
    assert mass(ws_bytes=need - 1) == -4
    assert mass(dd=desc(H=34, Hkv=2, d=34 * 128)) == -2                    # at most 16 query heads per kv head
    assert ea.attn_mass_workspace_bytes(d, 0, 4) == -1
    # fp32 pages of 48 tokens: the rows of e are rounded up to whole tiles
    assert ea.attn_mass_workspace_bytes(desc(dtype=ea.EA_F32, P=48), 1, 3) == 8 * (3 * 64 + 1088 + 3 * 2) * 4


def test_decode_attn_mass_rejects_bad_arguments_before_launching():
    lib, d = raw(), desc()

    def call(dd=d, q=OK_PTR, k=OK_PTR, out=OK_PTR, mass=OK_PTR, B=2, max_pages=4, pool=8, S=2, ws=OK_PTR, ws_bytes=1 << 30):
        return lib.ea_decode_attn_mass(ctypes.byref(dd), q, k, OK_PTR, OK_PTR, OK_PTR, out, mass, B, max_pages, pool, S,
                                       ws, ws_bytes, None)

    assert call(q=None) == -1 and call(mass=None) == -1 and call(B=0) == -1 and call(S=-1) == -1 and call(S=1025) == -1
    assert call(k=ODD_PTR) == -3 and call(mass=ODD_PTR) == -3
    assert call(ws=None) == -4                                             # needed for any split count
    need = ea.decode_attn_mass_workspace_bytes(d, 2, 4, 2)
    partials = 2 * 8 * 2 * (2 + 48)                                        # B H S (m, l, r_v_pad)
    assert need == (partials + 2 * 8 * (4 * 128 + 1088 + 2)) * 4           # + scores rows (padded) + (M, L) per row
    assert call(ws_bytes=need - 1) == -4
    assert call(dd=desc(dtype=ea.EA_F32, P=64)) == -2                      # bf16 layers only
    assert call(dd=desc(H=34, Hkv=2, d=34 * 128)) == -2
    assert ea.decode_attn_mass_workspace_bytes(d, 2, 4, 0) == -1           # the size depends on the split count


def test_rotary_entry_points_with_explicit_positions_reject_bad_arguments_before_launching():
    lib, d = raw(), desc()

    def call(dd=d, q=OK_PTR, u=OK_PTR, base=10000.0, pos=OK_PTR, stride=4 * 128, qpos=OK_PTR, out=OK_PTR, mass=False,
             B=2, max_pages=4, pool=8, S=1, ws=OK_PTR, ws_bytes=1 << 30):
        if mass is False:
            return lib.ea_decode_attn_rope_pos(ctypes.byref(dd), q, u, base, OK_PTR, OK_PTR, OK_PTR, OK_PTR, pos, stride,
                                               qpos, out, B, max_pages, pool, S, ws, ws_bytes, None)
        return lib.ea_decode_attn_mass_rope_pos(ctypes.byref(dd), q, u, base, OK_PTR, OK_PTR, OK_PTR, OK_PTR, pos, stride,
                                                qpos, out, mass, B, max_pages, pool, S, ws, ws_bytes, None)

    for m in (False, OK_PTR):
        assert call(q=None, mass=m) == -1 and call(pos=None, mass=m) == -1 and call(qpos=None, mass=m) == -1
        assert call(base=1.0, mass=m) == -1 and call(B=0, mass=m) == -1 and call(S=1025, mass=m) == -1
        assert call(stride=4 * 128 - 1, mass=m) == -1                       # shorter than the page table's capacity
        assert call(q=ODD_PTR, mass=m) == -3 and call(pos=0x10002, mass=m) == -3 and call(qpos=0x10002, mass=m) == -3   # int32 arrays: 4-byte aligned
        assert call(dd=desc(d_h=96, r_k=80), mass=m) == -2
    assert call(S=2, ws=None) == -4 and call(S=2, ws_bytes=ea.decode_workspace_bytes(d, 2, 2) - 1) == -4
    assert call(mass=None) == -1 and call(mass=ODD_PTR) == -3
    assert call(mass=OK_PTR, ws=None) == -4
    assert call(mass=OK_PTR, S=2, ws_bytes=ea.decode_attn_mass_workspace_bytes(d, 2, 4, 2) - 1) == -4
    assert call(mass=OK_PTR, dd=desc(dtype=ea.EA_F32, P=64)) == -2         # the statistic: bf16 layers only


@pytest.mark.parametrize("P,r_k,r_v,Hkv", [(128, 80, 80, 2), (256, 30, 33, 1), (384, 128, 16, 2)])
def test_q4_key_groups_of_128_tokens_share_one_block_of_scales(P, r_k, r_v, Hkv):
    """q4_key_group = 128: every code still has its own nibble, the two tiles of a pair point at the same scales
    (stored once, behind the codes of the pair's first tile), nothing overlaps, the page is shorter by one block of
    scales per pair, and the value side is untouched."""
    d = desc(Hkv=Hkv, H=Hkv, r_k=r_k, r_v=r_v, P=P)
    d64 = desc(Hkv=Hkv, H=Hkv, r_k=r_k, r_v=r_v, P=P)
    d.q4_key_group = 128
    d64.q4_key_group = 64
    lay, lay64, lay0 = ea.q4_layout_query(d), ea.q4_layout_query(d64), ea.q4_layout_query(desc(Hkv=Hkv, H=Hkv, r_k=r_k, r_v=r_v, P=P))
    assert (lay64.k_page_bytes, lay64.k_tile_bytes) == (lay0.k_page_bytes, lay0.k_tile_bytes)      # 0 means 64
    scales = 128 * (-(-lay.r_k_pad // 32))
    assert lay.k_tile_bytes == lay64.k_tile_bytes == 32 * lay.r_k_pad + scales
    assert lay.k_page_bytes == lay64.k_page_bytes - Hkv * (P // 128) * scales
    assert lay.v_page_bytes == lay64.v_page_bytes and lay.v_tile_bytes == lay64.v_tile_bytes
    page = 1
    used = np.zeros(lay.k_page_bytes * 2, np.int32)
    for h in range(Hkv):
        for t in range(P):
            for c in range(r_k):
                pos = ea.q4_k_code_pos(d, page, h, t, c)
                assert pos % 4 == 0
                used[pos // 4 - page * lay.k_page_bytes * 2] += 1
            assert ea.q4_v_code_pos(d, page, h, t, 0) == ea.q4_v_code_pos(d64, page, h, t, 0)
        for grp in range(P // 128):
            for c in range(r_k):
                sp = ea.q4_k_scale_pos(d, page, h, grp * 128, c) - page * lay.k_page_bytes
                assert all(ea.q4_k_scale_pos(d, page, h, grp * 128 + t, c) - page * lay.k_page_bytes == sp
                           for t in (1, 63, 64, 100, 127))
                for off in (sp, sp + 16):
                    used[2 * off:2 * off + 4] += 1
    assert used.max() == 1
    assert used.sum() == Hkv * P * r_k + Hkv * (P // 128) * r_k * 8
    # the first tile of a pair sits where a 64-token layout would put it if every earlier pair were one block of scales shorter
    codes = 32 * lay.r_k_pad
    assert ea.q4_k_code_pos(d, 0, 0, 64, 0) == (codes + scales) * 8
    assert ea.q4_k_scale_pos(d, 0, 0, 64, 0) == codes
    if P >= 256:
        assert ea.q4_k_code_pos(d, 0, 0, 128, 0) == (2 * codes + scales) * 8
        assert ea.q4_k_scale_pos(d, 0, 0, 200, 0) == 3 * codes + scales
    # groups of 128 tokens need pages of whole groups; other group lengths are not built
    bad = desc(P=192)
    bad.q4_key_group = 128
    assert ea.load_library().ea_q4_layout_query(ctypes.byref(bad), ctypes.byref(ea.Q4Layout())) == -2
    bad = desc()
    bad.q4_key_group = 32
    assert ea.load_library().ea_q4_layout_query(ctypes.byref(bad), ctypes.byref(ea.Q4Layout())) == -1


def test_prefill_over_the_q4_cache_rejects_bad_arguments_before_launching():
    lib, d = raw(), desc()

    def call(dd=d, q=OK_PTR, kq=OK_PTR, k=OK_PTR, tail=OK_PTR, out=OK_PTR, B=2, n=100, mq=4, qpool=8, mt=2, pool=8,
             ws=OK_PTR, ws_bytes=1 << 40):
        return lib.ea_prefill_attn_q4(ctypes.byref(dd), q, kq, OK_PTR, OK_PTR, OK_PTR, mq, qpool, k, OK_PTR, tail, OK_PTR,
                                      mt, pool, out, B, n, ws, ws_bytes, None)

    assert call(q=None) == -1 and call(tail=None) == -1 and call(k=None) == -1 and call(n=0) == -1 and call(mt=0) == -1
    assert call(kq=ODD_PTR) == -3 and call(out=ODD_PTR) == -3
    need = ea.prefill_q4_workspace_bytes(d, 2, 100)
    assert need == 2 * 2 * 100 * 8 * (48 + 2) * 4                          # two parts: output row, exponent, row sum
    assert call(ws=None) == -4 and call(ws_bytes=need - 1) == -4
    assert call(dd=desc(dtype=ea.EA_F32, P=64)) == -2                      # bf16 layers only
    assert ea.prefill_q4_workspace_bytes(d, 0, 100) == -1


def test_rotary_prefill_over_the_q4_cache_rejects_bad_arguments_before_launching():
    lib, d = raw(), desc()

    def call(dd=d, q=OK_PTR, u=OK_PTR, base=10000.0, kq=OK_PTR, k=OK_PTR, tail=OK_PTR, out=OK_PTR, B=2, n=100, mq=4,
             qpool=8, mt=2, pool=8, ws=OK_PTR, ws_bytes=1 << 40):
        return lib.ea_prefill_attn_rope_q4(ctypes.byref(dd), q, u, base, kq, OK_PTR, OK_PTR, OK_PTR, mq, qpool, k, OK_PTR,
                                           tail, OK_PTR, mt, pool, out, B, n, ws, ws_bytes, None)

    assert call(q=None) == -1 and call(u=None) == -1 and call(tail=None) == -1 and call(k=None) == -1
    assert call(n=0) == -1 and call(mt=0) == -1 and call(mq=0) == -1 and call(base=1.0) == -1
    assert call(kq=ODD_PTR) == -3 and call(out=ODD_PTR) == -3 and call(u=ODD_PTR) == -3
    need = ea.prefill_rope_q4_workspace_bytes(d, 2, 100, 4, 2)
    lay = ea.cache_layout_query(d)
    align = lambda x: -(-x // 256) * 256
    pages = 2 * (4 + 2)
    # the page lists and the staged table, two stage pools of bfloat16 pages, the rotary prefill's own workspace
    assert need == (align(4 * 2 * (3 * 6 + 1)) + align(pages * lay.k_page_elems * 2) + align(pages * lay.v_page_elems * 2)
                    + ea.prefill_rope_workspace_bytes(d, 2, 100, 6))
    assert call(ws=None) == -4 and call(ws_bytes=need - 1) == -4 and call(ws=OK_PTR + 16) == -4
    assert call(dd=desc(dtype=ea.EA_F32, P=64)) == -2                      # bf16 layers only
    assert call(dd=desc(d_h=96)) == -2                                     # d_head 64 or 128
    assert call(dd=desc(d_h=64, r_k=80)) == -2                             # r_k <= d_head
    assert ea.prefill_rope_q4_workspace_bytes(d, 0, 100, 4, 2) == -1
    # the position-free staged call: the same stage, no rotary workspace, the argument list of ea_prefill_attn_q4
    staged = ea.prefill_q4_staged_workspace_bytes(d, 2, 100, 4, 2)
    assert staged == need - ea.prefill_rope_workspace_bytes(d, 2, 100, 6)

    def call_staged(q=OK_PTR, tail=OK_PTR, n=100, mq=4, ws=OK_PTR, ws_bytes=1 << 40, dd=d):
        return lib.ea_prefill_attn_q4_staged(ctypes.byref(dd), q, OK_PTR, OK_PTR, OK_PTR, OK_PTR, mq, 8, OK_PTR, OK_PTR,
                                             tail, OK_PTR, 2, 8, OK_PTR, 2, n, ws, ws_bytes, None)

    assert call_staged(q=None) == -1 and call_staged(tail=None) == -1 and call_staged(n=0) == -1 and call_staged(mq=0) == -1
    assert call_staged(q=ODD_PTR) == -3
    assert call_staged(ws=None) == -4 and call_staged(ws_bytes=staged - 1) == -4 and call_staged(ws=OK_PTR + 16) == -4
    assert call_staged(dd=desc(dtype=ea.EA_F32, P=64)) == -2
    assert ea.prefill_q4_staged_workspace_bytes(d, 2, 0, 4, 2) == -1

    def call_alibi(q=OK_PTR, slopes=OK_PTR, ws=OK_PTR, ws_bytes=1 << 40):
        return lib.ea_prefill_attn_alibi_q4(ctypes.byref(d), q, slopes, OK_PTR, OK_PTR, OK_PTR, OK_PTR, 4, 8, OK_PTR,
                                            OK_PTR, OK_PTR, OK_PTR, 2, 8, OK_PTR, 2, 100, ws, ws_bytes, None)

    assert call_alibi(slopes=None) == -1 and call_alibi(q=None) == -1 and call_alibi(q=ODD_PTR) == -3
    assert call_alibi(ws_bytes=staged - 1) == -4 and call_alibi(ws=None) == -4
    assert ea.prefill_rope_q4_workspace_bytes(d, 1 << 20, 100, 1 << 10, 1 << 10) == -1      # 2^31 stage pages


@pytest.mark.parametrize("P,r_k,r_v,Hkv,group", [(64, 80, 80, 2, 64), (128, 30, 33, 1, 128), (192, 128, 16, 2, 64), (64, 8, 112, 1, 64)])
def test_q3_positions_tile_the_page_exactly(P, r_k, r_v, Hkv, group):
    """3-bit codes: every code has its own two low bits and its own high bit, every scale its own two bytes, nothing
    overlaps, everything lies inside the page, and the sizes are the documented ones."""
    d = desc(Hkv=Hkv, H=Hkv, r_k=r_k, r_v=r_v, P=P)
    d.q4_key_group, d.q4_bits = group, 3
    lay = ea.q4_layout_query(d)
    ncb = lay.r_v_pad // 16
    scales = 128 * (-(-lay.r_k_pad // 32))
    assert lay.k_tile_bytes == 24 * lay.r_k_pad + scales
    assert lay.v_tile_bytes == (ncb // 2) * 768 + (ncb % 2) * 512 + 256
    tpg = group // 64
    assert lay.k_page_bytes == Hkv * ((P // 64) * 24 * lay.r_k_pad + (P // 64 // tpg) * scales)
    assert lay.v_page_bytes == Hkv * (P // 64) * lay.v_tile_bytes
    assert ea.q4_k_code_pos(d, 0, 0, 0, 0) == -1 and ea.q4_v_code_pos(d, 0, 0, 0, 0) == -1     # the 4-bit functions decline
    d4 = desc(Hkv=Hkv, H=Hkv, r_k=r_k, r_v=r_v, P=P)
    assert ea.q3_k_code_pos(d4, 0, 0, 0, 0) is None
    page = 1
    used_k = np.zeros(lay.k_page_bytes * 8, np.int32)          # per bit
    used_v = np.zeros(lay.v_page_bytes * 8, np.int32)
    for h in range(Hkv):
        for t in range(P):
            for c in range(r_k):
                for pos in ea.q3_k_code_pos(d, page, h, t, c):
                    used_k[pos - page * lay.k_page_bytes * 8] += 1
            for c in range(r_v):
                for pos in ea.q3_v_code_pos(d, page, h, t, c):
                    used_v[pos - page * lay.v_page_bytes * 8] += 1
            sp = ea.q4_v_scale_pos(d, page, h, t) - page * lay.v_page_bytes
            for off in (sp, sp + 128):
                used_v[8 * off:8 * off + 16] += 1
        for grp in range(P // group):
            for c in range(r_k):
                sp = ea.q4_k_scale_pos(d, page, h, grp * group, c) - page * lay.k_page_bytes
                assert sp == ea.q4_k_scale_pos(d, page, h, grp * group + group - 1, c) - page * lay.k_page_bytes
                for off in (sp, sp + 16):
                    used_k[8 * off:8 * off + 16] += 1
    assert used_k.max() == 1 and used_v.max() == 1
    assert used_k.sum() == Hkv * P * r_k * 3 + Hkv * (P // group) * r_k * 32
    assert used_v.sum() == Hkv * P * r_v * 3 + Hkv * P * 32
    # the order inside a unit: token 16*tb + t, channel 32*kk + 8*quad + e -> unit (quad*16 + t) of run kk, group tb;
    # groups 0-2: dword tb, bits 3i + b of half word h (e = 2i + h); group 3: bit 3i + b of its half word lives in
    # nibble (3i + b) / 4, i.e. in bits 12-15 of half word h of that dword
    for (t, c) in [(0, 0), (17, min(9, r_k - 1)), (63, r_k - 1), (35, min(44, r_k - 1)), (50, min(13, r_k - 1))]:
        tb, tt, kk, quad, e = t // 16, t % 16, c // 32, (c // 8) % 4, c % 8
        unit = kk * 768 + (quad * 16 + tt) * 12
        i, hh = e // 2, e % 2
        want = []
        for b in range(3):
            sbit = 3 * i + b
            want.append((unit + 4 * tb) * 8 + 16 * hh + sbit if tb < 3 else
                        (unit + 4 * (sbit // 4)) * 8 + 16 * hh + 12 + sbit % 4)
        assert ea.q3_k_code_pos(d, 0, 0, t, c) == tuple(want)
    bad = desc()
    bad.q4_bits = 2
    assert ea.load_library().ea_q4_layout_query(ctypes.byref(bad), ctypes.byref(ea.Q4Layout())) == -1


def test_a_code_width_other_than_3_or_4_is_declined_by_every_call_that_reads_codes():
    lib, d = raw(), desc()
    d.q4_bits = 5
    rc = lib.ea_decode_attn_rope_q4(ctypes.byref(d), OK_PTR, OK_PTR, 10000.0, OK_PTR, OK_PTR, OK_PTR, OK_PTR, 4, 8, None,
                                    None, None, None, 0, 0, OK_PTR, 2, 1, OK_PTR, 1 << 30, None)
    assert rc == -1
    rc = lib.ea_prefill_attn_q4(ctypes.byref(d), OK_PTR, OK_PTR, OK_PTR, OK_PTR, OK_PTR, 4, 8, OK_PTR, OK_PTR, OK_PTR, OK_PTR,
                                2, 8, OK_PTR, 2, 100, OK_PTR, 1 << 40, None)
    assert rc == -1



def test_layer_step_entry_points_reject_bad_arguments_before_launching():
    lib = raw()
    d = desc(H=8, Hkv=2, r_k=80, r_v=48, P=64, d=512)

    def call(fn, dd=d, x=OK_PTR, wo=OK_PTR, y=OK_PTR, B=4, n_splits=2, ws=OK_PTR, ws_bytes=1 << 30, status=None):
        return fn(ctypes.byref(dd), x, OK_PTR, wo, OK_PTR, OK_PTR, OK_PTR, OK_PTR, y, B, 4, 16, n_splits, ws, ws_bytes,
                  status, None)

    for fn, need in ((lib.ea_decode_layer, ea.decode_layer_workspace_bytes(d, 4, 2)),
                     (lib.ea_decode_layer_fused, ea.decode_layer_fused_workspace_bytes(d, 4, 2))):
        assert call(fn, x=None) == -1 and call(fn, y=None) == -1 and call(fn, B=0) == -1 and call(fn, n_splits=1025) == -1
        assert call(fn, wo=ODD_PTR) == -3
        assert call(fn, ws=None) == -4 and call(fn, ws_bytes=need - 1) == -4
        assert call(fn, ws=OK_PTR + 16) == -4                              # the workspace must be 256-byte aligned
        assert call(fn, dd=desc(dtype=ea.EA_F32, P=64)) == -2              # bf16 layers only
        assert call(fn, dd=desc(H=8, Hkv=2, r_k=80, r_v=47, P=64, d=512)) == -2   # H * r_v must be a multiple of 32
    # the two-launch form: at most 16 sequences and 64 splits, and it brings its counters in the workspace
    assert call(lib.ea_decode_layer_fused, B=17, n_splits=1) == -2
    assert call(lib.ea_decode_layer_fused, n_splits=65) == -2
    assert ea.decode_layer_fused_workspace_bytes(d, 4, 2) == ea.decode_layer_workspace_bytes(d, 4, 2) + 256
    assert ea.decode_layer_fused_workspace_bytes(d, 17, 1) == -1
    assert call(lib.ea_decode_layer_fused, status=OK_PTR + 2) == -3
    assert lib.ea_set_wait_limit(0) == -1 and lib.ea_set_wait_limit(1 << 20) == 0
    # the ALiBi forms: the same checks behind one more pointer, which must be there

    def call_alibi(fn, slopes=OK_PTR, x=OK_PTR, B=4, n_splits=2, ws=OK_PTR, ws_bytes=1 << 30):
        return fn(ctypes.byref(d), x, OK_PTR, OK_PTR, slopes, OK_PTR, OK_PTR, OK_PTR, OK_PTR, OK_PTR, B, 4, 16, n_splits,
                  ws, ws_bytes, None, None)

    for fn, need in ((lib.ea_decode_layer_alibi, ea.decode_layer_workspace_bytes(d, 4, 2)),
                     (lib.ea_decode_layer_fused_alibi, ea.decode_layer_fused_workspace_bytes(d, 4, 2))):
        assert call_alibi(fn, slopes=None) == -1 and call_alibi(fn, x=None) == -1 and call_alibi(fn, B=0) == -1
        assert call_alibi(fn, ws=None) == -4 and call_alibi(fn, ws_bytes=need - 1) == -4
    assert call_alibi(lib.ea_decode_layer_fused_alibi, B=17, n_splits=1) == -2
    assert call_alibi(lib.ea_decode_layer_fused_alibi, n_splits=65) == -2
    header = open(os.path.join(ROOT, "include", "eigenattn.h")).read()
    assert re.search(r"#define\s+EA_STATUS_WAIT_EXPIRED\s+\(1 << 30\)", header) and ea.STATUS_WAIT_EXPIRED == 1 << 30


def _dispatch_model_finishes(n_wgs, n_work, slots_per_die, dies=8):
    """The second launch of the two-launch layer step as the chip runs it: workgroup i belongs to die i % dies, a die
    starts its workgroups in order as slots come free, the last n_work workgroups of the grid wait (holding their
    slot) until every workgroup has arrived, all others arrive and leave.  True if every workgroup gets to leave."""
    queue = [[i for i in range(n_wgs) if i % dies == x] for x in range(dies)]
    nxt = [0] * dies                       # next workgroup of each die's share to start
    held = [0] * dies                      # slots held by waiting workgroups
    arrived = 0
    while True:
        progress = False
        for x in range(dies):
            while nxt[x] < len(queue[x]) and held[x] < slots_per_die:
                wg = queue[x][nxt[x]]
                nxt[x] += 1
                arrived += 1
                progress = True
                if wg >= n_wgs - n_work:
                    held[x] += 1           # waits for the whole grid in its slot
        if arrived == n_wgs:
            return True                    # the waiting ones see the count and leave
        if not progress:
            return False                   # every free slot is held by a workgroup that waits for one not started


def test_workgroups_that_wait_never_block_the_ones_they_wait_for():
    # the rule the library applies (ea_decode_layer_fused_workers) keeps the waiting workgroups within half of the
    # resident slots: 2 per compute unit, 256 compute units in 8 dies on MI355X (also what the library assumes when it
    # cannot ask a device)
    slots_per_die = 2 * 256 // 8
    for d_model in (256, 4096, 8192, 16384):
        for Hkv in (2, 8, 32):
            for B in (1, 8, 16):
                for S in (1, 4, 8, 64):
                    dd = ea.LayerDesc(d_model, 32, Hkv, 128, 80, 80, ea.EA_BF16, 64)
                    n_work = ea.decode_layer_fused_workers(dd, B, S)
                    n_wgs = Hkv * S * B
                    assert 1 <= n_work <= min(d_model // 16, n_wgs, 256)
                    assert _dispatch_model_finishes(n_wgs, n_work, slots_per_die)
    # and the model does tell the difference: more waiting workgroups than a die has slots never finish ...
    assert not _dispatch_model_finishes(n_wgs=4096, n_work=1024, slots_per_die=slots_per_die)
    # ... while half the slots are safe however long the grid
    assert _dispatch_model_finishes(n_wgs=1 << 16, n_work=256, slots_per_die=slots_per_die)
    assert ea.decode_layer_fused_workers(desc(H=8, Hkv=3), 4, 1) == -1
