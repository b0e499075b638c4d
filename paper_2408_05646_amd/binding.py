"""ctypes binding of libeigenattn.so: same names as the C ABI, argument marshalling only.

Tensors are torch tensors living on the GPU (PyTorch is used for device memory
and streams, nothing else); every step of the path runs in the library's HIP
kernels.  There is no CPU fallback: if the library is missing, calls raise.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np

__all__ = [
    "EA_F32", "EA_BF16", "EigenAttnError", "LayerDesc", "CacheLayout", "library_path", "load_library",
    "cache_layout_query", "cache_k_index", "cache_v_index", "cache_slot", "cache_scatter", "cache_gather",
    "packed_weight_elems", "pack_weight", "project_qkv", "decode_auto_splits", "decode_workspace_bytes", "decode_attn", "prefill_attn", "out_proj",
    "strerror", "version", "alloc_pools", "EXPORTED_SYMBOLS", "decode_attn_rope", "project_qkv_rope", "prefill_attn_rope", "prefill_rope_workspace_bytes", "decode_attn_alibi", "prefill_attn_alibi", "decode_rope_auto_splits",
    "Q4Layout", "q4_layout_query", "q4_k_code_pos", "q4_v_code_pos", "q4_k_scale_pos", "q4_v_scale_pos", "alloc_q4_pools",
    "quantize_pages_q4", "dequantize_pages_q4", "decode_q4_workspace_bytes", "decode_attn_q4", "decode_attn_rope_q4", "decode_attn_alibi_q4",
    "attn_mass", "attn_mass_workspace_bytes", "decode_attn_mass", "decode_attn_mass_workspace_bytes",
    "decode_attn_static", "STATIC_SCRATCH_BYTES", "decode_layer_workspace_bytes", "decode_layer", "decode_layer_rope",
    "decode_layer_fused_workspace_bytes", "decode_layer_fused", "decode_layer_fused_rope", "set_wait_limit", "STATUS_WAIT_EXPIRED",
    "decode_layer_fused_workers", "decode_layer_alibi", "decode_layer_fused_alibi",
    "decode_attn_rope_pos", "decode_attn_mass_rope_pos", "prefill_attn_q4", "prefill_q4_workspace_bytes",
    "prefill_attn_rope_q4", "prefill_rope_q4_workspace_bytes", "prefill_q4_staged_workspace_bytes",
    "q3_k_code_pos", "q3_v_code_pos",
]

EA_F32, EA_BF16 = 0, 1

EXPORTED_SYMBOLS = (
    "ea_cache_layout_query", "ea_cache_k_index", "ea_cache_v_index", "ea_cache_slot", "ea_strerror", "ea_version",
    "ea_cache_scatter", "ea_cache_gather", "ea_packed_weight_elems", "ea_pack_weight", "ea_project_qkv", "ea_project_qkv_rope", "ea_decode_auto_splits", "ea_decode_workspace_bytes",
    "ea_decode_attn", "ea_decode_rope_auto_splits", "ea_decode_attn_rope", "ea_prefill_attn", "ea_prefill_rope_workspace_bytes", "ea_prefill_attn_rope",
    "ea_decode_attn_alibi", "ea_prefill_attn_alibi", "ea_out_proj",
    "ea_q4_layout_query", "ea_q4_k_code_pos", "ea_q4_v_code_pos", "ea_q4_k_scale_pos", "ea_q4_v_scale_pos",
    "ea_quantize_pages_q4", "ea_dequantize_pages_q4", "ea_decode_q4_workspace_bytes", "ea_decode_attn_q4", "ea_decode_attn_rope_q4", "ea_decode_attn_alibi_q4",
    "ea_attn_mass_workspace_bytes", "ea_attn_mass", "ea_decode_attn_mass_workspace_bytes", "ea_decode_attn_mass",
    "ea_decode_attn_static", "ea_decode_layer_workspace_bytes", "ea_decode_layer", "ea_decode_layer_rope",
    "ea_decode_layer_fused_workspace_bytes", "ea_decode_layer_fused", "ea_decode_layer_fused_rope", "ea_set_wait_limit",
    "ea_decode_layer_fused_workers", "ea_decode_layer_alibi", "ea_decode_layer_fused_alibi",
    "ea_decode_attn_rope_pos", "ea_decode_attn_mass_rope_pos", "ea_prefill_q4_workspace_bytes", "ea_prefill_attn_q4",
    "ea_prefill_rope_q4_workspace_bytes", "ea_prefill_attn_rope_q4",
    "ea_prefill_q4_staged_workspace_bytes", "ea_prefill_attn_q4_staged", "ea_prefill_attn_alibi_q4",
    "ea_q3_k_code_pos", "ea_q3_v_code_pos",
)

STATIC_SCRATCH_BYTES = 8 * 1024 * 1024      # EA_STATIC_SCRATCH_BYTES of the header
STATUS_WAIT_EXPIRED = 1 << 30               # EA_STATUS_WAIT_EXPIRED of the header


class EigenAttnError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {strerror(code)} ({code})")


class LayerDesc(ctypes.Structure):
    # q4_key_group (optional): tokens that share a key scale in the 4-bit cache, 64 (also meant by 0) or 128;
    # q4_bits (optional): width of a code of that cache, 4 (also meant by 0) or 3
    _fields_ = [(n, ctypes.c_int32) for n in
                ("d_model", "n_heads", "n_kv_heads", "d_head", "r_k", "r_v", "dtype", "page_tokens", "q4_key_group",
                 "q4_bits")]

    def __repr__(self):
        return "LayerDesc(" + ", ".join(f"{n}={getattr(self, n)}" for n, _ in self._fields_) + ")"


class CacheLayout(ctypes.Structure):
    _fields_ = [("layout_id", ctypes.c_int32), ("elem_bytes", ctypes.c_int32), ("r_k_pad", ctypes.c_int32),
                ("r_v_pad", ctypes.c_int32), ("k_slab_elems", ctypes.c_int64), ("v_slab_elems", ctypes.c_int64),
                ("k_page_elems", ctypes.c_int64), ("v_page_elems", ctypes.c_int64)]


class Q4Layout(ctypes.Structure):
    _fields_ = [("r_k_pad", ctypes.c_int32), ("r_v_pad", ctypes.c_int32), ("k_tile_bytes", ctypes.c_int64),
                ("v_tile_bytes", ctypes.c_int64), ("k_page_bytes", ctypes.c_int64), ("v_page_bytes", ctypes.c_int64)]


_LIB = None


def library_path() -> str:
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), "libeigenattn.so")


def load_library():
    """Loads libeigenattn.so (built by paper_2408_05646_amd/build.py).  Raises if it is not there."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = library_path()
    if not os.path.exists(path):
        raise RuntimeError(f"{path} not found: build it with `python -m paper_2408_05646_amd.build` "
                           "(there is no fallback path)")
    # PyTorch ships its own copy of the HIP runtime.  It must be in the process first, so that this
    # library binds to the SAME runtime that owns the tensors and streams handed to it.
    import torch  # noqa: F401
    lib = ctypes.CDLL(path)
    P, I32, I64, VP = ctypes.POINTER, ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p
    D = P(LayerDesc)
    lib.ea_version.restype = ctypes.c_int
    lib.ea_strerror.restype = ctypes.c_char_p
    lib.ea_strerror.argtypes = [ctypes.c_int]
    lib.ea_cache_layout_query.argtypes = [D, P(CacheLayout)]
    for f in (lib.ea_cache_k_index, lib.ea_cache_v_index):
        f.restype = I64
        f.argtypes = [D, I32, I32, I32, I32]
    lib.ea_cache_slot.restype = I64
    lib.ea_cache_slot.argtypes = [D, P(I32), I32, I32]
    lib.ea_cache_scatter.argtypes = [D, VP, VP, VP, VP, VP, I32, I32, I32, I32, I32, VP]
    lib.ea_cache_gather.argtypes = [D, VP, VP, VP, VP, VP, I32, I32, I32, I32, I32, VP]
    lib.ea_packed_weight_elems.restype = I64
    lib.ea_packed_weight_elems.argtypes = [I32, I32, I32]
    lib.ea_pack_weight.argtypes = [VP, VP, I32, I32, I32, VP]
    lib.ea_project_qkv.argtypes = [D, VP, VP, VP, I32, VP, VP, VP, VP, I32, I32, I32, I32, VP, VP]
    lib.ea_project_qkv_rope.argtypes = [D, VP, VP, VP, I32, VP, VP, VP, VP, I32, I32, I32, I32, VP, VP]
    lib.ea_decode_auto_splits.restype = I32
    lib.ea_decode_auto_splits.argtypes = [D, I32, I32]
    lib.ea_decode_workspace_bytes.restype = I64
    lib.ea_decode_rope_auto_splits.argtypes = [D, I32, I32]
    lib.ea_decode_rope_auto_splits.restype = I32
    lib.ea_decode_workspace_bytes.argtypes = [D, I32, I32]
    lib.ea_decode_attn.argtypes = [D, VP, VP, VP, VP, VP, VP, I32, I32, I32, I32, VP, I64, VP]
    lib.ea_decode_layer_workspace_bytes.restype = I64
    lib.ea_decode_layer_workspace_bytes.argtypes = [D, I32, I32, I32]
    lib.ea_decode_layer.argtypes = [D, VP, VP, VP, VP, VP, VP, VP, VP, I32, I32, I32, I32, VP, I64, VP, VP]
    lib.ea_decode_layer_fused.argtypes = lib.ea_decode_layer.argtypes
    lib.ea_decode_layer_alibi.argtypes = [D, VP, VP, VP, VP, VP, VP, VP, VP, VP, I32, I32, I32, I32, VP, I64, VP, VP]
    lib.ea_decode_layer_fused_alibi.argtypes = lib.ea_decode_layer_alibi.argtypes
    lib.ea_decode_layer_fused_workspace_bytes.restype = I64
    lib.ea_decode_layer_fused_workspace_bytes.argtypes = [D, I32, I32, I32]
    lib.ea_set_wait_limit.argtypes = [ctypes.c_uint32]
    lib.ea_decode_layer_fused_workers.restype = I32
    lib.ea_decode_layer_fused_workers.argtypes = [D, I32, I32]
    lib.ea_decode_layer_rope.argtypes = [D, VP, VP, VP, VP, ctypes.c_double, VP, VP, VP, VP, VP, I32, I32, I32, I32, VP,
                                         I64, VP, VP]
    lib.ea_decode_layer_fused_rope.argtypes = lib.ea_decode_layer_rope.argtypes
    lib.ea_decode_attn_static.argtypes = [D, VP, VP, VP, VP, VP, VP, I32, I32, I32, I32, VP]
    lib.ea_decode_attn_rope.argtypes = [D, VP, VP, ctypes.c_double, VP, VP, VP, VP, VP, I32, I32, I32, I32, VP, I64, VP]
    lib.ea_decode_attn_rope_pos.argtypes = [D, VP, VP, ctypes.c_double, VP, VP, VP, VP, VP, I32, VP, VP, I32, I32, I32, I32,
                                            VP, I64, VP]
    lib.ea_decode_attn_mass_rope_pos.argtypes = [D, VP, VP, ctypes.c_double, VP, VP, VP, VP, VP, I32, VP, VP, VP, I32, I32,
                                                 I32, I32, VP, I64, VP]
    lib.ea_decode_attn_alibi.argtypes = [D, VP, VP, VP, VP, VP, VP, VP, I32, I32, I32, I32, VP, I64, VP]
    lib.ea_prefill_attn_alibi.argtypes = [D, VP, VP, VP, VP, VP, VP, VP, I32, I32, I32, I32, VP]
    lib.ea_prefill_rope_workspace_bytes.argtypes = [D, I32, I32, I32]
    lib.ea_prefill_rope_workspace_bytes.restype = I64
    lib.ea_prefill_attn_rope.argtypes = [D, VP, VP, ctypes.c_double, VP, VP, VP, VP, VP, I32, I32, I32, I32, VP, I64, VP]
    lib.ea_prefill_attn.argtypes = [D, VP, VP, VP, VP, VP, VP, I32, I32, I32, I32, VP]
    lib.ea_out_proj.argtypes = [D, VP, I32, VP, VP, I32, VP]
    lib.ea_q4_layout_query.argtypes = [D, P(Q4Layout)]
    for f in (lib.ea_q4_k_code_pos, lib.ea_q4_v_code_pos, lib.ea_q4_k_scale_pos):
        f.restype = I64
        f.argtypes = [D, I32, I32, I32, I32]
    lib.ea_q4_v_scale_pos.restype = I64
    lib.ea_q4_v_scale_pos.argtypes = [D, I32, I32, I32]
    for f in (lib.ea_q3_k_code_pos, lib.ea_q3_v_code_pos):
        f.argtypes = [D, I32, I32, I32, I32, P(I64)]
    lib.ea_quantize_pages_q4.argtypes = [D, VP, VP, VP, VP, VP, VP, I32, I32, I32, VP]
    lib.ea_dequantize_pages_q4.argtypes = [D, VP, VP, VP, VP, VP, VP, I32, I32, I32, VP]
    lib.ea_decode_q4_workspace_bytes.restype = I64
    lib.ea_decode_q4_workspace_bytes.argtypes = [D, I32, I32]
    lib.ea_decode_attn_q4.argtypes = [D, VP, VP, VP, VP, VP, I32, I32, VP, VP, VP, VP, I32, I32, VP, I32, I32, VP, I64, VP]
    lib.ea_prefill_q4_workspace_bytes.restype = I64
    lib.ea_prefill_q4_workspace_bytes.argtypes = [D, I32, I32]
    lib.ea_prefill_attn_q4.argtypes = [D, VP, VP, VP, VP, VP, I32, I32, VP, VP, VP, VP, I32, I32, VP, I32, I32, VP, I64, VP]
    lib.ea_prefill_q4_staged_workspace_bytes.restype = I64
    lib.ea_prefill_q4_staged_workspace_bytes.argtypes = [D, I32, I32, I32, I32]
    lib.ea_prefill_attn_q4_staged.argtypes = lib.ea_prefill_attn_q4.argtypes
    lib.ea_prefill_attn_alibi_q4.argtypes = [D, VP, VP, VP, VP, VP, VP, I32, I32, VP, VP, VP, VP, I32, I32, VP, I32, I32, VP,
                                             I64, VP]
    lib.ea_prefill_rope_q4_workspace_bytes.restype = I64
    lib.ea_prefill_rope_q4_workspace_bytes.argtypes = [D, I32, I32, I32, I32]
    lib.ea_prefill_attn_rope_q4.argtypes = [D, VP, VP, ctypes.c_double, VP, VP, VP, VP, I32, I32, VP, VP, VP, VP, I32, I32,
                                            VP, I32, I32, VP, I64, VP]
    lib.ea_attn_mass_workspace_bytes.restype = I64
    lib.ea_attn_mass_workspace_bytes.argtypes = [D, I32, I32]
    lib.ea_attn_mass.argtypes = [D, VP, VP, VP, VP, VP, I32, I32, I32, VP, I64, VP]
    lib.ea_decode_attn_mass_workspace_bytes.restype = I64
    lib.ea_decode_attn_mass_workspace_bytes.argtypes = [D, I32, I32, I32]
    lib.ea_decode_attn_mass.argtypes = [D, VP, VP, VP, VP, VP, VP, VP, I32, I32, I32, I32, VP, I64, VP]
    lib.ea_decode_attn_alibi_q4.argtypes = [D, VP, VP, VP, VP, VP, VP, I32, I32, VP, VP, VP, VP, I32, I32, VP, I32, I32, VP, I64,
                                            VP]
    lib.ea_decode_attn_rope_q4.argtypes = [D, VP, VP, ctypes.c_double, VP, VP, VP, VP, I32, I32, VP, VP, VP, VP, I32, I32,
                                           VP, I32, I32, VP, I64, VP]
    _LIB = lib
    return lib


def strerror(code: int) -> str:
    return load_library().ea_strerror(int(code)).decode()


def version() -> int:
    return int(load_library().ea_version())


def _check(rc: int, where: str) -> None:
    if rc != 0:
        raise EigenAttnError(rc, where)


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("tensor must live on the GPU")
    if not t.is_contiguous():
        raise ValueError("tensor must be contiguous")
    return t.data_ptr()


def _stream(stream) -> int:
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return int(s.cuda_stream)


def _dt(t) -> int:
    import torch
    if t.dtype == torch.float32:
        return EA_F32
    if t.dtype == torch.bfloat16:
        return EA_BF16
    raise ValueError(f"unsupported tensor dtype {t.dtype}")


def _expect(t, desc_dtype: int, name: str) -> None:
    if _dt(t) != desc_dtype:
        raise ValueError(f"{name}: dtype {t.dtype} does not match the layer dtype")


def _i32(t, name: str) -> None:
    import torch
    if t.dtype != torch.int32:
        raise ValueError(f"{name} must be int32")


# ---- host helpers ------------------------------------------------------------
def cache_layout_query(desc: LayerDesc) -> CacheLayout:
    out = CacheLayout()
    _check(load_library().ea_cache_layout_query(ctypes.byref(desc), ctypes.byref(out)), "ea_cache_layout_query")
    return out


def cache_k_index(desc: LayerDesc, page: int, kv_head: int, token_in_page: int, channel: int) -> int:
    return int(load_library().ea_cache_k_index(ctypes.byref(desc), page, kv_head, token_in_page, channel))


def cache_v_index(desc: LayerDesc, page: int, kv_head: int, token_in_page: int, channel: int) -> int:
    return int(load_library().ea_cache_v_index(ctypes.byref(desc), page, kv_head, token_in_page, channel))


def cache_slot(desc: LayerDesc, page_table_row, pos: int) -> int:
    row = np.ascontiguousarray(page_table_row, dtype=np.int32)
    return int(load_library().ea_cache_slot(ctypes.byref(desc), row.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                                            int(row.shape[0]), int(pos)))


def alloc_pools(desc: LayerDesc, pool_pages: int, device="cuda", zero: bool = True):
    """Device memory for the K and V page pools of one layer: [pool_pages, page_elems] each."""
    import torch
    lay = cache_layout_query(desc)
    dt = torch.bfloat16 if desc.dtype == EA_BF16 else torch.float32
    mk = torch.zeros if zero else torch.empty
    return (mk((pool_pages, lay.k_page_elems), dtype=dt, device=device),
            mk((pool_pages, lay.v_page_elems), dtype=dt, device=device))


# ---- device calls ------------------------------------------------------------
def cache_scatter(desc, k_dense, v_dense, k_pool, v_pool, page_table, pos0: int = 0, stream=None) -> None:
    """k_dense [B, H_kv, n, r_k], v_dense [B, H_kv, n, r_v] -> pools (either dense tensor may be None)."""
    ref = k_dense if k_dense is not None else v_dense
    B, n = ref.shape[0], ref.shape[2]
    _i32(page_table, "page_table")
    for t, nm in ((k_dense, "k_dense"), (v_dense, "v_dense"), (k_pool, "k_pool"), (v_pool, "v_pool")):
        if t is not None:
            _expect(t, desc.dtype, nm)
    rc = load_library().ea_cache_scatter(ctypes.byref(desc), _ptr(k_dense), _ptr(v_dense), _ptr(k_pool), _ptr(v_pool),
                                         _ptr(page_table), B, n, pos0, page_table.shape[1],
                                         (k_pool if k_pool is not None else v_pool).shape[0], _stream(stream))
    _check(rc, "ea_cache_scatter")


def cache_gather(desc, k_dense, v_dense, k_pool, v_pool, page_table, pos0: int = 0, stream=None) -> None:
    ref = k_dense if k_dense is not None else v_dense
    B, n = ref.shape[0], ref.shape[2]
    _i32(page_table, "page_table")
    for t, nm in ((k_dense, "k_dense"), (v_dense, "v_dense"), (k_pool, "k_pool"), (v_pool, "v_pool")):
        if t is not None:
            _expect(t, desc.dtype, nm)
    rc = load_library().ea_cache_gather(ctypes.byref(desc), _ptr(k_dense), _ptr(v_dense), _ptr(k_pool), _ptr(v_pool),
                                        _ptr(page_table), B, n, pos0, page_table.shape[1],
                                        (k_pool if k_pool is not None else v_pool).shape[0], _stream(stream))
    _check(rc, "ea_cache_gather")


def packed_weight_elems(N: int, K: int, dtype: int) -> int:
    return int(load_library().ea_packed_weight_elems(N, K, dtype))


def pack_weight(w_t, stream=None):
    """Out-major weights w_t [N, K] (float32 or bfloat16, on the GPU) -> the packed order the projection calls read."""
    import torch
    N, K = w_t.shape
    dt = _dt(w_t)
    n = packed_weight_elems(N, K, dt)
    if n < 0:
        raise ValueError("weights cannot be packed (bfloat16 needs K % 32 == 0)")
    packed = torch.empty((n,), dtype=w_t.dtype, device=w_t.device)
    _check(load_library().ea_pack_weight(_ptr(w_t), _ptr(packed), N, K, dt, _stream(stream)), "ea_pack_weight")
    return packed


def _project_qkv(fn_name, q_dim, desc, x, wqkv, q, k_pool, v_pool, page_table, seq_len, T, stream, status):
    B = seq_len.shape[0]
    if x.shape[0] != B * T:
        raise ValueError("x must have B*T rows")
    _expect(x, desc.dtype, "x"); _expect(wqkv, desc.dtype, "wqkv")
    _expect(k_pool, desc.dtype, "k_pool"); _expect(v_pool, desc.dtype, "v_pool")
    _i32(page_table, "page_table"); _i32(seq_len, "seq_len")
    n_out = desc.n_heads * q_dim + desc.n_kv_heads * (desc.r_k + desc.r_v)
    if wqkv.numel() != packed_weight_elems(n_out, desc.d_model, desc.dtype) or x.shape[1] != desc.d_model:
        raise ValueError("packed weight / activation size does not match the layer")
    if q.numel() != B * T * desc.n_heads * q_dim:
        raise ValueError("q has the wrong size")
    if status is not None:
        _i32(status, "status")
    rc = getattr(load_library(), fn_name)(ctypes.byref(desc), _ptr(x), _ptr(wqkv), _ptr(q), _dt(q), _ptr(k_pool),
                                          _ptr(v_pool), _ptr(page_table), _ptr(seq_len), B, T, page_table.shape[1],
                                          k_pool.shape[0], _ptr(status), _stream(stream))
    _check(rc, fn_name)


def project_qkv(desc, x, wqkv, q_r, k_pool, v_pool, page_table, seq_len, T: int, stream=None, status=None) -> None:
    """x [B*T, d]; wqkv = pack_weight([N_qkv, d]); q_r [B*T, H, r_k] (float32 or bfloat16) is written,
    k and v go to the pools.  status: an int32 device tensor of one element to which the number of appends that
    could not be stored (cache full, bad page id) is added, or None."""
    _project_qkv("ea_project_qkv", desc.r_k, desc, x, wqkv, q_r, k_pool, v_pool, page_table, seq_len, T, stream,
                 status)


def project_qkv_rope(desc, x, wqkv, q, k_pool, v_pool, page_table, seq_len, T: int, stream=None, status=None) -> None:
    """Rotary variant: wqkv = pack_weight([H*d_head + H_kv*(r_k + r_v), d]); q [B*T, H, d_head] is written."""
    _project_qkv("ea_project_qkv_rope", desc.d_head, desc, x, wqkv, q, k_pool, v_pool, page_table, seq_len, T, stream,
                 status)


def decode_auto_splits(desc, B: int, max_seq_len: int) -> int:
    return int(load_library().ea_decode_auto_splits(ctypes.byref(desc), B, max_seq_len))


def decode_rope_auto_splits(desc, B: int, max_seq_len: int) -> int:
    return int(load_library().ea_decode_rope_auto_splits(ctypes.byref(desc), B, max_seq_len))


def decode_workspace_bytes(desc, B: int, n_splits: int) -> int:
    return int(load_library().ea_decode_workspace_bytes(ctypes.byref(desc), B, n_splits))


def decode_attn(desc, q_r, k_pool, v_pool, page_table, seq_len, out, n_splits: int = 0, ws=None, stream=None) -> None:
    """q_r [B, H, r_k] float32 -> out [B, H, r_v] float32 over the cached tokens of each sequence."""
    import torch
    B = seq_len.shape[0]
    if q_r.dtype != torch.float32 or out.dtype != torch.float32:
        raise ValueError("q_r and out must be float32")
    if q_r.numel() != B * desc.n_heads * desc.r_k or out.numel() != B * desc.n_heads * desc.r_v:
        raise ValueError("q_r / out have the wrong size")
    _expect(k_pool, desc.dtype, "k_pool"); _expect(v_pool, desc.dtype, "v_pool")
    _i32(page_table, "page_table"); _i32(seq_len, "seq_len")
    ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    rc = load_library().ea_decode_attn(ctypes.byref(desc), _ptr(q_r), _ptr(k_pool), _ptr(v_pool), _ptr(page_table),
                                       _ptr(seq_len), _ptr(out), B, page_table.shape[1], k_pool.shape[0], n_splits,
                                       _ptr(ws), ws_bytes, _stream(stream))
    _check(rc, "ea_decode_attn")


def decode_attn_static(desc, q_r, k_pool, v_pool, page_table, seq_len, out, n_splits: int = 0, stream=None) -> None:
    """decode_attn without a workspace argument: the split partials go to the library's built-in buffer
    (STATIC_SCRATCH_BYTES); nothing is allocated."""
    import torch
    B = seq_len.shape[0]
    if q_r.dtype != torch.float32 or out.dtype != torch.float32:
        raise ValueError("q_r and out must be float32")
    if q_r.numel() != B * desc.n_heads * desc.r_k or out.numel() != B * desc.n_heads * desc.r_v:
        raise ValueError("q_r / out have the wrong size")
    _expect(k_pool, desc.dtype, "k_pool"); _expect(v_pool, desc.dtype, "v_pool")
    _i32(page_table, "page_table"); _i32(seq_len, "seq_len")
    rc = load_library().ea_decode_attn_static(ctypes.byref(desc), _ptr(q_r), _ptr(k_pool), _ptr(v_pool),
                                              _ptr(page_table), _ptr(seq_len), _ptr(out), B, page_table.shape[1],
                                              k_pool.shape[0], n_splits, _stream(stream))
    _check(rc, "ea_decode_attn_static")


def decode_layer_workspace_bytes(desc, B: int, n_splits: int, rotary: bool = False) -> int:
    return int(load_library().ea_decode_layer_workspace_bytes(ctypes.byref(desc), B, n_splits, int(rotary)))


def decode_layer_fused_workspace_bytes(desc, B: int, n_splits: int, rotary: bool = False) -> int:
    return int(load_library().ea_decode_layer_fused_workspace_bytes(ctypes.byref(desc), B, n_splits, int(rotary)))


def decode_layer_fused_workers(desc, B: int, n_splits: int) -> int:
    return int(load_library().ea_decode_layer_fused_workers(ctypes.byref(desc), B, n_splits))


def set_wait_limit(polls: int) -> None:
    _check(load_library().ea_set_wait_limit(int(polls)), "ea_set_wait_limit")


def decode_layer(desc, x, wqkv, wo, k_pool, v_pool, page_table, seq_len, y, n_splits: int, ws, u_k=None,
                 rope_base: float = 10000.0, status=None, stream=None, fused: bool = False, alibi_slopes=None) -> None:
    """One generation step of a layer (projection + append, attention over seq_len + 1 tokens, output projection) in
    one call: x [B, d] -> y [B, d], both bfloat16.  With u_k ([d_head, r_k] bfloat16) the rotary form
    (ea_decode_layer_rope).  ws: decode_layer_workspace_bytes bytes.  fused: the two-launch form
    (ea_decode_layer_fused / ea_decode_layer_fused_rope; ws: decode_layer_fused_workspace_bytes bytes).
    With alibi_slopes ([H] float32, not together with u_k) the ALiBi form (ea_decode_layer_alibi /
    ea_decode_layer_fused_alibi)."""
    import torch
    B = seq_len.shape[0]
    _expect(x, desc.dtype, "x"); _expect(y, desc.dtype, "y"); _expect(wqkv, desc.dtype, "wqkv"); _expect(wo, desc.dtype, "wo")
    _expect(k_pool, desc.dtype, "k_pool"); _expect(v_pool, desc.dtype, "v_pool")
    _i32(page_table, "page_table"); _i32(seq_len, "seq_len")
    q_dim = desc.d_head if u_k is not None else desc.r_k
    n_out = desc.n_heads * q_dim + desc.n_kv_heads * (desc.r_k + desc.r_v)
    if (x.numel() != B * desc.d_model or y.numel() != B * desc.d_model
            or wqkv.numel() != packed_weight_elems(n_out, desc.d_model, desc.dtype)
            or wo.numel() != packed_weight_elems(desc.d_model, desc.n_heads * desc.r_v, desc.dtype)):
        raise ValueError("x / y / packed weight sizes do not match the layer")
    if status is not None:
        _i32(status, "status")
    ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    lib = load_library()
    if alibi_slopes is not None:
        if u_k is not None:
            raise ValueError("alibi_slopes and u_k exclude each other")
        if alibi_slopes.dtype != torch.float32 or alibi_slopes.numel() != desc.n_heads or not alibi_slopes.is_contiguous():
            raise ValueError("alibi_slopes must be a contiguous float32 [H] tensor")
        fn = lib.ea_decode_layer_fused_alibi if fused else lib.ea_decode_layer_alibi
        rc = fn(ctypes.byref(desc), _ptr(x), _ptr(wqkv), _ptr(wo), _ptr(alibi_slopes), _ptr(k_pool), _ptr(v_pool),
                _ptr(page_table), _ptr(seq_len), _ptr(y), B, page_table.shape[1], k_pool.shape[0],
                n_splits, _ptr(ws), ws_bytes, _ptr(status), _stream(stream))
        _check(rc, "ea_decode_layer_fused_alibi" if fused else "ea_decode_layer_alibi")
    elif u_k is None:
        fn = lib.ea_decode_layer_fused if fused else lib.ea_decode_layer
        rc = fn(ctypes.byref(desc), _ptr(x), _ptr(wqkv), _ptr(wo), _ptr(k_pool), _ptr(v_pool),
                _ptr(page_table), _ptr(seq_len), _ptr(y), B, page_table.shape[1], k_pool.shape[0],
                n_splits, _ptr(ws), ws_bytes, _ptr(status), _stream(stream))
        _check(rc, "ea_decode_layer_fused" if fused else "ea_decode_layer")
    else:
        _expect(u_k, desc.dtype, "u_k")
        if u_k.numel() != desc.d_head * desc.r_k or not u_k.is_contiguous():
            raise ValueError("u_k must be a contiguous [d_head, r_k] tensor")
        fn = lib.ea_decode_layer_fused_rope if fused else lib.ea_decode_layer_rope
        rc = fn(ctypes.byref(desc), _ptr(x), _ptr(wqkv), _ptr(wo), _ptr(u_k), float(rope_base),
                _ptr(k_pool), _ptr(v_pool), _ptr(page_table), _ptr(seq_len), _ptr(y), B,
                page_table.shape[1], k_pool.shape[0], n_splits, _ptr(ws), ws_bytes,
                _ptr(status), _stream(stream))
        _check(rc, "ea_decode_layer_fused_rope" if fused else "ea_decode_layer_rope")


def decode_layer_fused(desc, x, wqkv, wo, k_pool, v_pool, page_table, seq_len, y, n_splits: int, ws, status=None,
                       stream=None) -> None:
    decode_layer(desc, x, wqkv, wo, k_pool, v_pool, page_table, seq_len, y, n_splits, ws, status=status, stream=stream,
                 fused=True)


def decode_layer_fused_rope(desc, x, wqkv, wo, u_k, rope_base, k_pool, v_pool, page_table, seq_len, y, n_splits: int,
                            ws, status=None, stream=None) -> None:
    decode_layer(desc, x, wqkv, wo, k_pool, v_pool, page_table, seq_len, y, n_splits, ws, u_k=u_k, rope_base=rope_base,
                 status=status, stream=stream, fused=True)


def decode_layer_alibi(desc, x, wqkv, wo, alibi_slopes, k_pool, v_pool, page_table, seq_len, y, n_splits: int, ws,
                       status=None, stream=None, fused: bool = False) -> None:
    decode_layer(desc, x, wqkv, wo, k_pool, v_pool, page_table, seq_len, y, n_splits, ws, status=status, stream=stream,
                 fused=fused, alibi_slopes=alibi_slopes)


def decode_layer_fused_alibi(desc, x, wqkv, wo, alibi_slopes, k_pool, v_pool, page_table, seq_len, y, n_splits: int, ws,
                             status=None, stream=None) -> None:
    decode_layer_alibi(desc, x, wqkv, wo, alibi_slopes, k_pool, v_pool, page_table, seq_len, y, n_splits, ws,
                       status=status, stream=stream, fused=True)


def decode_layer_rope(desc, x, wqkv, wo, u_k, rope_base, k_pool, v_pool, page_table, seq_len, y, n_splits: int, ws,
                      status=None, stream=None) -> None:
    decode_layer(desc, x, wqkv, wo, k_pool, v_pool, page_table, seq_len, y, n_splits, ws, u_k=u_k, rope_base=rope_base,
                 status=status, stream=stream)


def decode_attn_rope(desc, q, u_k, rope_base: float, k_pool, v_pool, page_table, seq_len, out, n_splits: int = 0,
                     ws=None, stream=None) -> None:
    """q [B, H, d_head] float32 (not rotated), u_k [d_head, r_k] in the layer dtype -> out [B, H, r_v] float32."""
    import torch
    B = seq_len.shape[0]
    if q.dtype != torch.float32 or out.dtype != torch.float32:
        raise ValueError("q and out must be float32")
    _expect(u_k, desc.dtype, "u_k")
    if q.numel() != B * desc.n_heads * desc.d_head or out.numel() != B * desc.n_heads * desc.r_v:
        raise ValueError("q / out have the wrong size")
    if u_k.numel() != desc.d_head * desc.r_k or not u_k.is_contiguous():
        raise ValueError("u_k must be a contiguous [d_head, r_k] tensor")
    _expect(k_pool, desc.dtype, "k_pool"); _expect(v_pool, desc.dtype, "v_pool")
    _i32(page_table, "page_table"); _i32(seq_len, "seq_len")
    ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    rc = load_library().ea_decode_attn_rope(ctypes.byref(desc), _ptr(q), _ptr(u_k), float(rope_base), _ptr(k_pool),
                                            _ptr(v_pool), _ptr(page_table), _ptr(seq_len), _ptr(out), B,
                                            page_table.shape[1], k_pool.shape[0], n_splits, _ptr(ws), ws_bytes,
                                            _stream(stream))
    _check(rc, "ea_decode_attn_rope")


def decode_attn_rope_pos(desc, q, u_k, rope_base: float, k_pool, v_pool, page_table, seq_len, slot_pos, q_pos, out,
                         n_splits: int = 0, ws=None, mass=None, stream=None) -> None:
    """decode_attn_rope over a cache from which tokens have been dropped: slot_pos [B, >= max_pages * page_tokens]
    int32 holds the position in the text of the token in every cache slot, q_pos [B] int32 the query's.  With mass
    ([B, H_kv, max_pages * page_tokens] float32, bfloat16 layers) the probability every slot received is added to it
    (ea_decode_attn_mass_rope_pos; ws: decode_attn_mass_workspace_bytes, n_splits >= 1)."""
    import torch
    B = seq_len.shape[0]
    if q.dtype != torch.float32 or out.dtype != torch.float32:
        raise ValueError("q and out must be float32")
    _expect(u_k, desc.dtype, "u_k")
    if q.numel() != B * desc.n_heads * desc.d_head or out.numel() != B * desc.n_heads * desc.r_v:
        raise ValueError("q / out have the wrong size")
    if u_k.numel() != desc.d_head * desc.r_k or not u_k.is_contiguous():
        raise ValueError("u_k must be a contiguous [d_head, r_k] tensor")
    _expect(k_pool, desc.dtype, "k_pool"); _expect(v_pool, desc.dtype, "v_pool")
    _i32(page_table, "page_table"); _i32(seq_len, "seq_len"); _i32(slot_pos, "slot_pos"); _i32(q_pos, "q_pos")
    if slot_pos.dim() != 2 or slot_pos.shape[0] != B or not slot_pos.is_contiguous() or q_pos.numel() != B:
        raise ValueError("slot_pos must be a contiguous [B, stride] tensor, q_pos [B]")
    ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    lib = load_library()
    if mass is None:
        rc = lib.ea_decode_attn_rope_pos(ctypes.byref(desc), _ptr(q), _ptr(u_k), float(rope_base), _ptr(k_pool),
                                         _ptr(v_pool), _ptr(page_table), _ptr(seq_len), _ptr(slot_pos),
                                         slot_pos.shape[1], _ptr(q_pos), _ptr(out), B, page_table.shape[1],
                                         k_pool.shape[0], n_splits, _ptr(ws), ws_bytes, _stream(stream))
        _check(rc, "ea_decode_attn_rope_pos")
        return
    if mass.dtype != torch.float32 or mass.numel() != B * desc.n_kv_heads * page_table.shape[1] * desc.page_tokens:
        raise ValueError("mass must be float32 [B, H_kv, max_pages * page_tokens]")
    rc = lib.ea_decode_attn_mass_rope_pos(ctypes.byref(desc), _ptr(q), _ptr(u_k), float(rope_base), _ptr(k_pool),
                                          _ptr(v_pool), _ptr(page_table), _ptr(seq_len), _ptr(slot_pos),
                                          slot_pos.shape[1], _ptr(q_pos), _ptr(out), _ptr(mass), B, page_table.shape[1],
                                          k_pool.shape[0], n_splits, _ptr(ws), ws_bytes, _stream(stream))
    _check(rc, "ea_decode_attn_mass_rope_pos")


def decode_attn_mass_rope_pos(desc, q, u_k, rope_base: float, k_pool, v_pool, page_table, seq_len, slot_pos, q_pos, out,
                              mass, n_splits: int, ws, stream=None) -> None:
    decode_attn_rope_pos(desc, q, u_k, rope_base, k_pool, v_pool, page_table, seq_len, slot_pos, q_pos, out,
                         n_splits=n_splits, ws=ws, mass=mass, stream=stream)


def prefill_attn(desc, q_r, k_pool, v_pool, page_table, seq_len, out, stream=None) -> None:
    """q_r [B, n, H, r_k] -> out [B, n, H, r_v] (layer dtype), causal over each sequence's cache."""
    B, n = q_r.shape[0], q_r.shape[1]
    _expect(q_r, desc.dtype, "q_r"); _expect(out, desc.dtype, "out")
    _expect(k_pool, desc.dtype, "k_pool"); _expect(v_pool, desc.dtype, "v_pool")
    _i32(page_table, "page_table"); _i32(seq_len, "seq_len")
    if q_r.numel() != B * n * desc.n_heads * desc.r_k or out.numel() != B * n * desc.n_heads * desc.r_v:
        raise ValueError("q_r / out have the wrong size")
    rc = load_library().ea_prefill_attn(ctypes.byref(desc), _ptr(q_r), _ptr(k_pool), _ptr(v_pool), _ptr(page_table),
                                        _ptr(seq_len), _ptr(out), B, n, page_table.shape[1], k_pool.shape[0],
                                        _stream(stream))
    _check(rc, "ea_prefill_attn")


def _slopes(desc, slopes):
    import torch
    if slopes.dtype != torch.float32 or slopes.numel() != desc.n_heads or not slopes.is_contiguous():
        raise ValueError("slopes must be a contiguous float32 tensor with one entry per head")


def decode_attn_alibi(desc, q_r, slopes, k_pool, v_pool, page_table, seq_len, out, n_splits: int = 0, ws=None,
                      stream=None) -> None:
    """decode_attn with the ALiBi bias -slopes[h] * (distance of the key to the query) added to the scores."""
    import torch
    B = seq_len.shape[0]
    if q_r.dtype != torch.float32 or out.dtype != torch.float32:
        raise ValueError("q_r and out must be float32")
    if q_r.numel() != B * desc.n_heads * desc.r_k or out.numel() != B * desc.n_heads * desc.r_v:
        raise ValueError("q_r / out have the wrong size")
    _slopes(desc, slopes)
    _expect(k_pool, desc.dtype, "k_pool"); _expect(v_pool, desc.dtype, "v_pool")
    _i32(page_table, "page_table"); _i32(seq_len, "seq_len")
    ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    rc = load_library().ea_decode_attn_alibi(ctypes.byref(desc), _ptr(q_r), _ptr(slopes), _ptr(k_pool), _ptr(v_pool),
                                             _ptr(page_table), _ptr(seq_len), _ptr(out), B, page_table.shape[1],
                                             k_pool.shape[0], n_splits, _ptr(ws), ws_bytes, _stream(stream))
    _check(rc, "ea_decode_attn_alibi")


def prefill_attn_alibi(desc, q_r, slopes, k_pool, v_pool, page_table, seq_len, out, stream=None) -> None:
    """prefill_attn with the ALiBi bias."""
    B, n = q_r.shape[0], q_r.shape[1]
    _expect(q_r, desc.dtype, "q_r"); _expect(out, desc.dtype, "out")
    _expect(k_pool, desc.dtype, "k_pool"); _expect(v_pool, desc.dtype, "v_pool")
    _i32(page_table, "page_table"); _i32(seq_len, "seq_len")
    _slopes(desc, slopes)
    if q_r.numel() != B * n * desc.n_heads * desc.r_k or out.numel() != B * n * desc.n_heads * desc.r_v:
        raise ValueError("q_r / out have the wrong size")
    rc = load_library().ea_prefill_attn_alibi(ctypes.byref(desc), _ptr(q_r), _ptr(slopes), _ptr(k_pool), _ptr(v_pool),
                                              _ptr(page_table), _ptr(seq_len), _ptr(out), B, n, page_table.shape[1],
                                              k_pool.shape[0], _stream(stream))
    _check(rc, "ea_prefill_attn_alibi")


def prefill_rope_workspace_bytes(desc, B: int, n: int, max_pages: int) -> int:
    return int(load_library().ea_prefill_rope_workspace_bytes(ctypes.byref(desc), B, n, max_pages))


def prefill_attn_rope(desc, q, u_k, rope_base: float, k_pool, v_pool, page_table, seq_len, out, ws=None,
                      stream=None) -> None:
    """Rotary prefill: q [B, n, H, d_head] (layer dtype, not rotated) -> out [B, n, H, r_v], causal."""
    B, n = q.shape[0], q.shape[1]
    _expect(q, desc.dtype, "q"); _expect(out, desc.dtype, "out"); _expect(u_k, desc.dtype, "u_k")
    _expect(k_pool, desc.dtype, "k_pool"); _expect(v_pool, desc.dtype, "v_pool")
    _i32(page_table, "page_table"); _i32(seq_len, "seq_len")
    if q.numel() != B * n * desc.n_heads * desc.d_head or out.numel() != B * n * desc.n_heads * desc.r_v:
        raise ValueError("q / out have the wrong size")
    if u_k.numel() != desc.d_head * desc.r_k or not u_k.is_contiguous():
        raise ValueError("u_k must be a contiguous [d_head, r_k] tensor")
    ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    rc = load_library().ea_prefill_attn_rope(ctypes.byref(desc), _ptr(q), _ptr(u_k), float(rope_base), _ptr(k_pool),
                                             _ptr(v_pool), _ptr(page_table), _ptr(seq_len), _ptr(out), B, n,
                                             page_table.shape[1], k_pool.shape[0], _ptr(ws), ws_bytes,
                                             _stream(stream))
    _check(rc, "ea_prefill_attn_rope")


def out_proj(desc, o, wo, y, stream=None) -> None:
    """o [M, H*r_v] (float32 or bfloat16) x wo = pack_weight([d, H*r_v]) -> y [M, d] (layer dtype)."""
    M = y.shape[0]
    _expect(wo, desc.dtype, "wo"); _expect(y, desc.dtype, "y")
    if (wo.numel() != packed_weight_elems(desc.d_model, desc.n_heads * desc.r_v, desc.dtype)
            or o.numel() != M * desc.n_heads * desc.r_v):
        raise ValueError("o / packed wo size does not match the layer")
    rc = load_library().ea_out_proj(ctypes.byref(desc), _ptr(o), _dt(o), _ptr(wo), _ptr(y), M, _stream(stream))
    _check(rc, "ea_out_proj")


# ---- 4-bit group-quantised cache ----------------------------------------------
def q4_layout_query(desc: LayerDesc) -> Q4Layout:
    out = Q4Layout()
    _check(load_library().ea_q4_layout_query(ctypes.byref(desc), ctypes.byref(out)), "ea_q4_layout_query")
    return out


def q4_k_code_pos(desc, page: int, kv_head: int, token_in_page: int, channel: int) -> int:
    return int(load_library().ea_q4_k_code_pos(ctypes.byref(desc), page, kv_head, token_in_page, channel))


def q4_v_code_pos(desc, page: int, kv_head: int, token_in_page: int, channel: int) -> int:
    return int(load_library().ea_q4_v_code_pos(ctypes.byref(desc), page, kv_head, token_in_page, channel))


def q3_k_code_pos(desc, page: int, kv_head: int, token_in_page: int, channel: int):
    """3-bit codes (desc.q4_bits = 3): the bit offsets of the code's three bits, lowest first; None on bad arguments."""
    pos = (ctypes.c_int64 * 3)()
    rc = load_library().ea_q3_k_code_pos(ctypes.byref(desc), page, kv_head, token_in_page, channel, pos)
    return tuple(int(v) for v in pos) if rc == 0 else None


def q3_v_code_pos(desc, page: int, kv_head: int, token_in_page: int, channel: int):
    pos = (ctypes.c_int64 * 3)()
    rc = load_library().ea_q3_v_code_pos(ctypes.byref(desc), page, kv_head, token_in_page, channel, pos)
    return tuple(int(v) for v in pos) if rc == 0 else None


def q4_k_scale_pos(desc, page: int, kv_head: int, token_in_page: int, channel: int) -> int:
    return int(load_library().ea_q4_k_scale_pos(ctypes.byref(desc), page, kv_head, token_in_page, channel))


def q4_v_scale_pos(desc, page: int, kv_head: int, token_in_page: int) -> int:
    return int(load_library().ea_q4_v_scale_pos(ctypes.byref(desc), page, kv_head, token_in_page))


def alloc_q4_pools(desc: LayerDesc, q4_pool_pages: int, device="cuda", zero: bool = True):
    """Device memory for the 4-bit K and V page pools of one layer: uint8 [q4_pool_pages, page_bytes] each."""
    import torch
    lay = q4_layout_query(desc)
    mk = torch.zeros if zero else torch.empty
    return (mk((q4_pool_pages, lay.k_page_bytes), dtype=torch.uint8, device=device),
            mk((q4_pool_pages, lay.v_page_bytes), dtype=torch.uint8, device=device))


def _u8(t, name: str) -> None:
    import torch
    if t.dtype != torch.uint8:
        raise ValueError(f"{name} must be uint8")


def quantize_pages_q4(desc, k_pool, v_pool, src_pages, kq_pool, vq_pool, dst_pages, stream=None) -> None:
    """Full pages src_pages[i] of the bfloat16 pools -> pages dst_pages[i] of the 4-bit pools."""
    _expect(k_pool, desc.dtype, "k_pool"); _expect(v_pool, desc.dtype, "v_pool")
    _u8(kq_pool, "kq_pool"); _u8(vq_pool, "vq_pool")
    _i32(src_pages, "src_pages"); _i32(dst_pages, "dst_pages")
    if src_pages.numel() != dst_pages.numel():
        raise ValueError("src_pages and dst_pages must have the same length")
    rc = load_library().ea_quantize_pages_q4(ctypes.byref(desc), _ptr(k_pool), _ptr(v_pool), _ptr(src_pages),
                                             _ptr(kq_pool), _ptr(vq_pool), _ptr(dst_pages), src_pages.numel(),
                                             k_pool.shape[0], kq_pool.shape[0], _stream(stream))
    _check(rc, "ea_quantize_pages_q4")


def dequantize_pages_q4(desc, kq_pool, vq_pool, src_pages, k_pool, v_pool, dst_pages, stream=None) -> None:
    """Pages src_pages[i] of the 4-bit pools -> pages dst_pages[i] of the bfloat16 pools (export / inspection)."""
    _expect(k_pool, desc.dtype, "k_pool"); _expect(v_pool, desc.dtype, "v_pool")
    _u8(kq_pool, "kq_pool"); _u8(vq_pool, "vq_pool")
    _i32(src_pages, "src_pages"); _i32(dst_pages, "dst_pages")
    if src_pages.numel() != dst_pages.numel():
        raise ValueError("src_pages and dst_pages must have the same length")
    rc = load_library().ea_dequantize_pages_q4(ctypes.byref(desc), _ptr(kq_pool), _ptr(vq_pool), _ptr(src_pages),
                                               _ptr(k_pool), _ptr(v_pool), _ptr(dst_pages), src_pages.numel(),
                                               kq_pool.shape[0], k_pool.shape[0], _stream(stream))
    _check(rc, "ea_dequantize_pages_q4")


def decode_q4_workspace_bytes(desc, B: int, n_splits: int) -> int:
    return int(load_library().ea_decode_q4_workspace_bytes(ctypes.byref(desc), B, n_splits))


def decode_attn_q4(desc, q_r, kq_pool, vq_pool, q4_page_table, q4_len, k_pool, v_pool, tail_page_table, tail_len, out,
                   n_splits: int, ws, stream=None, alibi_slopes=None) -> None:
    """q_r [B, H, r_k] float32 -> out [B, H, r_v] float32 over q4_len[b] tokens of the 4-bit pools followed by
    tail_len[b] tokens of the bfloat16 pools (k_pool, v_pool, tail_page_table, tail_len may all be None).
    With alibi_slopes ([H] float32) the ALiBi bias is added (ea_decode_attn_alibi_q4)."""
    import torch
    if alibi_slopes is not None:
        _slopes(desc, alibi_slopes)
    B = q4_len.shape[0]
    if q_r.dtype != torch.float32 or out.dtype != torch.float32:
        raise ValueError("q_r and out must be float32")
    if q_r.numel() != B * desc.n_heads * desc.r_k or out.numel() != B * desc.n_heads * desc.r_v:
        raise ValueError("q_r / out have the wrong size")
    _u8(kq_pool, "kq_pool"); _u8(vq_pool, "vq_pool")
    _i32(q4_page_table, "q4_page_table"); _i32(q4_len, "q4_len")
    tail = tail_page_table is not None
    if tail:
        _expect(k_pool, desc.dtype, "k_pool"); _expect(v_pool, desc.dtype, "v_pool")
        _i32(tail_page_table, "tail_page_table"); _i32(tail_len, "tail_len")
    ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    rest = (_ptr(kq_pool), _ptr(vq_pool), _ptr(q4_page_table), _ptr(q4_len),
            q4_page_table.shape[1], kq_pool.shape[0], _ptr(k_pool) if tail else None, _ptr(v_pool) if tail else None,
            _ptr(tail_page_table), _ptr(tail_len) if tail else None, tail_page_table.shape[1] if tail else 0,
            k_pool.shape[0] if tail else 0, _ptr(out), B, n_splits, _ptr(ws), ws_bytes, _stream(stream))
    if alibi_slopes is None:
        _check(load_library().ea_decode_attn_q4(ctypes.byref(desc), _ptr(q_r), *rest), "ea_decode_attn_q4")
    else:
        _check(load_library().ea_decode_attn_alibi_q4(ctypes.byref(desc), _ptr(q_r), _ptr(alibi_slopes), *rest),
               "ea_decode_attn_alibi_q4")


def prefill_q4_workspace_bytes(desc, B: int, n: int) -> int:
    return int(load_library().ea_prefill_q4_workspace_bytes(ctypes.byref(desc), B, n))


def prefill_q4_staged_workspace_bytes(desc, B: int, n: int, max_q4_pages: int, max_tail_pages: int) -> int:
    return int(load_library().ea_prefill_q4_staged_workspace_bytes(ctypes.byref(desc), B, n, max_q4_pages,
                                                                   max_tail_pages))


def prefill_attn_q4(desc, q_r, kq_pool, vq_pool, q4_page_table, q4_len, k_pool, v_pool, tail_page_table, tail_len, out,
                    ws, stream=None, staged: bool = False, alibi_slopes=None) -> None:
    """Causal prefill attention of the last n tokens of every sequence: q_r [B, n, H, r_k] -> out [B, n, H, r_v]
    (bfloat16) over q4_len[b] tokens of the 4-bit pools followed by tail_len[b] >= n tokens of the bfloat16 pools.
    staged: ea_prefill_attn_q4_staged (codes dequantised into stage pools inside ws, which then must hold
    prefill_q4_staged_workspace_bytes bytes; q4_len in whole pages).  With alibi_slopes ([H] float32) the staged call
    with the ALiBi bias (ea_prefill_attn_alibi_q4; same workspace)."""
    import torch
    B, n = q_r.shape[0], q_r.shape[1]
    _expect(q_r, desc.dtype, "q_r"); _expect(out, desc.dtype, "out")
    if q_r.numel() != B * n * desc.n_heads * desc.r_k or out.numel() != B * n * desc.n_heads * desc.r_v:
        raise ValueError("q_r / out have the wrong size")
    _u8(kq_pool, "kq_pool"); _u8(vq_pool, "vq_pool")
    _expect(k_pool, desc.dtype, "k_pool"); _expect(v_pool, desc.dtype, "v_pool")
    for t, name in ((q4_page_table, "q4_page_table"), (q4_len, "q4_len"), (tail_page_table, "tail_page_table"),
                    (tail_len, "tail_len")):
        _i32(t, name)
    ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    lib = load_library()
    if alibi_slopes is not None:
        if alibi_slopes.dtype != torch.float32 or alibi_slopes.numel() != desc.n_heads or not alibi_slopes.is_contiguous():
            raise ValueError("alibi_slopes must be a contiguous float32 [H] tensor")
        rc = lib.ea_prefill_attn_alibi_q4(
            ctypes.byref(desc), _ptr(q_r), _ptr(alibi_slopes), _ptr(kq_pool), _ptr(vq_pool), _ptr(q4_page_table),
            _ptr(q4_len), q4_page_table.shape[1], kq_pool.shape[0], _ptr(k_pool), _ptr(v_pool), _ptr(tail_page_table),
            _ptr(tail_len), tail_page_table.shape[1], k_pool.shape[0], _ptr(out), B, n, _ptr(ws), ws_bytes,
            _stream(stream))
        _check(rc, "ea_prefill_attn_alibi_q4")
        return
    rc = (lib.ea_prefill_attn_q4_staged if staged else lib.ea_prefill_attn_q4)(
        ctypes.byref(desc), _ptr(q_r), _ptr(kq_pool), _ptr(vq_pool), _ptr(q4_page_table), _ptr(q4_len),
        q4_page_table.shape[1], kq_pool.shape[0], _ptr(k_pool), _ptr(v_pool), _ptr(tail_page_table), _ptr(tail_len),
        tail_page_table.shape[1], k_pool.shape[0], _ptr(out), B, n, _ptr(ws), ws_bytes, _stream(stream))
    _check(rc, "ea_prefill_attn_q4_staged" if staged else "ea_prefill_attn_q4")


def prefill_rope_q4_workspace_bytes(desc, B: int, n: int, max_q4_pages: int, max_tail_pages: int) -> int:
    return int(load_library().ea_prefill_rope_q4_workspace_bytes(ctypes.byref(desc), B, n, max_q4_pages,
                                                                 max_tail_pages))


def prefill_attn_rope_q4(desc, q, u_k, rope_base: float, kq_pool, vq_pool, q4_page_table, q4_len, k_pool, v_pool,
                         tail_page_table, tail_len, out, ws, stream=None) -> None:
    """Rotary variant of prefill_attn_q4: q [B, n, H, d_head] bfloat16 (not rotated), u_k [d_head, r_k] bfloat16;
    q4_len in whole pages; ws: prefill_rope_q4_workspace_bytes bytes."""
    B, n = q.shape[0], q.shape[1]
    _expect(q, desc.dtype, "q"); _expect(out, desc.dtype, "out"); _expect(u_k, desc.dtype, "u_k")
    if q.numel() != B * n * desc.n_heads * desc.d_head or out.numel() != B * n * desc.n_heads * desc.r_v:
        raise ValueError("q / out have the wrong size")
    if u_k.numel() != desc.d_head * desc.r_k or not u_k.is_contiguous():
        raise ValueError("u_k must be a contiguous [d_head, r_k] tensor")
    _u8(kq_pool, "kq_pool"); _u8(vq_pool, "vq_pool")
    _expect(k_pool, desc.dtype, "k_pool"); _expect(v_pool, desc.dtype, "v_pool")
    for t, name in ((q4_page_table, "q4_page_table"), (q4_len, "q4_len"), (tail_page_table, "tail_page_table"),
                    (tail_len, "tail_len")):
        _i32(t, name)
    ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    rc = load_library().ea_prefill_attn_rope_q4(
        ctypes.byref(desc), _ptr(q), _ptr(u_k), float(rope_base), _ptr(kq_pool), _ptr(vq_pool), _ptr(q4_page_table),
        _ptr(q4_len), q4_page_table.shape[1], kq_pool.shape[0], _ptr(k_pool), _ptr(v_pool), _ptr(tail_page_table),
        _ptr(tail_len), tail_page_table.shape[1], k_pool.shape[0], _ptr(out), B, n, _ptr(ws), ws_bytes,
        _stream(stream))
    _check(rc, "ea_prefill_attn_rope_q4")


def decode_attn_alibi_q4(desc, q_r, slopes, kq_pool, vq_pool, q4_page_table, q4_len, k_pool, v_pool, tail_page_table,
                         tail_len, out, n_splits: int, ws, stream=None) -> None:
    """decode_attn_q4 with the ALiBi bias -slopes[h] * (distance of the key to the newest token)."""
    decode_attn_q4(desc, q_r, kq_pool, vq_pool, q4_page_table, q4_len, k_pool, v_pool, tail_page_table, tail_len, out,
                   n_splits, ws, stream=stream, alibi_slopes=slopes)


def decode_attn_rope_q4(desc, q, u_k, rope_base: float, kq_pool, vq_pool, q4_page_table, q4_len, k_pool, v_pool,
                        tail_page_table, tail_len, out, n_splits: int, ws, stream=None) -> None:
    """Rotary variant of decode_attn_q4: q [B, H, d_head] float32 (not rotated), u_k [d_head, r_k] bfloat16."""
    import torch
    B = q4_len.shape[0]
    if q.dtype != torch.float32 or out.dtype != torch.float32:
        raise ValueError("q and out must be float32")
    if q.numel() != B * desc.n_heads * desc.d_head or out.numel() != B * desc.n_heads * desc.r_v:
        raise ValueError("q / out have the wrong size")
    _expect(u_k, desc.dtype, "u_k")
    if u_k.numel() != desc.d_head * desc.r_k or not u_k.is_contiguous():
        raise ValueError("u_k must be a contiguous [d_head, r_k] tensor")
    _u8(kq_pool, "kq_pool"); _u8(vq_pool, "vq_pool")
    _i32(q4_page_table, "q4_page_table"); _i32(q4_len, "q4_len")
    tail = tail_page_table is not None
    if tail:
        _expect(k_pool, desc.dtype, "k_pool"); _expect(v_pool, desc.dtype, "v_pool")
        _i32(tail_page_table, "tail_page_table"); _i32(tail_len, "tail_len")
    ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    rc = load_library().ea_decode_attn_rope_q4(
        ctypes.byref(desc), _ptr(q), _ptr(u_k), float(rope_base), _ptr(kq_pool), _ptr(vq_pool), _ptr(q4_page_table),
        _ptr(q4_len), q4_page_table.shape[1], kq_pool.shape[0], _ptr(k_pool) if tail else None,
        _ptr(v_pool) if tail else None, _ptr(tail_page_table), _ptr(tail_len) if tail else None,
        tail_page_table.shape[1] if tail else 0, k_pool.shape[0] if tail else 0, _ptr(out), B, n_splits, _ptr(ws),
        ws_bytes, _stream(stream))
    _check(rc, "ea_decode_attn_rope_q4")


# ---- attention statistics for token-eviction policies ---------------------------
def attn_mass_workspace_bytes(desc, B: int, max_pages: int) -> int:
    return int(load_library().ea_attn_mass_workspace_bytes(ctypes.byref(desc), B, max_pages))


def attn_mass(desc, q_r, k_pool, page_table, seq_len, mass, ws, stream=None) -> None:
    """mass [B, H_kv, max_pages * page_tokens] float32 += the softmax probability every cached token receives from
    the queries q_r [B, H, r_k] (summed over the query heads of each kv head)."""
    import torch
    B = seq_len.shape[0]
    if q_r.dtype != torch.float32 or mass.dtype != torch.float32:
        raise ValueError("q_r and mass must be float32")
    if q_r.numel() != B * desc.n_heads * desc.r_k:
        raise ValueError("q_r has the wrong size")
    if mass.numel() != B * desc.n_kv_heads * page_table.shape[1] * desc.page_tokens:
        raise ValueError("mass must be [B, H_kv, max_pages * page_tokens]")
    _expect(k_pool, desc.dtype, "k_pool")
    _i32(page_table, "page_table"); _i32(seq_len, "seq_len")
    ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    rc = load_library().ea_attn_mass(ctypes.byref(desc), _ptr(q_r), _ptr(k_pool), _ptr(page_table), _ptr(seq_len),
                                     _ptr(mass), B, page_table.shape[1], k_pool.shape[0], _ptr(ws), ws_bytes,
                                     _stream(stream))
    _check(rc, "ea_attn_mass")


def decode_attn_mass_workspace_bytes(desc, B: int, max_pages: int, n_splits: int) -> int:
    return int(load_library().ea_decode_attn_mass_workspace_bytes(ctypes.byref(desc), B, max_pages, n_splits))


def decode_attn_mass(desc, q_r, k_pool, v_pool, page_table, seq_len, out, mass, n_splits: int, ws, stream=None) -> None:
    """decode_attn and attn_mass in one pass over the cache (bfloat16 layers): out [B, H, r_v] float32 is written,
    mass [B, H_kv, max_pages * page_tokens] float32 is added to."""
    import torch
    B = seq_len.shape[0]
    if q_r.dtype != torch.float32 or out.dtype != torch.float32 or mass.dtype != torch.float32:
        raise ValueError("q_r, out and mass must be float32")
    if q_r.numel() != B * desc.n_heads * desc.r_k or out.numel() != B * desc.n_heads * desc.r_v:
        raise ValueError("q_r / out have the wrong size")
    if mass.numel() != B * desc.n_kv_heads * page_table.shape[1] * desc.page_tokens:
        raise ValueError("mass must be [B, H_kv, max_pages * page_tokens]")
    _expect(k_pool, desc.dtype, "k_pool"); _expect(v_pool, desc.dtype, "v_pool")
    _i32(page_table, "page_table"); _i32(seq_len, "seq_len")
    ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    rc = load_library().ea_decode_attn_mass(ctypes.byref(desc), _ptr(q_r), _ptr(k_pool), _ptr(v_pool), _ptr(page_table),
                                            _ptr(seq_len), _ptr(out), _ptr(mass), B, page_table.shape[1],
                                            k_pool.shape[0], n_splits, _ptr(ws), ws_bytes, _stream(stream))
    _check(rc, "ea_decode_attn_mass")
