"""Shared plumbing of the GPU parity tests: build inputs on the host, hand the same
values to the HIP path (through the C ABI) and to the fp64 oracle, compare."""
from __future__ import annotations

import numpy as np
import torch

import paper_2408_05646_amd as ea
from oracle import eigen_attention as ora
from paper_2408_05646_amd import synth

TOL_F32 = 1e-5     # relative L2, fp32 path
TOL_BF16 = 1e-2    # relative L2, bf16 cache with fp32 accumulation


def tdtype(desc):
    return torch.bfloat16 if desc.dtype == ea.EA_BF16 else torch.float32


def quantize(desc, a: np.ndarray) -> np.ndarray:
    """Values as the cache / activations will hold them (float64 view of the rounded numbers)."""
    a32 = np.asarray(a, np.float32)
    return (synth.round_to_bf16(a32) if desc.dtype == ea.EA_BF16 else a32).astype(np.float64)


def to_dev(desc, a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a, np.float32)).to(tdtype(desc)).cuda()


class DeviceCache:
    """Paged pools + page table on the GPU, filled from per-sequence dense arrays."""

    def __init__(self, desc, K_list, V_list, g: np.random.Generator, spare_pages: int = 3, extra_len: int = 0,
                 poison: bool = True):
        P = desc.page_tokens
        B = len(K_list)
        lens = [k.shape[1] for k in K_list]
        self.max_pages = max(1, -(-(max(lens) + extra_len) // P))
        self.pool_pages = B * self.max_pages + spare_pages
        self.k_pool, self.v_pool = ea.alloc_pools(desc, self.pool_pages)
        if poison:   # slots that are never written must not matter
            self.k_pool.fill_(float("nan"))
            self.v_pool.fill_(float("nan"))
        self.page_table_host = synth.random_page_table(g, B, self.max_pages, self.pool_pages)
        self.page_table = torch.from_numpy(self.page_table_host).cuda()
        self.seq_len = torch.tensor(lens, dtype=torch.int32).cuda()
        for b in range(B):
            if lens[b] == 0:
                continue
            ea.cache_scatter(desc, to_dev(desc, K_list[b][None]), to_dev(desc, V_list[b][None]), self.k_pool,
                             self.v_pool, self.page_table[b:b + 1].contiguous())
        torch.cuda.synchronize()


def random_cache(desc, lens, g, k_std=1.0):
    K = [quantize(desc, synth.gaussian(g, (desc.n_kv_heads, n, desc.r_k), k_std)) for n in lens]
    V = [quantize(desc, synth.gaussian(g, (desc.n_kv_heads, n, desc.r_v))) for n in lens]
    return K, V


def assert_close(got: np.ndarray, ref: np.ndarray, tol: float, what: str = ""):
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    err = ora.rel_l2(got, ref)
    rows_g = got.reshape(-1, got.shape[-1])
    rows_r = ref.reshape(-1, ref.shape[-1])
    row_err = np.linalg.norm(rows_g - rows_r, axis=1) / np.maximum(np.linalg.norm(rows_r, axis=1), 1e-300)
    assert err <= tol, f"{what}: rel-L2 {err:.3e} > {tol:.1e}"
    # no single (sequence, head) row may hide behind the others: measured worst rows are about 3e-3 (bf16), so 3x the
    # bar on the whole tensor is already generous
    assert row_err.max() <= 3 * tol, f"{what}: worst row rel-L2 {row_err.max():.3e}"
    return err
