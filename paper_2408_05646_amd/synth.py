"""Seeded synthetic inputs with the shapes and statistics of the paper's workloads.

This module only DRAWS inputs (Gaussian tensors, orthonormal bases, low-rank
plus noise samples, page tables) and converts number formats.  It contains none
of the method's arithmetic (no folding, no projection, no attention): both the
HIP path and the CPU checker are handed the arrays made here.

Random numbers come from numpy's counter-based Philox generator keyed by
(base seed, config index, stream ids), so any tensor can be regenerated alone.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Tuple

import numpy as np

BASE_SEED = 20240805


def rng(*stream: int) -> np.random.Generator:
    """Counter-based generator for the stream (config, layer, tensor id, ...)."""
    key = np.random.SeedSequence([BASE_SEED, *[int(s) for s in stream]]).generate_state(2, dtype=np.uint64)
    return np.random.Generator(np.random.Philox(key=key))


@dataclass(frozen=True)
class LayerShape:
    """Shape of one attention layer and of the batch it serves."""
    name: str
    d_model: int
    n_heads: int
    n_kv_heads: int
    d_head: int
    r_k: int
    r_v: int
    batch: int
    n_ctx: int
    dtype: str          # "f32" or "bf16"
    n_layers: int = 1


# The five workload shapes (Llama-2-7B-like attention layers; see the paper's
# Introduction for the B=16, n=32k example they are built around).
CFG1 = LayerShape("tiny-f32", 256, 4, 4, 64, 32, 32, 1, 256, "f32")
CFG1_FULL = LayerShape("tiny-f32-fullrank", 256, 4, 4, 64, 64, 64, 1, 256, "f32")
CFG2 = LayerShape("llama7b-decode-4k", 4096, 32, 32, 128, 80, 80, 16, 4096, "bf16")
CFG3 = LayerShape("llama7b-decode-32k", 4096, 32, 32, 128, 80, 80, 16, 32768, "bf16", n_layers=32)
CFG3_FULLRANK = LayerShape("llama7b-decode-32k-fullrank", 4096, 32, 32, 128, 128, 128, 16, 32768, "bf16")
CFG4 = LayerShape("llama7b-prefill-8k", 4096, 32, 32, 128, 64, 64, 4, 8192, "bf16")
CFG5 = LayerShape("gqa-hetero-16k", 4096, 32, 8, 128, 80, 80, 8, 16384, "bf16", n_layers=32)
CFG5_RANKS = (48, 64, 80, 96, 112)


def cfg5_layer_ranks(n_layers: int = 32) -> Tuple[Tuple[int, int], ...]:
    """Per-layer (r_k, r_v), drawn independently and uniformly from CFG5_RANKS."""
    g = rng(5, 0)
    rk = g.choice(CFG5_RANKS, size=n_layers)
    rv = g.choice(CFG5_RANKS, size=n_layers)
    return tuple((int(a), int(b)) for a, b in zip(rk, rv))


def gaussian(g: np.random.Generator, shape, std: float = 1.0) -> np.ndarray:
    return g.standard_normal(shape) * std


def orthonormal_basis(g: np.random.Generator, d_head: int, r: int) -> np.ndarray:
    """First r columns of Q from the QR factorisation of a Gaussian d_head x d_head
    matrix, signs fixed so that diag(R) > 0.  Columns are orthonormal."""
    q, rr = np.linalg.qr(g.standard_normal((d_head, d_head)))
    q = q * np.sign(np.diag(rr))[None, :]
    return np.ascontiguousarray(q[:, :r])


def lowrank_plus_noise(g: np.random.Generator, n: int, directions: np.ndarray, sigma: float) -> np.ndarray:
    """n samples z A + sigma eps: `directions` A is [r, d_head] with orthonormal rows,
    z ~ N(0, I_r) (variance 1 along each dominant direction), eps ~ N(0, I_d_head)."""
    r, d_head = directions.shape
    return g.standard_normal((n, r)) @ directions + sigma * g.standard_normal((n, d_head))


def top_singular_basis(samples: np.ndarray, r: int) -> np.ndarray:
    """[d_head, r]: the r leading right singular vectors of a [n_samples, d_head]
    sample matrix (no mean-centring), via LAPACK."""
    _, _, vt = np.linalg.svd(samples, full_matrices=False)
    return np.ascontiguousarray(vt[:r].T)


def random_page_table(g: np.random.Generator, batch: int, pages_per_seq: int, pool_pages: int) -> np.ndarray:
    """[batch, pages_per_seq] int32: distinct physical pages in seeded random order."""
    assert batch * pages_per_seq <= pool_pages
    perm = g.permutation(pool_pages)[:batch * pages_per_seq]
    return perm.reshape(batch, pages_per_seq).astype(np.int32)


# ---- number formats ---------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float -> bfloat16 bit patterns (uint16), round to nearest even; NaN stays NaN."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = (u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))) >> np.uint32(16)
    nan = (u & np.uint32(0x7FFFFFFF)) > np.uint32(0x7F800000)
    return np.where(nan, (u >> np.uint32(16)) | np.uint32(0x40), rounded).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Values of x rounded to the nearest bfloat16, returned as float32."""
    return bf16_bits_to_f32(f32_to_bf16_bits(x))
