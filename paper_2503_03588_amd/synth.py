"""Seeded synthetic inputs shared by the tests, the smoke check and the bench.

Holds no attention arithmetic: it only draws i.i.d. Gaussian tensors of the
requested shape on the CPU from a seeded generator, casts them to the storage
type, and converts storage between torch and NumPy views so that the GPU
library and the CPU checker see the same bits.
"""
from __future__ import annotations

import numpy as np
import torch

_DTYPES = {"bf16": torch.bfloat16, "f32": torch.float32}


def gaussian(shape, dtype: str, seed: int, std: float = 1.0) -> torch.Tensor:
    """CPU tensor ~ N(0, std^2) of `shape`, drawn in fp32 from `seed`, then
    rounded to `dtype` ("bf16" or "f32")."""
    gen = torch.Generator(device="cpu")
    gen.manual_seed(int(seed))
    x = torch.randn(tuple(shape), generator=gen, dtype=torch.float32)
    if std != 1.0:
        x = x * std
    return x.to(_DTYPES[dtype])


def qkv(batch, n_q_heads, n_kv_heads, seq_len, head_dim, dtype: str, seed: int, std: float = 1.0):
    """Q [b,Hq,N,D] and K, V [b,Hkv,N,D]; seeds seed, seed+10007, seed+20011."""
    q = gaussian((batch, n_q_heads, seq_len, head_dim), dtype, seed, std)
    k = gaussian((batch, n_kv_heads, seq_len, head_dim), dtype, seed + 10007, std)
    v = gaussian((batch, n_kv_heads, seq_len, head_dim), dtype, seed + 20011, std)
    return q, k, v


def decode_inputs(batch, n_q_heads, n_kv_heads, capacity, head_dim, dtype: str, seed: int):
    """q [b,Hq,D] and K/V caches [b,Hkv,capacity,D]."""
    q = gaussian((batch, n_q_heads, head_dim), dtype, seed)
    k = gaussian((batch, n_kv_heads, capacity, head_dim), dtype, seed + 10007)
    v = gaussian((batch, n_kv_heads, capacity, head_dim), dtype, seed + 20011)
    return q, k, v


def to_numpy_storage(t: torch.Tensor) -> np.ndarray:
    """CPU view of a tensor's stored bits: float32 arrays as they are,
    bfloat16 as uint16 bit patterns."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()
