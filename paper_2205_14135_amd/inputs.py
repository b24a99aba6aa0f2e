"""Seeded synthetic inputs for the attention tests and benchmarks.

This module only draws numbers and builds index structures; it contains none
of the attention arithmetic and is the one module that both the CPU oracle's
tests and the GPU path's callers use.

The paper's attention benchmarks run on random Q, K, V (Appendix E.6,
"Setup"); its model workloads (BERT-large, GPT-2, long-range tasks) are
represented here by i.i.d. N(0,1) tensors of the same shapes, rounded to the
kernel's input type so that the oracle and the GPU see identical values.
"""
from __future__ import annotations

import numpy as np

BASE_SEED = 20220527
BASE_DROPOUT_SEED = 0x5EED0000


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even); returns float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    lsb = (u >> np.uint64(16)) & np.uint64(1)
    u = (u + np.uint64(0x7FFF) + lsb) & np.uint64(0xFFFF0000)
    return u.astype(np.uint32).view(np.float32).reshape(x.shape)


def round_to_fp16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest float16; returns float32."""
    return np.asarray(x, dtype=np.float32).astype(np.float16).astype(np.float32)


def round_to(x: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "bf16":
        return round_to_bf16(x)
    if dtype == "fp16":
        return round_to_fp16(x)
    raise ValueError(f"unknown dtype {dtype!r}")


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of float32 values that are already bf16-representable."""
    return (np.ascontiguousarray(x, dtype=np.float32).view(np.uint32) >> 16).astype(np.uint16)


def gaussian_tensors(B, H, N, d, dtype, seed, names=("Q", "K", "V", "dO")):
    """i.i.d. N(0,1) tensors [B, H, N, d], rounded to `dtype`, as float32 arrays."""
    rng = np.random.default_rng(seed)
    out = {}
    for name in names:
        x = rng.standard_normal((B, H, N, d), dtype=np.float32)
        out[name] = round_to(x, dtype)
    return out


def butterfly_block_mask(T: int) -> np.ndarray:
    """uint8 [T, T] block mask: keep (i, j) iff |i-j| <= 1, or i xor j is a power of two, or j == 0."""
    i = np.arange(T)[:, None]
    j = np.arange(T)[None, :]
    x = i ^ j
    pow2 = (x != 0) & ((x & (x - 1)) == 0)
    keep = (np.abs(i - j) <= 1) | pow2 | (j == 0)
    return keep.astype(np.uint8)


def to_torch(x: np.ndarray, dtype: str, device="cpu"):
    """float32 array of representable values -> torch tensor of the 16-bit type."""
    import torch
    tdt = {"bf16": torch.bfloat16, "fp16": torch.float16}[dtype]
    return torch.from_numpy(np.ascontiguousarray(x)).to(device=device, dtype=tdt)


# The five benchmark configurations (shapes only; index = position in the list).
CONFIGS = {
    "C1": dict(B=1, H=1, N=128, d=64, dtype="fp16", causal=False, p_drop=0.0),
    "C2": dict(B=16, H=16, N=512, d=64, dtype="fp16", causal=False, p_drop=0.1),
    "C3": dict(B=8, H=16, N=1024, d=64, dtype="bf16", causal=True, p_drop=0.1),
    "C3_d128": dict(B=8, H=8, N=1024, d=128, dtype="bf16", causal=True, p_drop=0.1),
}


def sweep_points(tokens=16384, H=16):
    """(B, N) pairs of the sequence-length sweep with B*N fixed."""
    return [(tokens // n, n) for n in (128, 256, 512, 1024, 2048, 4096, 8192, 16384)]
