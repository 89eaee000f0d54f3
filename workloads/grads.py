"""Seeded gradient generators.

Every draw is addressed by (config id, replica r, micro-step k, parameter p),
so a test can regenerate any single tensor of a multi-gigabyte workload
without producing the rest.  Storage formats on the host:

    DT_FP32 -> numpy float32
    DT_FP16 -> numpy float16
    DT_BF16 -> numpy uint16 holding the upper 16 bits of a binary32 value

Only random draws and format packing happen here.
"""
from __future__ import annotations

import numpy as np

DT_FP32, DT_FP16, DT_BF16 = 0, 1, 2
ESIZE = {DT_FP32: 4, DT_FP16: 2, DT_BF16: 2}
NP_STORAGE = {DT_FP32: np.float32, DT_FP16: np.float16, DT_BF16: np.uint16}


def f32_to_storage_trunc(x: np.ndarray, dtype: int) -> np.ndarray:
    """Bring float32 samples into a storage format *for use as inputs*.
    fp16 uses numpy's conversion; bf16 keeps the upper 16 bits (truncation),
    which is enough to produce valid bf16 input values."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == DT_FP32:
        return x
    if dtype == DT_FP16:
        return x.astype(np.float16)
    if dtype == DT_BF16:
        return (x.view(np.uint32) >> np.uint32(16)).astype(np.uint16)
    raise ValueError(f"unknown dtype code {dtype}")


def _rng(config_id: int, r: int, k: int, p: int) -> np.random.Generator:
    return np.random.default_rng(np.random.SeedSequence([config_id, r, k, p]))


def gaussian_grad(config_id: int, r: int, k: int, p: int, numel: int,
                  sigma: float, dtype: int = DT_FP32) -> np.ndarray:
    """N(0, sigma^2) gradient of parameter p, replica r, micro-step k."""
    x = _rng(config_id, r, k, p).standard_normal(numel, dtype=np.float32)
    x *= np.float32(sigma)
    return f32_to_storage_trunc(x, dtype)


def gaussian_replica(config_id: int, r: int, k: int, numels, sigma: float,
                     dtype: int = DT_FP32):
    """All gradients of one replica, in registration order."""
    return [gaussian_grad(config_id, r, k, p, n, sigma, dtype)
            for p, n in enumerate(numels)]


def tag_grad(r: int, start: int, numel: int, dtype: int = DT_FP32) -> np.ndarray:
    """Unique finite tags: element j of a tensor whose first element has
    model-wide index `start` gets a bit pattern derived from (start + j, r).
    Used to show that packing and unpacking move every element to the right
    place.  No NaN or infinity is produced."""
    idx = np.arange(start, start + numel, dtype=np.uint64)
    if dtype == DT_FP32:
        # odd multiplier: a bijection of the index modulo 2^32
        b32 = ((idx * np.uint64(2654435761) + np.uint64(40503 * r + 1))
               & np.uint64(0xFFFFFFFF)).astype(np.uint32)
        expo_all_ones = (b32 & np.uint32(0x7F800000)) == np.uint32(0x7F800000)
        b32 = np.where(expo_all_ones, b32 & np.uint32(0xBFFFFFFF), b32).astype(np.uint32)
        return b32.view(np.float32)
    bits = ((idx * np.uint64(40503) + np.uint64(977 * r + 13)) & np.uint64(0xFFFF)).astype(np.uint16)
    if dtype == DT_FP16:
        expo_all_ones = (bits & np.uint16(0x7C00)) == np.uint16(0x7C00)
        bits = np.where(expo_all_ones, bits & np.uint16(0xBFFF), bits).astype(np.uint16)
        return bits.view(np.float16)
    if dtype == DT_BF16:
        expo_all_ones = (bits & np.uint16(0x7F80)) == np.uint16(0x7F80)
        return np.where(expo_all_ones, bits & np.uint16(0xBFFF), bits).astype(np.uint16)
    raise ValueError(f"unknown dtype code {dtype}")


def integer_grad(seed: int, r: int, k: int, p: int, numel: int, bound: int,
                 dtype: int = DT_FP32) -> np.ndarray:
    """Integer-valued gradients drawn uniformly from [-bound, bound]."""
    rng = np.random.default_rng(np.random.SeedSequence([seed, r, k, p, 7]))
    v = rng.integers(-bound, bound + 1, size=numel).astype(np.float32)
    return f32_to_storage_trunc(v, dtype)


def linear_regression_problem(seed: int, d: int = 16, batch: int = 64):
    """Inputs of the toy model y_hat = X w + b with mean-squared-error loss
    (the nn.Linear + MSELoss example of the paper's API section), float64."""
    rng = np.random.default_rng(np.random.SeedSequence([seed, 1001]))
    X = rng.standard_normal((batch, d))
    w = rng.standard_normal(d)
    b = float(rng.standard_normal())
    y = rng.standard_normal(batch)
    return X, w, b, y


def unused_param_set(seed: int, n: int, fraction: float = 0.1):
    """Seeded choice of parameters that never get a ready mark."""
    rng = np.random.default_rng(np.random.SeedSequence([seed, 2002]))
    size = int(n * fraction)
    return sorted(int(i) for i in rng.choice(n, size=size, replace=False))
