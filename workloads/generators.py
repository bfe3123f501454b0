"""Seeded, counter-based synthetic tensors for the GPTQ layer solver.

Every element is a pure function of (seed, tensor id, row, column), so any tile of any
tensor can be produced on its own, on the CPU or on the GPU, without materialising the rest.
Only integer arithmetic (which wraps identically on every device), exact int->float
conversion and single IEEE multiplications are used, so the CPU and the GPU produce the
same bit patterns.  This module holds none of the quantization method's arithmetic; it is
shared by the CPU oracle's tests and by the GPU path's tests and benchmark.

Distributions
  * "normal": Irwin-Hall(12) -- the sum of twelve independent 16-bit uniforms, centred and
    scaled to unit variance.  It stands in for N(0,1): same mean and variance, excess
    kurtosis -0.1, support clipped at |z| <= 6, resolution 2^-16.
  * channel scales: exp(sigma * z_c), one per input channel, always evaluated on the CPU in
    float64 and rounded to float32 (so both devices see the same float32 values).
  * outlier channels: the k channels whose hash is smallest.
  * post-ReLU-like: |z| with a seeded fraction of entries set to exactly zero.
"""
from __future__ import annotations

import numpy as np
import torch

_M64 = (1 << 64) - 1


def _s64(u: int) -> int:
    """Reinterpret an unsigned 64-bit integer as the signed value torch.int64 stores."""
    u &= _M64
    return u - (1 << 64) if u >= (1 << 63) else u


_C1 = _s64(0xBF58476D1CE4E5B9)
_C2 = _s64(0x94D049BB133111EB)
_GOLD = _s64(0x9E3779B97F4A7C15)


def _lshr(x: torch.Tensor, k: int) -> torch.Tensor:
    """Logical right shift of an int64 tensor."""
    return (x >> k) & ((1 << (64 - k)) - 1)


def _mix64(x: torch.Tensor) -> torch.Tensor:
    """splitmix64 finaliser on int64 tensors (two's-complement wraparound)."""
    x = (x ^ _lshr(x, 30)) * _C1
    x = (x ^ _lshr(x, 27)) * _C2
    return x ^ _lshr(x, 31)


def mix64_int(x: int) -> int:
    """The same finaliser on a Python integer (used for keys and by the generator's tests)."""
    x &= _M64
    x = ((x ^ (x >> 30)) * 0xBF58476D1CE4E5B9) & _M64
    x = ((x ^ (x >> 27)) * 0x94D049BB133111EB) & _M64
    return x ^ (x >> 31)


def _key(seed: int, tensor_id: int) -> int:
    return mix64_int(seed ^ mix64_int(tensor_id + 0x1234567))


def _counters(total_cols: int, row0: int, nrows: int, col0: int, ncols: int, device) -> torch.Tensor:
    r = torch.arange(row0, row0 + nrows, dtype=torch.int64, device=device).unsqueeze(1)
    c = torch.arange(col0, col0 + ncols, dtype=torch.int64, device=device).unsqueeze(0)
    return r * int(total_cols) + c


def random_bits(seed: int, tensor_id: int, total_cols: int, row0: int, nrows: int, col0: int, ncols: int,
                lane: int, device="cpu") -> torch.Tensor:
    """64 random bits (as int64) for each element of the tile; `lane` selects one of several
    independent words per element."""
    ctr = _counters(total_cols, row0, nrows, col0, ncols, device)
    k = _s64(_key(seed, tensor_id))
    return _mix64((ctr * 4 + lane) * _GOLD + k)


def normal_tile(seed: int, tensor_id: int, total_cols: int, row0: int, nrows: int, col0: int, ncols: int,
                device="cpu") -> torch.Tensor:
    """float32 tile of unit-variance Irwin-Hall(12) variates (exactly representable values)."""
    acc = torch.zeros((nrows, ncols), dtype=torch.int64, device=device)
    for lane in range(3):
        h = random_bits(seed, tensor_id, total_cols, row0, nrows, col0, ncols, lane, device)
        acc += (h & 0xFFFF) + (_lshr(h, 16) & 0xFFFF) + (_lshr(h, 32) & 0xFFFF) + _lshr(h, 48)
    # mean of the sum is 6*65535; variance of one 16-bit uniform is (2^32-1)/12 ~ 2^32/12
    return (acc - 6 * 65535).to(torch.float32) * (1.0 / 65536.0)


def zero_mask_tile(seed: int, tensor_id: int, total_cols: int, row0: int, nrows: int, col0: int, ncols: int,
                   zero_fraction: float, device="cpu") -> torch.Tensor:
    """Boolean tile, True where the entry is forced to zero (probability zero_fraction)."""
    h = random_bits(seed, tensor_id, total_cols, row0, nrows, col0, ncols, 3, device)
    thresh = int(round(zero_fraction * (1 << 24)))
    return (h & 0xFFFFFF) < thresh


def channel_scales(seed: int, tensor_id: int, n: int, sigma: float, n_outliers: int, outlier_gain: float) -> torch.Tensor:
    """float32 vector of per-channel multipliers: LogNormal(0, sigma) (sigma == 0 gives ones)
    times outlier_gain on the n_outliers channels with the smallest hash.  CPU only."""
    z = normal_tile(seed, tensor_id + 1000003, 1, 0, n, 0, 1, "cpu").double().numpy()[:, 0]
    s = np.exp(sigma * z) if sigma != 0.0 else np.ones(n)
    if n_outliers > 0:
        h = random_bits(seed, tensor_id + 2000003, 1, 0, n, 0, 1, 0, "cpu").numpy()[:, 0]
        order = np.argsort(h.view(np.uint64), kind="stable")
        s[order[:n_outliers]] *= outlier_gain
    return torch.from_numpy(s.astype(np.float32))


def weight_tile(seed: int, tensor_id: int, r: int, n: int, std: float, dtype: torch.dtype,
                row0: int = 0, nrows: int | None = None, device="cpu") -> torch.Tensor:
    """Rows [row0, row0+nrows) of the r x n weight matrix: dtype(float32(std) * z)."""
    nrows = r - row0 if nrows is None else nrows
    z = normal_tile(seed, tensor_id, n, row0, nrows, 0, n, device)
    return (z * float(np.float32(std))).to(dtype)


def activation_tile(seed: int, tensor_id: int, n: int, m: int, dtype: torch.dtype, scales: torch.Tensor | None,
                    kind: str = "normal", zero_fraction: float = 0.0,
                    row0: int = 0, nrows: int | None = None, col0: int = 0, ncols: int | None = None,
                    device="cpu") -> torch.Tensor:
    """Channels [row0, row0+nrows) x tokens [col0, col0+ncols) of the n x m activation matrix X
    (one row per input channel, tokens contiguous).

    kind "normal":   X = dtype(z * scale_c)
    kind "halfnorm": X = dtype(|z| * scale_c), with a seeded zero_fraction of entries set to 0.
    """
    nrows = n - row0 if nrows is None else nrows
    ncols = m - col0 if ncols is None else ncols
    z = normal_tile(seed, tensor_id, m, row0, nrows, col0, ncols, device)
    if kind == "halfnorm":
        z = z.abs()
        if zero_fraction > 0.0:
            z = torch.where(zero_mask_tile(seed, tensor_id, m, row0, nrows, col0, ncols, zero_fraction, device),
                            torch.zeros_like(z), z)
    elif kind != "normal":
        raise ValueError(kind)
    if scales is not None:
        z = z * scales[row0:row0 + nrows].to(device).unsqueeze(1)
    return z.to(dtype)
