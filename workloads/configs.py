"""The synthetic, paper-shaped layer workloads (shapes, distributions, seeds).

A `Layer` names one linear layer to quantize: its weight matrix, the activation matrix whose
Hessian it uses, and the quantization settings.  Shapes follow the public OPT / BLOOM model
dimensions; the calibration set is 128 sequences x 2048 tokens = 262144 tokens.  These tensors
stand in for C4-calibrated real layers.  No method arithmetic lives here.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import torch

from . import generators as g

BASE_SEED = 17323
TOKENS = 128 * 2048


@dataclass(frozen=True)
class Activations:
    tensor_id: int
    n: int                       # input channels (= d_col of the layer)
    m: int                       # tokens
    dtype: torch.dtype = torch.float16
    kind: str = "normal"         # "normal" | "halfnorm"
    zero_fraction: float = 0.0
    sigma: float = 0.0           # LogNormal(0, sigma) per-channel scale
    n_outliers: int = 0
    outlier_gain: float = 1.0

    def scales(self) -> torch.Tensor | None:
        if self.sigma == 0.0 and self.n_outliers == 0:
            return None
        return g.channel_scales(BASE_SEED, self.tensor_id, self.n, self.sigma, self.n_outliers, self.outlier_gain)

    def tile(self, row0=0, nrows=None, col0=0, ncols=None, device="cpu", scales=None) -> torch.Tensor:
        s = self.scales() if scales is None else scales
        return g.activation_tile(BASE_SEED, self.tensor_id, self.n, self.m, self.dtype, s, self.kind,
                                 self.zero_fraction, row0, nrows, col0, ncols, device)


@dataclass(frozen=True)
class Layer:
    name: str
    tensor_id: int
    r: int                       # d_row (output features)
    n: int                       # d_col (input features)
    x: Activations
    std: float = 0.02
    dtype: torch.dtype = torch.float16
    bits: int = 4
    grid: str = "minmax"         # "minmax" (asymmetric) | "ternary"
    group: int = 0               # 0 = one grid per row
    block: int = 128
    percdamp: float = 0.01

    def weights(self, row0=0, nrows=None, device="cpu") -> torch.Tensor:
        return g.weight_tile(BASE_SEED, self.tensor_id, self.r, self.n, self.std, self.dtype, row0, nrows, device)


def _lognormal_x(tid, n, m=TOKENS, outlier_frac=0.001, gain=30.0):
    return Activations(tid, n, m, sigma=0.5, n_outliers=max(1, round(outlier_frac * n)) if outlier_frac else 0,
                       outlier_gain=gain)


def _relu_x(tid, n, m=TOKENS):
    return Activations(tid, n, m, kind="halfnorm", zero_fraction=0.6)


def config1():
    x = Activations(101, 256, 4096, dtype=torch.float32, n_outliers=4, outlier_gain=20.0)
    return [Layer("tiny", 100, 256, 256, x, std=0.02, dtype=torch.float32, bits=4)]


def config2(m=TOKENS):
    return [Layer("opt6.7b_attn", 200, 4096, 4096, _lognormal_x(201, 4096, m), std=0.02, bits=4)]


def config3(m=TOKENS):
    return [
        Layer("opt175b_fc1", 300, 49152, 12288, _lognormal_x(301, 12288, m), std=0.015, bits=3),
        Layer("opt175b_fc2", 310, 12288, 49152, _relu_x(311, 49152, m), std=0.015, bits=3),
    ]


def config4(m=TOKENS):
    out = []
    for grid, bits in (("minmax", 2), ("ternary", 2)):
        out.append(Layer(f"bloom176b_qkv_{grid}", 400, 43008, 14336, _lognormal_x(401, 14336, m), std=0.015,
                         bits=bits, grid=grid, group=128))
        out.append(Layer(f"bloom176b_out_{grid}", 410, 14336, 14336, _lognormal_x(411, 14336, m), std=0.015,
                         bits=bits, grid=grid, group=128))
    return out


def config5(m=TOKENS, bits=3):
    xa = _lognormal_x(501, 12288, m)
    return [
        Layer("q", 500, 12288, 12288, xa, std=0.015, bits=bits),
        Layer("k", 502, 12288, 12288, xa, std=0.015, bits=bits),
        Layer("v", 504, 12288, 12288, xa, std=0.015, bits=bits),
        Layer("out", 510, 12288, 12288, _lognormal_x(511, 12288, m), std=0.015, bits=bits),
        Layer("fc1", 520, 49152, 12288, _lognormal_x(521, 12288, m), std=0.015, bits=bits),
        Layer("fc2", 530, 12288, 49152, _relu_x(531, 49152, m), std=0.015, bits=bits),
    ]


def scaled_twin(layer: Layer, n: int, r: int | None = None, m: int | None = None) -> Layer:
    """Same distributions and settings at a size a float64 CPU oracle finishes whole:
    n input channels, r rows (default: keep the aspect ratio), m = 16 n tokens."""
    r = max(1, layer.r * n // layer.n) if r is None else r
    m = 16 * n if m is None else m
    x = layer.x
    nout = 0 if x.n_outliers == 0 else max(1, round(x.n_outliers * n / x.n))
    return replace(layer, name=layer.name + f"_twin{n}", r=r, n=n, x=replace(x, n=n, m=m, n_outliers=nout))


def materialize(layer: Layer, device, max_elems: int = 1 << 27):
    """(W, X) of a layer as tensors on `device`, generated tile by tile so that the generator's
    int64 temporaries stay small (X of the largest layer is 24 GiB of fp16)."""
    scales = layer.x.scales()
    X = torch.empty((layer.n, layer.x.m), dtype=layer.x.dtype, device=device)
    rows = max(1, min(layer.n, max_elems // max(layer.x.m, 1)))
    for r0 in range(0, layer.n, rows):
        nr = min(rows, layer.n - r0)
        X[r0:r0 + nr] = layer.x.tile(row0=r0, nrows=nr, device=device, scales=scales)
    W = torch.empty((layer.r, layer.n), dtype=layer.dtype, device=device)
    rows = max(1, min(layer.r, max_elems // layer.n))
    for r0 in range(0, layer.r, rows):
        nr = min(rows, layer.r - r0)
        W[r0:r0 + nr] = layer.weights(row0=r0, nrows=nr, device=device)
    return W, X
