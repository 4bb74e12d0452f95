"""Seeded synthetic sparse-convolution layers (inputs only, no method arithmetic).

The paper evaluates on pruned ImageNet AlexNet / GoogLeNet / ResNet models
(Section 4); those weights are not available, so every layer here is a seeded
synthetic stand-in with the same shape, sparsity level and value distribution.
This module only draws random tensors and lays the nonzeros of the pruned filter
bank out as CSR, one row per output channel over C*R*S columns (Section 2.3, and
the M x CRS filter matrix of Section 2.2).  It is shared by the tests, the bench
and the CPU oracle's callers; it holds none of the convolution, stretching or
padding arithmetic.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

BASE_SEED = 1802_10280


@dataclass(frozen=True)
class LayerSpec:
    """Shape parameters in the paper's notation (Table 1) plus the generator recipe."""

    name: str
    config: int          # index into the workload list (0 = tiny ... 4 = sparsity sweep)
    index: int           # layer index inside that config (seed offset)
    N: int
    C: int
    H: int
    W: int
    M: int
    R: int
    S: int
    stride: int
    pad: int
    sparsity: float
    dist: str = "normal"     # "normal": N(0, sigma=0.05); "uniform": U[-1, 1]
    skew: bool = False       # power-law nnz per output channel (exponent 1.5)
    permute_rows: bool = False

    @property
    def Hp(self) -> int:
        return self.H + 2 * self.pad

    @property
    def Wp(self) -> int:
        return self.W + 2 * self.pad

    @property
    def E(self) -> int:
        return (self.Hp - self.R) // self.stride + 1

    @property
    def F(self) -> int:
        return (self.Wp - self.S) // self.stride + 1

    @property
    def seed(self) -> int:
        return BASE_SEED + self.config * 100 + self.index

    def with_batch(self, N: int) -> "LayerSpec":
        d = dict(self.__dict__)
        d["N"] = N
        return LayerSpec(**d)


def _L(name, config, index, N, C, HW, M, RS, stride, pad, sparsity, **kw):
    return LayerSpec(name, config, index, N, C, HW, HW, M, RS, RS, stride, pad, sparsity, **kw)


# name -> spec.  Config 0: tiny; 1: AlexNet-style; 2: GoogLeNet-style; 3: ResNet-50-style;
# 4: sparsity sweep on one layer (incl. the power-law-skewed variant).
LAYERS = {
    s.name: s
    for s in [
        _L("T1", 0, 0, 1, 16, 14, 32, 3, 1, 1, 0.80, dist="uniform"),
        _L("A1b1", 1, 0, 1, 256, 13, 384, 3, 1, 1, 0.65),
        _L("A2b1", 1, 1, 1, 384, 13, 384, 3, 1, 1, 0.65),
        _L("A3b1", 1, 2, 1, 384, 13, 256, 3, 1, 1, 0.65),
        _L("A1b64", 1, 0, 64, 256, 13, 384, 3, 1, 1, 0.65),
        _L("A2b64", 1, 1, 64, 384, 13, 384, 3, 1, 1, 0.65),
        _L("A3b64", 1, 2, 64, 384, 13, 256, 3, 1, 1, 0.65),
        _L("G1", 2, 0, 32, 192, 28, 64, 1, 1, 0, 0.70),
        _L("G3", 2, 1, 32, 96, 28, 128, 3, 1, 1, 0.70),
        _L("G5", 2, 2, 32, 16, 28, 32, 5, 1, 2, 0.70),
        _L("R56", 3, 0, 32, 64, 56, 64, 3, 1, 1, 0.80),
        _L("R28", 3, 1, 32, 128, 28, 128, 3, 1, 1, 0.80),
        _L("R14", 3, 2, 32, 256, 14, 256, 3, 1, 1, 0.80),
        _L("R7", 3, 3, 32, 512, 7, 512, 3, 1, 1, 0.80),
        _L("R56s2", 3, 4, 32, 128, 56, 128, 3, 2, 1, 0.80),
        # head of a three-layer chain (C56 -> R56s2 -> R28): each output is the next input
        _L("C56", 3, 5, 32, 64, 56, 128, 3, 1, 1, 0.80),
        _L("S50", 4, 0, 64, 256, 28, 256, 3, 1, 1, 0.50),
        _L("S70", 4, 1, 64, 256, 28, 256, 3, 1, 1, 0.70),
        _L("S80", 4, 2, 64, 256, 28, 256, 3, 1, 1, 0.80),
        _L("S90", 4, 3, 64, 256, 28, 256, 3, 1, 1, 0.90),
        _L("S95", 4, 4, 64, 256, 28, 256, 3, 1, 1, 0.95),
        _L("S80skew", 4, 5, 64, 256, 28, 256, 3, 1, 1, 0.80, skew=True),
        _L("S80skewperm", 4, 5, 64, 256, 28, 256, 3, 1, 1, 0.80, skew=True, permute_rows=True),
    ]
}

CONFIG_LAYERS = {
    "tiny": ["T1"],
    "alexnet_b1": ["A1b1", "A2b1", "A3b1"],
    "alexnet_b64": ["A1b64", "A2b64", "A3b64"],
    "googlenet": ["G1", "G3", "G5"],
    "resnet": ["R56", "R28", "R14", "R7", "R56s2"],
    "chain": ["C56", "R56s2", "R28"],
    "sweep": ["S50", "S70", "S80", "S90", "S95", "S80skew", "S80skewperm"],
}


@dataclass
class Layer:
    """A generated layer: dense pruned filter bank, its CSR form, and the input."""

    spec: LayerSpec
    weight: np.ndarray            # (M, C, R, S) float32, zeros where pruned
    rowptr: np.ndarray            # (M+1,) int32
    colidx: np.ndarray            # (nnz,) int32, column j = (c*R + r)*S + s, ascending per row
    value: np.ndarray             # (nnz,) float32
    input: np.ndarray             # (N, C, H, W) float32
    bias: np.ndarray = field(default=None)  # (M,) float32

    @property
    def nnz(self) -> int:
        return int(self.rowptr[-1])


def skewed_row_nnz(M: int, cols: int, total: int) -> np.ndarray:
    """nnz per row ~ K * (m+1)^-1.5, clipped to [1, cols], with K solved so the sum is `total`."""
    ranks = np.arange(1, M + 1, dtype=np.float64) ** -1.5

    def rows(K):
        return np.clip(np.rint(K * ranks), 1, cols).astype(np.int64)

    lo, hi = 1.0, float(cols) * M * 64.0
    for _ in range(200):
        mid = 0.5 * (lo + hi)
        if rows(mid).sum() < total:
            lo = mid
        else:
            hi = mid
    n = rows(hi)
    # fix the rounding residue on the smallest rows that can take it
    diff = int(n.sum() - total)
    i = M - 1
    while diff != 0 and i >= 0:
        step = -1 if diff > 0 else 1
        if 1 <= n[i] + step <= cols:
            n[i] += step
            diff += step
        i -= 1
    return n


def dense_to_csr(weight: np.ndarray):
    """CSR of the M x (C*R*S) filter matrix: the nonzeros of each output channel's filter,
    row-major over (c, r, s), ascending column index (Section 2.3)."""
    M = weight.shape[0]
    flat = weight.reshape(M, -1)
    rows, cols = np.nonzero(flat)            # row-major order: ascending cols inside each row
    rowptr = np.zeros(M + 1, dtype=np.int32)
    np.cumsum(np.bincount(rows, minlength=M), out=rowptr[1:])
    return rowptr, cols.astype(np.int32), flat[rows, cols].astype(np.float32)


def make_weight(spec: LayerSpec, rng: np.random.Generator) -> np.ndarray:
    M, cols = spec.M, spec.C * spec.R * spec.S
    if spec.skew:
        total = int(round(M * cols * (1.0 - spec.sparsity)))
        per_row = skewed_row_nnz(M, cols, total)
        if spec.permute_rows:
            per_row = per_row[rng.permutation(M)]
        mask = np.zeros((M, cols), dtype=bool)
        for m in range(M):
            mask[m, rng.choice(cols, size=int(per_row[m]), replace=False)] = True
    else:
        mask = rng.random((M, cols)) >= spec.sparsity
    if spec.dist == "uniform":
        vals = rng.uniform(-1.0, 1.0, size=(M, cols))
    else:
        vals = rng.normal(0.0, 0.05, size=(M, cols))
    w = np.where(mask, vals, 0.0).astype(np.float32)
    # a drawn value that rounds to exactly 0 would silently drop out of the CSR; keep it nonzero
    w[mask & (w == 0.0)] = np.float32(1e-3)
    return w.reshape(M, spec.C, spec.R, spec.S)


def make_input(spec: LayerSpec, rng: np.random.Generator, N: int | None = None) -> np.ndarray:
    """Post-ReLU look: U[0,1] with an independent Bernoulli(0.5) zero mask."""
    shape = (spec.N if N is None else N, spec.C, spec.H, spec.W)
    x = rng.random(shape, dtype=np.float32)
    x *= rng.random(shape, dtype=np.float32) >= 0.5
    return x


def make_layer(spec: LayerSpec | str, N: int | None = None, with_input: bool = True) -> Layer:
    if isinstance(spec, str):
        spec = LAYERS[spec]
    if N is not None:
        spec = spec.with_batch(N)
    rng = np.random.Generator(np.random.PCG64(spec.seed))
    w = make_weight(spec, rng)
    rowptr, colidx, value = dense_to_csr(w)
    bias = rng.normal(0.0, 0.1, size=spec.M).astype(np.float32)
    x = make_input(spec, rng) if with_input else None
    return Layer(spec, w, rowptr, colidx, value, x, bias)


def custom_layer(N, C, H, W, M, R, S, stride, pad, sparsity, seed, dist="uniform",
                 name="custom") -> Layer:
    spec = LayerSpec(name, 9, 0, N, C, H, W, M, R, S, stride, pad, sparsity, dist=dist)
    rng = np.random.Generator(np.random.PCG64(seed))
    w = make_weight(spec, rng)
    rowptr, colidx, value = dense_to_csr(w)
    bias = rng.normal(0.0, 0.1, size=M).astype(np.float32)
    return Layer(spec, w, rowptr, colidx, value, make_input(spec, rng), bias)
