"""Seeded synthetic inputs for the LSP compress / decompress-apply path.

This module only *draws inputs* (gradients, weights, sparse projectors in ELL
layout, subspace matrices).  It contains none of the method's arithmetic: no
projection, no accumulation.  Both the CPU oracle's tests and the HIP path's
tests/bench take their inputs from here so that the two sides see identical
bits; neither side's code is imported here.

Notation (this repository's letters; the paper swaps them):
    m x n   shape of the gradient G and the weight W
    r       subspace size  (columns of P and Q; S is r x r)   -- paper's "d"
    d       nonzeros per projector row                         -- paper's "r"

Projector construction follows the paper's random initialisation of
(d,r)-sparse projectors ("Learned sparse projectors" paragraph): every row gets
d nonzero positions drawn at random and Gaussian values.  The scale is read as
standard deviation 1/sqrt(d) (variance 1/d), the only reading under which
E[P P^T] = I, i.e. the unbiasedness that paragraph claims.

Storage types: fp32 arrays are numpy float32; fp16 arrays are numpy float16;
bf16 arrays are numpy uint16 holding the bf16 bit pattern (numpy has no bf16).
Everything is generated in fp32 and rounded to nearest-even once.
"""
from __future__ import annotations

import dataclasses
import math
from typing import List, Optional, Tuple

import numpy as np

DTYPES = ("f32", "f16", "bf16")
DTYPE_CODE = {"f32": 0, "f16": 1, "bf16": 2}   # matches lsp_dtype in include/lsp.h
DTYPE_SIZE = {"f32": 4, "f16": 2, "bf16": 2}


# --------------------------------------------------------------------------
# storage-type helpers (pure bit manipulation, no arithmetic of the method)
# --------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 -> bf16 (nearest, ties to even); returns uint16 bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    nan = np.isnan(x)
    rounded = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    out = rounded.astype(np.uint16)
    if nan.any():
        out = np.where(nan, np.uint16(0x7FC0), out)
    return out


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns (uint16) to float32."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32)


def to_storage(x32: np.ndarray, dtype: str) -> np.ndarray:
    """Round an fp32 array once into the storage type named by `dtype`."""
    if dtype == "f32":
        return np.ascontiguousarray(x32, dtype=np.float32)
    if dtype == "f16":
        return np.ascontiguousarray(x32, dtype=np.float32).astype(np.float16)
    if dtype == "bf16":
        return f32_to_bf16_bits(x32)
    raise ValueError(f"unknown dtype {dtype!r}")


def storage_to_f64(x: np.ndarray, dtype: str) -> np.ndarray:
    """Exact widening of a storage array to float64 (for checks, not for the oracle's C code)."""
    if dtype == "f32":
        return x.astype(np.float64)
    if dtype == "f16":
        return x.astype(np.float64)
    if dtype == "bf16":
        return bf16_bits_to_f32(x).astype(np.float64)
    raise ValueError(dtype)


def ulp_of(x64: np.ndarray, dtype: str) -> np.ndarray:
    """Spacing of the storage format at |x| (subnormal spacing below the smallest normal)."""
    p, emin = {"f32": (24, -126), "f16": (11, -14), "bf16": (8, -126)}[dtype]
    ax = np.abs(np.asarray(x64, dtype=np.float64))
    e = np.floor(np.log2(np.maximum(ax, 2.0 ** emin)))
    e = np.maximum(e, emin)
    return np.exp2(e - (p - 1))


# --------------------------------------------------------------------------
# projectors
# --------------------------------------------------------------------------
def _zipf_cdf(r: int, s: float) -> np.ndarray:
    w = np.arange(1, r + 1, dtype=np.float64) ** (-s)
    c = np.cumsum(w)
    return c / c[-1]


def ell_projector(rows: int, r: int, d: int, rng: np.random.Generator,
                  index_dist: str = "uniform", zipf_s: float = 1.1,
                  value_mode: str = "normal") -> Tuple[np.ndarray, np.ndarray]:
    """Draw one sparse projector in ELL layout: idx int32 [rows][d], val float32 [rows][d].

    index_dist:
      "distinct" d distinct columns per row, uniform without replacement
      "uniform"  d i.i.d. uniform columns per row (duplicates possible; they sum)
      "zipf"     d i.i.d. columns per row from a bounded Zipf law
                 Pr[col = k-1] ~ k^(-zipf_s), k = 1..r (hot columns are the low indices)
    value_mode:
      "normal"   N(0, variance 1/d)
      "ones"     all 1.0 (selection projectors when d == 1)
      "smallint" integers in [-3, 3] (exactly representable everywhere)
    """
    if d > r and index_dist == "distinct":
        raise ValueError("d distinct columns need d <= r")
    if index_dist == "distinct":
        # argsort of uniform keys = uniform random permutation; keep first d
        keys = rng.random((rows, r))
        idx = np.argsort(keys, axis=1, kind="stable")[:, :d]
    elif index_dist == "uniform":
        idx = rng.integers(0, r, size=(rows, d))
    elif index_dist == "zipf":
        cdf = _zipf_cdf(r, zipf_s)
        u = rng.random((rows, d))
        idx = np.minimum(np.searchsorted(cdf, u, side="left"), r - 1)
    else:
        raise ValueError(index_dist)
    if value_mode == "normal":
        val = rng.standard_normal((rows, d)) * (1.0 / math.sqrt(d))
    elif value_mode == "ones":
        val = np.ones((rows, d))
    elif value_mode == "smallint":
        val = rng.integers(-3, 4, size=(rows, d)).astype(np.float64)
    else:
        raise ValueError(value_mode)
    return (np.ascontiguousarray(idx, dtype=np.int32),
            np.ascontiguousarray(val, dtype=np.float32))


def permutation_projector(rows: int, rng: np.random.Generator) -> Tuple[np.ndarray, np.ndarray]:
    """d = 1, r = rows, value 1, the column map a permutation."""
    perm = rng.permutation(rows).astype(np.int32).reshape(rows, 1)
    return np.ascontiguousarray(perm), np.ones((rows, 1), dtype=np.float32)


# --------------------------------------------------------------------------
# dense operands
# --------------------------------------------------------------------------
def gaussian_matrix(m: int, n: int, std: float, dtype: str, rng: np.random.Generator,
                    heavy_row_frac: float = 0.0, heavy_row_scale: float = 100.0) -> np.ndarray:
    """m x n matrix ~ N(0, std^2) drawn in fp32, optional heavy rows, rounded once to `dtype`."""
    x = rng.standard_normal((m, n), dtype=np.float32) * np.float32(std)
    if heavy_row_frac > 0.0:
        k = int(math.ceil(heavy_row_frac * m))
        rows = rng.choice(m, size=k, replace=False)
        x[rows, :] *= np.float32(heavy_row_scale)
    return to_storage(x, dtype)


def integer_matrix(m: int, n: int, lo: int, hi: int, dtype: str, rng: np.random.Generator) -> np.ndarray:
    """Integer-valued matrix in [lo, hi]; exactly representable in every storage type when small."""
    x = rng.integers(lo, hi + 1, size=(m, n)).astype(np.float32)
    return to_storage(x, dtype)


# --------------------------------------------------------------------------
# one matrix problem, and the five benchmark configurations
# --------------------------------------------------------------------------
@dataclasses.dataclass
class Problem:
    """Everything one compress + decompress-apply call pair needs."""
    name: str
    m: int
    n: int
    r: int
    d: int
    dtype: str
    G: np.ndarray          # storage array m x n
    W: np.ndarray          # storage array m x n
    P_idx: np.ndarray      # int32 [m][d]
    P_val: np.ndarray      # float32 [m][d]
    Q_idx: np.ndarray      # int32 [n][d]
    Q_val: np.ndarray      # float32 [n][d]
    S_in: np.ndarray       # float32 r x r, an update to decompress that is independent of G

    @property
    def compress_bytes(self) -> int:
        sz = DTYPE_SIZE[self.dtype]
        return self.m * self.n * sz + (self.m + self.n) * self.d * 8 + self.r * self.r * 4

    @property
    def decompress_bytes(self) -> int:
        sz = DTYPE_SIZE[self.dtype]
        return 2 * self.m * self.n * sz + (self.m + self.n) * self.d * 8 + self.r * self.r * 4


def make_problem(name: str, m: int, n: int, r: int, d: int, dtype: str, seed: int,
                 g_std: float = 1e-3, w_std: float = 0.02, s_std: float = 1e-3,
                 index_dist: str = "uniform", heavy_row_frac: float = 0.0,
                 value_mode: str = "normal") -> Problem:
    """Draw one problem.  Order of draws is fixed: G, W, P, Q, S_in."""
    rng = np.random.default_rng(seed)
    G = gaussian_matrix(m, n, g_std, dtype, rng, heavy_row_frac=heavy_row_frac)
    W = gaussian_matrix(m, n, w_std, dtype, rng)
    P_idx, P_val = ell_projector(m, r, d, rng, index_dist=index_dist, value_mode=value_mode)
    Q_idx, Q_val = ell_projector(n, r, d, rng, index_dist=index_dist, value_mode=value_mode)
    S_in = (rng.standard_normal((r, r), dtype=np.float32) * np.float32(s_std)).astype(np.float32)
    return Problem(name, m, n, r, d, dtype, G, W, P_idx, P_val, Q_idx, Q_val, S_in)


def make_integer_problem(name: str, m: int, n: int, r: int, d: int, dtype: str, seed: int,
                         index_dist: str = "uniform", value_mode: str = "smallint") -> Problem:
    """All-integer operands of small magnitude: every partial sum is exact in fp32, so any
    correct implementation must reproduce the oracle bit for bit (pins the index handling)."""
    rng = np.random.default_rng(seed)
    G = integer_matrix(m, n, -8, 8, dtype, rng)
    W = integer_matrix(m, n, -64, 64, dtype, rng)
    P_idx, P_val = ell_projector(m, r, d, rng, index_dist=index_dist, value_mode=value_mode)
    Q_idx, Q_val = ell_projector(n, r, d, rng, index_dist=index_dist, value_mode=value_mode)
    S_in = rng.integers(-2, 3, size=(r, r)).astype(np.float32)
    return Problem(name, m, n, r, d, dtype, G, W, P_idx, P_val, Q_idx, Q_val, S_in)


# Shapes of one 6.7B-class transformer layer, in the order the backward pass reaches them
# (reverse of forward use): down, gate, up, o, v, k, q.
LAYER_67B: List[Tuple[str, int, int]] = [
    ("down", 11008, 4096), ("gate", 4096, 11008), ("up", 4096, 11008),
    ("o", 4096, 4096), ("v", 4096, 4096), ("k", 4096, 4096), ("q", 4096, 4096),
]


def config1() -> Problem:
    """Single small fp32 layer: 256x256, r=16, d=2 distinct columns per row."""
    return make_problem("cfg1", 256, 256, 16, 2, "f32", seed=0, g_std=1.0, w_std=0.02,
                        index_dist="distinct")


def config2() -> Problem:
    """1.3B-style attention projection: fp16 2048x2048, r=256, d=4."""
    return make_problem("cfg2", 2048, 2048, 256, 4, "f16", seed=2)


def config3() -> List[Problem]:
    """1.3B-style MLP pair, fp16, 1% of gradient rows scaled x100, r=512, d=4."""
    return [make_problem("cfg3_up", 2048, 8192, 512, 4, "f16", seed=3, heavy_row_frac=0.01),
            make_problem("cfg3_down", 8192, 2048, 512, 4, "f16", seed=30, heavy_row_frac=0.01)]


def config4_matrix(layer: int, which: int, scale_rows: Optional[int] = None) -> Problem:
    """One matrix of the 6.7B-style stack: bf16, r=512, d=8.  `which` indexes LAYER_67B."""
    name, m, n = LAYER_67B[which]
    return make_problem(f"cfg4_L{layer}_{name}", m, n, 512, 8, "bf16", seed=4000 + layer * 7 + which)


def config5_point(r: int, d: int, index: int = 0, m: int = 4096, n: int = 16384) -> Problem:
    """One point of the wide sweep: bf16 4096x16384, Zipf(1.1) projector columns."""
    return make_problem(f"cfg5_r{r}_d{d}", m, n, r, d, "bf16", seed=5000 + index, index_dist="zipf")
