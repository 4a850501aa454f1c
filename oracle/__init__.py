"""CPU oracle for the LSP compress / decompress-apply path, the estimation bias, the state re-projection and
the fitting gradient.  TEST INFRASTRUCTURE ONLY.

Thin ctypes wrapper around ``lsp_oracle.c`` (plain fp64 loops written from the paper's
two formulas: the compress step S = P^T G Q and the decompress-and-apply step
W <- W - P S Q^T of Alg. 1 / Alg. 3 with the (d,r)-sparse projectors of Def. 1, and the
estimation bias of Def. 2).

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py``
may import this package.  It imports nothing from the HIP package and the HIP package
imports nothing from here.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lsp_oracle.c")
_LIB = os.path.join(_HERE, "liblsp_oracle.so")

DTYPE_CODE = {"f32": 0, "f16": 1, "bf16": 2}
_NP_STORAGE = {"f32": np.float32, "f16": np.float16, "bf16": np.uint16}


def build(force: bool = False) -> str:
    """Compile the oracle's C file with gcc (no GPU toolchain involved)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-Wall", "-Wextra", "-shared", "-fPIC",
                               "-o", _LIB, _SRC, "-lm", "-lpthread"])
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
        proj = [vp, vp, vp, vp]
        lib.lsp_oracle_compress.argtypes = [vp, i32] + proj + [i64, i64, i32, i32, vp]
        lib.lsp_oracle_compress_dense.argtypes = lib.lsp_oracle_compress.argtypes
        lib.lsp_oracle_compress_mt.argtypes = lib.lsp_oracle_compress.argtypes + [i32]
        lib.lsp_oracle_decompress_apply.argtypes = [vp, i32, vp] + proj + [i64, i64, i32, i32, vp, vp]
        lib.lsp_oracle_decompress_apply_dense.argtypes = lib.lsp_oracle_decompress_apply.argtypes
        lib.lsp_oracle_decompress_apply_mt.argtypes = lib.lsp_oracle_decompress_apply.argtypes + [i32]
        lib.lsp_oracle_decompress_rows.argtypes = [vp, i32, vp] + proj + [i64, i64, i32, i32, vp, i64, vp]
        lib.lsp_oracle_compress_entries.argtypes = [vp, i32] + proj + [i64, i64, i32, i32, vp, vp, i64, vp]
        lib.lsp_oracle_bias.argtypes = [vp, i32] + proj + [i64, i64, i32, i32, vp]
        lib.lsp_oracle_bias_dense.argtypes = lib.lsp_oracle_bias.argtypes
        lib.lsp_oracle_bias_grad.argtypes = [vp, i32] + proj + [i64, i64, i32, i32, vp, vp]
        lib.lsp_oracle_bias_grad_dense.argtypes = lib.lsp_oracle_bias_grad.argtypes
        lib.lsp_oracle_reproject.argtypes = proj + proj + [i64, i64, i32, i32, vp, vp, vp, vp]
        lib.lsp_oracle_round_to_storage.argtypes = [ctypes.c_double, i32]
        lib.lsp_oracle_round_to_storage.restype = ctypes.c_double
        lib.lsp_oracle_widen.argtypes = [vp, i64, i32]
        lib.lsp_oracle_widen.restype = ctypes.c_double
        _lib = lib
    return _lib


def _p(a: np.ndarray) -> ctypes.c_void_p:
    return ctypes.c_void_p(a.ctypes.data)


def _storage(x: np.ndarray, dtype: str, shape: Tuple[int, int]) -> np.ndarray:
    want = _NP_STORAGE[dtype]
    if x.dtype != want:
        raise TypeError(f"storage for {dtype} must be numpy {want.__name__}, got {x.dtype}")
    if x.shape != shape:
        raise ValueError(f"expected shape {shape}, got {x.shape}")
    return np.ascontiguousarray(x)


def _proj(idx: np.ndarray, val: np.ndarray, rows: int, r: int, d: int):
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    val = np.ascontiguousarray(val, dtype=np.float32)
    if idx.shape != (rows, d) or val.shape != (rows, d):
        raise ValueError(f"projector arrays must be [{rows}][{d}], got {idx.shape} / {val.shape}")
    if idx.size and (idx.min() < 0 or idx.max() >= r):
        raise ValueError("projector column index out of [0, r)")
    return idx, val


def compress(G, dtype, P_idx, P_val, Q_idx, Q_val, r: int, *, dense: bool = False,
             threads: int = 0) -> np.ndarray:
    """S = P^T G Q as float64 [r][r].  dense=True evaluates the literal definition (tiny inputs)."""
    lib = _load()
    m, n = G.shape
    d = P_idx.shape[1]
    G = _storage(G, dtype, (m, n))
    P_idx, P_val = _proj(P_idx, P_val, m, r, d)
    Q_idx, Q_val = _proj(Q_idx, Q_val, n, r, d)
    S = np.empty((r, r), dtype=np.float64)
    args = [_p(G), DTYPE_CODE[dtype], _p(P_idx), _p(P_val), _p(Q_idx), _p(Q_val), m, n, r, d, _p(S)]
    if dense:
        rc = lib.lsp_oracle_compress_dense(*args)
    elif threads > 0:
        rc = lib.lsp_oracle_compress_mt(*args, threads)
    else:
        rc = lib.lsp_oracle_compress(*args)
    if rc != 0:
        raise RuntimeError(f"oracle compress failed rc={rc}")
    return S


def decompress_apply(W, dtype, S, P_idx, P_val, Q_idx, Q_val, *, dense: bool = False,
                     threads: int = 0, want_rounded: bool = True):
    """Returns (W' as float64 [m][n], W' rounded once to the storage type or None).  W is not modified."""
    lib = _load()
    m, n = W.shape
    d = P_idx.shape[1]
    S = np.ascontiguousarray(S, dtype=np.float32)
    r = S.shape[0]
    if S.shape != (r, r):
        raise ValueError("S must be square")
    W = _storage(W, dtype, (m, n))
    P_idx, P_val = _proj(P_idx, P_val, m, r, d)
    Q_idx, Q_val = _proj(Q_idx, Q_val, n, r, d)
    Wp = np.empty((m, n), dtype=np.float64)
    Wr = np.empty((m, n), dtype=_NP_STORAGE[dtype]) if want_rounded else None
    args = [_p(W), DTYPE_CODE[dtype], _p(S), _p(P_idx), _p(P_val), _p(Q_idx), _p(Q_val),
            m, n, r, d, _p(Wp), _p(Wr) if Wr is not None else None]
    if dense:
        rc = lib.lsp_oracle_decompress_apply_dense(*args)
    elif threads > 0:
        rc = lib.lsp_oracle_decompress_apply_mt(*args, threads)
    else:
        rc = lib.lsp_oracle_decompress_apply(*args)
    if rc != 0:
        raise RuntimeError(f"oracle decompress_apply failed rc={rc}")
    return Wp, Wr


def estimation_bias(G, dtype, P_idx, P_val, Q_idx, Q_val, r: int, *, dense: bool = False) -> Tuple[float, float]:
    """Def. 2: returns (||P P^T G Q Q^T - G||_F^2, ||G||_F^2) in float64; the bias is the square root of
    their ratio.  dense=True forms P P^T and Q Q^T as dense matrices first (tiny inputs)."""
    lib = _load()
    m, n = G.shape
    d = P_idx.shape[1]
    G = _storage(G, dtype, (m, n))
    P_idx, P_val = _proj(P_idx, P_val, m, r, d)
    Q_idx, Q_val = _proj(Q_idx, Q_val, n, r, d)
    out = np.zeros(2, dtype=np.float64)
    fn = lib.lsp_oracle_bias_dense if dense else lib.lsp_oracle_bias
    rc = fn(_p(G), DTYPE_CODE[dtype], _p(P_idx), _p(P_val), _p(Q_idx), _p(Q_val), m, n, r, d, _p(out))
    if rc != 0:
        raise RuntimeError(f"oracle estimation_bias failed rc={rc}")
    return float(out[0]), float(out[1])


def bias_gradient(G, dtype, P_idx, P_val, Q_idx, Q_val, r: int, *, dense: bool = False):
    """Gradient of F = 1/2 ||P P^T G Q Q^T - G||_F^2 (half the squared numerator of Def. 2's bias: the data
    term of the fitting objective of Eq. 2 / MaybeUpdate, Alg. 1) with respect to the stored projector
    values: returns (dF/dP_val [m][d], dF/dQ_val [n][d]) in float64.  dense=True evaluates the chain rule on
    dense m x m and n x n matrices (tiny inputs)."""
    lib = _load()
    m, n = G.shape
    d = P_idx.shape[1]
    G = _storage(G, dtype, (m, n))
    P_idx, P_val = _proj(P_idx, P_val, m, r, d)
    Q_idx, Q_val = _proj(Q_idx, Q_val, n, r, d)
    gP = np.zeros((m, d), dtype=np.float64)
    gQ = np.zeros((n, d), dtype=np.float64)
    fn = lib.lsp_oracle_bias_grad_dense if dense else lib.lsp_oracle_bias_grad
    rc = fn(_p(G), DTYPE_CODE[dtype], _p(P_idx), _p(P_val), _p(Q_idx), _p(Q_val), m, n, r, d, _p(gP), _p(gQ))
    if rc != 0:
        raise RuntimeError(f"oracle bias_gradient failed rc={rc}")
    return gP, gQ


def reproject_state(P_idx, P_val, Pp_idx, Pp_val, Q_idx, Q_val, Qp_idx, Qp_val, r: int, M, V):
    """Last two assignments of MaybeUpdate (Alg. 1): M' = (P^T P_prev) M (Q_prev^T Q) and
    V' = (P^T P_prev)^2 V (Q_prev^T Q)^2 with element-wise squares, in float64.  P, P_prev are [m][d]
    ELL pairs, Q, Q_prev [n][d]; M, V float32 [r][r]."""
    lib = _load()
    m, d = P_idx.shape
    n = Q_idx.shape[0]
    P_idx, P_val = _proj(P_idx, P_val, m, r, d)
    Pp_idx, Pp_val = _proj(Pp_idx, Pp_val, m, r, d)
    Q_idx, Q_val = _proj(Q_idx, Q_val, n, r, d)
    Qp_idx, Qp_val = _proj(Qp_idx, Qp_val, n, r, d)
    M = np.ascontiguousarray(M, dtype=np.float32)
    V = np.ascontiguousarray(V, dtype=np.float32)
    if M.shape != (r, r) or V.shape != (r, r):
        raise ValueError("M and V must be [r][r]")
    Mo = np.empty((r, r), dtype=np.float64)
    Vo = np.empty((r, r), dtype=np.float64)
    rc = lib.lsp_oracle_reproject(_p(P_idx), _p(P_val), _p(Pp_idx), _p(Pp_val), _p(Q_idx), _p(Q_val),
                                  _p(Qp_idx), _p(Qp_val), m, n, r, d, _p(M), _p(V), _p(Mo), _p(Vo))
    if rc != 0:
        raise RuntimeError(f"oracle reproject_state failed rc={rc}")
    return Mo, Vo


def decompress_rows(W, dtype, S, P_idx, P_val, Q_idx, Q_val, rows: Sequence[int]) -> np.ndarray:
    """W'[rows, :] as float64, for sampled checks at full benchmark sizes."""
    lib = _load()
    m, n = W.shape
    d = P_idx.shape[1]
    S = np.ascontiguousarray(S, dtype=np.float32)
    r = S.shape[0]
    W = _storage(W, dtype, (m, n))
    P_idx, P_val = _proj(P_idx, P_val, m, r, d)
    Q_idx, Q_val = _proj(Q_idx, Q_val, n, r, d)
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    out = np.empty((rows.size, n), dtype=np.float64)
    rc = lib.lsp_oracle_decompress_rows(_p(W), DTYPE_CODE[dtype], _p(S), _p(P_idx), _p(P_val),
                                        _p(Q_idx), _p(Q_val), m, n, r, d, _p(rows), rows.size, _p(out))
    if rc != 0:
        raise RuntimeError(f"oracle decompress_rows failed rc={rc}")
    return out


def compress_entries(G, dtype, P_idx, P_val, Q_idx, Q_val, r: int,
                     ea: Sequence[int], eb: Sequence[int]) -> np.ndarray:
    """Selected entries S[ea[t]][eb[t]] straight from the definition (no intermediate)."""
    lib = _load()
    m, n = G.shape
    d = P_idx.shape[1]
    G = _storage(G, dtype, (m, n))
    P_idx, P_val = _proj(P_idx, P_val, m, r, d)
    Q_idx, Q_val = _proj(Q_idx, Q_val, n, r, d)
    ea = np.ascontiguousarray(ea, dtype=np.int32)
    eb = np.ascontiguousarray(eb, dtype=np.int32)
    out = np.empty(ea.size, dtype=np.float64)
    rc = lib.lsp_oracle_compress_entries(_p(G), DTYPE_CODE[dtype], _p(P_idx), _p(P_val), _p(Q_idx),
                                         _p(Q_val), m, n, r, d, _p(ea), _p(eb), ea.size, _p(out))
    if rc != 0:
        raise RuntimeError(f"oracle compress_entries failed rc={rc}")
    return out


def round_to_storage(x: float, dtype: str) -> float:
    return float(_load().lsp_oracle_round_to_storage(float(x), DTYPE_CODE[dtype]))


def widen(arr: np.ndarray, k: int, dtype: str) -> float:
    arr = np.ascontiguousarray(arr)
    return float(_load().lsp_oracle_widen(_p(arr), int(k), DTYPE_CODE[dtype]))
