"""Dense-projector ablation of compress (lsp_compress_dense, matrix cores) against the oracle.

A dense m x r projector is the d = r case of Def. 1 (every column present), so the reference is the compress
oracle itself on ELL arrays with idx[i][k] = k.  The projector values handed to both sides are representable in
the storage type; what is left to differ is the rounding of T = G Q to the storage type between the two products
and the order of the fp32 sums."""
import numpy as np
import pytest
import torch

import lsp_synth as syn
import oracle
import paper_2406_10181_amd as L
from gpu_util import to_device

pytestmark = pytest.mark.gpu


def _round(x32, dtype):
    """values of the storage type, as fp32"""
    bits = syn.to_storage(x32.astype(np.float32), dtype)
    return syn.bf16_bits_to_f32(bits) if dtype == "bf16" else bits.astype(np.float32)


def _run(G32, P32, Q32, dtype):
    """G32 [m][n], P32 [m][r], Q32 [n][r]: fp32 arrays whose values the storage type holds exactly."""
    m, n = G32.shape
    r = P32.shape[1]
    code = syn.DTYPE_CODE[dtype]
    Gs = syn.to_storage(G32, dtype)
    G = to_device(Gs, dtype)
    Pt = to_device(syn.to_storage(np.ascontiguousarray(P32.T), dtype), dtype)
    Qt = to_device(syn.to_storage(np.ascontiguousarray(Q32.T), dtype), dtype)
    S = torch.full((r, r), float("nan"), dtype=torch.float32, device="cuda")
    wb = L.lsp_compress_dense_workspace_bytes(m, n, r)
    assert wb > 0
    ws = torch.empty(wb, dtype=torch.uint8, device="cuda")
    print(f"[case] dense compress m={m} n={n} r={r} {dtype}", flush=True)
    L.lsp_compress_dense(G, Pt, Qt, m, n, r, S, code, ws, wb, torch.cuda.current_stream())
    torch.cuda.synchronize()
    first = S.cpu().numpy().copy()
    S.fill_(float("nan"))
    L.lsp_compress_dense(G, Pt, Qt, m, n, r, S, code, ws, wb, torch.cuda.current_stream())
    torch.cuda.synchronize()
    assert np.array_equal(first, S.cpu().numpy()), "not bit-reproducible"
    idx_p = np.tile(np.arange(r, dtype=np.int32), (m, 1))
    idx_q = np.tile(np.arange(r, dtype=np.int32), (n, 1))
    S_o = oracle.compress(Gs, dtype, idx_p, P32, idx_q, Q32, r, threads=8)
    return first.astype(np.float64), S_o


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("m,n,r", [(128, 64, 128), (256, 192, 128), (384, 320, 256)])
def test_dense_compress_matches_oracle(m, n, r, dtype):
    rng = np.random.default_rng(m + n + r)
    G32 = _round(rng.standard_normal((m, n)) * 1e-2, dtype)
    P32 = _round(rng.standard_normal((m, r)) / np.sqrt(r), dtype)
    Q32 = _round(rng.standard_normal((n, r)) / np.sqrt(r), dtype)
    got, S_o = _run(G32, P32, Q32, dtype)
    # T is rounded once to the storage type (relative 2^-9 for bf16, 2^-12 for fp16; fp16 may also lose tiny values to
    # its subnormal range) before the second product: |dS[a][b]| <= eps * sum_i |P[i][a]| |T[i][b]| plus fp32 slack
    T = G32.astype(np.float64) @ Q32.astype(np.float64)
    eps = 2.0 ** -8 if dtype == "bf16" else 2.0 ** -11
    bound = eps * (np.abs(P32.astype(np.float64)).T @ (np.abs(T) + (6e-8 if dtype == "f16" else 0.0))) + 1e-5 * np.abs(S_o).max()
    err = np.abs(got - S_o)
    assert (err <= bound).all(), f"max excess {np.max(err - bound):.3e}"
    assert err.max() <= (6e-3 if dtype == "bf16" else 1e-3) * np.abs(S_o).max()


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_dense_compress_exact_on_small_integers(dtype):
    """Integer-valued operands whose intermediate T stays below 256 in magnitude: every product and sum is exact in
    both types, so the result must equal the oracle's bit for bit (any slip in the tile or lane indexing shows)."""
    m, n, r = 256, 128, 128
    rng = np.random.default_rng(11)
    G32 = rng.integers(-2, 3, size=(m, n)).astype(np.float32)
    Q32 = np.zeros((n, r), dtype=np.float32)
    P32 = np.zeros((m, r), dtype=np.float32)
    for j in range(n):
        Q32[j, rng.choice(r, size=4, replace=False)] = rng.choice([-1.0, 1.0], size=4)
    for i in range(m):
        P32[i, rng.choice(r, size=4, replace=False)] = rng.choice([-1.0, 1.0, 2.0], size=4)
    assert np.abs(G32.astype(np.float64) @ Q32).max() < 256
    got, S_o = _run(G32, P32, Q32, dtype)
    assert np.array_equal(got, S_o)
