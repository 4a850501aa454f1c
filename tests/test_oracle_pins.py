"""Pins for the CPU oracle (no GPU).  Each test fixes the oracle against something that is
not the oracle: hand-worked numbers, the literal dense definition, independent few-line
loops, algebraic identities, numpy's fp64 GEMM, numpy's own fp16 conversion.

They are chosen so that a plausible mistake (dropped term, wrong sign, transposed or
mis-paired projector, wrong index stride, double rounding) fails at least one of them.
"""
import os

import numpy as np
import pytest

import lsp_synth as syn
import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rng(seed):
    return np.random.default_rng(seed)


def _dense(idx, val, r):
    rows, d = idx.shape
    D = np.zeros((rows, r), dtype=np.float64)
    for i in range(rows):
        for k in range(d):
            D[i, idx[i, k]] += float(val[i, k])
    return D


# ---------------------------------------------------------------- hand-worked example
def _read_golden(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, *vals = line.split()
            out[key] = np.array([float(v) for v in vals])
    return out


def test_hand_worked_example():
    gold = _read_golden("hand_case_2x3.txt")
    G = np.array([[1, 2, 3], [4, 5, 6]], dtype=np.float32)
    P_idx = np.array([[1], [0]], dtype=np.int32)
    P_val = np.array([[2], [3]], dtype=np.float32)
    Q_idx = np.array([[0], [1], [0]], dtype=np.int32)
    Q_val = np.array([[1], [-1], [0.5]], dtype=np.float32)
    for dense in (False, True):
        S = oracle.compress(G, "f32", P_idx, P_val, Q_idx, Q_val, 2, dense=dense)
        assert np.array_equal(S.ravel(), gold["S"])
        S2 = np.array([[1, 0], [0, 2]], dtype=np.float32)
        W0 = np.zeros((2, 3), dtype=np.float32)
        Wp, Wr = oracle.decompress_apply(W0, "f32", S2, P_idx, P_val, Q_idx, Q_val, dense=dense)
        assert np.array_equal(Wp.ravel(), gold["W"])
        assert np.array_equal(Wr.ravel().astype(np.float64), gold["W"])


def test_hand_worked_asymmetry_is_detected():
    """The example is not symmetric under P<->Q or transposition, so a mis-paired operand
    cannot give the same numbers (guards the fixture's power, on the CPU)."""
    gold = _read_golden("hand_case_2x3.txt")
    G = np.array([[1, 2, 3], [4, 5, 6]], dtype=np.float64)
    Ph = np.array([[0, 2], [3, 0]], dtype=np.float64)
    Qh = np.array([[1, 0], [0, -1], [0.5, 0]], dtype=np.float64)
    right = Ph.T @ G @ Qh
    assert np.array_equal(right.ravel(), gold["S"])
    assert not np.array_equal((Ph.T @ G @ Qh).T.ravel(), gold["S"])


# ---------------------------------------------------------------- pin 1: literal definition
@pytest.mark.parametrize("m,n,r,d,dist,dtype", [
    (5, 7, 3, 2, "uniform", "f32"),
    (12, 9, 6, 3, "uniform", "f32"),
    (7, 12, 4, 4, "distinct", "f32"),      # d == r
    (6, 6, 5, 3, "zipf", "f32"),           # duplicates certain
    (9, 5, 6, 2, "uniform", "bf16"),
    (8, 11, 4, 1, "uniform", "f16"),
    (1, 1, 1, 1, "uniform", "f32"),
])
def test_working_form_equals_literal_definition(m, n, r, d, dist, dtype):
    pb = syn.make_problem("t", m, n, r, d, dtype, seed=100 + m * n, g_std=1.0, w_std=1.0, s_std=1.0,
                          index_dist=dist)
    S_w = oracle.compress(pb.G, dtype, pb.P_idx, pb.P_val, pb.Q_idx, pb.Q_val, r)
    S_d = oracle.compress(pb.G, dtype, pb.P_idx, pb.P_val, pb.Q_idx, pb.Q_val, r, dense=True)
    np.testing.assert_allclose(S_w, S_d, rtol=0, atol=1e-12 * max(1.0, np.abs(S_d).max()))
    Wp_w, Wr_w = oracle.decompress_apply(pb.W, dtype, pb.S_in, pb.P_idx, pb.P_val, pb.Q_idx, pb.Q_val)
    Wp_d, Wr_d = oracle.decompress_apply(pb.W, dtype, pb.S_in, pb.P_idx, pb.P_val, pb.Q_idx, pb.Q_val,
                                         dense=True)
    np.testing.assert_allclose(Wp_w, Wp_d, rtol=0, atol=1e-12 * max(1.0, np.abs(Wp_d).max()))


# ---------------------------------------------------------------- pin 6: numpy fp64 GEMM
@pytest.mark.parametrize("maker", [syn.config1,
                                   lambda: syn.make_problem("t", 96, 160, 32, 4, "bf16", 7),
                                   lambda: syn.make_problem("t", 200, 72, 24, 3, "f16", 8,
                                                            index_dist="zipf")])
def test_against_numpy_gemm(maker):
    pb = maker()
    Ph, Qh = _dense(pb.P_idx, pb.P_val, pb.r), _dense(pb.Q_idx, pb.Q_val, pb.r)
    G64 = syn.storage_to_f64(pb.G, pb.dtype)
    W64 = syn.storage_to_f64(pb.W, pb.dtype)
    S = oracle.compress(pb.G, pb.dtype, pb.P_idx, pb.P_val, pb.Q_idx, pb.Q_val, pb.r)
    ref = Ph.T @ G64 @ Qh
    np.testing.assert_allclose(S, ref, rtol=0, atol=1e-12 * np.abs(ref).max())
    Wp, Wr = oracle.decompress_apply(pb.W, pb.dtype, pb.S_in, pb.P_idx, pb.P_val, pb.Q_idx, pb.Q_val)
    refW = W64 - Ph @ pb.S_in.astype(np.float64) @ Qh.T
    np.testing.assert_allclose(Wp, refW, rtol=0, atol=1e-13)
    # the rounded output is the fp64 value rounded once to the storage type
    back = syn.storage_to_f64(Wr, pb.dtype)
    assert np.all(np.abs(back - Wp) <= 0.5 * syn.ulp_of(Wp, pb.dtype) * (1 + 1e-12))


# ---------------------------------------------------------------- pin 2: selection projectors
@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
def test_selection_projectors_give_block_sums(dtype):
    rng = _rng(11)
    m, n, r = 37, 53, 6
    G = syn.integer_matrix(m, n, -8, 8, dtype, rng)
    p = rng.integers(0, r, size=m).astype(np.int32)
    q = rng.integers(0, r, size=n).astype(np.int32)
    ones_m = np.ones((m, 1), dtype=np.float32)
    ones_n = np.ones((n, 1), dtype=np.float32)
    S = oracle.compress(G, dtype, p.reshape(m, 1), ones_m, q.reshape(n, 1), ones_n, r)
    G64 = syn.storage_to_f64(G, dtype)
    ref = np.zeros((r, r))
    for i in range(m):                      # independent: plain block sums of G
        for j in range(n):
            ref[p[i], q[j]] += G64[i, j]
    assert np.array_equal(S, ref)


# ---------------------------------------------------------------- pin 3: linearity
def test_linearity_exact_on_integers():
    rng = _rng(12)
    m, n, r, d = 40, 33, 8, 3
    P_idx, P_val = syn.ell_projector(m, r, d, rng, "uniform", value_mode="smallint")
    Q_idx, Q_val = syn.ell_projector(n, r, d, rng, "uniform", value_mode="smallint")
    G1 = syn.integer_matrix(m, n, -8, 8, "f32", rng)
    G2 = syn.integer_matrix(m, n, -8, 8, "f32", rng)
    S1 = oracle.compress(G1, "f32", P_idx, P_val, Q_idx, Q_val, r)
    S2 = oracle.compress(G2, "f32", P_idx, P_val, Q_idx, Q_val, r)
    S12 = oracle.compress((2 * G1 - 4 * G2).astype(np.float32), "f32", P_idx, P_val, Q_idx, Q_val, r)
    assert np.array_equal(S12, 2 * S1 - 4 * S2)
    # decompress is affine in S: W - P(2A-4B)Q^T = W - 2(PAQ^T) + 4(PBQ^T)
    A = rng.integers(-2, 3, size=(r, r)).astype(np.float32)
    B = rng.integers(-2, 3, size=(r, r)).astype(np.float32)
    Z = np.zeros((m, n), dtype=np.float32)
    dA, _ = oracle.decompress_apply(Z, "f32", A, P_idx, P_val, Q_idx, Q_val)
    dB, _ = oracle.decompress_apply(Z, "f32", B, P_idx, P_val, Q_idx, Q_val)
    dAB, _ = oracle.decompress_apply(Z, "f32", 2 * A - 4 * B, P_idx, P_val, Q_idx, Q_val)
    assert np.array_equal(dAB, 2 * dA - 4 * dB)


# ---------------------------------------------------------------- pin 4: permutation round trip
def test_permutation_round_trip():
    rng = _rng(13)
    m, n = 19, 23
    G = rng.standard_normal((m, n)).astype(np.float32)
    p_idx, p_val = syn.permutation_projector(m, rng)
    # r is shared by P and Q, so use r = max(m, n) and an injective map for the shorter side
    r = max(m, n)
    q_idx, q_val = syn.permutation_projector(n, rng)
    S = oracle.compress(G, "f32", p_idx, p_val, q_idx, q_val, r)
    for i in range(m):
        for j in range(n):
            assert S[p_idx[i, 0], q_idx[j, 0]] == float(G[i, j])
    assert np.count_nonzero(S) <= m * n
    Wp, _ = oracle.decompress_apply(np.zeros((m, n), np.float32), "f32", S.astype(np.float32),
                                    p_idx, p_val, q_idx, q_val)
    assert np.array_equal(Wp, -G.astype(np.float64))      # bias b^{P,Q}(G) = P P^T G Q Q^T - G = 0


# ---------------------------------------------------------------- pin 5: adjoint identity
@pytest.mark.parametrize("dist", ["uniform", "zipf"])
def test_adjoint_identity(dist):
    pb = syn.make_problem("t", 45, 61, 12, 3, "f32", seed=14, g_std=1.0, s_std=1.0, index_dist=dist)
    S = oracle.compress(pb.G, "f32", pb.P_idx, pb.P_val, pb.Q_idx, pb.Q_val, pb.r)
    Z = np.zeros((pb.m, pb.n), dtype=np.float32)
    D, _ = oracle.decompress_apply(Z, "f32", pb.S_in, pb.P_idx, pb.P_val, pb.Q_idx, pb.Q_val)
    lhs = np.sum(S * pb.S_in.astype(np.float64))                  # <P^T G Q, S'>
    rhs = np.sum(pb.G.astype(np.float64) * (-D))                  # <G, P S' Q^T>
    assert abs(lhs - rhs) <= 1e-12 * max(abs(lhs), abs(rhs), 1.0)


# ---------------------------------------------------------------- pin 7: zero / padding / duplicates
def test_zero_padding_and_duplicates():
    rng = _rng(15)
    m, n, r, d = 14, 17, 5, 3
    pb = syn.make_problem("t", m, n, r, d, "bf16", seed=16, g_std=1.0, w_std=1.0, s_std=1.0)
    Zs = np.zeros((r, r), dtype=np.float32)
    # G = 0 -> S = 0
    S0 = oracle.compress(np.zeros((m, n), np.uint16), "bf16", pb.P_idx, pb.P_val, pb.Q_idx, pb.Q_val, r)
    assert not S0.any()
    # S = 0 -> W unchanged bit for bit
    Wp, Wr = oracle.decompress_apply(pb.W, "bf16", Zs, pb.P_idx, pb.P_val, pb.Q_idx, pb.Q_val)
    assert np.array_equal(Wr, pb.W)
    # padding entries (val = 0, any index) change nothing
    P_idx2 = np.concatenate([pb.P_idx, rng.integers(0, r, size=(m, 2)).astype(np.int32)], axis=1)
    P_val2 = np.concatenate([pb.P_val, np.zeros((m, 2), np.float32)], axis=1)
    Q_idx2 = np.concatenate([pb.Q_idx, rng.integers(0, r, size=(n, 2)).astype(np.int32)], axis=1)
    Q_val2 = np.concatenate([pb.Q_val, np.zeros((n, 2), np.float32)], axis=1)
    S_a = oracle.compress(pb.G, "bf16", pb.P_idx, pb.P_val, pb.Q_idx, pb.Q_val, r)
    S_b = oracle.compress(pb.G, "bf16", P_idx2, P_val2, Q_idx2, Q_val2, r)
    np.testing.assert_allclose(S_a, S_b, rtol=0, atol=1e-13 * np.abs(S_a).max())
    # a duplicated index pair (a, v1), (a, v2) equals a single (a, v1 + v2)
    Pi = np.array([[2, 2]] * m, dtype=np.int32)
    Pv = np.array([[0.5, 1.5]] * m, dtype=np.float32)
    Qi = pb.Q_idx[:, :2].copy()
    Qv = pb.Q_val[:, :2].copy()
    S_dup = oracle.compress(pb.G, "bf16", Pi, Pv, Qi, Qv, r)
    Pi_eq = np.array([[2, 0]] * m, dtype=np.int32)
    Pv_eq = np.array([[2.0, 0.0]] * m, dtype=np.float32)
    S_eq = oracle.compress(pb.G, "bf16", Pi_eq, Pv_eq, Qi, Qv, r)
    np.testing.assert_allclose(S_dup, S_eq, rtol=0, atol=1e-13 * max(np.abs(S_eq).max(), 1e-300))


# ---------------------------------------------------------------- pin 9: separability
def test_rank_one_separability():
    rng = _rng(17)
    m, n, r, d = 50, 41, 9, 3
    P_idx, P_val = syn.ell_projector(m, r, d, rng)
    Q_idx, Q_val = syn.ell_projector(n, r, d, rng)
    u = rng.standard_normal(m).astype(np.float32)
    v = rng.standard_normal(n).astype(np.float32)
    G = np.outer(u.astype(np.float64), v.astype(np.float64)).astype(np.float32)
    G64 = G.astype(np.float64)
    S = oracle.compress(G, "f32", P_idx, P_val, Q_idx, Q_val, r)
    # two independent sparse mat-vecs on the fp32-rounded outer product's factors would differ by
    # the rounding of G; use the rounded G's own row/column structure instead: S = Phat^T G Qhat
    pu = np.zeros(r)
    for i in range(m):
        for k in range(d):
            pu[P_idx[i, k]] += float(P_val[i, k]) * float(u[i])
    qv = np.zeros(r)
    for j in range(n):
        for k in range(d):
            qv[Q_idx[j, k]] += float(Q_val[j, k]) * float(v[j])
    approx = np.outer(pu, qv)
    # G was rounded to fp32 element-wise: relative perturbation <= 2^-24 per term
    bound = 2.0 ** -23 * (np.abs(_dense(P_idx, P_val, r)).T @ np.abs(G64) @ np.abs(_dense(Q_idx, Q_val, r)))
    assert np.all(np.abs(S - approx) <= bound + 1e-15)


# ---------------------------------------------------------------- pin 8: generator scale (unbiasedness)
def test_generator_unbiasedness_pins_variance_reading():
    """E[Phat Phat^T] = I holds only if the values have variance 1/d (the reading of the
    paper's N(0, 1/sqrt(d)) as a standard deviation).  Also pins mean(decompress(compress(G))) -> G."""
    m, n, r, d = 12, 10, 24, 4
    G = _rng(18).standard_normal((m, n)).astype(np.float32)
    acc = np.zeros((m, m))
    accG = np.zeros((m, n))
    trials = 600
    for t in range(trials):
        rng = _rng(1000 + t)
        P_idx, P_val = syn.ell_projector(m, r, d, rng, "distinct")
        Q_idx, Q_val = syn.ell_projector(n, r, d, rng, "distinct")
        Ph = _dense(P_idx, P_val, r)
        acc += Ph @ Ph.T
        S = oracle.compress(G, "f32", P_idx, P_val, Q_idx, Q_val, r)
        D, _ = oracle.decompress_apply(np.zeros((m, n), np.float32), "f32", S.astype(np.float32),
                                       P_idx, P_val, Q_idx, Q_val)
        accG += -D
    acc /= trials
    accG /= trials
    assert np.abs(np.diag(acc) - 1.0).max() < 0.15
    off = acc - np.diag(np.diag(acc))
    assert np.abs(off).max() < 0.15
    # variance 1/d^2 or 1 (the other readings) would put the diagonal at 1/d or d: far outside
    rel = np.linalg.norm(accG - G) / np.linalg.norm(G)
    assert rel < 0.35


# ---------------------------------------------------------------- storage conversions
def test_widening_and_rounding_against_numpy():
    rng = _rng(19)
    # every fp16 bit pattern widens exactly as numpy widens it
    bits = np.arange(0, 1 << 16, dtype=np.uint16)
    h = bits.view(np.float16)
    sample = rng.choice(bits.size, size=4000, replace=False)
    for k in sample:
        a = oracle.widen(h, int(k), "f16")
        b = float(h[k])
        assert (np.isnan(a) and np.isnan(b)) or a == b
    # bf16 widening = bits << 16
    bb = rng.integers(0, 1 << 16, size=2000).astype(np.uint16)
    f = syn.bf16_bits_to_f32(bb)
    for k in range(0, 2000, 7):
        a = oracle.widen(bb, k, "bf16")
        assert (np.isnan(a) and np.isnan(f[k])) or a == float(f[k])
    # rounding fp64 -> fp16 equals numpy's direct float64 -> float16 conversion (single rounding)
    xs = np.concatenate([rng.standard_normal(3000) * 10.0 ** rng.integers(-9, 5, size=3000),
                         np.array([0.0, -0.0, 65504.0, 65519.9, 65520.0, 1e6, 6e-8, 2.98e-8, 2.99e-8,
                                   6.103515625e-05, 6.1e-05, 1.0 + 2 ** -11, 1.0 + 3 * 2 ** -11])])
    for x in xs:
        a = oracle.round_to_storage(float(x), "f16")
        b = float(np.float64(x).astype(np.float16))
        assert a == b, (x, a, b)
    # rounding fp64 -> bf16: ties to even on hand-picked cases, and agreement with the
    # integer bit trick on values that are exactly fp32
    assert oracle.round_to_storage(1.0 + 2 ** -8, "bf16") == 1.0            # tie -> even (1.0)
    assert oracle.round_to_storage(1.0 + 3 * 2 ** -8, "bf16") == 1.0 + 2 ** -6   # tie -> even
    assert oracle.round_to_storage(1.0 + 2 ** -8 + 2 ** -30, "bf16") == 1.0 + 2 ** -7
    x32 = (rng.standard_normal(3000) * 10.0 ** rng.integers(-6, 6, size=3000)).astype(np.float32)
    via_bits = syn.bf16_bits_to_f32(syn.f32_to_bf16_bits(x32))
    for k in range(x32.size):
        assert oracle.round_to_storage(float(x32[k]), "bf16") == float(via_bits[k])
    # double rounding trap: x just above a bf16 tie but rounding to the tie in fp32
    x = 1.0 + 2 ** -8 + 2 ** -40
    assert float(np.float32(x)) == 1.0 + 2 ** -8                 # fp32 lands on the tie
    assert oracle.round_to_storage(x, "bf16") == 1.0 + 2 ** -7   # single rounding goes up


# ---------------------------------------------------------------- helpers agree with the full forms
def test_sampled_forms_match_full_forms():
    pb = syn.make_problem("t", 64, 80, 16, 3, "bf16", seed=21)
    S = oracle.compress(pb.G, pb.dtype, pb.P_idx, pb.P_val, pb.Q_idx, pb.Q_val, pb.r)
    ea = np.array([0, 3, 15, 7, 7], dtype=np.int32)
    eb = np.array([0, 9, 15, 2, 7], dtype=np.int32)
    ent = oracle.compress_entries(pb.G, pb.dtype, pb.P_idx, pb.P_val, pb.Q_idx, pb.Q_val, pb.r, ea, eb)
    np.testing.assert_allclose(ent, S[ea, eb], rtol=0, atol=1e-13 * np.abs(S).max())
    Wp, _ = oracle.decompress_apply(pb.W, pb.dtype, pb.S_in, pb.P_idx, pb.P_val, pb.Q_idx, pb.Q_val)
    rows = [0, 63, 17, 17]
    sub = oracle.decompress_rows(pb.W, pb.dtype, pb.S_in, pb.P_idx, pb.P_val, pb.Q_idx, pb.Q_val, rows)
    assert np.array_equal(sub, Wp[rows])


def test_threaded_driver_matches_single_thread():
    pb = syn.make_problem("t", 130, 96, 32, 4, "f16", seed=22)
    S1 = oracle.compress(pb.G, pb.dtype, pb.P_idx, pb.P_val, pb.Q_idx, pb.Q_val, pb.r)
    S4 = oracle.compress(pb.G, pb.dtype, pb.P_idx, pb.P_val, pb.Q_idx, pb.Q_val, pb.r, threads=4)
    np.testing.assert_allclose(S4, S1, rtol=0, atol=1e-13 * np.abs(S1).max())
    W1, R1 = oracle.decompress_apply(pb.W, pb.dtype, pb.S_in, pb.P_idx, pb.P_val, pb.Q_idx, pb.Q_val)
    W4, R4 = oracle.decompress_apply(pb.W, pb.dtype, pb.S_in, pb.P_idx, pb.P_val, pb.Q_idx, pb.Q_val,
                                     threads=4)
    assert np.array_equal(W1, W4) and np.array_equal(R1, R4)


# ---------------------------------------------------------------- the generators themselves
def test_generators_are_deterministic_and_shaped():
    a, b = syn.config1(), syn.config1()
    for f in ("G", "W", "P_idx", "P_val", "Q_idx", "Q_val", "S_in"):
        assert np.array_equal(getattr(a, f), getattr(b, f))
    assert a.P_idx.shape == (256, 2) and a.Q_idx.shape == (256, 2)
    assert all(len(set(row)) == 2 for row in a.P_idx.tolist())          # without replacement
    assert a.P_idx.min() >= 0 and a.P_idx.max() < 16
    # ELL storage is (m + n) d values plus as many indices: the GPU-memory row of Table 2
    assert a.P_val.size + a.Q_val.size == (a.m + a.n) * a.d
    z = syn.ell_projector(4000, 512, 8, _rng(5), "zipf")[0]
    frac0 = np.mean(z == 0)
    H = np.sum(np.arange(1, 513, dtype=np.float64) ** -1.1)
    assert abs(frac0 - 1.0 / H) < 0.02                                   # hottest column ~ 1/H
    pb = syn.make_problem("t", 200, 64, 8, 2, "f16", 3, heavy_row_frac=0.01)
    rowmax = np.abs(pb.G.astype(np.float64)).max(axis=1)
    assert np.sum(rowmax > 0.02) == 2                                    # ceil(1% of 200) heavy rows


# ---------------------------------------------------------------- estimation bias (Def. 2)
def _bias(G, dtype, P_idx, P_val, Q_idx, Q_val, r, **kw):
    num, den = oracle.estimation_bias(G, dtype, P_idx, P_val, Q_idx, Q_val, r, **kw)
    return num, den


@pytest.mark.parametrize("m,n,r,d,dist,dtype", [
    (5, 7, 3, 2, "uniform", "f32"),
    (12, 9, 6, 3, "uniform", "f32"),
    (6, 6, 5, 3, "zipf", "f32"),           # duplicates certain
    (9, 5, 6, 2, "uniform", "bf16"),
    (8, 11, 4, 1, "uniform", "f16"),
])
def test_bias_working_form_equals_definition_and_numpy(m, n, r, d, dist, dtype):
    """The working form (S = P^T G Q first, then P S Q^T) against Def. 2 with P P^T and Q Q^T formed
    first, and both against numpy's dense products."""
    pb = syn.make_problem("t", m, n, r, d, dtype, seed=300 + m * n, g_std=1.0, index_dist=dist)
    nw, dw = _bias(pb.G, dtype, pb.P_idx, pb.P_val, pb.Q_idx, pb.Q_val, r)
    nd, dd = _bias(pb.G, dtype, pb.P_idx, pb.P_val, pb.Q_idx, pb.Q_val, r, dense=True)
    Ph, Qh = _dense(pb.P_idx, pb.P_val, r), _dense(pb.Q_idx, pb.Q_val, r)
    G64 = syn.storage_to_f64(pb.G, dtype)
    R = Ph @ Ph.T @ G64 @ Qh @ Qh.T
    ref_n, ref_d = float(((R - G64) ** 2).sum()), float((G64 ** 2).sum())
    for got_n, got_d in ((nw, dw), (nd, dd)):
        assert abs(got_n - ref_n) <= 1e-11 * max(1.0, ref_n) and abs(got_d - ref_d) <= 1e-12 * ref_d


def test_bias_of_selection_projectors_is_the_dropped_energy():
    """Projectors that select rows and columns (one unit entry per row, distinct targets; the other
    rows zero) have orthonormal columns, so P P^T G Q Q^T keeps the selected block of G and zeroes
    the rest: the squared bias is the energy outside the block over the total energy."""
    rng = _rng(21)
    m, n, r = 23, 31, 7
    G = syn.integer_matrix(m, n, -8, 8, "f32", rng)
    rows = rng.permutation(m)[:r]; cols = rng.permutation(n)[:r]
    P_idx = np.zeros((m, 1), dtype=np.int32); P_val = np.zeros((m, 1), dtype=np.float32)
    Q_idx = np.zeros((n, 1), dtype=np.int32); Q_val = np.zeros((n, 1), dtype=np.float32)
    P_idx[rows, 0] = np.arange(r); P_val[rows, 0] = 1.0
    Q_idx[cols, 0] = rng.permutation(r); Q_val[cols, 0] = 1.0
    num, den = _bias(G, "f32", P_idx, P_val, Q_idx, Q_val, r)
    G64 = G.astype(np.float64)
    kept = float((G64[np.ix_(rows, cols)] ** 2).sum())
    assert den == float((G64 ** 2).sum())
    assert num == den - kept                    # integers: exact


def test_bias_closed_forms():
    rng = _rng(22)
    m, n = 9, 13
    G = syn.integer_matrix(m, n, -8, 8, "f32", rng)
    # identity projectors (r = m = n would be needed on both sides; use a square case): bias 0
    Gs = syn.integer_matrix(6, 6, -8, 8, "f32", rng)
    eye_i = np.arange(6, dtype=np.int32).reshape(6, 1); eye_v = np.ones((6, 1), dtype=np.float32)
    num, den = _bias(Gs, "f32", eye_i, eye_v, eye_i, eye_v, 6)
    assert num == 0.0 and den == float((Gs.astype(np.float64) ** 2).sum())
    # a projector of zeros reconstructs nothing: bias exactly 1
    r, d = 4, 2
    P_idx = rng.integers(0, r, size=(m, d)).astype(np.int32); Q_idx = rng.integers(0, r, size=(n, d)).astype(np.int32)
    Q_val = rng.standard_normal((n, d)).astype(np.float32)
    num, den = _bias(G, "f32", P_idx, np.zeros((m, d), dtype=np.float32), Q_idx, Q_val, r)
    assert num == den > 0
    # rank one (r = 1): P P^T G Q Q^T = (p^T G q) p q^T
    p = rng.standard_normal((m, 1)).astype(np.float32); q = rng.standard_normal((n, 1)).astype(np.float32)
    z_m = np.zeros((m, 1), dtype=np.int32); z_n = np.zeros((n, 1), dtype=np.int32)
    num, den = _bias(G, "f32", z_m, p, z_n, q, 1)
    G64, p64, q64 = G.astype(np.float64), p.astype(np.float64)[:, 0], q.astype(np.float64)[:, 0]
    s = p64 @ G64 @ q64
    ref = float(((s * np.outer(p64, q64) - G64) ** 2).sum())
    assert abs(num - ref) <= 1e-12 * ref
    # the bias does not change when G is scaled (by a power of two: exactly)
    G4 = (G * np.float32(4.0)).astype(np.float32)
    P_val = rng.standard_normal((m, d)).astype(np.float32)
    n1, d1 = _bias(G, "f32", P_idx, P_val, Q_idx, Q_val, r)
    n4, d4 = _bias(G4, "f32", P_idx, P_val, Q_idx, Q_val, r)
    assert n4 == 16.0 * n1 and d4 == 16.0 * d1


def test_bias_a_transposed_reconstruction_is_detected():
    """With m != n a reconstruction that swapped the roles of P and Q could not even be formed; on a
    square case it can, and gives a different number: the pin above is not blind to it."""
    pb = syn.make_problem("t", 8, 8, 4, 2, "f32", seed=5, g_std=1.0)
    num, den = _bias(pb.G, "f32", pb.P_idx, pb.P_val, pb.Q_idx, pb.Q_val, 4)
    Ph, Qh = _dense(pb.P_idx, pb.P_val, 4), _dense(pb.Q_idx, pb.Q_val, 4)
    G64 = pb.G.astype(np.float64)
    wrong = Qh @ Qh.T @ G64 @ Ph @ Ph.T
    assert abs(float(((wrong - G64) ** 2).sum()) - num) > 1e-3 * num


# ---------------------------------------------------------------- optimiser-state re-projection (Alg. 1, MaybeUpdate)
def _two_projector_pairs(m, n, r, d, seed, dist="uniform"):
    rng = _rng(seed)
    return [syn.ell_projector(rows, r, d, rng, dist) for rows in (m, m, n, n)]      # P, P_prev, Q, Q_prev


@pytest.mark.parametrize("m,n,r,d,dist", [(9, 7, 4, 2, "uniform"), (20, 33, 6, 3, "zipf"), (5, 5, 5, 1, "distinct")])
def test_reproject_against_numpy(m, n, r, d, dist):
    (P_idx, P_val), (Pp_idx, Pp_val), (Q_idx, Q_val), (Qp_idx, Qp_val) = _two_projector_pairs(m, n, r, d, 500 + m, dist)
    rng = _rng(501 + m)
    M = rng.standard_normal((r, r)).astype(np.float32)
    V = (rng.standard_normal((r, r)) ** 2).astype(np.float32)
    Mo, Vo = oracle.reproject_state(P_idx, P_val, Pp_idx, Pp_val, Q_idx, Q_val, Qp_idx, Qp_val, r, M, V)
    A = _dense(P_idx, P_val, r).T @ _dense(Pp_idx, Pp_val, r)
    B = _dense(Qp_idx, Qp_val, r).T @ _dense(Q_idx, Q_val, r)
    refM = A @ M.astype(np.float64) @ B
    refV = (A * A) @ V.astype(np.float64) @ (B * B)
    np.testing.assert_allclose(Mo, refM, rtol=0, atol=1e-12 * max(1.0, np.abs(refM).max()))
    np.testing.assert_allclose(Vo, refV, rtol=0, atol=1e-12 * max(1.0, np.abs(refV).max()))
    assert Vo.min() >= 0.0                                  # a second moment stays non-negative


def test_reproject_closed_forms():
    rng = _rng(510)
    m = n = r = 6
    M = rng.standard_normal((r, r)).astype(np.float32)
    V = (rng.standard_normal((r, r)) ** 2).astype(np.float32)
    one = np.ones((m, 1), dtype=np.float32)
    ident = np.arange(r, dtype=np.int32).reshape(r, 1)
    # unchanged orthonormal projectors: P^T P_prev = I on both sides, the state is kept
    Mo, Vo = oracle.reproject_state(ident, one, ident, one, ident, one, ident, one, r, M, V)
    assert np.array_equal(Mo, M.astype(np.float64)) and np.array_equal(Vo, V.astype(np.float64))
    # the new projectors are a relabelling of the old columns: the state is permuted the same way
    pa, pb = rng.permutation(r).astype(np.int32), rng.permutation(r).astype(np.int32)
    Mo, Vo = oracle.reproject_state(pa.reshape(r, 1), one, ident, one, pb.reshape(r, 1), one, ident, one, r, M, V)
    # A[pa[i], i] = 1 and B[j, pb[j]] = 1:  M'[pa[i], pb[j]] = M[i, j]
    refM = np.zeros((r, r)); refV = np.zeros((r, r))
    refM[np.ix_(pa, pb)] = M; refV[np.ix_(pa, pb)] = V
    assert np.array_equal(Mo, refM) and np.array_equal(Vo, refV)
    # doubling the new P doubles M' and quadruples V' (element-wise squares; a matrix square would not)
    (P_idx, P_val), (Pp_idx, Pp_val), (Q_idx, Q_val), (Qp_idx, Qp_val) = _two_projector_pairs(8, 9, 4, 2, 511)
    M4 = rng.standard_normal((4, 4)).astype(np.float32); V4 = (rng.standard_normal((4, 4)) ** 2).astype(np.float32)
    M1, V1 = oracle.reproject_state(P_idx, P_val, Pp_idx, Pp_val, Q_idx, Q_val, Qp_idx, Qp_val, 4, M4, V4)
    M2, V2 = oracle.reproject_state(P_idx, 2 * P_val, Pp_idx, Pp_val, Q_idx, Q_val, Qp_idx, Qp_val, 4, M4, V4)
    assert np.array_equal(M2, 2 * M1) and np.array_equal(V2, 4 * V1)
    # the roles of the old and the new projector are not interchangeable
    M3, _ = oracle.reproject_state(Pp_idx, Pp_val, P_idx, P_val, Q_idx, Q_val, Qp_idx, Qp_val, 4, M4, V4)
    assert np.abs(M3 - M1).max() > 1e-6 * np.abs(M1).max()


# ---------------------------------------------------------------- fitting gradient (Eq. 2 / MaybeUpdate)
def _grad(G, dtype, P_idx, P_val, Q_idx, Q_val, r, **kw):
    return oracle.bias_gradient(G, dtype, P_idx, P_val, Q_idx, Q_val, r, **kw)


def _half_bias_sq(G, dtype, P_idx, P_val, Q_idx, Q_val, r):
    """F = 1/2 ||P P^T G Q Q^T - G||_F^2 from the (separately pinned) bias oracle."""
    return 0.5 * oracle.estimation_bias(G, dtype, P_idx, P_val, Q_idx, Q_val, r, dense=True)[0]


@pytest.mark.parametrize("m,n,r,d,dist", [
    (5, 7, 3, 2, "uniform"),
    (6, 4, 4, 3, "zipf"),                  # duplicate columns inside rows
    (4, 9, 2, 1, "uniform"),
])
def test_gradient_against_finite_differences_of_the_bias(m, n, r, d, dist):
    """F is a polynomial of degree four in every single projector value (the value enters P P^T twice and F is
    quadratic in P P^T), so the five-point central difference
        (-F(x+2h) + 8 F(x+h) - 8 F(x-h) + F(x-2h)) / (12 h)
    is its derivative exactly, up to fp64 rounding.  Values are multiples of 2^-6 and h = 2^-3, so every
    perturbed value is an exact float32.  F comes from the bias oracle's literal form (Def. 2), which knows
    nothing about gradients."""
    rng = _rng(900 + m * n + r)
    G = syn.integer_matrix(m, n, -8, 8, "f32", rng)
    P_idx, _ = syn.ell_projector(m, r, d, rng, dist)
    Q_idx, _ = syn.ell_projector(n, r, d, rng, dist)
    P_val = (rng.integers(-48, 49, size=(m, d)) / 64.0).astype(np.float32)
    Q_val = (rng.integers(-48, 49, size=(n, d)) / 64.0).astype(np.float32)
    h = 0.125
    for dense in (True, False):
        gP, gQ = _grad(G, "f32", P_idx, P_val, Q_idx, Q_val, r, dense=dense)
        scale = max(np.abs(gP).max(), np.abs(gQ).max())
        for (val, grad, which) in ((P_val, gP, "P"), (Q_val, gQ, "Q")):
            for (i, k) in [(0, 0), (val.shape[0] - 1, d - 1), (val.shape[0] // 2, d // 2)]:
                F = {}
                for s in (-2, -1, 1, 2):
                    v2 = val.copy()
                    v2[i, k] = np.float32(val[i, k] + s * h)
                    args = (P_idx, v2, Q_idx, Q_val) if which == "P" else (P_idx, P_val, Q_idx, v2)
                    F[s] = _half_bias_sq(G, "f32", *args, r)
                fd = (-F[2] + 8 * F[1] - 8 * F[-1] + F[-2]) / (12 * h)
                assert abs(fd - grad[i, k]) <= 1e-9 * scale, (which, i, k, dense, fd, grad[i, k])


@pytest.mark.parametrize("m,n,r,d,dist,dtype", [
    (12, 9, 6, 3, "uniform", "f32"),
    (9, 14, 5, 2, "zipf", "bf16"),
    (40, 33, 8, 4, "uniform", "f16"),
])
def test_gradient_working_form_equals_dense_form_and_numpy(m, n, r, d, dist, dtype):
    """Sparse working form (T_R S^T + T_G Z^T, Y_R S + Y_G Z) against the chain rule on dense m x m / n x n
    matrices, and both against numpy's matrix products on densified projectors."""
    pb = syn.make_problem("g", m, n, r, d, dtype, seed=700 + m * n, g_std=1.0, index_dist=dist)
    gPw, gQw = _grad(pb.G, dtype, pb.P_idx, pb.P_val, pb.Q_idx, pb.Q_val, r)
    gPd, gQd = _grad(pb.G, dtype, pb.P_idx, pb.P_val, pb.Q_idx, pb.Q_val, r, dense=True)
    Ph, Qh = _dense(pb.P_idx, pb.P_val, r), _dense(pb.Q_idx, pb.Q_val, r)
    G64 = syn.storage_to_f64(pb.G, dtype)
    A, B = Ph @ Ph.T, Qh @ Qh.T
    R = A @ G64 @ B - G64
    X = R @ B @ G64.T
    Y = G64.T @ A @ R
    refP = ((X + X.T) @ Ph)[np.arange(m)[:, None], pb.P_idx]
    refQ = ((Y + Y.T) @ Qh)[np.arange(n)[:, None], pb.Q_idx]
    scale = max(np.abs(refP).max(), np.abs(refQ).max())
    for gP, gQ in ((gPw, gQw), (gPd, gQd)):
        assert np.abs(gP - refP).max() <= 1e-11 * scale and np.abs(gQ - refQ).max() <= 1e-11 * scale


def test_gradient_closed_forms():
    rng = _rng(31)
    # (1) projectors that reproduce G exactly (identity on both sides): R = 0, so the gradient vanishes
    G = syn.integer_matrix(6, 6, -8, 8, "f32", rng)
    eye_i = np.arange(6, dtype=np.int32).reshape(6, 1); eye_v = np.ones((6, 1), dtype=np.float32)
    gP, gQ = _grad(G, "f32", eye_i, eye_v, eye_i, eye_v, 6)
    assert not gP.any() and not gQ.any()
    # (2) G inside the span of orthonormal selection projectors: R = 0 again, although r < m, n
    m, n, r = 11, 13, 4
    rows = rng.permutation(m)[:r]; cols = rng.permutation(n)[:r]
    P_idx = np.zeros((m, 1), dtype=np.int32); P_val = np.zeros((m, 1), dtype=np.float32)
    Q_idx = np.zeros((n, 1), dtype=np.int32); Q_val = np.zeros((n, 1), dtype=np.float32)
    P_idx[rows, 0] = np.arange(r); P_val[rows, 0] = 1.0
    Q_idx[cols, 0] = np.arange(r); Q_val[cols, 0] = 1.0
    G = np.zeros((m, n), dtype=np.float32)
    G[np.ix_(rows, cols)] = rng.integers(-8, 9, size=(r, r))
    gP, gQ = _grad(G, "f32", P_idx, P_val, Q_idx, Q_val, r)
    assert not gP.any() and not gQ.any()
    # (3) Euler's relation along the ray t -> F(t P, Q):  <dF/dP_val, P_val> = d/dt F(tP, Q) at t = 1
    #     = <R, 2 (R + G)> = 2 (||R||^2 + ||S||^2 - ||G||^2)   with S = P^T G Q  (since <P S Q^T, G> = ||S||^2),
    #     all three norms from the compress and bias oracles; the same for Q.
    pb = syn.make_problem("e", 17, 23, 6, 3, "f32", seed=32, g_std=1.0)
    gP, gQ = _grad(pb.G, "f32", pb.P_idx, pb.P_val, pb.Q_idx, pb.Q_val, pb.r)
    num, den = oracle.estimation_bias(pb.G, "f32", pb.P_idx, pb.P_val, pb.Q_idx, pb.Q_val, pb.r)
    S = oracle.compress(pb.G, "f32", pb.P_idx, pb.P_val, pb.Q_idx, pb.Q_val, pb.r)
    want = 2.0 * (num + float((S ** 2).sum()) - den)
    assert abs(float((gP * pb.P_val).sum()) - want) <= 1e-10 * abs(want)
    assert abs(float((gQ * pb.Q_val).sum()) - want) <= 1e-10 * abs(want)
    # (4) duplicated columns inside a row are one dense entry: their stored values get the same derivative
    P_idx = pb.P_idx.copy(); P_idx[:, 1] = P_idx[:, 0]
    gP, _ = _grad(pb.G, "f32", P_idx, pb.P_val, pb.Q_idx, pb.Q_val, pb.r)
    assert np.array_equal(gP[:, 0], gP[:, 1])
    # (5) a zero G gives a zero gradient; doubling G quadruples F and hence the gradient (exactly: power of two)
    gP1, gQ1 = _grad(pb.G, "f32", pb.P_idx, pb.P_val, pb.Q_idx, pb.Q_val, pb.r)
    gP2, gQ2 = _grad((pb.G * np.float32(2.0)).astype(np.float32), "f32", pb.P_idx, pb.P_val, pb.Q_idx, pb.Q_val, pb.r)
    assert np.array_equal(gP2, 4.0 * gP1) and np.array_equal(gQ2, 4.0 * gQ1)
    gP0, gQ0 = _grad(np.zeros_like(pb.G), "f32", pb.P_idx, pb.P_val, pb.Q_idx, pb.Q_val, pb.r)
    assert not gP0.any() and not gQ0.any()


def test_gradient_of_the_transposed_problem_swaps_the_roles():
    """F(P, Q; G) = F(Q, P; G^T): the gradient with respect to Q's values is the gradient with respect to the
    left projector of the transposed problem.  A routine that mixed up the two sides would fail here (m != n)."""
    pb = syn.make_problem("t", 10, 15, 5, 2, "f32", seed=33, g_std=1.0)
    gP, gQ = _grad(pb.G, "f32", pb.P_idx, pb.P_val, pb.Q_idx, pb.Q_val, pb.r)
    Gt = np.ascontiguousarray(pb.G.T)
    gQ_t, gP_t = _grad(Gt, "f32", pb.Q_idx, pb.Q_val, pb.P_idx, pb.P_val, pb.r)
    scale = max(np.abs(gP).max(), np.abs(gQ).max())
    assert np.abs(gP - gP_t).max() <= 1e-12 * scale and np.abs(gQ - gQ_t).max() <= 1e-12 * scale
    assert np.abs(gP).max() > 0 and np.abs(gQ).max() > 0
