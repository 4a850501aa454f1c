"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle, element by
element on the same seeded inputs."""
import numpy as np
import pytest

import lsp_synth as syn
import oracle

pytestmark = pytest.mark.gpu

THREADS = 16


def _dp(pb):
    from gpu_util import DeviceProblem
    return DeviceProblem(pb)


def _full_check(pb, tight=5e-5, raw=True):
    import gpu_util as gu
    print(f"[case] {pb.name} m={pb.m} n={pb.n} r={pb.r} d={pb.d} {pb.dtype}", flush=True)
    dp = _dp(pb)
    S_o = oracle.compress(pb.G, pb.dtype, pb.P_idx, pb.P_val, pb.Q_idx, pb.Q_val, pb.r, threads=THREADS)
    S_p = dp.compress_planned()
    e1 = gu.check_compress(S_p, S_o, pb.name + " planned", tight)
    if raw:
        S_r = dp.compress_raw()
        gu.check_compress(S_r, S_o, pb.name + " raw", tight)
    Wp, Wr = oracle.decompress_apply(pb.W, pb.dtype, pb.S_in, pb.P_idx, pb.P_val, pb.Q_idx, pb.Q_val,
                                     threads=THREADS)
    W_g = dp.decompress(pb.S_in)
    mism = gu.check_decompress(W_g, pb.W, Wp, Wr, pb.dtype, pb.name)
    # fp32 storage: the last bit of an fp32 evaluation legitimately differs from the rounded fp64 value
    assert pb.dtype == "f32" or mism < 0.02, f"{pb.name}: {mism:.4f} of W differs from the singly rounded oracle"
    print(f"[ok]   {pb.name} compress rel err {e1:.2e}, W mismatch fraction {mism:.2e}", flush=True)
    return dp


# ------------------------------------------------------------------ the five benchmark configurations
def test_config1_fp32_small():
    dp = _full_check(syn.config1(), tight=2e-6)
    # round trip: decompress the compressed gradient (what MaybeUpdate's bias test composes)
    import gpu_util as gu
    pb = dp.pb
    S_g = dp.compress_planned()
    Wp, Wr = oracle.decompress_apply(pb.W, pb.dtype, S_g, pb.P_idx, pb.P_val, pb.Q_idx, pb.Q_val)
    gu.check_decompress(dp.decompress(S_g), pb.W, Wp, Wr, pb.dtype, "cfg1 round trip")


def test_config2_fp16_attention():
    _full_check(syn.config2())


def test_config3_fp16_mlp_heavy_rows():
    for pb in syn.config3():
        _full_check(pb)


@pytest.mark.parametrize("which", [0, 1, 3])      # down 11008x4096, gate 4096x11008, o 4096x4096
def test_config4_bf16_layer_shapes(which):
    _full_check(syn.config4_matrix(31, which), raw=(which == 3))


@pytest.mark.parametrize("r,d", [(r, d) for r in (256, 512, 1024) for d in (2, 4, 8, 16)])
def test_config5_bf16_zipf_wide(r, d):
    # skewed columns: lists are cut into pieces and summed with atomics; accumulation error grows
    # with the number of terms per entry (up to ~2.6e5), still far below the bar
    _full_check(syn.config5_point(r, d, index=r + d), tight=2e-4, raw=False)


# ------------------------------------------------------------------ bit-exact index handling
@pytest.mark.parametrize("m,n,r,d,dtype,dist", [
    (256, 2048, 64, 4, "bf16", "uniform"),
    (100, 3000, 16, 2, "f16", "distinct"),       # ragged rows, three chunks
    (64, 1040, 8, 8, "bf16", "zipf"),            # cut lists, atomic pieces
    (48, 1000, 20, 3, "f32", "uniform"),         # generic decompress kernel (d = 3)
    (37, 53, 6, 1, "f32", "uniform"),            # selection-like, everything ragged
])
def test_integer_inputs_bit_exact(m, n, r, d, dtype, dist):
    pb = syn.make_integer_problem("int", m, n, r, d, dtype, seed=900 + m, index_dist=dist)
    print(f"[case] integer m={m} n={n} r={r} d={d} {dtype} {dist}", flush=True)
    dp = _dp(pb)
    S_o = oracle.compress(pb.G, dtype, pb.P_idx, pb.P_val, pb.Q_idx, pb.Q_val, r)
    assert np.abs(S_o).max() < 2 ** 24                       # exactly representable in fp32
    assert np.array_equal(dp.compress_planned().astype(np.float64), S_o)
    assert np.array_equal(dp.compress_raw().astype(np.float64), S_o)
    Wp, Wr = oracle.decompress_apply(pb.W, dtype, pb.S_in, pb.P_idx, pb.P_val, pb.Q_idx, pb.Q_val)
    W_g = dp.decompress(pb.S_in)
    if dtype == "f32":
        assert np.array_equal(W_g, Wr)
    else:
        # the fp32 update is exact on integers, so the single rounding to 16 bits must agree bit for bit
        assert np.array_equal(W_g.view(np.uint16), Wr.view(np.uint16))


def test_selection_projectors_block_sums_bit_exact():
    rng = np.random.default_rng(5)
    m, n, r = 300, 2500, 32
    G = syn.integer_matrix(m, n, -8, 8, "bf16", rng)
    p = rng.integers(0, r, size=(m, 1)).astype(np.int32)
    q = rng.integers(0, r, size=(n, 1)).astype(np.int32)
    pb = syn.Problem("sel", m, n, r, 1, "bf16", G, G.copy(), p, np.ones((m, 1), np.float32), q,
                     np.ones((n, 1), np.float32), np.zeros((r, r), np.float32))
    G64 = syn.storage_to_f64(G, "bf16")
    ref = np.zeros((r, r))
    np.add.at(ref, (p[:, 0][:, None], q[:, 0][None, :]), G64)       # plain block sums of G
    dp = _dp(pb)
    assert np.array_equal(dp.compress_planned().astype(np.float64), ref)
    assert np.array_equal(dp.compress_raw().astype(np.float64), ref)


# ------------------------------------------------------------------ edge shapes
@pytest.mark.parametrize("m,n,r,d,dtype", [
    (1, 1, 1, 1, "f32"),
    (1, 8, 4, 2, "bf16"),
    (17, 9, 5, 5, "f16"),            # d == r, nothing aligned
    (16, 1024, 16, 2, "bf16"),       # exactly one tile, one chunk
    (15, 1025, 12, 4, "bf16"),       # one row short, one column over a chunk
    (130, 4100, 256, 4, "f16"),
    (40, 2048, 2048, 8, "bf16"),     # largest subspace (two-plane kernels)
    (33, 520, 1030, 2, "bf16"),      # r not a multiple of 4 above 1024
    (24, 64, 1000, 16, "f32"),
])
def test_edge_shapes(m, n, r, d, dtype):
    pb = syn.make_problem(f"edge_{m}x{n}_r{r}_d{d}", m, n, r, d, dtype, seed=300 + m + n, g_std=0.5,
                          index_dist="uniform" if d < r else "distinct")
    _full_check(pb)


def test_zero_and_identity_cases():
    pb = syn.make_problem("zero", 64, 2048, 128, 4, "bf16", seed=42)
    dp = _dp(pb)
    # S = 0 leaves W unchanged bit for bit
    W_g = dp.decompress(np.zeros((pb.r, pb.r), np.float32))
    assert np.array_equal(W_g, pb.W)
    # G = 0 gives S = 0 exactly (and S is overwritten, not accumulated: it was NaN-filled)
    dp.G.zero_()
    assert not dp.compress_planned().any()
    assert not dp.compress_raw().any()


def test_planned_path_is_reproducible_and_plan_reusable():
    pb = syn.config2()
    dp = _dp(pb)
    a = dp.compress_planned()
    b = dp.compress_planned()
    assert np.array_equal(a, b)                      # no atomics on this path for uniform projectors
    # a second gradient through the same plan (projectors fixed between refreshes)
    G2 = syn.gaussian_matrix(pb.m, pb.n, 1e-3, pb.dtype, np.random.default_rng(99))
    import gpu_util as gu
    dp.G.copy_(gu.to_device(G2, pb.dtype))
    S2 = dp.compress_planned()
    S2_o = oracle.compress(G2, pb.dtype, pb.P_idx, pb.P_val, pb.Q_idx, pb.Q_val, pb.r, threads=THREADS)
    gu.check_compress(S2, S2_o, "cfg2 second gradient")


def test_plan_of_another_problem_is_not_followed():
    """A plan built for other sizes, or a buffer that holds no plan: the kernels follow none of its offsets,
    write nothing but S, and S comes back filled with NaN; the next correct call works."""
    import torch
    import gpu_util as gu
    import paper_2406_10181_amd as L
    pb = syn.make_problem("mismatch", 200, 2304, 128, 4, "bf16", seed=77)
    dp = _dp(pb)
    stream = torch.cuda.current_stream()
    others = [(264, 2304, 128, 4), (200, 4096, 128, 4), (200, 2304, 256, 4), (200, 2304, 128, 8)]   # m, n, r, d differ in turn
    plans = []
    for (m2, n2, r2, d2) in others:
        rng = np.random.default_rng(m2 + n2 + r2 + d2)
        pi, pv = syn.ell_projector(m2, r2, d2, rng)
        qi, qv = syn.ell_projector(n2, r2, d2, rng)
        nb = L.lsp_plan_bytes(m2, n2, r2, d2)
        host = np.zeros(nb, dtype=np.uint8)
        L.lsp_plan_build_host(pi, pv, qi, qv, m2, n2, r2, d2, host, nb)
        plans.append(torch.from_numpy(host).cuda())
    plans.append(torch.zeros(4096, dtype=torch.uint8, device="cuda"))          # no plan at all
    for k, plan in enumerate(plans):
        print(f"[case] foreign plan {k}", flush=True)
        dp.S.fill_(1.0)
        dp.ws.fill_(0x5A)
        rc = L.lsp_compress_planned(dp.G, plan, pb.m, pb.n, pb.r, pb.d, dp.S, dp.code, dp.ws, dp.ws_bytes, stream, check=False)
        torch.cuda.synchronize()
        assert rc == 0
        assert torch.isnan(dp.S).all(), "S must be NaN-filled when the plan does not belong to the problem"
        assert (dp.ws == 0x5A).all(), "nothing but S may be written"
    S_o = oracle.compress(pb.G, pb.dtype, pb.P_idx, pb.P_val, pb.Q_idx, pb.Q_val, pb.r)
    gu.check_compress(dp.compress_planned(), S_o, "after the foreign plans")


def _grouped_case(pbs, tight=5e-5, reordered_q=False):
    """Grouped calls against the oracle, and bit for bit against the single calls.  reordered_q: the expand
    side gets the copy of Q made by lsp_projector_reorder_host (the same projector, so the oracle keeps the
    original arrays)."""
    import torch
    import gpu_util as gu
    import paper_2406_10181_amd as L
    r, d, code = pbs[0].r, pbs[0].d, syn.DTYPE_CODE[pbs[0].dtype]
    dps = [_dp(pb) for pb in pbs]
    if reordered_q:
        for dp in dps:
            dp.use_reordered_q()
    for dp in dps:
        dp.build_plan()
    singles = [dp.compress_planned() for dp in dps]
    for dp in dps:
        dp.S.fill_(float("nan"))
    stream = torch.cuda.current_stream()
    items = L.compress_items([(dp.G, dp.plan, dp.S, dp.ws, dp.ws_bytes, dp.pb.m, dp.pb.n) for dp in dps])
    L.lsp_compress_planned_grouped(items, len(dps), r, d, code, stream)
    torch.cuda.synchronize()
    for dp, single in zip(dps, singles):
        pb = dp.pb
        print(f"[case] grouped {pb.name} m={pb.m} n={pb.n} r={pb.r} d={pb.d} {pb.dtype}", flush=True)
        S_g = dp.S.cpu().numpy()
        S_o = oracle.compress(pb.G, pb.dtype, pb.P_idx, pb.P_val, pb.Q_idx, pb.Q_val, pb.r, threads=THREADS)
        gu.check_compress(S_g, S_o, pb.name + " grouped", tight)
        assert np.array_equal(S_g, single), f"{pb.name}: grouped compress differs from the single call"
    W_single = [dp.decompress(dp.pb.S_in) for dp in dps]
    Wd = [dp.W.clone() for dp in dps]
    Sd = [torch.from_numpy(np.ascontiguousarray(dp.pb.S_in, dtype=np.float32)).cuda() for dp in dps]
    aitems = L.apply_items([(w, s, dp.P_idx, dp.P_val, dp.Qx_idx, dp.Qx_val, dp.pb.m, dp.pb.n)
                            for w, s, dp in zip(Wd, Sd, dps)])
    L.lsp_decompress_apply_grouped(aitems, len(dps), r, d, code, stream)
    torch.cuda.synchronize()
    for dp, w, ws in zip(dps, Wd, W_single):
        pb = dp.pb
        W_g = gu.to_host(w, pb.dtype)
        Wp, Wr = oracle.decompress_apply(pb.W, pb.dtype, pb.S_in, pb.P_idx, pb.P_val, pb.Q_idx, pb.Q_val, threads=THREADS)
        gu.check_decompress(W_g, pb.W, Wp, Wr, pb.dtype, pb.name + " grouped")
        assert np.array_equal(W_g, ws), f"{pb.name}: grouped decompress differs from the single call"


def test_grouped_calls_mixed_shapes():
    # three problems of different shapes (tall, wide with a ragged row block, small) in one launch per kernel
    pbs = [syn.make_problem("grp_a", 300, 4096, 256, 4, "bf16", seed=901),
           syn.make_problem("grp_b", 70, 6152, 256, 4, "bf16", seed=902),
           syn.make_problem("grp_c", 16, 2048, 256, 4, "bf16", seed=903)]
    _grouped_case(pbs)


def test_grouped_calls_fall_back_when_kernel_variants_differ():
    # n % 8 != 0 in one problem (element-wise loads, generic decompress): the call serves them one by one
    pbs = [syn.make_problem("grpmix_a", 64, 1030, 64, 3, "f16", seed=911),
           syn.make_problem("grpmix_b", 40, 2048, 64, 3, "f16", seed=912)]
    _grouped_case(pbs)


def test_big_grid_with_ragged_last_row_block():
    # 1027 blocks of 16 rows (the last one with 5 rows): the big-grid geometry of both kernels (several row
    # blocks per workgroup in compress, 32-row workgroups in decompress) with an odd block count and a ragged tail
    pb = syn.make_problem("big_ragged", 16 * 1026 + 5, 2048, 512, 4, "bf16", seed=921)
    _grouped_case([pb])
    _full_check(pb, raw=False)


def test_big_grid_with_an_odd_number_of_passes():
    # 32-row apply workgroups of 512 threads take 1024 columns per pass: three passes here, and the last row
    # blocks of the launch are shared by two workgroups with two passes and one
    pb = syn.make_problem("big_odd", 16 * 1030 + 9, 3072, 512, 8, "bf16", seed=925)
    _grouped_case([pb])
    _full_check(pb, raw=False)


@pytest.mark.parametrize("n,r,d,dist", [
    (1024, 1024, 2, "uniform"),       # two columns per lane, none shared
    (2048, 600, 4, "zipf"),           # hot columns split between lanes: several slots and the ordered merge
])
def test_big_grid_with_several_columns_per_lane(n, r, d, dist):
    # a workgroup walks two row blocks while every lane owns several columns of T
    pb = syn.make_problem("big_slots", 16 * 1030 + 3, n, r, d, "bf16", seed=930 + d, index_dist=dist)
    _full_check(pb, tight=2e-4, raw=False)


@pytest.mark.parametrize("m,n,r,d,dtype", [
    (4096, 4096, 2048, 8, "bf16"),    # subspace 2048 with 8 entries per row on a 4096-wide layer
    (2048, 2048, 1280, 4, "f16"),     # subspace 1280 with 4 entries per row on a 2048-wide layer
])
def test_paper_sized_subspaces(m, n, r, d, dtype):
    """The subspace sizes the paper trained with (its experiments section), at full matrix size."""
    pb = syn.make_problem("paper_r", m, n, r, d, dtype, seed=940 + d)
    _full_check(pb, raw=False)
    _bias_check(syn.make_problem("paper_r_bias", m, n, r, d, dtype, seed=950 + d, g_std=1.0))


@pytest.mark.parametrize("layer", [31, 16, 0])
def test_grouped_layer_of_config4(layer):
    # all seven matrices of a layer of the 6.7B-style stack, at full size, in one grouped call per kernel family
    # with the reordered copy of Q on the expand side -- the launches bench.py times: every element against
    # the oracle, and bit for bit against the single calls
    pbs = [syn.config4_matrix(layer, which) for which in range(7)]
    _grouped_case(pbs, reordered_q=True)


def test_fp16_subnormals_are_not_flushed():
    m, n, r, d = 32, 1024, 16, 2
    rng = np.random.default_rng(7)
    # gradients entirely below the fp16 minimum normal (6.1e-5): flushing them would give S = 0
    G = (rng.integers(1, 1023, size=(m, n)).astype(np.uint16)).view(np.float16)
    P_idx, P_val = syn.ell_projector(m, r, d, rng, value_mode="smallint")
    Q_idx, Q_val = syn.ell_projector(n, r, d, rng, value_mode="smallint")
    pb = syn.Problem("sub", m, n, r, d, "f16", G, G.copy(), P_idx, P_val, Q_idx, Q_val,
                     np.zeros((r, r), np.float32))
    S_o = oracle.compress(G, "f16", P_idx, P_val, Q_idx, Q_val, r)
    assert np.abs(S_o).max() > 0
    import gpu_util as gu
    dp = _dp(pb)
    gu.check_compress(dp.compress_planned(), S_o, "fp16 subnormal", tight=1e-6)
    gu.check_compress(dp.compress_raw(), S_o, "fp16 subnormal raw", tight=1e-6)


def test_validate_projector_and_plan_index_error():
    import torch
    import paper_2406_10181_amd as L
    pb = syn.make_problem("val", 64, 64, 16, 2, "f32", seed=1)
    dp = _dp(pb)
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    assert L.lsp_validate_projector(dp.Q_idx, 64, 2, 16, flag) == 0
    bad = dp.Q_idx.clone()
    bad[5, 1] = 16
    assert L.lsp_validate_projector(bad, 64, 2, 16, flag) == -6
    plan = torch.empty(L.lsp_plan_bytes(64, 64, 16, 2), dtype=torch.uint8, device="cuda")
    rc = L.lsp_plan_build(dp.P_idx, dp.P_val, bad, dp.Q_val, 64, 64, 16, 2, plan, plan.numel(), check=False)
    assert rc == -6


# ------------------------------------------------------------------ estimation bias (Def. 2)
BIAS_NUM_RTOL = 2e-4      # on || P S Q^T - G ||_F^2, relative to itself
BIAS_NUM_FLOOR = 2e-6     # plus this fraction of || G ||_F^2


def _bias_check(pb, tol=2e-4):
    print(f"[case] bias {pb.name} m={pb.m} n={pb.n} r={pb.r} d={pb.d} {pb.dtype}", flush=True)
    num, den = oracle.estimation_bias(pb.G, pb.dtype, pb.P_idx, pb.P_val, pb.Q_idx, pb.Q_val, pb.r)
    got = _dp(pb).estimation_bias()
    assert abs(got[1] - den) <= 1e-5 * den, f"{pb.name}: ||G||^2 {got[1]} vs {den}"
    # relative to the numerator itself (it is small when the projectors fit well), with a floor for the fp32
    # evaluation of P S Q^T - G, whose absolute error scales with G, not with the difference
    assert abs(got[0] - num) <= BIAS_NUM_RTOL * num + BIAS_NUM_FLOOR * den, f"{pb.name}: numerator {got[0]} vs {num}"
    want = np.sqrt(num / den)
    assert abs(got[2] - want) <= tol * want + 1e-6, f"{pb.name}: bias {got[2]} vs {want}"
    print(f"[ok]   bias {pb.name}: {got[2]:.6f} (oracle {want:.6f})", flush=True)
    return got


@pytest.mark.parametrize("m,n,r,d,dtype,dist", [
    (256, 256, 16, 2, "f32", "distinct"),        # config 1
    (512, 2048, 256, 4, "f16", "uniform"),
    (203, 3000, 512, 8, "bf16", "uniform"),      # ragged last row block, several passes over the columns
    (100, 1030, 64, 3, "bf16", "uniform"),       # generic kernel (d = 3, n % 4 != 0)
    (96, 1024, 1500, 2, "bf16", "uniform"),      # 8 rows per workgroup
    (64, 2048, 256, 16, "f16", "zipf"),          # d = 16: one pass in registers
])
def test_estimation_bias_against_oracle(m, n, r, d, dtype, dist):
    _bias_check(syn.make_problem("bias", m, n, r, d, dtype, seed=4000 + m + n, g_std=1.0, index_dist=dist))


def test_estimation_bias_config4_shape():
    _bias_check(syn.config4_matrix(31, 3))         # 4096 x 4096 bf16, r = 512, d = 8


def test_estimation_bias_exact_on_integers():
    """Small integers and selection projectors: every sum is an integer below 2^24, so the two
    squared norms are exact, and the reconstruction keeps exactly the selected block."""
    rng = np.random.default_rng(77)
    m, n, r = 203, 1000, 7
    G = syn.integer_matrix(m, n, -8, 8, "bf16", rng)
    rows = rng.permutation(m)[:r]; cols = rng.permutation(n)[:r]
    P_idx = np.zeros((m, 1), dtype=np.int32); P_val = np.zeros((m, 1), dtype=np.float32)
    Q_idx = np.zeros((n, 1), dtype=np.int32); Q_val = np.zeros((n, 1), dtype=np.float32)
    P_idx[rows, 0] = np.arange(r); P_val[rows, 0] = 1.0
    Q_idx[cols, 0] = rng.permutation(r); Q_val[cols, 0] = 1.0
    pb = syn.make_problem("sel", m, n, r, 1, "bf16", seed=1)
    pb.G, pb.P_idx, pb.P_val, pb.Q_idx, pb.Q_val = G, P_idx, P_val, Q_idx, Q_val
    num, den = oracle.estimation_bias(G, "bf16", P_idx, P_val, Q_idx, Q_val, r)
    got = _dp(pb).estimation_bias(planned=False)
    assert den < 2 ** 24 and float(got[0]) == num and float(got[1]) == den


def test_estimation_bias_is_reproducible_and_checks_arguments():
    import torch
    import paper_2406_10181_amd as L
    pb = syn.make_problem("rep", 300, 2048, 128, 4, "bf16", seed=9, g_std=1.0)
    dp = _dp(pb)
    a, b = dp.estimation_bias(), dp.estimation_bias()
    assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
    nb = L.lsp_estimation_bias_workspace_bytes(pb.m, pb.n, pb.r, pb.d)
    ws = torch.empty(nb, dtype=torch.uint8, device="cuda"); out = torch.zeros(3, device="cuda")
    args = (dp.G, dp.S, dp.P_idx, dp.P_val, dp.Q_idx, dp.Q_val, pb.m, pb.n, pb.r, pb.d, out)
    assert L.lsp_estimation_bias(*args, ws, nb - 1, dp.code, None, check=False) == -4
    assert L.lsp_estimation_bias(*args, ws, nb, 7, None, check=False) == -3


# ------------------------------------------------------------------ optimiser-state re-projection (MaybeUpdate)
@pytest.mark.parametrize("m,n,r,d,dist,with_v", [
    (300, 200, 64, 4, "uniform", True),
    (257, 131, 50, 3, "zipf", True),             # r not a multiple of the 64 x 64 tile, duplicates
    (128, 128, 16, 2, "distinct", False),        # first moment only
    (4096, 4096, 512, 8, "uniform", True),       # config-4 size
    (200, 160, 1100, 4, "uniform", True),        # r past 1024 and not a multiple of the tiles of the r x r products
])
def test_reproject_state_against_oracle(m, n, r, d, dist, with_v):
    import torch
    import paper_2406_10181_amd as L
    print(f"[case] reproject m={m} n={n} r={r} d={d} {dist}", flush=True)
    rng = np.random.default_rng(6000 + m + r)
    prj = [syn.ell_projector(rows, r, d, rng, dist) for rows in (m, m, n, n)]     # P, P_prev, Q, Q_prev
    M = rng.standard_normal((r, r)).astype(np.float32)
    V = (rng.standard_normal((r, r)) ** 2).astype(np.float32)
    Mo, Vo = oracle.reproject_state(*prj[0], *prj[1], *prj[2], *prj[3], r, M, V)
    dev = [torch.from_numpy(x).cuda() for pair in prj for x in pair]
    Md, Vd = torch.from_numpy(M).cuda(), torch.from_numpy(V).cuda()
    nb = L.lsp_reproject_state_workspace_bytes(r)
    ws = torch.empty(nb, dtype=torch.uint8, device="cuda")
    L.lsp_reproject_state(*dev, m, n, r, d, Md, Vd if with_v else None, ws, nb, torch.cuda.current_stream())
    torch.cuda.synchronize()
    eM = np.abs(Md.cpu().numpy() - Mo).max() / np.abs(Mo).max()
    assert eM <= 2e-5, f"M: {eM}"
    if with_v:
        Vg = Vd.cpu().numpy()
        eV = np.abs(Vg - Vo).max() / np.abs(Vo).max()
        assert eV <= 2e-5 and Vg.min() >= 0.0, f"V: {eV}"
    else:
        assert np.array_equal(Vd.cpu().numpy(), V)
    print(f"[ok]   reproject: M rel err {eM:.2e}", flush=True)


def test_reproject_state_concentrated_columns():
    """Every row of P and of P_prev has its first entry in column 0: one row block of P^T P_prev receives more
    products than the workgroup's queue holds, so the rest takes the kernel's direct path."""
    import torch
    import paper_2406_10181_amd as L
    m, n, r, d = 5000, 40, 32, 2
    print(f"[case] reproject concentrated m={m} n={n} r={r} d={d}", flush=True)
    rng = np.random.default_rng(6077)
    prj = [syn.ell_projector(rows, r, d, rng, "uniform") for rows in (m, m, n, n)]
    prj[0][0][:, 0] = 0
    prj[1][0][:, 0] = 0
    M = rng.standard_normal((r, r)).astype(np.float32)
    V = (rng.standard_normal((r, r)) ** 2).astype(np.float32)
    Mo, Vo = oracle.reproject_state(*prj[0], *prj[1], *prj[2], *prj[3], r, M, V)
    dev = [torch.from_numpy(np.ascontiguousarray(x)).cuda() for pair in prj for x in pair]
    Md, Vd = torch.from_numpy(M).cuda(), torch.from_numpy(V).cuda()
    nb = L.lsp_reproject_state_workspace_bytes(r)
    ws = torch.empty(nb, dtype=torch.uint8, device="cuda")
    L.lsp_reproject_state(*dev, m, n, r, d, Md, Vd, ws, nb, torch.cuda.current_stream())
    torch.cuda.synchronize()
    eM = np.abs(Md.cpu().numpy() - Mo).max() / np.abs(Mo).max()
    eV = np.abs(Vd.cpu().numpy() - Vo).max() / np.abs(Vo).max()
    print(f"[ok]   reproject concentrated: rel err M {eM:.2e} V {eV:.2e}", flush=True)
    assert eM <= 2e-5 and eV <= 2e-5, (eM, eV)


def test_reproject_state_exact_on_relabelled_projectors():
    """New projectors that relabel the old columns: P^T P_prev and Q_prev^T Q are permutation matrices and
    the moments are permuted, bit for bit."""
    import torch
    import paper_2406_10181_amd as L
    rng = np.random.default_rng(61)
    r = 96
    M = rng.standard_normal((r, r)).astype(np.float32)
    V = (rng.standard_normal((r, r)) ** 2).astype(np.float32)
    ident = np.arange(r, dtype=np.int32).reshape(r, 1); one = np.ones((r, 1), dtype=np.float32)
    pa, pb = rng.permutation(r).astype(np.int32), rng.permutation(r).astype(np.int32)
    host = [pa.reshape(r, 1), one, ident, one, pb.reshape(r, 1), one, ident, one]
    Mo, Vo = oracle.reproject_state(*host, r, M, V)
    dev = [torch.from_numpy(np.ascontiguousarray(x)).cuda() for x in host]
    Md, Vd = torch.from_numpy(M).cuda(), torch.from_numpy(V).cuda()
    nb = L.lsp_reproject_state_workspace_bytes(r)
    ws = torch.empty(nb, dtype=torch.uint8, device="cuda")
    L.lsp_reproject_state(*dev, r, r, r, 1, Md, Vd, ws, nb, torch.cuda.current_stream())
    torch.cuda.synchronize()
    assert np.array_equal(Md.cpu().numpy().astype(np.float64), Mo) and np.array_equal(Vd.cpu().numpy().astype(np.float64), Vo)


# ------------------------------------------------------------------ seeded sweep over odd shapes
def _sweep_cases():
    rng = np.random.default_rng(20240611)
    cases = []
    for k in range(40):
        r = int(rng.choice([1, 3, 16, 50, 128, 300, 512, 513, 700, 1100]))
        d = int(min(r, rng.choice([1, 2, 3, 4, 8, 16])))
        m = int(rng.integers(1, 180)) if k < 24 else int(rng.choice([15, 16, 17, 31, 33, 255, 257, 640]))
        n = int(rng.choice([1, 7, 8, 64, 1000, 2048, 2056, 4100, 4104, 6200]))
        dtype = str(rng.choice(["f32", "f16", "bf16"]))
        dist = str(rng.choice(["uniform", "zipf"]))
        cases.append((m, n, r, d, dtype, dist, 7000 + k))
    return cases


@pytest.mark.parametrize("m,n,r,d,dtype,dist,seed", _sweep_cases())
def test_seeded_shape_sweep(m, n, r, d, dtype, dist, seed):
    """Shapes nobody would pick by hand: one column, one row, r = 1, chunk boundaries +-8, more columns of T than
    lanes, every storage type; compress (plan), decompress-apply and the estimation bias against the oracle."""
    import gpu_util as gu
    import paper_2406_10181_amd as L
    pb = syn.make_problem("sweep", m, n, r, d, dtype, seed=seed, g_std=1.0, w_std=1.0, s_std=1.0, index_dist=dist)
    try:
        _full_check(pb, tight=2e-4, raw=False)
    except L.LspError as e:
        # columns used too unevenly for a plan: the raw entry point is the documented way out
        assert "unevenly" in str(e), e
        S_o = oracle.compress(pb.G, pb.dtype, pb.P_idx, pb.P_val, pb.Q_idx, pb.Q_val, pb.r, threads=THREADS)
        gu.check_compress(_dp(pb).compress_raw(), S_o, "sweep raw", 2e-4)
        got = _dp(pb).estimation_bias(planned=False)
        num, den = oracle.estimation_bias(pb.G, pb.dtype, pb.P_idx, pb.P_val, pb.Q_idx, pb.Q_val, pb.r)
        assert abs(got[0] - num) <= BIAS_NUM_RTOL * num + BIAS_NUM_FLOOR * den and abs(got[1] - den) <= 1e-5 * den
        return
    _bias_check(pb)


# ------------------------------------------------------------------ reordered projector rows on the expand side
@pytest.mark.parametrize("m,n,r,d,dtype", [(100, 3000, 512, 8, "bf16"), (64, 1030, 64, 3, "f16"), (40, 2048, 2048, 8, "bf16")])
def test_decompress_with_reordered_projector_rows(m, n, r, d, dtype):
    """The copy of Q made by lsp_projector_reorder_host is the same projector: decompress-apply and the bias with
    it meet the oracle's result for the original arrays."""
    import dataclasses
    import paper_2406_10181_amd as L
    import gpu_util as gu
    pb = syn.make_problem("reord", m, n, r, d, dtype, seed=8100 + n, g_std=1.0)
    qi, qv = np.empty_like(pb.Q_idx), np.empty_like(pb.Q_val)
    L.lsp_projector_reorder_host(pb.Q_idx, pb.Q_val, n, d, r, qi, qv)
    pb2 = dataclasses.replace(pb, Q_idx=qi, Q_val=qv)
    Wp, Wr = oracle.decompress_apply(pb.W, pb.dtype, pb.S_in, pb.P_idx, pb.P_val, pb.Q_idx, pb.Q_val, threads=THREADS)
    mism = gu.check_decompress(_dp(pb2).decompress(pb.S_in), pb.W, Wp, Wr, pb.dtype, "reordered Q")
    assert pb.dtype == "f32" or mism < 0.02
    num, den = oracle.estimation_bias(pb.G, pb.dtype, pb.P_idx, pb.P_val, pb.Q_idx, pb.Q_val, pb.r)
    got = _dp(pb2).estimation_bias()
    assert abs(got[0] - num) <= BIAS_NUM_RTOL * num + BIAS_NUM_FLOOR * den and abs(got[1] - den) <= 1e-5 * den


def test_projector_reorder_on_device_arrays_equals_host():
    import torch
    import paper_2406_10181_amd as L
    rng = np.random.default_rng(8300)
    idx, val = syn.ell_projector(1000, 300, 8, rng, "uniform")
    hi, hv = np.empty_like(idx), np.empty_like(val)
    L.lsp_projector_reorder_host(idx, val, 1000, 8, 300, hi, hv)
    di, dv = torch.from_numpy(idx).cuda(), torch.from_numpy(val).cuda()
    oi, ov = torch.empty_like(di), torch.empty_like(dv)
    L.lsp_projector_reorder(di, dv, 1000, 8, 300, oi, ov, torch.cuda.current_stream())
    assert np.array_equal(oi.cpu().numpy(), hi) and np.array_equal(ov.cpu().numpy(), hv)
    assert L.lsp_projector_reorder(di, dv, 1000, 8, 300, di, ov, None, check=False) == -2


def test_decompress_with_reordered_rows_exact_on_integers():
    import dataclasses
    import paper_2406_10181_amd as L
    pb = syn.make_integer_problem("reord_int", 70, 2100, 48, 4, "bf16", seed=8200, index_dist="zipf")
    qi, qv = np.empty_like(pb.Q_idx), np.empty_like(pb.Q_val)
    L.lsp_projector_reorder_host(pb.Q_idx, pb.Q_val, pb.n, pb.d, pb.r, qi, qv)
    a = _dp(pb).decompress(pb.S_in)
    b = _dp(dataclasses.replace(pb, Q_idx=qi, Q_val=qv)).decompress(pb.S_in)
    assert np.array_equal(a, b)
