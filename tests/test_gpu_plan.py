"""The device-side plan build against the host builder: the same bytes, for every shape class the plan has
(one slot with dealt lists, several slots, shared columns, spare lanes, cut rows of P^T, ragged chunks), and
its error reporting."""
import numpy as np
import pytest

import lsp_synth as syn

pytestmark = pytest.mark.gpu


def _both(m, n, r, d, dist, seed):
    import torch
    import paper_2406_10181_amd as L
    rng = np.random.default_rng(seed)
    P_idx, P_val = syn.ell_projector(m, r, d, rng, dist)
    Q_idx, Q_val = syn.ell_projector(n, r, d, rng, dist)
    nb = L.lsp_plan_bytes(m, n, r, d)
    host = np.zeros(nb, dtype=np.uint8)
    rc_host = L.lsp_plan_build_host(P_idx, P_val, Q_idx, Q_val, m, n, r, d, host, nb, check=False)
    dev = [torch.from_numpy(x).cuda() for x in (P_idx, P_val, Q_idx, Q_val)]
    plan = torch.full((nb,), 0xA5, dtype=torch.uint8, device="cuda")
    wb = L.lsp_plan_build_workspace_bytes(m, n, r, d)
    ws = torch.empty(wb, dtype=torch.uint8, device="cuda")
    status = torch.full((1,), 77, dtype=torch.int32, device="cuda")
    L.lsp_plan_build_async(*dev, m, n, r, d, plan, nb, ws, wb, status, torch.cuda.current_stream())
    torch.cuda.synchronize()
    return rc_host, host, int(status.item()), plan.cpu().numpy(), dev


@pytest.mark.parametrize("m,n,r,d,dist", [
    (48, 4200, 16, 2, "distinct"),      # three chunks, ragged last chunk, spare lanes handed out
    (40, 2048, 64, 4, "uniform"),
    (33, 2500, 96, 8, "zipf"),          # hot columns get several owners; long rows of P^T are cut
    (2000, 64, 4, 2, "uniform"),        # every row of P^T has ~1000 entries -> pieces + atomic flag
    (24, 3000, 600, 2, "uniform"),      # more columns than lanes: two slots
    (10, 7, 3, 1, "uniform"),
    (1, 1, 1, 1, "uniform"),
    (300, 6152, 256, 4, "uniform"),     # spare lanes: half the columns get a second owner
    (2048, 2048, 1280, 4, "uniform"),   # three slots
    (4096, 4096, 512, 8, "uniform"),    # a square matrix of the 6.7B-style stack
    (4096, 11008, 512, 8, "uniform"),   # its wide matrix
    (11008, 4096, 512, 8, "uniform"),   # its tall matrix
    (4096, 16384, 256, 16, "zipf"),     # wide sweep, most skewed point
    (4096, 16384, 1024, 2, "zipf"),
    (4096, 4096, 2048, 8, "uniform"),   # four slots
])
def test_device_plan_equals_host_plan(m, n, r, d, dist):
    print(f"[case] device plan m={m} n={n} r={r} d={d} {dist}", flush=True)
    rc_host, host, rc_dev, dev_plan, _ = _both(m, n, r, d, dist, seed=8800 + m + n + r)
    assert rc_host == 0 and rc_dev == 0
    bad = np.flatnonzero(host != dev_plan)
    assert bad.size == 0, f"{bad.size} bytes differ, first at offset {bad[:4]}"


def test_device_plan_reports_skew_and_bad_indices():
    import torch
    import paper_2406_10181_amd as L
    # r = 2048 uniformly used columns fill all 4 x 512 lanes; one hot column on top needs owners that do not exist
    m, n, r, d = 8, 2048, 2048, 16
    rng = np.random.default_rng(3)
    P_idx, P_val = syn.ell_projector(m, r, d, rng)
    Q_idx, Q_val = syn.ell_projector(n, r, d, rng, "distinct")
    Q_idx[:, 0] = 0
    nb = L.lsp_plan_bytes(m, n, r, d)
    host = np.zeros(nb, dtype=np.uint8)
    assert L.lsp_plan_build_host(P_idx, P_val, Q_idx, Q_val, m, n, r, d, host, nb, check=False) == -8
    dev = [torch.from_numpy(x).cuda() for x in (P_idx, P_val, Q_idx, Q_val)]
    plan = torch.full((nb,), 0xA5, dtype=torch.uint8, device="cuda")
    assert L.lsp_plan_build(*dev, m, n, r, d, plan, nb, torch.cuda.current_stream(), check=False) == -8
    assert int(plan[:4].view(torch.int32).item()) == 0, "a failed build leaves no plan behind"
    # the raw entry serves such projectors through its scatter form, chosen on the device
    import oracle
    import gpu_util as gu
    G = syn.gaussian_matrix(m, n, 1.0, "bf16", rng)
    pb = syn.Problem("skew", m, n, r, d, "bf16", G, G.copy(), P_idx, P_val, Q_idx, Q_val, np.zeros((r, r), np.float32))
    S_o = oracle.compress(G, "bf16", P_idx, P_val, Q_idx, Q_val, r)
    gu.check_compress(gu.DeviceProblem(pb).compress_raw(), S_o, "raw entry on unplannable projectors", 2e-4)
    # an index outside [0, r)
    bad = dev[2].clone()
    bad[5, 1] = r
    assert L.lsp_plan_build(dev[0], dev[1], bad, dev[3], m, n, r, d, plan, nb, torch.cuda.current_stream(), check=False) == -6
    assert int(plan[:4].view(torch.int32).item()) == 0
