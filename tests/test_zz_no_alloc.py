"""The entry point that allocates nothing (lsp_compress_planned_static) against the entry it mirrors
(lsp_compress_planned), through the C ABI: two calls in a row on one stream, the second on a smaller
problem, each compared bit for bit (the kernels are the same and, for uniformly drawn projectors, free of
atomics) and against the oracle."""
import numpy as np
import pytest

import lsp_synth as syn
import oracle

pytestmark = pytest.mark.gpu


def test_static_scratch_entry_matches_workspace_entry_two_calls_in_a_row():
    import torch
    import gpu_util as gu
    import paper_2406_10181_amd as L
    big = syn.make_problem("noalloc_big", 1100, 4104, 512, 8, "bf16", seed=9901)     # several tiles, ragged tail
    small = syn.make_problem("noalloc_small", 70, 1032, 96, 4, "f16", seed=9902)     # smaller: reuses the array's head
    assert L.lsp_static_scratch_bytes() == 24 << 20
    stream = torch.cuda.current_stream()
    dps = [gu.DeviceProblem(pb) for pb in (big, small)]
    want = [dp.compress_planned() for dp in dps]                   # the existing entry (caller's workspace)
    for dp in dps:
        dp.S.fill_(float("nan"))
    before = torch.cuda.memory_allocated()
    for dp in dps:                                                 # back to back, no sync in between
        pb = dp.pb
        print(f"[case] static scratch {pb.name} m={pb.m} n={pb.n} r={pb.r} d={pb.d} {pb.dtype}", flush=True)
        L.lsp_compress_planned_static(dp.G, dp.plan, pb.m, pb.n, pb.r, pb.d, dp.S, dp.code, stream)
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    for dp, ref in zip(dps, want):
        pb = dp.pb
        got = dp.S.cpu().numpy()
        assert np.array_equal(got, ref), f"{pb.name}: differs from lsp_compress_planned"
        S_o = oracle.compress(pb.G, pb.dtype, pb.P_idx, pb.P_val, pb.Q_idx, pb.Q_val, pb.r, threads=16)
        gu.check_compress(got, S_o, pb.name + " static scratch")


def test_static_scratch_entry_refuses_what_does_not_fit():
    import paper_2406_10181_amd as L
    fake = 0x1000
    # 16384 x 512 x 4 bytes = 32 MiB of T: above the 24 MiB the library holds
    assert L.lsp_compress_planned_static(fake, fake, 16384, 4096, 512, 8, fake, 2, None, check=False) == -9
    assert "scratch" in L.lsp_strerror(-9)
    assert L.lsp_compress_planned_static(None, fake, 64, 64, 16, 2, fake, 2, None, check=False) == -1
    assert L.lsp_compress_planned_static(fake, fake, 64, 64, 4, 8, fake, 2, None, check=False) == -2
    assert L.lsp_compress_planned_static(fake, fake, 64, 64, 16, 2, fake, 5, None, check=False) == -3
    assert L.lsp_compress_planned_static(fake + 2, fake, 64, 64, 16, 2, fake, 2, None, check=False) == -7
