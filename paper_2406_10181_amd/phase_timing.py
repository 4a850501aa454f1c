"""Per-phase cycle counts of compress kernel A (bf16, one column per lane) on one matrix.

Development aid.  Needs the library variant with the counters compiled in:

    python paper_2406_10181_amd/build.py --phase-timing
    python -m paper_2406_10181_amd.phase_timing 4096 11008 [r d]

Every wave of the kernel adds up the core-clock cycles it spends in each phase of a chunk (fetch of the next
chunk, the batches of plan rows before the staging, staging, the remaining batches, exchange of the partial
sums) and the script prints the means per wave position.  Inputs are random (uniform columns); nothing is checked
here, parity is the business of the tests."""
from __future__ import annotations

import ctypes
import sys

import numpy as np


def main(argv):
    import torch
    from . import binding as B
    from .build import PHASE_LIB
    B._LIB_PATH = PHASE_LIB                       # before the first call: the binding loads the library lazily
    import paper_2406_10181_amd as L

    m, n = int(argv[0]), int(argv[1])
    r = int(argv[2]) if len(argv) > 2 else 512
    d = int(argv[3]) if len(argv) > 3 else 8
    rows_per_block, waves, slots = 8, 8, 16
    dev = torch.device("cuda:0")
    stream = torch.cuda.current_stream()
    rng = np.random.default_rng(1)

    def projector(rows):
        idx = rng.integers(0, r, size=(rows, d), dtype=np.int32)
        val = (rng.standard_normal((rows, d)) / np.sqrt(d)).astype(np.float32)
        return torch.from_numpy(idx).to(dev), torch.from_numpy(val).to(dev)

    P_idx, P_val = projector(m)
    Q_idx, Q_val = projector(n)
    Gs = [(torch.randn(m, n, device=dev) * 1e-3).to(torch.bfloat16) for _ in range(4)]
    S = torch.empty(r, r, device=dev)
    pb = L.lsp_plan_bytes(m, n, r, d)
    plan = torch.empty(pb, dtype=torch.uint8, device=dev)
    L.lsp_plan_build(P_idx, P_val, Q_idx, Q_val, m, n, r, d, plan, pb, stream)
    wb = L.lsp_compress_planned_workspace_bytes(m, n, r, d)
    ws = torch.empty(wb, dtype=torch.uint8, device=dev)
    for G in Gs:
        L.lsp_compress_planned(G, plan, m, n, r, d, S, 2, ws, wb, stream)
    torch.cuda.synchronize()

    lib = ctypes.CDLL(PHASE_LIB)
    nwg = (m + rows_per_block - 1) // rows_per_block
    raw = np.zeros((nwg * waves, slots), dtype=np.uint64)
    rc = lib.lsp_dev_phase_read(raw.ctypes.data_as(ctypes.c_void_p), ctypes.c_size_t(raw.nbytes))
    if rc != 0:
        raise RuntimeError(f"lsp_dev_phase_read: hip error {rc}")
    b = raw.astype(np.float64).reshape(nwg, waves, slots)
    names = {0: "first stage", 1: "top of chunk", 2: "fetch + segment", 3: "first batches", 4: "stage", 6: "rest", 9: "exchange",
             12: "total", 5: "batches"}
    show = [0, 1, 2, 3, 4, 6, 9, 12, 5]
    print(f"{m} x {n}, r = {r}, d = {d}: {nwg} workgroups of {rows_per_block} rows; core clock cycles per wave, mean over workgroups")
    print("wave  " + "  ".join(f"{names[k]:>15s}" for k in show))
    for w in list(range(waves)) + [None]:
        sel = b[:, w, :] if w is not None else b.reshape(-1, slots)
        print(f"{'mean' if w is None else w:>4}  " + "  ".join(f"{sel[:, k].mean():15.0f}" for k in show))
    ghz = b[:, :, 12].mean() / (b[:, :, 14].mean() * 10.0)        # wall clock ticks at 100 MHz
    print(f"core clock {ghz:.2f} GHz; cycles per batch of 4 plan rows: before the staging {b[:, :, 3].sum() / b[:, :, 7].sum():.0f}, "
          f"after it {b[:, :, 6].sum() / b[:, :, 8].sum():.0f}")
    entry = b[:, :, 15].min(axis=1)
    end = (b[:, :, 15] + b[:, :, 14]).max(axis=1)
    print(f"workgroup loop: mean {b[:, 0, 14].mean() / 100:.1f} us, min {b[:, 0, 14].min() / 100:.1f}, max {b[:, 0, 14].max() / 100:.1f}; "
          f"first loop start to last loop end {(end.max() - entry.min()) / 100:.1f} us")


if __name__ == "__main__":
    main(sys.argv[1:])
