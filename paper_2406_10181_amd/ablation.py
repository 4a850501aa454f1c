"""What each piece of the two hot kernels costs: grouped launches of one 6.7B-style layer (benchmark configuration 4:
seven matrices, bf16, r = 512, d = 8) timed with library variants in which one piece is compiled out.

Development aid.  The variants compute wrong results by design; nothing is checked here.

    python paper_2406_10181_amd/build.py --ablations
    python -m paper_2406_10181_amd.ablation [layers] [repetitions]

Every variant runs in a process of its own (the binding loads one library per process) and prints the time of one
grouped compress call (kernel A + kernel B) and one grouped decompress-apply call per layer, from HIP events
around `repetitions` passes over `layers` layers of distinct buffers."""
from __future__ import annotations

import os
import subprocess
import sys


def measure(lib_path: str | None, layers: int, reps: int):
    import numpy as np
    import torch
    import lsp_synth as syn
    from . import binding as B
    if lib_path:
        B._LIB_PATH = lib_path                    # before the first call: the binding loads the library lazily
    import paper_2406_10181_amd as L
    dev = torch.device("cuda:0")
    stream = torch.cuda.current_stream()
    r, d, code = 512, 8, 2
    citems, aitems, keep = [], [], []
    for layer in range(layers):
        c, a = [], []
        for which, (_, m, n) in enumerate(syn.LAYER_67B):
            rng = np.random.default_rng(100 + layer * 7 + which)
            G = (torch.randn(m, n, device=dev) * 1e-3).to(torch.bfloat16)
            P_idx, P_val = syn.ell_projector(m, r, d, rng, "uniform")
            Q_idx, Q_val = syn.ell_projector(n, r, d, rng, "uniform")
            qi, qv = np.empty_like(Q_idx), np.empty_like(Q_val)
            L.lsp_projector_reorder_host(Q_idx, Q_val, n, d, r, qi, qv)
            t = [torch.from_numpy(x).to(dev) for x in (P_idx, P_val, Q_idx, Q_val, qi, qv)]
            pb = L.lsp_plan_bytes(m, n, r, d)
            plan = torch.empty(pb, dtype=torch.uint8, device=dev)
            L.lsp_plan_build(t[0], t[1], t[2], t[3], m, n, r, d, plan, pb, stream)
            ws = torch.empty(L.lsp_compress_planned_workspace_bytes(m, n, r, d), dtype=torch.uint8, device=dev)
            S, Su = torch.empty(r, r, device=dev), torch.randn(r, r, device=dev) * 1e-3
            keep.append((G, t, plan, ws, S, Su))
            c.append((G, plan, S, ws, ws.numel(), m, n))
            a.append((G, Su, t[0], t[1], t[4], t[5], m, n))
        citems.append(L.compress_items(c))
        aitems.append(L.apply_items(a))

    def run(fn):
        for _ in range(5):
            for li in range(layers):
                fn(li)
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(stream)
        for _ in range(reps):
            for li in range(layers):
                fn(li)
        b.record(stream)
        torch.cuda.synchronize()
        return a.elapsed_time(b) * 1e3 / (reps * layers)

    tc = run(lambda li: L.lsp_compress_planned_grouped(citems[li], 7, r, d, code, stream))
    td = run(lambda li: L.lsp_decompress_apply_grouped(aitems[li], 7, r, d, code, stream))
    return tc, td


def main(argv):
    from .build import ABLATIONS, ablation_lib
    layers = int(argv[0]) if len(argv) > 0 else 4
    reps = int(argv[1]) if len(argv) > 1 else 30
    if len(argv) > 2:                             # child: one variant
        tc, td = measure(argv[2] if argv[2] != "-" else None, layers, reps)
        print(f"RESULT {tc:.1f} {td:.1f}", flush=True)
        return
    print(f"grouped calls of one layer (7 matrices), us per call; {layers} layers of buffers, {reps} repetitions")
    print(f"{'variant':28s} {'compress (A + B)':>18s} {'decompress-apply':>18s}")
    for name in ["normal build"] + [n for n in ABLATIONS if os.path.exists(ablation_lib(n))]:
        lib = "-" if name == "normal build" else ablation_lib(name)
        out = subprocess.run([sys.executable, "-m", "paper_2406_10181_amd.ablation", str(layers), str(reps), lib],
                             capture_output=True, text=True, timeout=600)
        line = [l for l in out.stdout.splitlines() if l.startswith("RESULT")]
        if not line:
            print(f"{name:28s} failed: {out.stderr.strip().splitlines()[-1] if out.stderr.strip() else 'no output'}", flush=True)
            continue
        tc, td = line[0].split()[1:]
        shown_c = tc if not name.startswith("d_") else "-"
        shown_d = td if not name.startswith("a_") else "-"
        print(f"{name:28s} {shown_c:>18s} {shown_d:>18s}", flush=True)


if __name__ == "__main__":
    main(sys.argv[1:])
