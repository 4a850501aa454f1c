"""Helpers for the GPU parity tests: move a synthetic Problem to the device, call the C ABI
through the binding, bring results back as numpy."""
from __future__ import annotations

import numpy as np
import torch

import lsp_synth as syn
import paper_2406_10181_amd as L

_TORCH_STORAGE = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}


def to_device(arr: np.ndarray, dtype: str | None = None) -> torch.Tensor:
    """numpy storage array -> cuda tensor with the same bits."""
    if dtype == "bf16":
        return torch.from_numpy(arr.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(arr).cuda()


def to_host(t: torch.Tensor, dtype: str) -> np.ndarray:
    if dtype == "bf16":
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


class DeviceProblem:
    def __init__(self, pb: syn.Problem):
        self.pb = pb
        self.code = syn.DTYPE_CODE[pb.dtype]
        self.G = to_device(pb.G, pb.dtype)
        self.W = to_device(pb.W, pb.dtype)
        self.P_idx, self.P_val = to_device(pb.P_idx), to_device(pb.P_val)
        self.Q_idx, self.Q_val = to_device(pb.Q_idx), to_device(pb.Q_val)
        self.S = torch.full((pb.r, pb.r), float("nan"), dtype=torch.float32, device="cuda")
        self.ws_bytes = max(L.lsp_compress_workspace_bytes(pb.m, pb.n, pb.r, pb.d),
                            L.lsp_compress_planned_workspace_bytes(pb.m, pb.n, pb.r, pb.d))
        self.ws = torch.empty(self.ws_bytes, dtype=torch.uint8, device="cuda")
        self.plan = None
        self.plan_bytes = 0
        self.Qx_idx, self.Qx_val = self.Q_idx, self.Q_val        # what the expand side (decompress, bias) is handed

    def use_reordered_q(self):
        """The expand side gets the copy of Q with each row's entries ordered against LDS bank conflicts."""
        pb = self.pb
        qi, qv = np.empty_like(pb.Q_idx), np.empty_like(pb.Q_val)
        L.lsp_projector_reorder_host(pb.Q_idx, pb.Q_val, pb.n, pb.d, pb.r, qi, qv)
        self.Qx_idx, self.Qx_val = to_device(qi), to_device(qv)

    def build_plan(self):
        pb = self.pb
        self.plan_bytes = L.lsp_plan_bytes(pb.m, pb.n, pb.r, pb.d)
        self.plan = torch.empty(self.plan_bytes, dtype=torch.uint8, device="cuda")
        L.lsp_plan_build(self.P_idx, self.P_val, self.Q_idx, self.Q_val, pb.m, pb.n, pb.r, pb.d,
                         self.plan, self.plan_bytes, torch.cuda.current_stream())

    def compress_raw(self) -> np.ndarray:
        pb = self.pb
        self.S.fill_(float("nan"))
        L.lsp_compress(self.G, self.P_idx, self.P_val, self.Q_idx, self.Q_val, pb.m, pb.n, pb.r, pb.d,
                       self.S, self.code, self.ws, self.ws_bytes, torch.cuda.current_stream())
        torch.cuda.synchronize()
        return self.S.cpu().numpy().copy()

    def compress_planned(self) -> np.ndarray:
        pb = self.pb
        if self.plan is None:
            self.build_plan()
        self.S.fill_(float("nan"))
        L.lsp_compress_planned(self.G, self.plan, pb.m, pb.n, pb.r, pb.d, self.S, self.code,
                               self.ws, self.ws_bytes, torch.cuda.current_stream())
        torch.cuda.synchronize()
        return self.S.cpu().numpy().copy()

    def decompress(self, S_in: np.ndarray) -> np.ndarray:
        """Applies onto a fresh copy of W; returns the updated W as a numpy storage array."""
        pb = self.pb
        Wd = self.W.clone()
        Sd = torch.from_numpy(np.ascontiguousarray(S_in, dtype=np.float32)).cuda()
        L.lsp_decompress_apply(Wd, Sd, self.P_idx, self.P_val, self.Qx_idx, self.Qx_val, pb.m, pb.n, pb.r, pb.d,
                               self.code, torch.cuda.current_stream())
        torch.cuda.synchronize()
        return to_host(Wd, pb.dtype)


    def estimation_bias(self, planned: bool = True) -> np.ndarray:
        """Compress G, then the bias pass over G: returns the three floats of lsp_estimation_bias.
        G must come back untouched."""
        pb = self.pb
        before = self.G.clone()
        if planned:
            self.compress_planned()
        else:
            self.compress_raw()
        nb = L.lsp_estimation_bias_workspace_bytes(pb.m, pb.n, pb.r, pb.d)
        ws = torch.empty(nb, dtype=torch.uint8, device="cuda")
        out = torch.full((3,), float("nan"), dtype=torch.float32, device="cuda")
        L.lsp_estimation_bias(self.G, self.S, self.P_idx, self.P_val, self.Qx_idx, self.Qx_val, pb.m, pb.n, pb.r, pb.d,
                              out, ws, nb, self.code, torch.cuda.current_stream())
        torch.cuda.synchronize()
        assert torch.equal(before.view(torch.uint8), self.G.view(torch.uint8)), "the bias pass must not write G"
        return out.cpu().numpy()


# ------------------------------------------------------------------ parity criteria
def check_compress(S_gpu: np.ndarray, S_ora: np.ndarray, what: str, tight: float = 5e-5):
    """Norm-wise bar of the task: max |S_gpu - S_o| <= 1e-3 max |S_o|.  fp32 accumulation of a few
    thousand terms is expected to sit near 1e-6, so a much tighter bound is asserted as well."""
    assert np.isfinite(S_gpu).all(), f"{what}: non-finite S"
    scale = np.abs(S_ora).max()
    err = np.abs(S_gpu.astype(np.float64) - S_ora).max()
    if scale == 0.0:
        assert err == 0.0, what
        return 0.0
    assert err <= 1e-3 * scale, f"{what}: rel err {err / scale:.3e} above the 1e-3 bar"
    assert err <= tight * scale, f"{what}: rel err {err / scale:.3e} above the fp32-accumulation bound {tight}"
    return err / scale


def check_decompress(W_gpu: np.ndarray, W_in: np.ndarray, Wp_ora: np.ndarray, Wr_ora: np.ndarray, dtype: str,
                     what: str):
    """|float(W_gpu) - W'_o| <= 1/2 ulp(W'_o) + 1e-3 max|Delta_o|, stated on the pre-rounding
    value because one ulp of bf16 (2^-8 relative) already exceeds 1e-3; plus the fraction of
    elements that differ from the oracle's singly rounded result must be small."""
    Wg = syn.storage_to_f64(W_gpu, dtype)
    delta = syn.storage_to_f64(W_in, dtype) - Wp_ora
    dmax = np.abs(delta).max()
    bound = 0.5 * syn.ulp_of(Wp_ora, dtype) * (1 + 1e-9) + 1e-3 * dmax
    bad = np.abs(Wg - Wp_ora) > bound
    assert not bad.any(), f"{what}: {bad.sum()} elements outside 1/2 ulp + 1e-3 max|delta|"
    # tighter, arithmetic bound: fp32 evaluation of the update
    bound2 = 0.5 * syn.ulp_of(Wp_ora, dtype) * (1 + 1e-9) + 2e-5 * dmax + 2.0 ** -23 * np.abs(Wp_ora)
    bad2 = np.abs(Wg - Wp_ora) > bound2
    assert not bad2.any(), f"{what}: {bad2.sum()} elements outside the fp32-arithmetic bound"
    mism = np.mean(W_gpu.view(np.uint8) != Wr_ora.view(np.uint8)) if W_gpu.dtype != np.float32 else \
        np.mean(W_gpu != Wr_ora)
    return float(mism)
