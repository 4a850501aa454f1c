"""ctypes binding with the same names as the C ABI (argument marshalling only)."""
from __future__ import annotations

import ctypes
import os
from typing import Optional

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "liblsp_hip.so")

DTYPE_CODE = {"f32": 0, "f16": 1, "bf16": 2}


class lsp_compress_item(ctypes.Structure):
    """One problem of lsp_compress_planned_grouped (field for field the C struct)."""
    _fields_ = [("G", ctypes.c_void_p), ("plan", ctypes.c_void_p), ("S", ctypes.c_void_p),
                ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t),
                ("m", ctypes.c_int64), ("n", ctypes.c_int64)]


class lsp_apply_item(ctypes.Structure):
    """One problem of lsp_decompress_apply_grouped (field for field the C struct)."""
    _fields_ = [("W", ctypes.c_void_p), ("S", ctypes.c_void_p), ("P_idx", ctypes.c_void_p), ("P_val", ctypes.c_void_p),
                ("Q_idx", ctypes.c_void_p), ("Q_val", ctypes.c_void_p), ("m", ctypes.c_int64), ("n", ctypes.c_int64)]


class LspError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {lsp_strerror(code)} (status {code}, hip error {lib().lsp_last_hip_error()})")


_lib = None


def lib_path() -> str:
    return _LIB_PATH


def lib() -> ctypes.CDLL:
    """Loads the in-tree HIP library.  There is no fallback: a missing library is an error."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(
                f"{_LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()' "
                "or python paper_2406_10181_amd/build.py)")
        L = ctypes.CDLL(_LIB_PATH)
        vp, i64, i32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_size_t
        L.lsp_compress.argtypes = [vp, vp, vp, vp, vp, i64, i64, i32, i32, vp, i32, vp, sz, vp]
        L.lsp_compress.restype = ctypes.c_int
        L.lsp_compress_workspace_bytes.argtypes = [i64, i64, i32, i32]
        L.lsp_compress_workspace_bytes.restype = sz
        L.lsp_workspace_bytes.argtypes = [i64, i64, i32, i32, i32]
        L.lsp_workspace_bytes.restype = sz
        L.lsp_plan_bytes.argtypes = [i64, i64, i32, i32]
        L.lsp_plan_bytes.restype = sz
        L.lsp_plan_build.argtypes = [vp, vp, vp, vp, i64, i64, i32, i32, vp, sz, vp]
        L.lsp_plan_build.restype = ctypes.c_int
        L.lsp_plan_build_async.argtypes = [vp, vp, vp, vp, i64, i64, i32, i32, vp, sz, vp, sz, vp, vp]
        L.lsp_plan_build_async.restype = ctypes.c_int
        L.lsp_plan_build_workspace_bytes.argtypes = [i64, i64, i32, i32]
        L.lsp_plan_build_workspace_bytes.restype = sz
        L.lsp_plan_build_host.argtypes = [vp, vp, vp, vp, i64, i64, i32, i32, vp, sz]
        L.lsp_plan_build_host.restype = ctypes.c_int
        L.lsp_compress_planned.argtypes = [vp, vp, i64, i64, i32, i32, vp, i32, vp, sz, vp]
        L.lsp_compress_planned.restype = ctypes.c_int
        L.lsp_compress_planned_static.argtypes = [vp, vp, i64, i64, i32, i32, vp, i32, vp]
        L.lsp_compress_planned_static.restype = ctypes.c_int
        L.lsp_static_scratch_bytes.argtypes = []
        L.lsp_static_scratch_bytes.restype = sz
        L.lsp_compress_planned_workspace_bytes.argtypes = [i64, i64, i32, i32]
        L.lsp_compress_planned_workspace_bytes.restype = sz
        L.lsp_decompress_apply.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, i32, i32, i32, vp]
        L.lsp_decompress_apply.restype = ctypes.c_int
        L.lsp_compress_planned_grouped.argtypes = [vp, i32, i32, i32, i32, vp]
        L.lsp_compress_planned_grouped.restype = ctypes.c_int
        L.lsp_decompress_apply_grouped.argtypes = [vp, i32, i32, i32, i32, vp]
        L.lsp_decompress_apply_grouped.restype = ctypes.c_int
        L.lsp_compress_dense_workspace_bytes.argtypes = [i64, i64, i32]
        L.lsp_compress_dense_workspace_bytes.restype = sz
        L.lsp_compress_dense.argtypes = [vp, vp, vp, i64, i64, i32, vp, i32, vp, sz, vp]
        L.lsp_compress_dense.restype = ctypes.c_int
        L.lsp_estimation_bias.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, i32, i32, vp, vp, ctypes.c_size_t, i32, vp]
        L.lsp_estimation_bias.restype = ctypes.c_int
        L.lsp_projector_reorder_host.argtypes = [vp, vp, i64, i32, i32, vp, vp]
        L.lsp_projector_reorder_host.restype = ctypes.c_int
        L.lsp_projector_reorder.argtypes = [vp, vp, i64, i32, i32, vp, vp, vp]
        L.lsp_projector_reorder.restype = ctypes.c_int
        L.lsp_reproject_state.argtypes = [vp] * 8 + [i64, i64, i32, i32, vp, vp, vp, ctypes.c_size_t, vp]
        L.lsp_reproject_state.restype = ctypes.c_int
        L.lsp_reproject_state_workspace_bytes.argtypes = [i32]
        L.lsp_reproject_state_workspace_bytes.restype = ctypes.c_size_t
        L.lsp_estimation_bias_workspace_bytes.argtypes = [i64, i64, i32, i32]
        L.lsp_estimation_bias_workspace_bytes.restype = ctypes.c_size_t
        L.lsp_plan_refresh_values.argtypes = [vp, vp, vp, i64, i64, i32, i32, vp]
        L.lsp_plan_refresh_values.restype = ctypes.c_int
        L.lsp_bias_gradient.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, i32, i32, vp, vp, vp, sz, i32, vp]
        L.lsp_bias_gradient.restype = ctypes.c_int
        L.lsp_bias_gradient_workspace_bytes.argtypes = [i64, i64, i32, i32]
        L.lsp_bias_gradient_workspace_bytes.restype = sz
        L.lsp_hbm_probe_workspace_bytes.argtypes = [sz]
        L.lsp_hbm_probe_workspace_bytes.restype = sz
        L.lsp_hbm_probe_read.argtypes = [vp, sz, vp, sz, vp]
        L.lsp_hbm_probe_read.restype = ctypes.c_int
        L.lsp_hbm_probe_rmw.argtypes = [vp, sz, ctypes.c_float, vp]
        L.lsp_hbm_probe_rmw.restype = ctypes.c_int
        L.lsp_validate_projector.argtypes = [vp, i64, i32, i32, vp, vp]
        L.lsp_validate_projector.restype = ctypes.c_int
        L.lsp_strerror.argtypes = [ctypes.c_int]
        L.lsp_strerror.restype = ctypes.c_char_p
        L.lsp_last_hip_error.restype = ctypes.c_int
        L.lsp_version.restype = ctypes.c_int
        _lib = L
    return _lib


def _ptr(x) -> Optional[int]:
    """Device (or host) address of a torch tensor / numpy array / raw int; None stays NULL."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if hasattr(x, "data_ptr"):
        return x.data_ptr()
    if hasattr(x, "ctypes"):
        return x.ctypes.data
    raise TypeError(f"cannot take the address of {type(x)!r}")


def _stream(stream) -> Optional[int]:
    if stream is None:
        return None
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream          # torch.cuda.Stream


def torch_dtype_code(t) -> int:
    import torch
    return {torch.float32: 0, torch.float16: 1, torch.bfloat16: 2}[t]


def _check(rc: int, where: str) -> None:
    if rc != 0:
        raise LspError(rc, where)


def lsp_strerror(code: int) -> str:
    return lib().lsp_strerror(code).decode()


def lsp_version() -> int:
    return lib().lsp_version()


def lsp_compress_workspace_bytes(m, n, r, d) -> int:
    return lib().lsp_compress_workspace_bytes(m, n, r, d)


def lsp_workspace_bytes(m, n, r, d, dtype: int) -> int:
    return int(lib().lsp_workspace_bytes(m, n, r, d, dtype))


def lsp_compress_planned_workspace_bytes(m, n, r, d) -> int:
    return lib().lsp_compress_planned_workspace_bytes(m, n, r, d)


def lsp_plan_bytes(m, n, r, d) -> int:
    return lib().lsp_plan_bytes(m, n, r, d)


def lsp_compress(G, P_idx, P_val, Q_idx, Q_val, m, n, r, d, S, dtype: int, workspace, workspace_bytes, stream=None,
                 check: bool = True) -> int:
    rc = lib().lsp_compress(_ptr(G), _ptr(P_idx), _ptr(P_val), _ptr(Q_idx), _ptr(Q_val), m, n, r, d, _ptr(S),
                            dtype, _ptr(workspace), workspace_bytes, _stream(stream))
    if check:
        _check(rc, "lsp_compress")
    return rc


def lsp_plan_build(P_idx, P_val, Q_idx, Q_val, m, n, r, d, plan, plan_bytes, stream=None, check: bool = True) -> int:
    rc = lib().lsp_plan_build(_ptr(P_idx), _ptr(P_val), _ptr(Q_idx), _ptr(Q_val), m, n, r, d, _ptr(plan),
                              plan_bytes, _stream(stream))
    if check:
        _check(rc, "lsp_plan_build")
    return rc


def lsp_plan_build_workspace_bytes(m, n, r, d) -> int:
    return int(lib().lsp_plan_build_workspace_bytes(m, n, r, d))


def lsp_plan_build_async(P_idx, P_val, Q_idx, Q_val, m, n, r, d, plan, plan_bytes, workspace, workspace_bytes, status=None,
                         stream=None, check: bool = True) -> int:
    rc = lib().lsp_plan_build_async(_ptr(P_idx), _ptr(P_val), _ptr(Q_idx), _ptr(Q_val), m, n, r, d, _ptr(plan), plan_bytes,
                                    _ptr(workspace), workspace_bytes, _ptr(status), _stream(stream))
    if check:
        _check(rc, "lsp_plan_build_async")
    return rc


def lsp_plan_build_host(P_idx, P_val, Q_idx, Q_val, m, n, r, d, plan_host, plan_bytes, check: bool = True) -> int:
    rc = lib().lsp_plan_build_host(_ptr(P_idx), _ptr(P_val), _ptr(Q_idx), _ptr(Q_val), m, n, r, d,
                                   _ptr(plan_host), plan_bytes)
    if check:
        _check(rc, "lsp_plan_build_host")
    return rc


def lsp_compress_planned(G, plan, m, n, r, d, S, dtype: int, workspace, workspace_bytes, stream=None,
                         check: bool = True) -> int:
    rc = lib().lsp_compress_planned(_ptr(G), _ptr(plan), m, n, r, d, _ptr(S), dtype, _ptr(workspace),
                                    workspace_bytes, _stream(stream))
    if check:
        _check(rc, "lsp_compress_planned")
    return rc


def lsp_static_scratch_bytes() -> int:
    return int(lib().lsp_static_scratch_bytes())


def lsp_compress_planned_static(G, plan, m, n, r, d, S, dtype: int, stream=None, check: bool = True) -> int:
    rc = lib().lsp_compress_planned_static(_ptr(G), _ptr(plan), m, n, r, d, _ptr(S), dtype, _stream(stream))
    if check:
        _check(rc, "lsp_compress_planned_static")
    return rc


def lsp_decompress_apply(W, S, P_idx, P_val, Q_idx, Q_val, m, n, r, d, dtype: int, stream=None,
                         check: bool = True) -> int:
    rc = lib().lsp_decompress_apply(_ptr(W), _ptr(S), _ptr(P_idx), _ptr(P_val), _ptr(Q_idx), _ptr(Q_val),
                                    m, n, r, d, dtype, _stream(stream))
    if check:
        _check(rc, "lsp_decompress_apply")
    return rc


def lsp_estimation_bias_workspace_bytes(m, n, r, d) -> int:
    return int(lib().lsp_estimation_bias_workspace_bytes(m, n, r, d))


def lsp_estimation_bias(G, S, P_idx, P_val, Q_idx, Q_val, m, n, r, d, out, workspace, workspace_bytes,
                        dtype: int, stream=None, check: bool = True) -> int:
    rc = lib().lsp_estimation_bias(_ptr(G), _ptr(S), _ptr(P_idx), _ptr(P_val), _ptr(Q_idx), _ptr(Q_val),
                                   m, n, r, d, _ptr(out), _ptr(workspace), workspace_bytes, dtype, _stream(stream))
    if check:
        _check(rc, "lsp_estimation_bias")
    return rc


def lsp_projector_reorder_host(idx, val, rows, d, r, idx_out, val_out, check: bool = True) -> int:
    """Host arrays (numpy int32 / float32, [rows][d]) in and out."""
    rc = lib().lsp_projector_reorder_host(_ptr(idx), _ptr(val), rows, d, r, _ptr(idx_out), _ptr(val_out))
    if check:
        _check(rc, "lsp_projector_reorder_host")
    return rc


def lsp_projector_reorder(idx, val, rows, d, r, idx_out, val_out, stream=None, check: bool = True) -> int:
    """Device arrays in and out; waits for the stream."""
    rc = lib().lsp_projector_reorder(_ptr(idx), _ptr(val), rows, d, r, _ptr(idx_out), _ptr(val_out), _stream(stream))
    if check:
        _check(rc, "lsp_projector_reorder")
    return rc


def lsp_reproject_state_workspace_bytes(r) -> int:
    return int(lib().lsp_reproject_state_workspace_bytes(r))


def lsp_reproject_state(P_idx, P_val, Pprev_idx, Pprev_val, Q_idx, Q_val, Qprev_idx, Qprev_val, m, n, r, d, M, V,
                        workspace, workspace_bytes, stream=None, check: bool = True) -> int:
    rc = lib().lsp_reproject_state(_ptr(P_idx), _ptr(P_val), _ptr(Pprev_idx), _ptr(Pprev_val), _ptr(Q_idx), _ptr(Q_val),
                                   _ptr(Qprev_idx), _ptr(Qprev_val), m, n, r, d, _ptr(M), _ptr(V),
                                   _ptr(workspace), workspace_bytes, _stream(stream))
    if check:
        _check(rc, "lsp_reproject_state")
    return rc


def compress_items(problems):
    """Host array of lsp_compress_item from (G, plan, S, workspace, workspace_bytes, m, n) tuples."""
    arr = (lsp_compress_item * len(problems))()
    for k, (G, plan, S, ws, ws_bytes, m, n) in enumerate(problems):
        arr[k] = lsp_compress_item(_ptr(G), _ptr(plan), _ptr(S), _ptr(ws), ws_bytes, m, n)
    return arr


def apply_items(problems):
    """Host array of lsp_apply_item from (W, S, P_idx, P_val, Q_idx, Q_val, m, n) tuples."""
    arr = (lsp_apply_item * len(problems))()
    for k, (W, S, P_idx, P_val, Q_idx, Q_val, m, n) in enumerate(problems):
        arr[k] = lsp_apply_item(_ptr(W), _ptr(S), _ptr(P_idx), _ptr(P_val), _ptr(Q_idx), _ptr(Q_val), m, n)
    return arr


def lsp_compress_planned_grouped(items, count, r, d, dtype: int, stream=None, check: bool = True) -> int:
    """items: a ctypes array from compress_items() (kept alive by the caller for the call)."""
    rc = lib().lsp_compress_planned_grouped(ctypes.addressof(items) if items is not None else None, count, r, d, dtype,
                                            _stream(stream))
    if check:
        _check(rc, "lsp_compress_planned_grouped")
    return rc


def lsp_decompress_apply_grouped(items, count, r, d, dtype: int, stream=None, check: bool = True) -> int:
    """items: a ctypes array from apply_items()."""
    rc = lib().lsp_decompress_apply_grouped(ctypes.addressof(items) if items is not None else None, count, r, d, dtype,
                                            _stream(stream))
    if check:
        _check(rc, "lsp_decompress_apply_grouped")
    return rc


def lsp_compress_dense_workspace_bytes(m, n, r) -> int:
    return int(lib().lsp_compress_dense_workspace_bytes(m, n, r))


def lsp_compress_dense(G, Pt, Qt, m, n, r, S, dtype: int, workspace, workspace_bytes, stream=None, check: bool = True) -> int:
    """Pt, Qt: the transposed dense projectors [r][m], [r][n] in the storage type of G."""
    rc = lib().lsp_compress_dense(_ptr(G), _ptr(Pt), _ptr(Qt), m, n, r, _ptr(S), dtype, _ptr(workspace), workspace_bytes,
                                  _stream(stream))
    if check:
        _check(rc, "lsp_compress_dense")
    return rc


def lsp_plan_refresh_values(plan, P_val, Q_val, m, n, r, d, stream=None, check: bool = True) -> int:
    rc = lib().lsp_plan_refresh_values(_ptr(plan), _ptr(P_val), _ptr(Q_val), m, n, r, d, _stream(stream))
    if check:
        _check(rc, "lsp_plan_refresh_values")
    return rc


def lsp_bias_gradient_workspace_bytes(m, n, r, d) -> int:
    return int(lib().lsp_bias_gradient_workspace_bytes(m, n, r, d))


def lsp_bias_gradient(G, plan, P_idx, P_val, Q_idx, Q_val, m, n, r, d, gP, gQ, workspace, workspace_bytes,
                      dtype: int, stream=None, check: bool = True) -> int:
    rc = lib().lsp_bias_gradient(_ptr(G), _ptr(plan), _ptr(P_idx), _ptr(P_val), _ptr(Q_idx), _ptr(Q_val), m, n, r, d,
                                 _ptr(gP), _ptr(gQ), _ptr(workspace), workspace_bytes, dtype, _stream(stream))
    if check:
        _check(rc, "lsp_bias_gradient")
    return rc


def lsp_hbm_probe_workspace_bytes(nbytes: int) -> int:
    return int(lib().lsp_hbm_probe_workspace_bytes(nbytes))


def lsp_hbm_probe_read(buf, nbytes: int, workspace, workspace_bytes: int, stream=None, check: bool = True) -> int:
    rc = lib().lsp_hbm_probe_read(_ptr(buf), nbytes, _ptr(workspace), workspace_bytes, _stream(stream))
    if check:
        _check(rc, "lsp_hbm_probe_read")
    return rc


def lsp_hbm_probe_rmw(buf, nbytes: int, c: float, stream=None, check: bool = True) -> int:
    rc = lib().lsp_hbm_probe_rmw(_ptr(buf), nbytes, c, _stream(stream))
    if check:
        _check(rc, "lsp_hbm_probe_rmw")
    return rc


def lsp_validate_projector(idx, rows, d, r, flag, stream=None, check: bool = False) -> int:
    rc = lib().lsp_validate_projector(_ptr(idx), rows, d, r, _ptr(flag), _stream(stream))
    if check:
        _check(rc, "lsp_validate_projector")
    return rc
