"""ctypes binding of libmoe_hip.so: argument marshalling only, same names as the C ABI."""
from __future__ import annotations

import ctypes
import dataclasses
import os
from typing import Dict, Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_NAME = "libmoe_hip.so"
_lib = None

MOE_F32, MOE_BF16 = 0, 1
MOE_GATE_SOFTMAX, MOE_GATE_SIGMOID = 0, 1
EXPORTS = ["moe_abi_version", "moe_last_error", "moe_route_bwd", "moe_router_fwd", "moe_router_bwd",
           "moe_router_fwd_workspace_bytes", "moe_router_bwd_workspace_bytes", "moe_dispatch_workspace_bytes", "moe_expert_fwd_workspace_bytes",
           "moe_expert_bwd_workspace_bytes", "moe_route", "moe_dispatch", "moe_expert_fwd", "moe_expert_bwd",
           "moe_combine", "moe_combine_bwd", "moe_profile_enable", "moe_profile_report", "moe_copy_probe",
           "moe_aux_loss_workspace_bytes", "moe_aux_loss", "moe_aux_loss_bwd",
           "moe_plan_overlap_degree", "moe_plan_predict_load", "moe_plan_materialize", "moe_plan_dispatch",
           "moe_dispatch_static", "moe_mfma_probe", "moe_expert_fwd_gather", "moe_expert_bwd_gather",
           "moe_route_dispatch_workspace_bytes", "moe_route_dispatch", "moe_route_aux_bwd"]


class MoEError(RuntimeError):
    pass


class _CShape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("T", "d", "E", "k", "d_ff", "dtype", "gate", "renorm")]


@dataclasses.dataclass(frozen=True)
class MoEShape:
    T: int
    d: int
    E: int
    k: int
    d_ff: int
    dtype: str = "bf16"      # "f32" | "bf16"
    gate: str = "softmax"    # "softmax" | "sigmoid"
    renorm: bool = True

    def c(self) -> _CShape:
        return _CShape(self.T, self.d, self.E, self.k, self.d_ff, MOE_F32 if self.dtype == "f32" else MOE_BF16,
                       MOE_GATE_SOFTMAX if self.gate == "softmax" else MOE_GATE_SIGMOID, int(self.renorm))

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.float32 if self.dtype == "f32" else torch.bfloat16


def lib_path() -> str:
    return os.path.join(_HERE, _LIB_NAME)


def load_library():
    """Loads the in-tree library; raises if it has not been built (there is no fallback path)."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        raise MoEError(f"{path} is missing: build it with `python -m paper_2502_02581_amd.build` "
                       "(hipcc, gfx950); this package has no CPU or PyTorch fallback")
    lib = ctypes.CDLL(path)
    vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
    shp = ctypes.POINTER(_CShape)
    lib.moe_abi_version.restype = ctypes.c_int
    lib.moe_abi_version.argtypes = []
    lib.moe_last_error.restype = ctypes.c_char_p
    lib.moe_last_error.argtypes = []
    lib.moe_dispatch_workspace_bytes.restype = sz
    lib.moe_dispatch_workspace_bytes.argtypes = [shp]
    for f in (lib.moe_expert_fwd_workspace_bytes, lib.moe_expert_bwd_workspace_bytes):
        f.restype = sz
        f.argtypes = [shp, i32, i32, i32]
    lib.moe_route.restype = ctypes.c_int
    lib.moe_route.argtypes = [shp, vp, vp, vp, vp]
    for f in (lib.moe_router_fwd_workspace_bytes, lib.moe_router_bwd_workspace_bytes, lib.moe_aux_loss_workspace_bytes):
        f.restype = sz
        f.argtypes = [shp]
    lib.moe_aux_loss.restype = ctypes.c_int
    lib.moe_aux_loss.argtypes = [shp, vp, vp, ctypes.c_float, vp, vp, vp, sz, vp]
    lib.moe_aux_loss_bwd.restype = ctypes.c_int
    lib.moe_aux_loss_bwd.argtypes = [shp, vp, vp, ctypes.c_float, ctypes.c_float, i32, vp, vp]
    dbl = ctypes.c_double
    lib.moe_plan_overlap_degree.restype = ctypes.c_int
    lib.moe_plan_overlap_degree.argtypes = [dbl, dbl, dbl, ctypes.POINTER(ctypes.c_int32)]
    lib.moe_plan_predict_load.restype = ctypes.c_int
    lib.moe_plan_predict_load.argtypes = [vp, i32, i32, i32, vp]
    lib.moe_plan_materialize.restype = ctypes.c_int
    lib.moe_plan_materialize.argtypes = [i32, i32, i32, vp, vp, i32, i32, vp]
    lib.moe_plan_dispatch.restype = ctypes.c_int
    lib.moe_plan_dispatch.argtypes = [i32, i32, i32, vp, vp, vp]
    lib.moe_router_fwd.restype = ctypes.c_int
    lib.moe_router_fwd.argtypes = [shp, vp, vp, vp, vp, sz, vp]
    lib.moe_router_bwd.restype = ctypes.c_int
    lib.moe_router_bwd.argtypes = [shp, vp, vp, vp, vp, vp, i32, vp, sz, vp]
    lib.moe_route_bwd.restype = ctypes.c_int
    lib.moe_route_bwd.argtypes = [shp, vp, vp, vp, vp, vp]
    lib.moe_dispatch.restype = ctypes.c_int
    lib.moe_dispatch.argtypes = [shp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.moe_route_dispatch_workspace_bytes.restype = sz
    lib.moe_route_dispatch_workspace_bytes.argtypes = [shp]
    lib.moe_route_dispatch.restype = ctypes.c_int
    lib.moe_route_dispatch.argtypes = [shp, vp, vp, ctypes.c_float] + [vp] * 10 + [sz, vp]
    lib.moe_route_aux_bwd.restype = ctypes.c_int
    lib.moe_route_aux_bwd.argtypes = [shp, vp, vp, vp, vp, ctypes.c_float, ctypes.c_float, vp, vp]
    lib.moe_dispatch_static.restype = ctypes.c_int
    lib.moe_dispatch_static.argtypes = [shp, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.moe_expert_fwd.restype = ctypes.c_int
    lib.moe_expert_fwd.argtypes = [shp, i32, vp, i32] + [vp] * 9 + [sz, vp]
    lib.moe_expert_bwd.restype = ctypes.c_int
    lib.moe_expert_bwd.argtypes = [shp, i32, vp, i32] + [vp] * 15 + [sz, vp]
    lib.moe_expert_fwd_gather.restype = ctypes.c_int
    lib.moe_expert_fwd_gather.argtypes = [shp] + [vp] * 11 + [sz, vp]
    lib.moe_expert_bwd_gather.restype = ctypes.c_int
    lib.moe_expert_bwd_gather.argtypes = [shp] + [vp] * 19 + [sz, vp]
    lib.moe_combine.restype = ctypes.c_int
    lib.moe_combine.argtypes = [shp, vp, vp, vp, vp, vp, vp]
    lib.moe_combine_bwd.restype = ctypes.c_int
    lib.moe_combine_bwd.argtypes = [shp, vp, vp, vp, vp, vp, vp, vp]
    lib.moe_profile_enable.restype = ctypes.c_int
    lib.moe_profile_enable.argtypes = [ctypes.c_int]
    lib.moe_profile_report.restype = sz
    lib.moe_profile_report.argtypes = [ctypes.c_char_p, sz]
    lib.moe_copy_probe.restype = ctypes.c_int
    lib.moe_copy_probe.argtypes = [vp, vp, sz, vp]
    lib.moe_mfma_probe.restype = ctypes.c_int
    lib.moe_mfma_probe.argtypes = [i32, i32, vp, ctypes.POINTER(ctypes.c_double), vp]
    _lib = lib
    return lib


def _ptr(t: Optional[torch.Tensor], dtype=None, what="tensor"):
    if t is None:
        return None
    if not t.is_cuda:
        raise MoEError(f"{what} must live on the GPU")
    if not t.is_contiguous():
        raise MoEError(f"{what} must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise MoEError(f"{what} must be {dtype}, got {t.dtype}")
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream) -> ctypes.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _check(rc: int, who: str):
    if rc != 0:
        raise MoEError(f"{who} failed ({rc}): {load_library().moe_last_error().decode()}")


def moe_abi_version() -> int:
    return load_library().moe_abi_version()


def moe_last_error() -> str:
    return load_library().moe_last_error().decode()


def moe_dispatch_workspace_bytes(shape: MoEShape) -> int:
    return load_library().moe_dispatch_workspace_bytes(ctypes.byref(shape.c()))


def moe_expert_fwd_workspace_bytes(shape: MoEShape, n_groups: int, n_rows: int, shared: bool) -> int:
    return load_library().moe_expert_fwd_workspace_bytes(ctypes.byref(shape.c()), n_groups, n_rows, int(shared))


def moe_expert_bwd_workspace_bytes(shape: MoEShape, n_groups: int, n_rows: int, shared: bool) -> int:
    return load_library().moe_expert_bwd_workspace_bytes(ctypes.byref(shape.c()), n_groups, n_rows, int(shared))


def moe_route(shape: MoEShape, logits, topk_idx, topk_w, stream=None):
    rc = load_library().moe_route(ctypes.byref(shape.c()), _ptr(logits, torch.float32, "logits"),
                                  _ptr(topk_idx, torch.int32, "topk_idx"), _ptr(topk_w, torch.float32, "topk_w"),
                                  _stream(stream))
    _check(rc, "moe_route")


def moe_router_fwd_workspace_bytes(shape: MoEShape) -> int:
    return int(load_library().moe_router_fwd_workspace_bytes(ctypes.byref(shape.c())))


def moe_router_bwd_workspace_bytes(shape: MoEShape) -> int:
    return int(load_library().moe_router_bwd_workspace_bytes(ctypes.byref(shape.c())))


def moe_router_fwd(shape: MoEShape, X, Wr, logits, ws, stream=None):
    dt = shape.torch_dtype
    rc = load_library().moe_router_fwd(ctypes.byref(shape.c()), _ptr(X, dt, "X"), _ptr(Wr, dt, "Wr"),
                                       _ptr(logits, torch.float32, "logits"), _ptr(ws, None, "ws"),
                                       ws.numel() * ws.element_size(), _stream(stream))
    _check(rc, "moe_router_fwd")


def moe_router_bwd(shape: MoEShape, X, Wr, dlogits, dWr, dX, accumulate: bool, ws, stream=None):
    dt = shape.torch_dtype
    rc = load_library().moe_router_bwd(ctypes.byref(shape.c()), _ptr(X, dt, "X"), _ptr(Wr, dt, "Wr"),
                                       _ptr(dlogits, torch.float32, "dlogits"), _ptr(dWr, dt, "dWr"), _ptr(dX, dt, "dX"),
                                       int(bool(accumulate)), _ptr(ws, None, "ws"), ws.numel() * ws.element_size(),
                                       _stream(stream))
    _check(rc, "moe_router_bwd")


def moe_route_bwd(shape: MoEShape, logits, topk_idx, dw, dlogits, stream=None):
    rc = load_library().moe_route_bwd(ctypes.byref(shape.c()), _ptr(logits, torch.float32, "logits"),
                                      _ptr(topk_idx, torch.int32, "topk_idx"), _ptr(dw, torch.float32, "dw"),
                                      _ptr(dlogits, torch.float32, "dlogits"), _stream(stream))
    _check(rc, "moe_route_bwd")


def moe_aux_loss_workspace_bytes(shape: MoEShape) -> int:
    return int(load_library().moe_aux_loss_workspace_bytes(ctypes.byref(shape.c())))


def moe_aux_loss(shape: MoEShape, logits, counts, alpha, P, loss, ws, stream=None):
    rc = load_library().moe_aux_loss(ctypes.byref(shape.c()), _ptr(logits, torch.float32, "logits"),
                                     _ptr(counts, torch.int32, "counts"), float(alpha), _ptr(P, torch.float32, "P"),
                                     _ptr(loss, torch.float32, "loss"), _ptr(ws, None, "ws"),
                                     ws.numel() * ws.element_size(), _stream(stream))
    _check(rc, "moe_aux_loss")


def moe_aux_loss_bwd(shape: MoEShape, logits, counts, alpha, dloss, accumulate, dlogits, stream=None):
    rc = load_library().moe_aux_loss_bwd(ctypes.byref(shape.c()), _ptr(logits, torch.float32, "logits"),
                                         _ptr(counts, torch.int32, "counts"), float(alpha), float(dloss),
                                         int(bool(accumulate)), _ptr(dlogits, torch.float32, "dlogits"), _stream(stream))
    _check(rc, "moe_aux_loss_bwd")


# ---- host-side planners: numpy arrays in host memory, no GPU involved
def _host(a, dtype, shape, what):
    import numpy as np

    a = np.ascontiguousarray(a, dtype=dtype)
    if a.shape != tuple(shape):
        raise MoEError(f"{what} must have shape {tuple(shape)}, got {a.shape}")
    return a


def moe_plan_overlap_degree(t_attn: float, bw: float, psi: float) -> int:
    out = ctypes.c_int32(0)
    _check(load_library().moe_plan_overlap_degree(float(t_attn), float(bw), float(psi), ctypes.byref(out)),
           "moe_plan_overlap_degree")
    return int(out.value)


def moe_plan_predict_load(history, w: int = 5):
    import numpy as np

    h = np.ascontiguousarray(history, dtype=np.float64)
    if h.ndim != 2:
        raise MoEError("history must be [n_iters, E]")
    F = np.empty(h.shape[1], dtype=np.float64)
    _check(load_library().moe_plan_predict_load(h.ctypes.data, h.shape[0], h.shape[1], int(w), F.ctypes.data),
           "moe_plan_predict_load")
    return F


def moe_plan_materialize(P, F, t: int, m: int, dpn: int):
    import numpy as np

    P = np.ascontiguousarray(P, dtype=np.uint8)
    if P.ndim != 2:
        raise MoEError("P must be [E, D]")
    E, D = P.shape
    F = _host(F, np.float64, (E,), "F")
    out = np.empty_like(P)
    _check(load_library().moe_plan_materialize(E, D, int(dpn), P.ctypes.data, F.ctypes.data, int(t), int(m),
                                               out.ctypes.data), "moe_plan_materialize")
    return out


def moe_plan_dispatch(Pm, T, dpn: int):
    import numpy as np

    Pm = np.ascontiguousarray(Pm, dtype=np.uint8)
    if Pm.ndim != 2:
        raise MoEError("Pm must be [E, D]")
    E, D = Pm.shape
    T = _host(T, np.int32, (E, D), "T")
    R = np.empty((E, D, D), dtype=np.int32)
    _check(load_library().moe_plan_dispatch(E, D, int(dpn), Pm.ctypes.data, T.ctypes.data, R.ctypes.data),
           "moe_plan_dispatch")
    return R


def moe_dispatch(shape: MoEShape, X, topk_idx, counts, offsets, row_of, src_of, Xp, ws, stream=None):
    dt = shape.torch_dtype
    rc = load_library().moe_dispatch(ctypes.byref(shape.c()), _ptr(X, dt, "X"), _ptr(topk_idx, torch.int32, "topk_idx"),
                                     _ptr(counts, torch.int32, "counts"), _ptr(offsets, torch.int32, "offsets"),
                                     _ptr(row_of, torch.int32, "row_of"), _ptr(src_of, torch.int32, "src_of"),
                                     _ptr(Xp, dt, "Xp"), _ptr(ws, None, "ws"), ws.numel() * ws.element_size(),
                                     _stream(stream))
    _check(rc, "moe_dispatch")


def moe_route_dispatch_workspace_bytes(shape: MoEShape) -> int:
    return int(load_library().moe_route_dispatch_workspace_bytes(ctypes.byref(shape.c())))


def moe_route_dispatch(shape: MoEShape, logits, X, aux_alpha, topk_idx, topk_w, counts, offsets, row_of, src_of, Xp,
                       aux_P, aux_loss, ws, stream=None):
    """moe_route + moe_dispatch (+ moe_aux_loss when aux_P and aux_loss are given) in one call."""
    dt = shape.torch_dtype
    rc = load_library().moe_route_dispatch(
        ctypes.byref(shape.c()), _ptr(logits, torch.float32, "logits"), _ptr(X, dt, "X"), float(aux_alpha),
        _ptr(topk_idx, torch.int32, "topk_idx"), _ptr(topk_w, torch.float32, "topk_w"), _ptr(counts, torch.int32, "counts"),
        _ptr(offsets, torch.int32, "offsets"), _ptr(row_of, torch.int32, "row_of"), _ptr(src_of, torch.int32, "src_of"),
        _ptr(Xp, dt, "Xp"), _ptr(aux_P, torch.float32, "aux_P"), _ptr(aux_loss, torch.float32, "aux_loss"),
        _ptr(ws, None, "ws"), ws.numel() * ws.element_size(), _stream(stream))
    _check(rc, "moe_route_dispatch")


def moe_route_aux_bwd(shape: MoEShape, logits, topk_idx, dw, counts, alpha, dloss, dlogits, stream=None):
    """moe_route_bwd + moe_aux_loss_bwd(accumulate) in one kernel."""
    rc = load_library().moe_route_aux_bwd(ctypes.byref(shape.c()), _ptr(logits, torch.float32, "logits"),
                                          _ptr(topk_idx, torch.int32, "topk_idx"), _ptr(dw, torch.float32, "dw"),
                                          _ptr(counts, torch.int32, "counts"), float(alpha), float(dloss),
                                          _ptr(dlogits, torch.float32, "dlogits"), _stream(stream))
    _check(rc, "moe_route_aux_bwd")


def moe_dispatch_static(shape: MoEShape, X, topk_idx, counts, offsets, row_of, src_of, Xp, stream=None):
    """moe_dispatch without a workspace argument (the library's built-in scratch array; allocates nothing)."""
    dt = shape.torch_dtype
    rc = load_library().moe_dispatch_static(ctypes.byref(shape.c()), _ptr(X, dt, "X"),
                                            _ptr(topk_idx, torch.int32, "topk_idx"), _ptr(counts, torch.int32, "counts"),
                                            _ptr(offsets, torch.int32, "offsets"), _ptr(row_of, torch.int32, "row_of"),
                                            _ptr(src_of, torch.int32, "src_of"), _ptr(Xp, dt, "Xp"), _stream(stream))
    _check(rc, "moe_dispatch_static")


def moe_expert_fwd(shape: MoEShape, n_groups, offsets, n_rows, Xin, Wg, Wu, Wd, G, U, H, Yout, ws, stream=None):
    dt = shape.torch_dtype
    rc = load_library().moe_expert_fwd(
        ctypes.byref(shape.c()), n_groups, _ptr(offsets, torch.int32, "offsets"), n_rows, _ptr(Xin, dt, "Xin"),
        _ptr(Wg, dt, "Wg"), _ptr(Wu, dt, "Wu"), _ptr(Wd, dt, "Wd"), _ptr(G, dt, "G"), _ptr(U, dt, "U"),
        _ptr(H, dt, "H"), _ptr(Yout, dt, "Yout"), _ptr(ws, None, "ws"), ws.numel() * ws.element_size(),
        _stream(stream))
    _check(rc, "moe_expert_fwd")


def moe_expert_bwd(shape: MoEShape, n_groups, offsets, n_rows, Xin, Wg, Wu, Wd, G, U, H, dYin, dXin, active_ids,
                   n_active, dWg_c, dWu_c, dWd_c, ws, stream=None):
    dt = shape.torch_dtype
    rc = load_library().moe_expert_bwd(
        ctypes.byref(shape.c()), n_groups, _ptr(offsets, torch.int32, "offsets"), n_rows, _ptr(Xin, dt, "Xin"),
        _ptr(Wg, dt, "Wg"), _ptr(Wu, dt, "Wu"), _ptr(Wd, dt, "Wd"), _ptr(G, dt, "G"), _ptr(U, dt, "U"),
        _ptr(H, dt, "H"), _ptr(dYin, dt, "dYin"), _ptr(dXin, dt, "dXin"), _ptr(active_ids, torch.int32, "active_ids"),
        _ptr(n_active, torch.int32, "n_active"), _ptr(dWg_c, dt, "dWg_c"), _ptr(dWu_c, dt, "dWu_c"),
        _ptr(dWd_c, dt, "dWd_c"), _ptr(ws, None, "ws"), ws.numel() * ws.element_size(), _stream(stream))
    _check(rc, "moe_expert_bwd")


def moe_expert_fwd_gather(shape: MoEShape, offsets, src_of, X, Wg, Wu, Wd, G, U, H, Yout, ws, stream=None):
    dt = shape.torch_dtype
    rc = load_library().moe_expert_fwd_gather(
        ctypes.byref(shape.c()), _ptr(offsets, torch.int32, "offsets"), _ptr(src_of, torch.int32, "src_of"),
        _ptr(X, dt, "X"), _ptr(Wg, dt, "Wg"), _ptr(Wu, dt, "Wu"), _ptr(Wd, dt, "Wd"), _ptr(G, dt, "G"), _ptr(U, dt, "U"),
        _ptr(H, dt, "H"), _ptr(Yout, dt, "Yout"), _ptr(ws, None, "ws"), ws.numel() * ws.element_size(), _stream(stream))
    _check(rc, "moe_expert_fwd_gather")


def moe_expert_bwd_gather(shape: MoEShape, offsets, src_of, Xp, Wg, Wu, Wd, G, U, H, dY, topk_w, dYp, dXp, active_ids,
                          n_active, dWg_c, dWu_c, dWd_c, ws, stream=None):
    dt = shape.torch_dtype
    rc = load_library().moe_expert_bwd_gather(
        ctypes.byref(shape.c()), _ptr(offsets, torch.int32, "offsets"), _ptr(src_of, torch.int32, "src_of"),
        _ptr(Xp, dt, "Xp"), _ptr(Wg, dt, "Wg"), _ptr(Wu, dt, "Wu"), _ptr(Wd, dt, "Wd"), _ptr(G, dt, "G"), _ptr(U, dt, "U"),
        _ptr(H, dt, "H"), _ptr(dY, dt, "dY"), _ptr(topk_w, torch.float32, "topk_w"), _ptr(dYp, dt, "dYp"),
        _ptr(dXp, dt, "dXp"), _ptr(active_ids, torch.int32, "active_ids"), _ptr(n_active, torch.int32, "n_active"),
        _ptr(dWg_c, dt, "dWg_c"), _ptr(dWu_c, dt, "dWu_c"), _ptr(dWd_c, dt, "dWd_c"), _ptr(ws, None, "ws"),
        ws.numel() * ws.element_size(), _stream(stream))
    _check(rc, "moe_expert_bwd_gather")


def moe_combine(shape: MoEShape, Yp, row_of, topk_w, Yadd, Y, stream=None):
    dt = shape.torch_dtype
    rc = load_library().moe_combine(ctypes.byref(shape.c()), _ptr(Yp, dt, "Yp"), _ptr(row_of, torch.int32, "row_of"),
                                    _ptr(topk_w, torch.float32, "topk_w"), _ptr(Yadd, dt, "Yadd"), _ptr(Y, dt, "Y"),
                                    _stream(stream))
    _check(rc, "moe_combine")


def moe_combine_bwd(shape: MoEShape, dY, Yp, row_of, topk_w, dYp, dw, stream=None):
    dt = shape.torch_dtype
    rc = load_library().moe_combine_bwd(ctypes.byref(shape.c()), _ptr(dY, dt, "dY"), _ptr(Yp, dt, "Yp"),
                                        _ptr(row_of, torch.int32, "row_of"), _ptr(topk_w, torch.float32, "topk_w"),
                                        _ptr(dYp, dt, "dYp"), _ptr(dw, torch.float32, "dw"), _stream(stream))
    _check(rc, "moe_combine_bwd")


def moe_copy_probe(src: torch.Tensor, dst: torch.Tensor):
    """Copies src to dst (same byte size) with the library's plain copy kernel; calibrates profiler counters."""
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes:
        raise MoEError("moe_copy_probe: sizes differ")
    rc = load_library().moe_copy_probe(_ptr(src), _ptr(dst), ctypes.c_size_t(nbytes), _stream(None))
    _check(rc, "moe_copy_probe")


def moe_mfma_probe(n_blocks: int, iters: int, sink: torch.Tensor) -> float:
    """Launches the register-resident matrix loop once; returns the FLOPs of the launch (time it outside)."""
    if sink.numel() < n_blocks * 256:
        raise MoEError("moe_mfma_probe: sink needs n_blocks * 256 floats")
    flops = ctypes.c_double(0.0)
    rc = load_library().moe_mfma_probe(int(n_blocks), int(iters), _ptr(sink, torch.float32, "sink"), ctypes.byref(flops),
                                       _stream(None))
    _check(rc, "moe_mfma_probe")
    return float(flops.value)


def moe_profile_enable(on: bool):
    load_library().moe_profile_enable(int(on))


def moe_profile_report() -> Dict[str, tuple]:
    """{kernel label: (launches, total milliseconds)} of the launches recorded since enable."""
    lib = load_library()
    buf = ctypes.create_string_buffer(1 << 16)
    lib.moe_profile_report(buf, len(buf))
    out = {}
    for line in buf.value.decode().splitlines():
        label, n, ms = line.split()
        out[label] = (int(n), float(ms))
    return out


class MoEHotPath:
    """Owns the device buffers of one layer and chains the C calls of a training step.

    forward():  moe_route -> moe_dispatch -> moe_expert_fwd (routed, then shared) -> moe_combine
    backward(): moe_combine_bwd -> moe_expert_bwd (routed, then shared) -> moe_combine (unit weights)
                -> moe_route_bwd (gradient of the router logits)
    With aux_alpha > 0, forward() also evaluates the auxiliary load-balancing loss (moe_aux_loss, after
    the dispatch has counted the loads) and backward() adds its gradient to dlogits (moe_aux_loss_bwd).
    With fused (the default), gate + dispatch + loss go through moe_route_dispatch and the two backward
    calls of the gate through moe_route_aux_bwd: the same results from four launches fewer.
    No arithmetic happens here; tensors are only allocated and handed to the library.

    The shared experts depend on nothing the routed experts produce, so with overlap_shared their
    calls go to a second stream of the same (default) priority and join before the combine: their
    blocks then fill the CUs that the tail of a routed launch leaves idle (about 1 % of a step on the
    DeepSeek-V3-shaped workload; off by default because per-kernel durations then overlap).
    """

    def __init__(self, shape: MoEShape, n_shared: int = 0, d_ff_shared: int = 0, device="cuda:0",
                 overlap_shared: bool = False, aux_alpha: float = 0.0, gather: bool = False, fused: bool = True):
        self.shape, self.S, self.Fs, self.device = shape, n_shared, d_ff_shared, torch.device(device)
        self.gather = bool(gather)  # routed experts read X and dY through src_of (moe_expert_*_gather)
        # gate, dispatch and auxiliary loss through moe_route_dispatch / moe_route_aux_bwd (fewer launches)
        self.fused = bool(fused)
        self.aux_alpha = float(aux_alpha)
        self.overlap = bool(overlap_shared and n_shared)
        s, dt, dev = shape, shape.torch_dtype, self.device
        A = s.T * s.k
        i32 = dict(dtype=torch.int32, device=dev)
        f = dict(dtype=dt, device=dev)
        self.b: Dict[str, torch.Tensor] = {
            "topk_idx": torch.empty(s.T, s.k, **i32), "topk_w": torch.empty(s.T, s.k, dtype=torch.float32, device=dev),
            "counts": torch.empty(s.E, **i32), "offsets": torch.empty(s.E + 1, **i32),
            "row_of": torch.empty(A, **i32), "src_of": torch.empty(A, **i32),
            "Xp": torch.empty(A, s.d, **f), "G": torch.empty(A, s.d_ff, **f), "U": torch.empty(A, s.d_ff, **f),
            "H": torch.empty(A, s.d_ff, **f), "Yp": torch.empty(A, s.d, **f), "Y": torch.empty(s.T, s.d, **f),
            "dYp": torch.empty(A, s.d, **f), "dw": torch.empty(s.T, s.k, dtype=torch.float32, device=dev),
            "dlogits": torch.empty(s.T, s.E, dtype=torch.float32, device=dev),
            "dXp": torch.empty(A, s.d, **f), "dX": torch.empty(s.T, s.d, **f),
            "active_ids": torch.empty(s.E, **i32), "n_active": torch.empty(1, **i32),
            "dWg_c": torch.empty(s.E, s.d, s.d_ff, **f), "dWu_c": torch.empty(s.E, s.d, s.d_ff, **f),
            "dWd_c": torch.empty(s.E, s.d_ff, s.d, **f),
        }
        ws = max(moe_dispatch_workspace_bytes(s), moe_route_dispatch_workspace_bytes(s),
                 moe_expert_fwd_workspace_bytes(s, s.E, A, False), moe_expert_bwd_workspace_bytes(s, s.E, A, False))
        if n_shared:
            self.sshape = dataclasses.replace(s, d_ff=d_ff_shared)
            S, Fs = n_shared, d_ff_shared
            self.b.update({
                "Gs": torch.empty(S, s.T, Fs, **f), "Us": torch.empty(S, s.T, Fs, **f), "Hs": torch.empty(S, s.T, Fs, **f),
                "Ysh": torch.empty(s.T, s.d, **f), "dXsh": torch.empty(s.T, s.d, **f),
                "s_active_ids": torch.empty(S, **i32), "s_n_active": torch.empty(1, **i32),
                "dWsg": torch.empty(S, s.d, Fs, **f), "dWsu": torch.empty(S, s.d, Fs, **f),
                "dWsd": torch.empty(S, Fs, s.d, **f),
            })
            ws = max(ws, moe_expert_fwd_workspace_bytes(self.sshape, S, s.T, True),
                     moe_expert_bwd_workspace_bytes(self.sshape, S, s.T, True))
        if self.aux_alpha > 0:
            self.b.update({"aux_P": torch.empty(s.E, dtype=torch.float32, device=dev),
                           "aux_loss": torch.empty(1, dtype=torch.float32, device=dev)})
            ws = max(ws, moe_aux_loss_workspace_bytes(s))
        self.ws = torch.empty(ws, dtype=torch.uint8, device=dev)
        self.ws_shared = self.ws
        if self.overlap:  # concurrent calls need a workspace each
            self.ws_shared = torch.empty(max(moe_expert_fwd_workspace_bytes(self.sshape, n_shared, s.T, True),
                                             moe_expert_bwd_workspace_bytes(self.sshape, n_shared, s.T, True)),
                                         dtype=torch.uint8, device=dev)
            self.side = torch.cuda.Stream(device=dev)
            self.ev_fork, self.ev_join = torch.cuda.Event(), torch.cuda.Event()

    def _fork(self, stream):
        """The side stream starts after everything already queued on the main stream."""
        main = stream if stream is not None else torch.cuda.current_stream(self.device)
        self.ev_fork.record(main)
        self.side.wait_event(self.ev_fork)
        return main

    def _join(self, main):
        self.ev_join.record(self.side)
        main.wait_event(self.ev_join)

    def forward(self, logits, X, Wg, Wu, Wd, Wsg=None, Wsu=None, Wsd=None, stream=None):
        s, b = self.shape, self.b
        A = s.T * s.k
        self._logits = logits  # the gate's backward reads them again
        if self.overlap:
            main = self._fork(stream)
            moe_expert_fwd(self.sshape, self.S, None, s.T, X, Wsg, Wsu, Wsd, b["Gs"], b["Us"], b["Hs"], b["Ysh"],
                           self.ws_shared, self.side)
        if self.fused:
            moe_route_dispatch(s, logits, X, self.aux_alpha, b["topk_idx"], b["topk_w"], b["counts"], b["offsets"],
                               b["row_of"], b["src_of"], b["Xp"], b.get("aux_P"), b.get("aux_loss"), self.ws, stream)
        else:
            moe_route(s, logits, b["topk_idx"], b["topk_w"], stream)
            moe_dispatch(s, X, b["topk_idx"], b["counts"], b["offsets"], b["row_of"], b["src_of"], b["Xp"], self.ws,
                         stream)
            if self.aux_alpha > 0:
                moe_aux_loss(s, logits, b["counts"], self.aux_alpha, b["aux_P"], b["aux_loss"], self.ws, stream)
        if self.gather:
            moe_expert_fwd_gather(s, b["offsets"], b["src_of"], X, Wg, Wu, Wd, b["G"], b["U"], b["H"], b["Yp"], self.ws,
                                  stream)
        else:
            moe_expert_fwd(s, s.E, b["offsets"], A, b["Xp"], Wg, Wu, Wd, b["G"], b["U"], b["H"], b["Yp"], self.ws, stream)
        if self.overlap:
            self._join(main)
        elif self.S:
            moe_expert_fwd(self.sshape, self.S, None, s.T, X, Wsg, Wsu, Wsd, b["Gs"], b["Us"], b["Hs"], b["Ysh"],
                           self.ws, stream)
        moe_combine(s, b["Yp"], b["row_of"], b["topk_w"], b["Ysh"] if self.S else None, b["Y"], stream)
        return b["Y"]

    def backward(self, dY, X, Wg, Wu, Wd, Wsg=None, Wsu=None, Wsd=None, stream=None):
        s, b = self.shape, self.b
        A = s.T * s.k
        if self.overlap:
            main = self._fork(stream)
            moe_expert_bwd(self.sshape, self.S, None, s.T, X, Wsg, Wsu, Wsd, b["Gs"], b["Us"], b["Hs"], dY, b["dXsh"],
                           b["s_active_ids"], b["s_n_active"], b["dWsg"], b["dWsu"], b["dWsd"], self.ws_shared, self.side)
        moe_combine_bwd(s, dY, b["Yp"], b["row_of"], b["topk_w"], b["dYp"], b["dw"], stream)
        if self.gather:
            moe_expert_bwd_gather(s, b["offsets"], b["src_of"], b["Xp"], Wg, Wu, Wd, b["G"], b["U"], b["H"], dY,
                                  b["topk_w"], b["dYp"], b["dXp"], b["active_ids"], b["n_active"], b["dWg_c"],
                                  b["dWu_c"], b["dWd_c"], self.ws, stream)
        else:
            moe_expert_bwd(s, s.E, b["offsets"], A, b["Xp"], Wg, Wu, Wd, b["G"], b["U"], b["H"], b["dYp"], b["dXp"],
                           b["active_ids"], b["n_active"], b["dWg_c"], b["dWu_c"], b["dWd_c"], self.ws, stream)
        if self.overlap:
            self._join(main)
        elif self.S:
            moe_expert_bwd(self.sshape, self.S, None, s.T, X, Wsg, Wsu, Wsd, b["Gs"], b["Us"], b["Hs"], dY, b["dXsh"],
                           b["s_active_ids"], b["s_n_active"], b["dWsg"], b["dWsu"], b["dWsd"], self.ws, stream)
        moe_combine(s, b["dXp"], b["row_of"], None, b["dXsh"] if self.S else None, b["dX"], stream)
        if self.fused and self.aux_alpha > 0:
            moe_route_aux_bwd(s, self._logits, b["topk_idx"], b["dw"], b["counts"], self.aux_alpha, 1.0, b["dlogits"],
                              stream)
        else:
            moe_route_bwd(s, self._logits, b["topk_idx"], b["dw"], b["dlogits"], stream)
            if self.aux_alpha > 0:
                moe_aux_loss_bwd(s, self._logits, b["counts"], self.aux_alpha, 1.0, True, b["dlogits"], stream)
        return b["dX"]
