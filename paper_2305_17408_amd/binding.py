"""ctypes binding of libadaptgear.so: argument marshalling only.

Every function has the name and meaning of its C entry point in
include/adaptgear.h.  Feature matrices are torch CUDA tensors (torch only
provides device memory and the current HIP stream); host-side matrices are
numpy arrays.  There is no CPU fallback: if the library is missing, import of
the native part fails loudly.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libadaptgear.so")

AG_OK = 0
AG_ERR_INVALID, AG_ERR_NOMEM, AG_ERR_HIP, AG_ERR_UNSUPPORTED = -1, -2, -3, -4
AG_LAYOUT_ORIGINAL, AG_LAYOUT_REORDERED = 0, 1
AG_FLAG_HOST_ONLY = 1
AG_METHOD_LABEL_PROPAGATION, AG_METHOD_MODULARITY = 0, 1
AG_CLS_BLOCKS_DENSE, AG_CLS_BLOCKS_SPARSE, AG_CLS_REMAINDER, AG_CLS_COMPOSE = 0, 1, 2, 3
AG_NUM_CLS = 4
AG_K_BLOCK_SPARSE, AG_K_BLOCK_DENSE, AG_K_BLOCK_DENSE_BF16X3 = 0, 1, 2
AG_MIN_BLOCKS_OWN_LAUNCH = 256
AG_K_CSR_NARROW, AG_K_CSR_WIDE, AG_K_COO = 0, 1, 2
AG_COMPOSE_SPLIT, AG_COMPOSE_FUSED, AG_COMPOSE_FULL_CSR, AG_COMPOSE_FULL_CSR_WIDE = 0, 1, 2, 3
AG_DIR_FWD, AG_DIR_BWD = 0, 1
AG_STATIC_SCRATCH_BYTES = 32 << 20

_i32p = C.POINTER(C.c_int32)
_f32p = C.POINTER(C.c_float)


class ag_csr(C.Structure):
    _fields_ = [("n", C.c_int64), ("nnz", C.c_int64), ("rowptr", _i32p), ("colidx", _i32p),
                ("vals", _f32p)]


class ag_options(C.Structure):
    _fields_ = [("block_cap", C.c_int32), ("num_communities", C.c_int32), ("min_block", C.c_int32),
                ("sweeps", C.c_int32),
                ("max_levels", C.c_int32), ("order_levels", C.c_int32), ("trials", C.c_int32),
                ("layout", C.c_int32),
                ("flags", C.c_int32), ("dense_density", C.c_float),
                ("dev_alloc", C.c_void_p), ("dev_free", C.c_void_p), ("user", C.c_void_p),
                ("row_scale", C.c_void_p), ("col_scale", C.c_void_p), ("method", C.c_int32),
                ("reuse_perm", C.c_void_p), ("reuse_blk_ptr", C.c_void_p), ("reuse_n_blocks", C.c_int32)]


class ag_selector_info(C.Structure):
    _fields_ = [("frozen", C.c_int32), ("calls", C.c_int32), ("choice", C.c_int32 * AG_NUM_CLS),
                ("trial_ms", (C.c_float * 4) * AG_NUM_CLS), ("total_trial_ms", C.c_float)]


class ag_export(C.Structure):
    _fields_ = [("n", C.c_int64), ("nnz_intra", C.c_int64), ("nnz_inter", C.c_int64),
                ("n_blocks", C.c_int32),
                ("perm", _i32p), ("iperm", _i32p), ("blk_ptr", _i32p),
                ("intra_rowptr", _i32p), ("intra_col", _i32p), ("intra_val", _f32p),
                ("inter_rowptr", _i32p), ("inter_col", _i32p), ("inter_val", _f32p)]


class ag_stats(C.Structure):
    _fields_ = [("n", C.c_int64), ("nnz", C.c_int64), ("nnz_intra", C.c_int64), ("nnz_inter", C.c_int64),
                ("F", C.c_int32), ("n_blocks", C.c_int32), ("n_block_rows", C.c_int32),
                ("n_dense_blocks", C.c_int32), ("symmetric", C.c_int32), ("unit_weights", C.c_int32),
                ("n_long_rows", C.c_int64), ("n_long_segments", C.c_int64),
                ("density_full", C.c_double), ("density_intra", C.c_double), ("density_inter", C.c_double),
                ("sec_reorder", C.c_double), ("sec_split", C.c_double), ("sec_build", C.c_double),
                ("sec_upload", C.c_double), ("device_bytes", C.c_int64),
                ("block_density_hist", C.c_int32 * 8),
                ("dense_rows", C.c_int64), ("nnz_intra_dense", C.c_int64),
                ("nnz_inter_dense_rows", C.c_int64), ("nnz_inter_block_rows", C.c_int64),
                ("factored", C.c_int32)]


class ag_profile(C.Structure):
    _fields_ = [("calls", C.c_int64), ("class_ms", C.c_double * 3), ("total_ms", C.c_double),
                ("compose", C.c_int32)]


AG_GIN_MAX_LAYERS = 8


class ag_gin_io(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("width", C.c_int32 * (AG_GIN_MAX_LAYERS + 1)), ("eps", C.c_float),
                ("W", C.c_void_p * AG_GIN_MAX_LAYERS), ("b", C.c_void_p * AG_GIN_MAX_LAYERS),
                ("dW", C.c_void_p * AG_GIN_MAX_LAYERS), ("db", C.c_void_p * AG_GIN_MAX_LAYERS),
                ("loss", C.c_void_p), ("logits", C.c_void_p)]


class ag_gcn_io(C.Structure):
    _fields_ = [("f_in", C.c_int32), ("hidden", C.c_int32), ("n_class", C.c_int32),
                ("W1", C.c_void_p), ("b1", C.c_void_p), ("W2", C.c_void_p), ("b2", C.c_void_p),
                ("dW1", C.c_void_p), ("db1", C.c_void_p), ("dW2", C.c_void_p), ("db2", C.c_void_p),
                ("loss", C.c_void_p), ("logits", C.c_void_p)]


EXPORTS = ["ag_plan_create", "ag_plan_clone_for_width", "ag_plan_destroy", "ag_aggregate",
           "ag_aggregate_t", "ag_permute_rows", "ag_plan_force_kernels", "ag_plan_selector_info",
           "ag_plan_export", "ag_plan_stats", "ag_plan_set_profiling", "ag_plan_profile", "ag_last_error", "ag_gin_layer", "ag_gin_layer_t",
           "ag_gcn_workspace_bytes", "ag_gcn_step", "ag_gin_workspace_bytes", "ag_gin_step", "ag_aggregate_max", "ag_aggregate_max_t", "ag_aggregate_static"]

_lib = None


def lib() -> C.CDLL:
    """Load libadaptgear.so (built by build.py); raises if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            # nothing built yet: compile once with hipcc; there is no CPU fallback
            try:
                from . import build as _build
                _build.build()
            except Exception as exc:
                raise ImportError(f"{LIB_PATH} is missing and could not be built with hipcc: {exc}") from exc
        L = C.CDLL(LIB_PATH)
        vp = C.c_void_p
        L.ag_plan_create.argtypes = [C.POINTER(ag_csr), C.c_int64, C.c_int32, C.POINTER(ag_options), C.POINTER(vp)]
        L.ag_plan_clone_for_width.argtypes = [vp, C.c_int32, C.POINTER(vp)]
        L.ag_plan_destroy.argtypes = [vp]
        L.ag_plan_destroy.restype = None
        L.ag_aggregate.argtypes = [vp, vp, vp, vp]
        L.ag_aggregate_t.argtypes = [vp, vp, vp, vp]
        L.ag_aggregate_static.argtypes = [vp, vp, vp, vp]
        L.ag_permute_rows.argtypes = [vp, vp, vp, C.c_int32, C.c_int32, vp]
        L.ag_plan_force_kernels.argtypes = [vp, C.c_int32, C.c_int32, C.c_int32]
        L.ag_plan_selector_info.argtypes = [vp, C.c_int32, C.POINTER(ag_selector_info)]
        L.ag_plan_export.argtypes = [vp, C.POINTER(ag_export)]
        L.ag_plan_stats.argtypes = [vp, C.POINTER(ag_stats)]
        L.ag_plan_set_profiling.argtypes = [vp, C.c_int32]
        L.ag_plan_profile.argtypes = [vp, C.c_int32, C.POINTER(ag_profile)]
        L.ag_last_error.restype = C.c_char_p
        L.ag_gin_layer.argtypes = [vp, C.c_float, vp, vp, vp]
        L.ag_gin_layer_t.argtypes = [vp, C.c_float, vp, vp, vp]
        L.ag_gcn_workspace_bytes.argtypes = [C.c_int64, C.c_int32, C.c_int32, C.c_int32]
        L.ag_gcn_workspace_bytes.restype = C.c_size_t
        L.ag_aggregate_max.argtypes = [vp, vp, vp, vp, vp]
        L.ag_aggregate_max_t.argtypes = [vp, vp, vp, vp, vp]
        L.ag_gin_workspace_bytes.argtypes = [C.c_int64, C.POINTER(ag_gin_io)]
        L.ag_gin_workspace_bytes.restype = C.c_size_t
        L.ag_gin_step.argtypes = [C.POINTER(vp), C.POINTER(ag_gin_io), vp, vp, vp, C.c_size_t, vp]
        L.ag_gcn_step.argtypes = [vp, vp, C.POINTER(ag_gcn_io), vp, vp, vp, C.c_size_t, vp]
        _lib = L
    return _lib


class AdaptGearError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"adaptgear error {code}: {msg}")
        self.code = code


def _check(rc: int) -> None:
    if rc != AG_OK:
        raise AdaptGearError(rc, ag_last_error())


def ag_last_error() -> str:
    return (lib().ag_last_error() or b"").decode()


def _ptr(t):
    """Device pointer of a torch tensor (must be contiguous fp32/int32 on the GPU)."""
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous CUDA tensor")
    return C.c_void_p(t.data_ptr())


def _stream(stream=None):
    if stream is None:
        import torch
        stream = torch.cuda.current_stream().cuda_stream
    elif hasattr(stream, "cuda_stream"):
        stream = stream.cuda_stream
    return C.c_void_p(int(stream))


# --------------------------------------------------------------------------- #
# entry points, same names as the C ABI
# --------------------------------------------------------------------------- #
def ag_plan_create(rowptr, colidx, vals, N: int, F: int, **options):
    """-> opaque plan handle (c_void_p).  rowptr/colidx/vals are host numpy arrays."""
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int32)
    colidx = np.ascontiguousarray(colidx, dtype=np.int32)
    vals = None if vals is None else np.ascontiguousarray(vals, dtype=np.float32)
    a = ag_csr(int(rowptr.size - 1), int(colidx.size), rowptr.ctypes.data_as(_i32p),
               colidx.ctypes.data_as(_i32p), None if vals is None else vals.ctypes.data_as(_f32p))
    o = ag_options()
    keep = []                                            # host arrays borrowed by the call
    reuse = options.pop("reuse", None)                   # (perm, blk_ptr) of an earlier ag_plan_export
    if reuse is not None:
        perm = np.ascontiguousarray(reuse[0], dtype=np.int32)
        blk_ptr = np.ascontiguousarray(reuse[1], dtype=np.int32)
        if perm.size != int(N) or blk_ptr.size < 1:
            raise ValueError("reuse = (perm with N entries, blk_ptr with n_blocks + 1 entries)")
        keep += [perm, blk_ptr]
        o.reuse_perm, o.reuse_blk_ptr, o.reuse_n_blocks = perm.ctypes.data, blk_ptr.ctypes.data, int(blk_ptr.size - 1)
    for k, v in options.items():
        if not hasattr(o, k):
            raise TypeError(f"unknown option {k}")
        if k in ("row_scale", "col_scale"):
            if v is None:
                continue
            v = np.ascontiguousarray(v, dtype=np.float32)
            if v.size != int(N):
                raise ValueError(f"{k} must have N entries")
            keep.append(v)
            v = v.ctypes.data
        setattr(o, k, v)
    out = C.c_void_p()
    _check(lib().ag_plan_create(C.byref(a), int(N), int(F), C.byref(o), C.byref(out)))
    return out


def ag_plan_clone_for_width(plan, F2: int):
    out = C.c_void_p()
    _check(lib().ag_plan_clone_for_width(plan, int(F2), C.byref(out)))
    return out


def ag_plan_destroy(plan) -> None:
    lib().ag_plan_destroy(plan)


def ag_aggregate(plan, H, Y, stream=None) -> None:
    _check(lib().ag_aggregate(plan, _ptr(H), _ptr(Y), _stream(stream)))


def ag_aggregate_static(plan, H, Y, stream=None) -> None:
    _check(lib().ag_aggregate_static(plan, _ptr(H), _ptr(Y), _stream(stream)))


def ag_aggregate_t(plan, G, dH, stream=None) -> None:
    _check(lib().ag_aggregate_t(plan, _ptr(G), _ptr(dH), _stream(stream)))


def ag_permute_rows(plan, src, dst, F: int, inverse: bool, stream=None) -> None:
    _check(lib().ag_permute_rows(plan, _ptr(src), _ptr(dst), int(F), 1 if inverse else 0, _stream(stream)))


def ag_plan_force_kernels(plan, cls: int, direction: int, kernel_id: int) -> None:
    _check(lib().ag_plan_force_kernels(plan, int(cls), int(direction), int(kernel_id)))


def ag_plan_selector_info(plan, direction: int) -> dict:
    s = ag_selector_info()
    _check(lib().ag_plan_selector_info(plan, int(direction), C.byref(s)))
    return dict(frozen=bool(s.frozen), calls=int(s.calls), choice=list(s.choice),
                trial_ms=[list(r) for r in s.trial_ms], total_trial_ms=float(s.total_trial_ms))


def ag_plan_export(plan) -> dict:
    """Copies of the plan's host-side decomposition as numpy arrays."""
    e = ag_export()
    _check(lib().ag_plan_export(plan, C.byref(e)))
    n, nb = int(e.n), int(e.n_blocks)

    def arr(p, count, dt):
        if not p or count == 0:
            return np.empty(0, dt)
        return np.ctypeslib.as_array(p, shape=(count,)).astype(dt, copy=True)

    ni, no = int(e.nnz_intra), int(e.nnz_inter)
    unit = bool(ag_plan_stats(plan)["unit_weights"])      # unit weights: no value arrays at all
    return dict(
        n=n, n_blocks=nb, perm=arr(e.perm, n, np.int32), iperm=arr(e.iperm, n, np.int32),
        blk_ptr=arr(e.blk_ptr, nb + 1, np.int32),
        intra_rowptr=arr(e.intra_rowptr, n + 1, np.int32), intra_col=arr(e.intra_col, ni, np.int32),
        intra_val=None if unit else arr(e.intra_val, ni, np.float32),
        inter_rowptr=arr(e.inter_rowptr, n + 1, np.int32), inter_col=arr(e.inter_col, no, np.int32),
        inter_val=None if unit else arr(e.inter_val, no, np.float32))


def ag_plan_stats(plan) -> dict:
    s = ag_stats()
    _check(lib().ag_plan_stats(plan, C.byref(s)))
    d = {k: getattr(s, k) for k, _ in ag_stats._fields_}
    d["block_density_hist"] = list(s.block_density_hist)
    return d


def ag_plan_set_profiling(plan, on: bool) -> None:
    _check(lib().ag_plan_set_profiling(plan, 1 if on else 0))


def ag_plan_profile(plan, direction: int) -> dict:
    s = ag_profile()
    _check(lib().ag_plan_profile(plan, int(direction), C.byref(s)))
    return dict(calls=int(s.calls), class_ms=list(s.class_ms), total_ms=float(s.total_ms),
                compose=int(s.compose))


def ag_gin_layer(plan, eps: float, H, Y, stream=None) -> None:
    _check(lib().ag_gin_layer(plan, float(eps), _ptr(H), _ptr(Y), _stream(stream)))


def ag_gin_layer_t(plan, eps: float, G, dH, stream=None) -> None:
    _check(lib().ag_gin_layer_t(plan, float(eps), _ptr(G), _ptr(dH), _stream(stream)))


def ag_aggregate_max(plan, H, Y, arg=None, stream=None) -> None:
    _check(lib().ag_aggregate_max(plan, _ptr(H), _ptr(Y), _ptr(arg), _stream(stream)))


def ag_aggregate_max_t(plan, G, arg, dH, stream=None) -> None:
    _check(lib().ag_aggregate_max_t(plan, _ptr(G), _ptr(arg), _ptr(dH), _stream(stream)))


def _gin_io(widths, eps=0.0, W=(), b=(), dW=(), db=(), loss=None, logits=None) -> ag_gin_io:
    io = ag_gin_io()
    io.n_layers = len(widths) - 1
    for i, w in enumerate(widths[:AG_GIN_MAX_LAYERS + 1]):
        io.width[i] = int(w)
    io.eps = float(eps)
    for name, seq in (("W", W), ("b", b), ("dW", dW), ("db", db)):
        arr = getattr(io, name)
        for i, t in enumerate(seq[:AG_GIN_MAX_LAYERS]):
            arr[i] = t.data_ptr() if t is not None else None
    io.loss = loss.data_ptr() if loss is not None else None
    io.logits = logits.data_ptr() if logits is not None else None
    return io


def ag_gin_workspace_bytes(n: int, widths) -> int:
    io = _gin_io(list(widths))
    return int(lib().ag_gin_workspace_bytes(int(n), C.byref(io)))


def ag_gin_step(plans, *, widths, eps, W, b, dW, db, loss, logits, X, labels, workspace, stream=None) -> None:
    """plans[l] has F = widths[l] for l = 0..L (clones of one topology); see the C header."""
    widths = list(widths)
    for t in list(W) + list(b) + list(dW) + list(db) + [loss, X, labels, workspace]:
        _ptr(t)                                           # validates device / contiguity
    io = _gin_io(widths, eps, W, b, dW, db, loss, logits)
    arr = (C.c_void_p * len(plans))(*plans)
    _check(lib().ag_gin_step(arr, C.byref(io), _ptr(X), _ptr(labels), _ptr(workspace),
                             int(workspace.numel() * workspace.element_size()), _stream(stream)))


def ag_gcn_workspace_bytes(n: int, f_in: int, hidden: int, n_class: int) -> int:
    return int(lib().ag_gcn_workspace_bytes(int(n), int(f_in), int(hidden), int(n_class)))


def ag_gcn_step(plan_in, plan_out, *, f_in, hidden, n_class, W1, b1, W2, b2, dW1, db1, dW2, db2,
                loss, logits, X, labels, workspace, stream=None) -> None:
    io = ag_gcn_io(int(f_in), int(hidden), int(n_class), _ptr(W1), _ptr(b1), _ptr(W2), _ptr(b2),
                   _ptr(dW1), _ptr(db1), _ptr(dW2), _ptr(db2), _ptr(loss), _ptr(logits))
    _check(lib().ag_gcn_step(plan_in, plan_out, C.byref(io), _ptr(X), _ptr(labels), _ptr(workspace),
                             int(workspace.numel() * workspace.element_size()), _stream(stream)))
