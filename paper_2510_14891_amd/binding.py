"""Thin ctypes binding of the C-ABI library ``libmttkrp_hip.so``.

Argument marshalling only: every step of the MTTKRP runs in the HIP kernels of
``csrc/mttkrp.hip``.  PyTorch appears here solely as the owner of device memory
and of the HIP stream.  There is no CPU fallback: if the library has not been
built (``python -m paper_2510_14891_amd.build``) every entry point raises.
Function names follow ``include/mttkrp.h``.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmttkrp_hip.so")

MTTKRP_OK = 0
MTTKRP_ERR_INVALID_ARG = 1
MTTKRP_ERR_UNSUPPORTED = 2
MTTKRP_ERR_WORKSPACE = 3
MTTKRP_ERR_DEVICE = 4
MTTKRP_ERR_NUMERICAL = 5
MTTKRP_MAX_NDIM = 8

# every symbol include/mttkrp.h declares
EXPORTED = (
    "mttkrp_dense_f64", "mttkrp_dense_f32", "mttkrp_dense_workspace_bytes",
    "mttkrp_dense_f64_ws", "mttkrp_dense_f32_ws", "mttkrp_dense_ex_workspace_bytes",
    "mttkrp_dense_f64_ex", "mttkrp_dense_f32_ex", "mttkrp_status_string",
    "mttkrp_version", "mttkrp_release", "mttkrp_timing_enable",
    "mttkrp_timing_count", "mttkrp_timing_get", "mttkrp_timing_last",
    "mttkrp_tune_set", "mttkrp_plan_describe",
    "mttkrp_ablation_f64", "mttkrp_ablation_f32", "mttkrp_tile_volume",
    "mttkrp_dense_all_modes_f64", "mttkrp_dense_all_modes_f32", "mttkrp_cpals_f64",
    "mttkrp_calibrate_stream", "mttkrp_calibrate_mfma",
    "mttkrp_dense_f64_ld", "mttkrp_dense_f32_ld", "mttkrp_dense_f64_noalloc",
    "mttkrp_contract_leading_workspace_bytes", "mttkrp_contract_leading_f64", "mttkrp_contract_leading_f32",
    "mttkrp_dense_all_modes_shared_bytes", "mttkrp_dense_all_modes_shared_f64",
    "mttkrp_dense_all_modes_shared_f32", "mttkrp_cpals_shared_f64",
)

MTTKRP_SCHEDULE_ELEM = 1
MTTKRP_SCHEDULE_SUB = 2
MTTKRP_SCHEDULE_TILE = 3

_lib = None


class MttkrpError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__("mttkrp: %s (status %d)" % (text, status))
        self.status = status


def lib() -> ctypes.CDLL:
    """Load the library once; raise loudly if it is not there."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            "HIP library %s is missing: build it with "
            "`python -m paper_2510_14891_amd.build` (there is no CPU fallback)" % LIB_PATH)
    L = ctypes.CDLL(LIB_PATH)
    i64p = ctypes.POINTER(ctypes.c_int64)
    vpp = ctypes.POINTER(ctypes.c_void_p)
    core = [ctypes.c_int, i64p, ctypes.c_void_p, vpp, ctypes.c_int, ctypes.c_int,
            ctypes.c_void_p, ctypes.c_void_p]
    core_ws = core[:-1] + [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    for name in ("mttkrp_dense_f64", "mttkrp_dense_f32", "mttkrp_dense_f64_noalloc"):
        getattr(L, name).restype = ctypes.c_int
        getattr(L, name).argtypes = core
    for name in ("mttkrp_dense_f64_ws", "mttkrp_dense_f32_ws"):
        getattr(L, name).restype = ctypes.c_int
        getattr(L, name).argtypes = core_ws
    L.mttkrp_dense_workspace_bytes.restype = ctypes.c_size_t
    L.mttkrp_dense_workspace_bytes.argtypes = [ctypes.c_int, i64p, ctypes.c_int,
                                               ctypes.c_int, ctypes.c_int]
    L.mttkrp_dense_ex_workspace_bytes.restype = ctypes.c_size_t
    L.mttkrp_dense_ex_workspace_bytes.argtypes = L.mttkrp_dense_workspace_bytes.argtypes
    ex = [ctypes.c_int, i64p, ctypes.c_void_p, vpp, ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
    L.mttkrp_dense_f64_ex.restype = ctypes.c_int
    L.mttkrp_dense_f64_ex.argtypes = ex + [ctypes.c_double, ctypes.c_void_p, ctypes.c_void_p,
                                           ctypes.c_size_t, ctypes.c_void_p]
    L.mttkrp_dense_f32_ex.restype = ctypes.c_int
    L.mttkrp_dense_f32_ex.argtypes = ex + [ctypes.c_float, ctypes.c_void_p, ctypes.c_void_p,
                                           ctypes.c_size_t, ctypes.c_void_p]
    L.mttkrp_status_string.restype = ctypes.c_char_p
    L.mttkrp_status_string.argtypes = [ctypes.c_int]
    L.mttkrp_version.restype = ctypes.c_int
    L.mttkrp_release.restype = None
    L.mttkrp_timing_enable.restype = ctypes.c_int
    L.mttkrp_timing_enable.argtypes = [ctypes.c_int]
    L.mttkrp_timing_last.restype = ctypes.c_int
    L.mttkrp_timing_last.argtypes = [ctypes.POINTER(ctypes.c_float),
                                     ctypes.POINTER(ctypes.c_float)]
    L.mttkrp_timing_count.restype = ctypes.c_int64
    L.mttkrp_timing_get.restype = ctypes.c_int
    L.mttkrp_timing_get.argtypes = [ctypes.c_int64, ctypes.POINTER(ctypes.c_float),
                                    ctypes.POINTER(ctypes.c_float)]
    L.mttkrp_tune_set.restype = ctypes.c_int
    L.mttkrp_tune_set.argtypes = [ctypes.c_char_p, ctypes.c_int64]
    L.mttkrp_plan_describe.restype = ctypes.c_int
    L.mttkrp_plan_describe.argtypes = [ctypes.c_int, i64p, ctypes.c_int, ctypes.c_int,
                                       ctypes.c_int, ctypes.c_char_p, ctypes.c_size_t]
    abl = [ctypes.c_int, ctypes.c_int, i64p, ctypes.c_void_p, vpp, ctypes.c_int, ctypes.c_int,
           ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p]
    for name in ("mttkrp_ablation_f64", "mttkrp_ablation_f32"):
        getattr(L, name).restype = ctypes.c_int
        getattr(L, name).argtypes = abl
    L.mttkrp_tile_volume.restype = ctypes.c_int
    L.mttkrp_tile_volume.argtypes = [ctypes.c_int, i64p, ctypes.c_int64, ctypes.c_int, ctypes.c_int64,
                                     i64p, i64p]
    for name in ("mttkrp_dense_all_modes_f64", "mttkrp_dense_all_modes_f32"):
        getattr(L, name).restype = ctypes.c_int
        getattr(L, name).argtypes = [ctypes.c_int, i64p, ctypes.c_void_p, vpp, ctypes.c_int, vpp,
                                     ctypes.c_void_p]
    for name in ("mttkrp_cpals_f64", "mttkrp_cpals_shared_f64"):
        getattr(L, name).restype = ctypes.c_int
        getattr(L, name).argtypes = [ctypes.c_int, i64p, ctypes.c_void_p, vpp, ctypes.c_void_p, ctypes.c_int,
                                     ctypes.c_int, ctypes.c_double, ctypes.POINTER(ctypes.c_int),
                                     ctypes.POINTER(ctypes.c_double), ctypes.c_void_p]
    for name in ("mttkrp_dense_all_modes_shared_f64", "mttkrp_dense_all_modes_shared_f32"):
        getattr(L, name).restype = ctypes.c_int
        getattr(L, name).argtypes = [ctypes.c_int, i64p, ctypes.c_void_p, vpp, ctypes.c_int, vpp,
                                     ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    L.mttkrp_dense_all_modes_shared_bytes.restype = ctypes.c_size_t
    L.mttkrp_dense_all_modes_shared_bytes.argtypes = [ctypes.c_int, i64p, ctypes.c_int, ctypes.c_int]
    L.mttkrp_contract_leading_workspace_bytes.restype = ctypes.c_size_t
    L.mttkrp_contract_leading_workspace_bytes.argtypes = [ctypes.c_int64, ctypes.c_int64, ctypes.c_int, ctypes.c_int]
    for name in ("mttkrp_contract_leading_f64", "mttkrp_contract_leading_f32"):
        getattr(L, name).restype = ctypes.c_int
        getattr(L, name).argtypes = [ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p,
                                     ctypes.c_int64, ctypes.c_int, ctypes.c_void_p, ctypes.c_int64,
                                     ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    ldargs = [ctypes.c_int, i64p, ctypes.c_void_p, vpp, i64p, ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
    L.mttkrp_dense_f64_ld.restype = ctypes.c_int
    L.mttkrp_dense_f64_ld.argtypes = ldargs + [ctypes.c_double, ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p,
                                               ctypes.c_size_t, ctypes.c_void_p]
    L.mttkrp_dense_f32_ld.restype = ctypes.c_int
    L.mttkrp_dense_f32_ld.argtypes = ldargs + [ctypes.c_float, ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p,
                                               ctypes.c_size_t, ctypes.c_void_p]
    L.mttkrp_calibrate_stream.restype = ctypes.c_int
    L.mttkrp_calibrate_stream.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int,
                                          ctypes.POINTER(ctypes.c_float), ctypes.c_void_p]
    L.mttkrp_calibrate_mfma.restype = ctypes.c_int
    L.mttkrp_calibrate_mfma.argtypes = [ctypes.c_int, ctypes.c_double, ctypes.c_int,
                                        ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_double),
                                        ctypes.c_void_p]
    _lib = L
    return L


def mttkrp_status_string(status: int) -> str:
    return lib().mttkrp_status_string(int(status)).decode()


def _check(status: int) -> None:
    if status != MTTKRP_OK:
        raise MttkrpError(status, mttkrp_status_string(status))


def mttkrp_version() -> int:
    return int(lib().mttkrp_version())


def mttkrp_release() -> None:
    lib().mttkrp_release()


def mttkrp_timing_enable(enable: bool) -> None:
    _check(lib().mttkrp_timing_enable(1 if enable else 0))


def mttkrp_timing_last():
    """(stream_ms, combine_ms) of the most recent call on the current device."""
    a, b = ctypes.c_float(0), ctypes.c_float(0)
    _check(lib().mttkrp_timing_last(ctypes.byref(a), ctypes.byref(b)))
    return float(a.value), float(b.value)


def mttkrp_timing_count() -> int:
    return int(lib().mttkrp_timing_count())


def mttkrp_timing_get(index: int):
    """(stream_ms, combine_ms) of timed call ``index`` on the current device."""
    a, b = ctypes.c_float(0), ctypes.c_float(0)
    _check(lib().mttkrp_timing_get(int(index), ctypes.byref(a), ctypes.byref(b)))
    return float(a.value), float(b.value)


def mttkrp_tune_set(key: str, value: int) -> None:
    _check(lib().mttkrp_tune_set(key.encode(), int(value)))


def _dims_array(dims: Sequence[int]):
    return (ctypes.c_int64 * len(dims))(*[int(v) for v in dims])


def mttkrp_plan_describe(dims: Sequence[int], R: int, k: int, dtype_bytes: int) -> str:
    buf = ctypes.create_string_buffer(512)
    _check(lib().mttkrp_plan_describe(len(dims), _dims_array(dims), int(R), int(k),
                                      int(dtype_bytes), buf, len(buf)))
    return buf.value.decode()


def mttkrp_dense_workspace_bytes(dims: Sequence[int], R: int, k: int, dtype_bytes: int) -> int:
    n = lib().mttkrp_dense_workspace_bytes(len(dims), _dims_array(dims), int(R), int(k),
                                           int(dtype_bytes))
    if n == ctypes.c_size_t(-1).value:
        raise MttkrpError(MTTKRP_ERR_INVALID_ARG, "invalid argument")
    return int(n)


def mttkrp_dense_ex_workspace_bytes(dims: Sequence[int], R: int, k: int, dtype_bytes: int) -> int:
    n = lib().mttkrp_dense_ex_workspace_bytes(len(dims), _dims_array(dims), int(R), int(k),
                                              int(dtype_bytes))
    if n == ctypes.c_size_t(-1).value:
        raise MttkrpError(MTTKRP_ERR_INVALID_ARG, "invalid argument")
    return int(n)


def _marshal(X, dims, factors, k, M, stream):
    """Checks the tensors of one call and returns (suffix, d, factor pointer
    array, R, M, stream) ready for the C entry points."""
    import torch
    if not X.is_cuda:
        raise ValueError("X must live on the GPU")
    if X.dtype == torch.float64:
        suffix, sbytes = "f64", 8
    elif X.dtype == torch.float32:
        suffix, sbytes = "f32", 4
    else:
        raise TypeError("X must be float64 or float32")
    d = len(dims)
    if not X.is_contiguous():
        raise ValueError("X must be contiguous (flat, first index fastest)")
    n = 1
    for v in dims:
        n *= int(v)
    if X.numel() != n:
        raise ValueError("X has %d values, dims say %d" % (X.numel(), n))
    if len(factors) != d:
        raise ValueError("need one factor slot per mode")
    R = None
    ptrs = (ctypes.c_void_p * d)()
    for m in range(d):
        A = factors[m]
        if A is None:
            ptrs[m] = None
            continue
        if A.dtype != X.dtype or A.device != X.device or not A.is_contiguous():
            raise ValueError("factor %d: wrong dtype/device or not contiguous" % m)
        if A.dim() != 2 or A.shape[0] != int(dims[m]):
            raise ValueError("factor %d has shape %s" % (m, tuple(A.shape)))
        if R is None:
            R = int(A.shape[1])
        elif int(A.shape[1]) != R:
            raise ValueError("factors disagree on R")
        ptrs[m] = A.data_ptr()
    if R is None:
        raise ValueError("no factor given")
    if M is None:
        M = torch.empty((int(dims[k]), R), dtype=X.dtype, device=X.device)
    else:
        if (M.dtype != X.dtype or M.device != X.device or not M.is_contiguous()
                or tuple(M.shape) != (int(dims[k]), R)):
            raise ValueError("M must be a contiguous (I_k, R) tensor like X")
    if stream is None:
        stream = torch.cuda.current_stream(X.device).cuda_stream
    return suffix, d, ptrs, R, M, stream


def mttkrp_dense(X, dims: Sequence[int], factors: Sequence, k: int, M=None,
                 workspace=None, stream: Optional[int] = None, lam=None, beta=None):
    """M = X_(k) (Khatri-Rao of all factors but the k-th), on the GPU.

    X        flat torch tensor on a HIP device, prod(dims) values, first index
             fastest; float64 or float32
    dims     extents (I_0, ..., I_{d-1})
    factors  d torch tensors, factors[m] of shape (I_m, R), contiguous, same
             dtype/device as X; factors[k] may be None
    k        0-based mode
    M        optional output tensor (I_k, R); allocated when None
    workspace  optional torch tensor to use as caller-owned workspace (selects
             the *_ws entry point)
    lam, beta  optional weight vector (torch tensor of R values on the device)
             and accumulation factor; either selects the *_ex entry point:
             M = beta * M + result * diag(lam)
    stream   raw hipStream_t value; default: torch's current stream
    Returns M.  The call is asynchronous on the stream.
    """
    import torch
    L = lib()
    suffix, d, ptrs, R, M, stream = _marshal(X, dims, factors, k, M, stream)
    if lam is not None and (lam.dtype != X.dtype or lam.device != X.device
                            or not lam.is_contiguous() or lam.numel() != R):
        raise ValueError("lam must be a contiguous device vector of R values like X")
    with torch.cuda.device(X.device):
        if lam is not None or beta is not None:
            rc = getattr(L, "mttkrp_dense_" + suffix + "_ex")(
                d, _dims_array(dims), X.data_ptr(), ptrs, R, int(k),
                lam.data_ptr() if lam is not None else None,
                float(beta) if beta is not None else 0.0, M.data_ptr(),
                workspace.data_ptr() if workspace is not None else None,
                workspace.numel() * workspace.element_size() if workspace is not None else 0,
                ctypes.c_void_p(stream))
        elif workspace is None:
            rc = getattr(L, "mttkrp_dense_" + suffix)(
                d, _dims_array(dims), X.data_ptr(), ptrs, R, int(k), M.data_ptr(),
                ctypes.c_void_p(stream))
        else:
            rc = getattr(L, "mttkrp_dense_" + suffix + "_ws")(
                d, _dims_array(dims), X.data_ptr(), ptrs, R, int(k), M.data_ptr(),
                workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                ctypes.c_void_p(stream))
    _check(rc)
    return M


def mttkrp_dense_noalloc(X, dims: Sequence[int], factors: Sequence, k: int, M, stream: Optional[int] = None):
    """mttkrp_dense_f64_noalloc: the fp64 MTTKRP into the caller's ``M`` with the library's fixed
    scratch array as workspace (no device allocation; see include/mttkrp.h for the limit)."""
    import torch
    if X.dtype != torch.float64:
        raise TypeError("the no-allocation entry point is float64 only")
    if M is None:
        raise ValueError("M must be given: this entry point allocates nothing")
    suffix, d, ptrs, R, M, stream = _marshal(X, dims, factors, k, M, stream)
    with torch.cuda.device(X.device):
        rc = lib().mttkrp_dense_f64_noalloc(d, _dims_array(dims), X.data_ptr(), ptrs, R, int(k), M.data_ptr(),
                                            ctypes.c_void_p(stream))
    _check(rc)
    return M


def mttkrp_ablation(schedule: int, X, dims: Sequence[int], factors: Sequence, k: int,
                    tile_width: int = 0, M=None, stream: Optional[int] = None):
    """The same M by one of the paper's own schedules (ELEM, SUB, TILE); see
    include/mttkrp_ablation.h.  Arguments as for mttkrp_dense; ``tile_width``
    is the TILE schedule's entries per tile along each mode other than k."""
    import torch
    L = lib()
    suffix, d, ptrs, R, M, stream = _marshal(X, dims, factors, k, M, stream)
    with torch.cuda.device(X.device):
        rc = getattr(L, "mttkrp_ablation_" + suffix)(
            int(schedule), d, _dims_array(dims), X.data_ptr(), ptrs, R, int(k), int(tile_width),
            M.data_ptr(), ctypes.c_void_p(stream))
    _check(rc)
    return M


def mttkrp_tile_volume(dims: Sequence[int], cache_bytes: int, value_bytes: int,
                       tiles_per_unit: int):
    """(width, N_T) of the paper's tile-volume heuristic; host arithmetic only."""
    w, v = ctypes.c_int64(0), ctypes.c_int64(0)
    _check(lib().mttkrp_tile_volume(len(dims), _dims_array(dims), int(cache_bytes), int(value_bytes),
                                    int(tiles_per_unit), ctypes.byref(w), ctypes.byref(v)))
    return int(w.value), int(v.value)


def mttkrp_dense_all_modes(X, dims: Sequence[int], factors: Sequence, M_out=None,
                           stream: Optional[int] = None):
    """[M_0, ..., M_{d-1}]: the MTTKRP of every mode on the same resident X."""
    import torch
    L = lib()
    d = len(dims)
    suffix, d, ptrs, R, M0, stream = _marshal(X, dims, factors, 0, None if M_out is None else M_out[0], stream)
    if any(f is None for f in factors):
        raise ValueError("every factor is read by the all-modes sweep")
    if M_out is None:
        M_out = [M0] + [torch.empty((int(dims[k]), R), dtype=X.dtype, device=X.device) for k in range(1, d)]
    outs = (ctypes.c_void_p * d)()
    for k in range(d):
        M = M_out[k]
        if (M.dtype != X.dtype or M.device != X.device or not M.is_contiguous()
                or tuple(M.shape) != (int(dims[k]), R)):
            raise ValueError("M_out[%d] must be a contiguous (I_k, R) tensor like X" % k)
        outs[k] = M.data_ptr()
    with torch.cuda.device(X.device):
        rc = getattr(L, "mttkrp_dense_all_modes_" + suffix)(d, _dims_array(dims), X.data_ptr(), ptrs, R, outs,
                                                            ctypes.c_void_p(stream))
    _check(rc)
    return list(M_out)


_scratch_buffers = {}


def _scratch(device, stream, nbytes):
    """A caller-owned workspace for the calls that take one: kept per (device, stream) and
    grown on demand, so that it outlives the kernels that use it."""
    import torch
    key = (str(device), int(stream))
    buf = _scratch_buffers.get(key)
    if buf is None or buf.numel() < nbytes:
        if buf is not None:
            torch.cuda.synchronize(device)
        buf = torch.empty(int(nbytes), dtype=torch.uint8, device=device)
        _scratch_buffers[key] = buf
    return buf


def mttkrp_dense_all_modes_shared_bytes(dims: Sequence[int], R: int, dtype_bytes: int) -> int:
    """Bytes of workspace the shared sweep needs; 0 when the shape has no supported cut."""
    return int(lib().mttkrp_dense_all_modes_shared_bytes(len(dims), _dims_array(dims), int(R), int(dtype_bytes)))


def mttkrp_dense_all_modes_shared(X, dims: Sequence[int], factors: Sequence, M_out=None,
                                  stream: Optional[int] = None, workspace=None):
    """[M_0, ..., M_{d-1}] from two passes over X (partial contractions shared between the
    modes); see mttkrp_dense_all_modes_shared_f64 in include/mttkrp_cpals.h.  ``workspace``: an
    optional torch tensor of at least mttkrp_dense_all_modes_shared_bytes(...) bytes on X's
    device (default: a buffer this module keeps per stream)."""
    import torch
    L = lib()
    suffix, d, ptrs, R, M0, stream = _marshal(X, dims, factors, 0, None if M_out is None else M_out[0], stream)
    if any(f is None for f in factors):
        raise ValueError("every factor is read by the all-modes sweep")
    if M_out is None:
        M_out = [M0] + [torch.empty((int(dims[k]), R), dtype=X.dtype, device=X.device) for k in range(1, d)]
    outs = (ctypes.c_void_p * d)()
    for k in range(d):
        M = M_out[k]
        if (M.dtype != X.dtype or M.device != X.device or not M.is_contiguous()
                or tuple(M.shape) != (int(dims[k]), R)):
            raise ValueError("M_out[%d] must be a contiguous (I_k, R) tensor like X" % k)
        outs[k] = M.data_ptr()
    nbytes = mttkrp_dense_all_modes_shared_bytes(dims, R, X.element_size())
    if nbytes == 0:
        raise MttkrpError(MTTKRP_ERR_UNSUPPORTED, "no supported cut for this shape")
    if workspace is not None:
        if workspace.device != X.device or not workspace.is_contiguous() \
                or workspace.numel() * workspace.element_size() < nbytes:
            raise ValueError("workspace must be a contiguous tensor of at least %d bytes on X's device" % nbytes)
        ws = workspace
    else:
        ws = _scratch(X.device, stream, nbytes)
    with torch.cuda.device(X.device):
        rc = getattr(L, "mttkrp_dense_all_modes_shared_" + suffix)(
            d, _dims_array(dims), X.data_ptr(), ptrs, R, outs, ws.data_ptr(), nbytes, ctypes.c_void_p(stream))
    _check(rc)
    return list(M_out)


def mttkrp_contract_leading(X, P: int, Q: int, K, T_out=None, stream: Optional[int] = None):
    """T (Q x R) = X^T K for X read as a P x Q matrix, first index fastest, and K (P x R);
    see mttkrp_contract_leading_f64 in include/mttkrp.h."""
    import torch
    L = lib()
    if X.dtype not in (torch.float64, torch.float32) or not X.is_cuda or not X.is_contiguous():
        raise ValueError("X must be a contiguous float64/float32 tensor on the GPU")
    if X.numel() != int(P) * int(Q):
        raise ValueError("X must hold P * Q values")
    if (K.dtype != X.dtype or K.device != X.device or K.dim() != 2 or K.shape[0] != int(P)
            or K.stride(1) != 1):
        raise ValueError("K must be a (P, R) tensor like X with unit column stride")
    R = int(K.shape[1])
    if T_out is None:
        T_out = torch.empty((int(Q), R), dtype=X.dtype, device=X.device)
    if (T_out.dtype != X.dtype or T_out.device != X.device or tuple(T_out.shape) != (int(Q), R)
            or T_out.stride(1) != 1):
        raise ValueError("T_out must be a (Q, R) tensor like X with unit column stride")
    suffix = "f64" if X.dtype == torch.float64 else "f32"
    if stream is None:
        stream = torch.cuda.current_stream(X.device).cuda_stream
    nbytes = int(L.mttkrp_contract_leading_workspace_bytes(int(P), int(Q), R, X.element_size()))
    if nbytes == ctypes.c_size_t(-1).value:
        raise MttkrpError(MTTKRP_ERR_UNSUPPORTED, "unsupported shape")
    ws = _scratch(X.device, stream, max(nbytes, 1))
    with torch.cuda.device(X.device):
        rc = getattr(L, "mttkrp_contract_leading_" + suffix)(
            int(P), int(Q), X.data_ptr(), K.data_ptr(), int(K.stride(0)), R, T_out.data_ptr(),
            int(T_out.stride(0)), ws.data_ptr() if nbytes else None, nbytes, ctypes.c_void_p(stream))
    _check(rc)
    return T_out


def mttkrp_cpals(X, dims: Sequence[int], factors: Sequence, max_iters: int, tol: float,
                 stream: Optional[int] = None, shared: bool = False):
    """CP-ALS in fp64 on the GPU.  ``factors`` (initial guess) are updated in place.
    ``shared``: sweeps share partial contractions between the modes (two passes over X).
    Returns (lambda tensor, list of fits per sweep)."""
    import torch
    L = lib()
    if X.dtype != torch.float64:
        raise TypeError("CP-ALS runs in float64")
    suffix, d, ptrs, R, _, stream = _marshal(X, dims, factors, 0, None, stream)
    if any(f is None for f in factors):
        raise ValueError("CP-ALS needs an initial guess for every factor")
    lam = torch.empty(R, dtype=X.dtype, device=X.device)
    iters = ctypes.c_int(0)
    fits = (ctypes.c_double * int(max_iters))()
    with torch.cuda.device(X.device):
        fn = L.mttkrp_cpals_shared_f64 if shared else L.mttkrp_cpals_f64
        rc = fn(d, _dims_array(dims), X.data_ptr(), ptrs, lam.data_ptr(), R, int(max_iters),
                float(tol), ctypes.byref(iters), fits, ctypes.c_void_p(stream))
    _check(rc)
    return lam, [float(fits[i]) for i in range(iters.value)]


def mttkrp_calibrate_stream(buf, launches: int = 10, stream: Optional[int] = None) -> float:
    """GB/s of a read-only pass over the torch tensor ``buf`` (see include/mttkrp_calibrate.h)."""
    import torch
    nbytes = buf.numel() * buf.element_size()
    nbytes -= nbytes % 16
    if stream is None:
        stream = torch.cuda.current_stream(buf.device).cuda_stream
    ms = ctypes.c_float(0)
    with torch.cuda.device(buf.device):
        _check(lib().mttkrp_calibrate_stream(buf.data_ptr(), nbytes, int(launches), ctypes.byref(ms),
                                             ctypes.c_void_p(stream)))
    return nbytes / ms.value / 1e6


def mttkrp_calibrate_mfma(dtype_bytes: int, gflop_per_launch: float, launches: int = 10,
                          stream: Optional[int] = None) -> float:
    """TFLOP/s of back-to-back 16x16x4 MFMAs of the data type (see include/mttkrp_calibrate.h)."""
    import torch
    if stream is None:
        stream = torch.cuda.current_stream().cuda_stream
    ms, flop = ctypes.c_float(0), ctypes.c_double(0)
    _check(lib().mttkrp_calibrate_mfma(int(dtype_bytes), float(gflop_per_launch), int(launches),
                                       ctypes.byref(ms), ctypes.byref(flop), ctypes.c_void_p(stream)))
    return flop.value / ms.value / 1e9


def mttkrp_dense_ld(X, dims: Sequence[int], factors: Sequence, k: int, M, R: int, lam=None,
                    beta: float = 0.0, stream: Optional[int] = None):
    """The MTTKRP on blocks of wider arrays: ``factors[m]`` are 2-D torch tensors
    (I_m, >= R) whose rows may be strided (stride(1) == 1), of which the first R
    columns are the factor; ``M`` likewise (I_k, >= R), of which the first R
    columns are written.  See mttkrp_dense_f64_ld in include/mttkrp.h."""
    import torch
    L = lib()
    d = len(dims)
    suffix = "f64" if X.dtype == torch.float64 else "f32"
    if X.dtype not in (torch.float64, torch.float32) or not X.is_cuda or not X.is_contiguous():
        raise ValueError("X must be a contiguous float64/float32 tensor on the GPU")
    ptrs = (ctypes.c_void_p * d)()
    lds = (ctypes.c_int64 * d)()
    for m in range(d):
        A = factors[m]
        if A is None:
            ptrs[m] = None
            lds[m] = R
            continue
        if (A.dtype != X.dtype or A.device != X.device or A.dim() != 2 or A.shape[0] != int(dims[m])
                or A.shape[1] < R or (A.shape[1] > 1 and A.stride(1) != 1)):
            raise ValueError("factor %d: wrong dtype/device/shape/strides" % m)
        ptrs[m] = A.data_ptr()
        lds[m] = A.stride(0) if A.shape[0] > 1 else max(R, A.shape[1])
    if (M.dtype != X.dtype or M.device != X.device or M.dim() != 2 or M.shape[0] != int(dims[k])
            or M.shape[1] < R or (M.shape[1] > 1 and M.stride(1) != 1)):
        raise ValueError("M: wrong dtype/device/shape/strides")
    ldM = M.stride(0) if M.shape[0] > 1 else max(R, M.shape[1])
    if stream is None:
        stream = torch.cuda.current_stream(X.device).cuda_stream
    with torch.cuda.device(X.device):
        rc = getattr(L, "mttkrp_dense_" + suffix + "_ld")(
            d, _dims_array(dims), X.data_ptr(), ptrs, lds, int(R), int(k),
            lam.data_ptr() if lam is not None else None, float(beta), M.data_ptr(), int(ldM),
            None, 0, ctypes.c_void_p(stream))
    _check(rc)
    return M
