"""ctypes binding of libosdp: same names as the C ABI, argument marshalling only.

PyTorch supplies device memory (``tensor.data_ptr()``) and streams
(``torch.cuda.Stream().cuda_stream`` is a ``hipStream_t`` on ROCm builds); every
step of the path runs inside the library's HIP kernels.  There is no CPU or
PyTorch fallback: if the library is missing the import of this module fails.
"""
from __future__ import annotations

import ctypes
from dataclasses import dataclass
from typing import Optional, Sequence

from . import build as _build

OSDP_OK = 0
OSDP_ERR_INVALID_ARG = -1
OSDP_ERR_UNSUPPORTED = -2
OSDP_ERR_WORKSPACE = -3
OSDP_ERR_HIP = -4

OSDP_STAGING_AUTO = 0
OSDP_STAGING_SINGLE = 1
OSDP_STAGING_DOUBLE = 2
OSDP_STAGING_HALF = 3

OSDP_SPLIT_OUT_FEATURES = 0
OSDP_SPLIT_IN_FEATURES = 1
OSDP_SPLIT_LONGER = 2
OSDP_SPLIT_PER_PASS = 3

OSDP_NOALLOC_SCRATCH_BYTES = 64 << 20

OSDP_KERNEL_GATHER = 0
OSDP_KERNEL_GEMM_FWD = 1
OSDP_KERNEL_GEMM_DW = 2
OSDP_KERNEL_GEMM_DX = 3
OSDP_KERNEL_GATHER_CARRIED = 4
OSDP_KERNEL_GEMM_PERSISTENT = 5
OSDP_KERNEL_KINDS = 6
KERNEL_NAMES = ("gather", "gemm_fwd", "gemm_dw", "gemm_dx", "gather_carried", "gemm_persistent")

EXPORTS = (
    "osdp_slice_range", "osdp_row_slice_range", "osdp_split_linear_gather_slice",
    "osdp_split_linear_gather_row_slice", "osdp_split_linear_workspace_bytes", "osdp_split_linear_fwd",
    "osdp_split_linear_bwd", "osdp_split_linear_fwd_noalloc", "osdp_split_linear_fwd_mixed", "osdp_split_linear_bwd_mixed",
    "osdp_granularity_candidates", "osdp_granularity_measure",
    "osdp_granularity_select", "osdp_cost_model", "osdp_plan_search", "osdp_profile_begin", "osdp_profile_end", "osdp_profile_overlap",
    "osdp_debug_option", "osdp_strerror", "osdp_last_error", "osdp_version",
)


class osdp_shape(ctypes.Structure):
    _fields_ = [("T", ctypes.c_int64), ("I", ctypes.c_int64), ("O", ctypes.c_int64),
                ("N", ctypes.c_int32), ("k", ctypes.c_int32)]


class osdp_plan(ctypes.Structure):
    _fields_ = [("n_ops", ctypes.c_int32), ("k_per_op", ctypes.POINTER(ctypes.c_int32)),
                ("zdp_mask", ctypes.POINTER(ctypes.c_uint64)), ("staging", ctypes.c_int32),
                ("split_dim_per_op", ctypes.POINTER(ctypes.c_uint8)),
                ("staging_per_op", ctypes.POINTER(ctypes.c_int32))]


class osdp_granularity_candidate(ctypes.Structure):
    _fields_ = [("k", ctypes.c_int32), ("staging", ctypes.c_int32), ("split_dim", ctypes.c_int32),
                ("reserved", ctypes.c_int32), ("peak_weight_staging", ctypes.c_size_t),
                ("workspace", ctypes.c_size_t), ("ms", ctypes.c_double)]


class osdp_operator_cost(ctypes.Structure):
    _fields_ = [("m_model", ctypes.c_double), ("m_act", ctypes.c_double), ("m_extra", ctypes.c_double),
                ("s_bytes", ctypes.c_double), ("gamma", ctypes.c_double)]


class osdp_device_info(ctypes.Structure):
    _fields_ = [("N", ctypes.c_int32), ("b_max", ctypes.c_int32), ("alpha", ctypes.c_double),
                ("beta", ctypes.c_double), ("m_limit", ctypes.c_double)]


class osdp_search_result(ctypes.Structure):
    _fields_ = [("found", ctypes.c_int32), ("b", ctypes.c_int32), ("time_per_sample", ctypes.c_double),
                ("memory", ctypes.c_double), ("batch_sizes_tried", ctypes.c_int32), ("exact", ctypes.c_int32),
                ("reserved", ctypes.c_int32), ("plans_visited", ctypes.c_uint64)]


class osdp_kernel_stats(ctypes.Structure):
    _fields_ = [("launches", ctypes.c_int64), ("ms", ctypes.c_double), ("flops", ctypes.c_double),
                ("bytes", ctypes.c_double)]


class OsdpError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"libosdp status {status}: {message}")
        self.status = status


def _load() -> ctypes.CDLL:
    path = _build.LIB
    if not path.exists():
        raise ImportError(
            f"{path} is missing: build it first (python paper_2209_13258_amd/build.py); "
            "there is no fallback path")
    lib = ctypes.CDLL(str(path))
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
    shp, pln = ctypes.POINTER(osdp_shape), ctypes.POINTER(osdp_plan)
    lib.osdp_slice_range.argtypes = [shp, i32, ctypes.POINTER(i64), ctypes.POINTER(i64)]
    lib.osdp_row_slice_range.argtypes = [shp, i32, ctypes.POINTER(i64), ctypes.POINTER(i64)]
    lib.osdp_split_linear_gather_slice.argtypes = [shp, i32, vp, vp, vp]
    lib.osdp_split_linear_gather_row_slice.argtypes = [shp, i32, vp, vp, vp]
    lib.osdp_split_linear_workspace_bytes.argtypes = [shp, pln, i32, i32, ctypes.POINTER(ctypes.c_size_t),
                                                      ctypes.POINTER(ctypes.c_size_t)]
    lib.osdp_split_linear_fwd.argtypes = [shp, pln, i32, vp, i64, vp, vp, i64, vp, ctypes.c_size_t, vp, vp]
    lib.osdp_split_linear_fwd_noalloc.argtypes = [shp, pln, i32, vp, i64, vp, vp, i64, vp]
    lib.osdp_split_linear_fwd_noalloc.restype = ctypes.c_int
    lib.osdp_split_linear_bwd.argtypes = [shp, pln, i32, vp, i64, vp, i64, vp, vp, i64, vp, vp,
                                          ctypes.c_size_t, vp, vp]
    lib.osdp_split_linear_fwd_mixed.argtypes = [shp, pln, i32, vp, i64, vp, vp, i64, vp, i64, vp, ctypes.c_size_t, vp, vp]
    lib.osdp_split_linear_bwd_mixed.argtypes = [shp, pln, i32, vp, i64, vp, i64, vp, vp, i64, vp, i64, vp, vp, vp,
                                                ctypes.c_size_t, vp, vp]
    cnd = ctypes.POINTER(osdp_granularity_candidate)
    lib.osdp_granularity_candidates.argtypes = [shp, ctypes.POINTER(i32), i32, cnd, i32, ctypes.POINTER(i32)]
    lib.osdp_granularity_measure.argtypes = [shp, vp, i64, vp, i64, vp, vp, i64, vp, i64, vp, vp, ctypes.c_size_t,
                                             vp, vp, cnd, i32, i32, i32]
    lib.osdp_granularity_select.argtypes = [cnd, i32, ctypes.c_size_t, ctypes.c_size_t, ctypes.c_double,
                                            ctypes.POINTER(i32)]
    opc, dvi = ctypes.POINTER(osdp_operator_cost), ctypes.POINTER(osdp_device_info)
    lib.osdp_cost_model.argtypes = [opc, i32, dvi, ctypes.POINTER(ctypes.c_uint8), i32,
                                    ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]
    lib.osdp_plan_search.argtypes = [opc, i32, dvi, ctypes.POINTER(ctypes.c_uint8), ctypes.POINTER(osdp_search_result)]
    lib.osdp_debug_option.argtypes = [ctypes.c_char_p, i32]
    lib.osdp_debug_option.restype = ctypes.c_int
    lib.osdp_profile_begin.argtypes = [i32]
    lib.osdp_profile_end.argtypes = [ctypes.POINTER(osdp_kernel_stats)]
    lib.osdp_profile_overlap.argtypes = [ctypes.POINTER(ctypes.c_double)] * 3
    lib.osdp_profile_overlap.restype = ctypes.c_int
    for name in ("osdp_slice_range", "osdp_row_slice_range", "osdp_split_linear_gather_slice",
                 "osdp_split_linear_gather_row_slice", "osdp_split_linear_workspace_bytes",
                 "osdp_split_linear_fwd", "osdp_split_linear_bwd", "osdp_split_linear_fwd_mixed",
                 "osdp_split_linear_bwd_mixed", "osdp_granularity_candidates",
                 "osdp_granularity_measure", "osdp_granularity_select", "osdp_cost_model", "osdp_plan_search",
                 "osdp_profile_begin", "osdp_profile_end"):
        getattr(lib, name).restype = ctypes.c_int
    lib.osdp_strerror.argtypes = [ctypes.c_int]
    lib.osdp_strerror.restype = ctypes.c_char_p
    lib.osdp_last_error.restype = ctypes.c_char_p
    lib.osdp_version.restype = ctypes.c_char_p
    return lib


lib = _load()


def _check(status: int) -> None:
    if status != OSDP_OK:
        msg = lib.osdp_last_error().decode() or lib.osdp_strerror(status).decode()
        raise OsdpError(status, msg)


@dataclass
class Plan:
    """Per-operator slice granularities (and, optionally, ZDP masks and split dimensions) plus the staging mode."""
    k_per_op: Sequence[int]
    staging: int = OSDP_STAGING_AUTO
    zdp_mask: Optional[Sequence[int]] = None
    split_dim_per_op: Optional[Sequence[int]] = None
    staging_per_op: Optional[Sequence[int]] = None

    def to_c(self):
        n = len(self.k_per_op)
        ks = (ctypes.c_int32 * n)(*self.k_per_op)
        mask = (ctypes.c_uint64 * n)(*self.zdp_mask) if self.zdp_mask is not None else None
        dims = (ctypes.c_uint8 * n)(*self.split_dim_per_op) if self.split_dim_per_op is not None else None
        modes = (ctypes.c_int32 * n)(*self.staging_per_op) if self.staging_per_op is not None else None
        p = osdp_plan(n, ctypes.cast(ks, ctypes.POINTER(ctypes.c_int32)),
                      ctypes.cast(mask, ctypes.POINTER(ctypes.c_uint64)) if mask is not None else None,
                      self.staging,
                      ctypes.cast(dims, ctypes.POINTER(ctypes.c_uint8)) if dims is not None else None,
                      ctypes.cast(modes, ctypes.POINTER(ctypes.c_int32)) if modes is not None else None)
        return p, (ks, mask, dims, modes)  # keep the arrays alive with the struct


def _shape(T, I, O, N, k):
    return osdp_shape(int(T), int(I), int(O), int(N), int(k))


def _plan_ref(plan: Optional[Plan]):
    if plan is None:
        return None, None
    p, keep = plan.to_c()
    return ctypes.byref(p), (p, keep)


def _ptrs(tensors):
    return (ctypes.c_void_p * len(tensors))(*[int(t.data_ptr()) for t in tensors])


def _stream(s) -> Optional[int]:
    if s is None:
        return None
    return int(getattr(s, "cuda_stream", s))


def osdp_version() -> str:
    return lib.osdp_version().decode()


def osdp_slice_range(O: int, k: int, j: int, T: int = 1, I: int = 8, N: int = 1):
    c0, c1 = ctypes.c_int64(), ctypes.c_int64()
    shape = _shape(T, I, O, N, k)
    _check(lib.osdp_slice_range(ctypes.byref(shape), j, ctypes.byref(c0), ctypes.byref(c1)))
    return c0.value, c1.value


def osdp_row_slice_range(I: int, k: int, j: int, T: int = 1, O: int = 8, N: int = 1):
    r0, r1 = ctypes.c_int64(), ctypes.c_int64()
    shape = _shape(T, I, O, N, k)
    _check(lib.osdp_row_slice_range(ctypes.byref(shape), j, ctypes.byref(r0), ctypes.byref(r1)))
    return r0.value, r1.value


def osdp_split_linear_workspace_bytes(T, I, O, N, k, is_bwd: bool, plan: Optional[Plan] = None, op_index: int = 0):
    """Returns (total workspace bytes, peak gathered-weight staging bytes)."""
    shape = _shape(T, I, O, N, k)
    total, peak = ctypes.c_size_t(), ctypes.c_size_t()
    pref, _keep = _plan_ref(plan)
    _check(lib.osdp_split_linear_workspace_bytes(ctypes.byref(shape), pref, op_index, int(bool(is_bwd)),
                                                 ctypes.byref(total), ctypes.byref(peak)))
    return total.value, peak.value


def osdp_split_linear_gather_slice(I, O, k, j, w_shards, staging, stream=None, T: int = 1):
    """Gathers column slice j of k from the shard tensors into ``staging`` (dense [I x w_j])."""
    shape = _shape(T, I, O, len(w_shards), k)
    _check(lib.osdp_split_linear_gather_slice(ctypes.byref(shape), j, _ptrs(w_shards),
                                              int(staging.data_ptr()), _stream(stream)))


def osdp_split_linear_gather_row_slice(I, O, k, j, w_shards, staging, stream=None, T: int = 1):
    """Gathers row slice j of k from the shard tensors into ``staging`` (dense [h_j x O])."""
    shape = _shape(T, I, O, len(w_shards), k)
    _check(lib.osdp_split_linear_gather_row_slice(ctypes.byref(shape), j, _ptrs(w_shards),
                                                  int(staging.data_ptr()), _stream(stream)))


def osdp_split_linear_fwd(X, w_shards, Y, k, workspace, *, plan: Optional[Plan] = None, op_index: int = 0,
                          stream_compute=None, stream_copy=None):
    """Y[T x O] = X[T x I] . W, W given as N shard tensors; X, Y 2-D bf16 tensors (row stride = ld)."""
    T, I = X.shape
    O = Y.shape[1]
    shape = _shape(T, I, O, len(w_shards), k)
    pref, _keep = _plan_ref(plan)
    _check(lib.osdp_split_linear_fwd(ctypes.byref(shape), pref, op_index, int(X.data_ptr()), X.stride(0),
                                     _ptrs(w_shards), int(Y.data_ptr()), Y.stride(0),
                                     int(workspace.data_ptr()), workspace.numel() * workspace.element_size(),
                                     _stream(stream_compute), _stream(stream_copy)))


def osdp_split_linear_fwd_noalloc(X, w_shards, Y, k, *, plan: Optional[Plan] = None, op_index: int = 0, stream=None):
    """The forward on one stream with the library's built-in scratch array in place of a workspace."""
    T, I = X.shape
    O = Y.shape[1]
    shape = _shape(T, I, O, len(w_shards), k)
    pref, _keep = _plan_ref(plan)
    _check(lib.osdp_split_linear_fwd_noalloc(ctypes.byref(shape), pref, op_index, int(X.data_ptr()), X.stride(0),
                                             _ptrs(w_shards), int(Y.data_ptr()), Y.stride(0), _stream(stream)))


def osdp_split_linear_bwd(X, dY, w_shards, dX, dw_shards, k, workspace, *, plan: Optional[Plan] = None,
                          op_index: int = 0, stream_compute=None, stream_copy=None):
    """dX[T x I] and the shard-major dW from X[T x I], dY[T x O] and the weight shards."""
    T, I = X.shape
    O = dY.shape[1]
    shape = _shape(T, I, O, len(w_shards), k)
    pref, _keep = _plan_ref(plan)
    _check(lib.osdp_split_linear_bwd(ctypes.byref(shape), pref, op_index, int(X.data_ptr()), X.stride(0),
                                     int(dY.data_ptr()), dY.stride(0), _ptrs(w_shards),
                                     int(dX.data_ptr()), dX.stride(0), _ptrs(dw_shards),
                                     int(workspace.data_ptr()), workspace.numel() * workspace.element_size(),
                                     _stream(stream_compute), _stream(stream_copy)))


def _opt_ptrs(tensors):
    """Array of device pointers in which None stands for a slice that has no replica (ZDP mode)."""
    if tensors is None:
        return None
    return (ctypes.c_void_p * len(tensors))(*[None if t is None else int(t.data_ptr()) for t in tensors])


def osdp_split_linear_fwd_mixed(X, w_shards, w_dp, ld_dp, Y, k, workspace, *, plan: Optional[Plan] = None,
                                op_index: int = 0, stream_compute=None, stream_copy=None):
    """Forward with every slice in its own mode: ``w_dp[j]`` is the replica of DP slice j (None for ZDP slices)."""
    T, I = X.shape
    O = Y.shape[1]
    shape = _shape(T, I, O, len(w_shards), k)
    pref, _keep = _plan_ref(plan)
    _check(lib.osdp_split_linear_fwd_mixed(ctypes.byref(shape), pref, op_index, int(X.data_ptr()), X.stride(0),
                                           _ptrs(w_shards), _opt_ptrs(w_dp), int(ld_dp), int(Y.data_ptr()), Y.stride(0),
                                           int(workspace.data_ptr()), workspace.numel() * workspace.element_size(),
                                           _stream(stream_compute), _stream(stream_copy)))


def osdp_split_linear_bwd_mixed(X, dY, w_shards, w_dp, ld_dp, dX, dw_shards, dw_dp, k, workspace, *,
                                plan: Optional[Plan] = None, op_index: int = 0, stream_compute=None, stream_copy=None):
    """Backward with every slice in its own mode: DP slices' gradients go to ``dw_dp[j]``, ZDP ones to the shards."""
    T, I = X.shape
    O = dY.shape[1]
    shape = _shape(T, I, O, len(w_shards), k)
    pref, _keep = _plan_ref(plan)
    _check(lib.osdp_split_linear_bwd_mixed(ctypes.byref(shape), pref, op_index, int(X.data_ptr()), X.stride(0),
                                           int(dY.data_ptr()), dY.stride(0), _ptrs(w_shards), _opt_ptrs(w_dp), int(ld_dp),
                                           int(dX.data_ptr()), dX.stride(0), _ptrs(dw_shards), _opt_ptrs(dw_dp),
                                           int(workspace.data_ptr()), workspace.numel() * workspace.element_size(),
                                           _stream(stream_compute), _stream(stream_copy)))


def osdp_granularity_candidates(T, I, O, N, k_list: Optional[Sequence[int]] = None):
    """The (k, staging mode, split dimension) combinations the kernels take for this shape, as a ctypes array."""
    shape = _shape(T, I, O, N, 0)
    ks = (ctypes.c_int32 * len(k_list))(*k_list) if k_list is not None else None
    nk = len(k_list) if k_list is not None else 0
    count = ctypes.c_int32()
    _check(lib.osdp_granularity_candidates(ctypes.byref(shape), ks, nk, None, 0, ctypes.byref(count)))
    out = (osdp_granularity_candidate * max(count.value, 1))()
    _check(lib.osdp_granularity_candidates(ctypes.byref(shape), ks, nk, out, count.value, ctypes.byref(count)))
    return (osdp_granularity_candidate * count.value).from_buffer(out) if count.value else \
        (osdp_granularity_candidate * 0)()


def osdp_granularity_measure(X, dY, w_shards, Y, dX, dw_shards, workspace, cands, *, warmup: int = 2, reps: int = 5,
                             stream_compute=None, stream_copy=None) -> None:
    """Times one forward + backward per candidate on the GPU and fills ``cands[i].ms``."""
    T, I = X.shape
    O = dY.shape[1]
    shape = _shape(T, I, O, len(w_shards), 0)
    _check(lib.osdp_granularity_measure(ctypes.byref(shape), int(X.data_ptr()), X.stride(0), int(dY.data_ptr()),
                                        dY.stride(0), _ptrs(w_shards), int(Y.data_ptr()), Y.stride(0),
                                        int(dX.data_ptr()), dX.stride(0), _ptrs(dw_shards),
                                        int(workspace.data_ptr()), workspace.numel() * workspace.element_size(),
                                        _stream(stream_compute), _stream(stream_copy), cands, len(cands), warmup, reps))


def osdp_granularity_select(cands, staging_budget: int = 0, workspace_budget: int = 0,
                            max_slowdown: float = 0.0) -> int:
    """Index of the candidate the selection rule picks."""
    chosen = ctypes.c_int32(-1)
    _check(lib.osdp_granularity_select(cands, len(cands), int(staging_budget), int(workspace_budget),
                                       float(max_slowdown), ctypes.byref(chosen)))
    return chosen.value


def _costs(ops):
    """ops: sequence of (m_model, m_act, m_extra, s_bytes, gamma)."""
    return (osdp_operator_cost * len(ops))(*[osdp_operator_cost(*map(float, o)) for o in ops])


def _device(N, alpha, beta, m_limit, b_max=0):
    return osdp_device_info(int(N), int(b_max), float(alpha), float(beta), float(m_limit))


def osdp_cost_model(ops, N, alpha, beta, m_limit, modes, b):
    """(M(p, b), T(p, b)) of Section 3.1 for the plan ``modes`` (0 = DP, 1 = ZDP per operator)."""
    mem, t = ctypes.c_double(), ctypes.c_double()
    dev = _device(N, alpha, beta, m_limit)
    m = (ctypes.c_uint8 * len(modes))(*modes)
    _check(lib.osdp_cost_model(_costs(ops), len(ops), ctypes.byref(dev), m, int(b), ctypes.byref(mem), ctypes.byref(t)))
    return mem.value, t.value


def osdp_plan_search(ops, N, alpha, beta, m_limit, b_max=0):
    """Algorithm 1.  Returns None when nothing fits, else dict(modes, b, time_per_sample, memory, ...)."""
    dev = _device(N, alpha, beta, m_limit, b_max)
    modes = (ctypes.c_uint8 * len(ops))()
    res = osdp_search_result()
    _check(lib.osdp_plan_search(_costs(ops), len(ops), ctypes.byref(dev), modes, ctypes.byref(res)))
    if not res.found:
        return None
    return dict(modes=list(modes), b=res.b, time_per_sample=res.time_per_sample, memory=res.memory,
                batch_sizes_tried=res.batch_sizes_tried, plans_visited=res.plans_visited, exact=bool(res.exact))


def osdp_debug_option(name: str, value: int) -> None:
    """Sets one of the library's process-wide test and debug switches (-1: back to the library's own choice)."""
    _check(lib.osdp_debug_option(name.encode(), int(value)))


def osdp_profile_begin(max_launches: int = 1 << 16) -> None:
    _check(lib.osdp_profile_begin(max_launches))


def osdp_profile_end():
    """Returns {kernel name: dict(launches, ms, flops, bytes)}."""
    stats = (osdp_kernel_stats * OSDP_KERNEL_KINDS)()
    _check(lib.osdp_profile_end(stats))
    return {KERNEL_NAMES[i]: dict(launches=stats[i].launches, ms=stats[i].ms, flops=stats[i].flops,
                                  bytes=stats[i].bytes) for i in range(OSDP_KERNEL_KINDS)}


def osdp_profile_overlap():
    """After osdp_profile_end: dict(span_ms, idle_ms, gather_exposed_ms) of the profiled region."""
    span, idle, exposed = ctypes.c_double(), ctypes.c_double(), ctypes.c_double()
    _check(lib.osdp_profile_overlap(ctypes.byref(span), ctypes.byref(idle), ctypes.byref(exposed)))
    return dict(span_ms=span.value, idle_ms=idle.value, gather_exposed_ms=exposed.value)
