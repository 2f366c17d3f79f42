"""CPU oracle for the operator-split linear layer (arXiv 2209.13258, Section 3.3).

TEST INFRASTRUCTURE ONLY: imported by tests, the smoke check and the bench's
cpu_baseline leg.  The GPU package never imports this module and this module
never imports the GPU package.

The arithmetic lives in ``osdp_oracle.c`` (plain C, fp64, textbook loops);
this file builds it with gcc and marshals numpy arrays into it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "osdp_oracle.c"
_LIB = _HERE / "libosdp_oracle.so"
_lib = None

_i64 = ctypes.c_int64
_p = ctypes.c_void_p


def build(force: bool = False) -> Path:
    """Compile the C oracle into ``oracle/libosdp_oracle.so`` with gcc."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        tmp = _LIB.with_suffix(f".so.tmp{os.getpid()}")
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-fvisibility=hidden",
               "-std=c11", "-Wall", "-Wextra", "-o", str(tmp), str(_SRC)]
        subprocess.run(cmd, check=True)
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        # OSDP_ORACLE_LIB: another build of osdp_oracle.c (the mutation test loads deliberately broken ones)
        override = os.environ.get("OSDP_ORACLE_LIB")
        if not override:
            build()
        lib = ctypes.CDLL(override or str(_LIB))
        lib.osdp_oracle_bf16_to_f64.restype = ctypes.c_double
        lib.osdp_oracle_bf16_to_f64.argtypes = [ctypes.c_uint16]
        lib.osdp_oracle_threads.restype = ctypes.c_int
        lib.osdp_oracle_weight_bytes.restype = _i64
        lib.osdp_oracle_weight_bytes.argtypes = [_i64] * 3
        lib.osdp_oracle_slice_range.restype = None
        lib.osdp_oracle_slice_range.argtypes = [_i64, _i64, _i64, _p, _p]
        lib.osdp_oracle_peak_staging_bytes.restype = _i64
        lib.osdp_oracle_peak_staging_bytes.argtypes = [_i64] * 5
        lib.osdp_oracle_shard_len.restype = _i64
        lib.osdp_oracle_shard_len.argtypes = [_i64] * 3
        lib.osdp_oracle_locate.restype = None
        lib.osdp_oracle_locate.argtypes = [_i64] * 5 + [_p, _p]
        lib.osdp_oracle_assemble.restype = None
        lib.osdp_oracle_assemble.argtypes = [_i64] * 3 + [_p, _p]
        lib.osdp_oracle_shard.restype = None
        lib.osdp_oracle_shard.argtypes = [_i64] * 3 + [_p, _p]
        lib.osdp_oracle_gather_slice.restype = None
        lib.osdp_oracle_gather_slice.argtypes = [_i64] * 5 + [_p, _p]
        lib.osdp_oracle_matmul_fwd.restype = None
        lib.osdp_oracle_matmul_fwd.argtypes = [_i64, _i64, _i64, _p, _i64, _p, _i64, _p]
        lib.osdp_oracle_matmul_dx.restype = None
        lib.osdp_oracle_matmul_dx.argtypes = [_i64, _i64, _i64, _p, _i64, _p, _i64, _p]
        lib.osdp_oracle_matmul_dw.restype = None
        lib.osdp_oracle_matmul_dw.argtypes = [_i64, _i64, _i64, _p, _i64, _p, _i64, _p]
        lib.osdp_oracle_linear.restype = ctypes.c_int
        lib.osdp_oracle_linear.argtypes = [_i64] * 4 + [_p] * 6
        lib.osdp_oracle_split_fwd.restype = ctypes.c_int
        lib.osdp_oracle_split_fwd.argtypes = [_i64] * 5 + [_p] * 4
        lib.osdp_oracle_split_bwd.restype = ctypes.c_int
        lib.osdp_oracle_split_bwd.argtypes = [_i64] * 5 + [_p] * 6
        lib.osdp_oracle_row_slice_range.restype = None
        lib.osdp_oracle_row_slice_range.argtypes = [_i64, _i64, _i64, _p, _p]
        lib.osdp_oracle_gather_row_slice.restype = None
        lib.osdp_oracle_gather_row_slice.argtypes = [_i64] * 5 + [_p, _p]
        lib.osdp_oracle_peak_staging_bytes_rows.restype = _i64
        lib.osdp_oracle_peak_staging_bytes_rows.argtypes = [_i64] * 5
        lib.osdp_oracle_split_fwd_rows.restype = ctypes.c_int
        lib.osdp_oracle_split_fwd_rows.argtypes = [_i64] * 5 + [_p] * 4
        lib.osdp_oracle_split_bwd_rows.restype = ctypes.c_int
        lib.osdp_oracle_split_bwd_rows.argtypes = [_i64] * 5 + [_p] * 6
        lib.osdp_oracle_split_fwd_mixed.restype = ctypes.c_int
        lib.osdp_oracle_split_fwd_mixed.argtypes = [_i64] * 5 + [ctypes.c_int, ctypes.c_uint64, _p, _p, _p, _i64, _p, _p]
        lib.osdp_oracle_split_bwd_mixed.restype = ctypes.c_int
        lib.osdp_oracle_split_bwd_mixed.argtypes = [_i64] * 5 + [ctypes.c_int, ctypes.c_uint64, _p, _p, _p, _p, _i64,
                                                                 _p, _p, _p, _p]
        lib.osdp_oracle_sample_y.restype = None
        lib.osdp_oracle_sample_y.argtypes = [_i64] * 4 + [_p, _p, _i64, _p, _p, _p]
        lib.osdp_oracle_sample_dx.restype = None
        lib.osdp_oracle_sample_dx.argtypes = [_i64] * 4 + [_p, _p, _i64, _p, _p, _p]
        lib.osdp_oracle_sample_dw.restype = None
        lib.osdp_oracle_sample_dw.argtypes = [_i64] * 3 + [_p, _p, _i64, _p, _p, _p]
        _lib = lib
    return _lib


# ---------------------------------------------------------------- marshalling
def _u16(a, shape=None) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.uint16)
    if shape is not None and a.shape != tuple(shape):
        raise ValueError(f"expected shape {tuple(shape)}, got {a.shape}")
    return a


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _ptr_array(arrs):
    return (ctypes.c_void_p * len(arrs))(*[a.ctypes.data for a in arrs])


def _check_shards(shards, I, O, N):
    L = shard_len(I, O, N)
    if len(shards) != N:
        raise ValueError(f"expected {N} shards, got {len(shards)}")
    out = [_u16(s).reshape(-1) for s in shards]
    for s in out:
        if s.size != L:
            raise ValueError(f"each shard must hold {L} elements, got {s.size}")
    return out


# ------------------------------------------------------------------ scalars
def threads() -> int:
    """Number of host threads the oracle's loops run on."""
    return int(_load().osdp_oracle_threads())


def bf16_to_f64(bits) -> np.ndarray:
    """Widen bf16 bit patterns exactly to float64 (scalar loop through the C routine)."""
    lib = _load()
    bits = np.asarray(bits, dtype=np.uint16)
    flat = [lib.osdp_oracle_bf16_to_f64(int(b)) for b in bits.reshape(-1)]
    return np.array(flat, dtype=np.float64).reshape(bits.shape)


def weight_bytes(I: int, O: int, elem_bytes: int) -> int:
    """Gathered size of one MatMul's weight (Section 3.3)."""
    return int(_load().osdp_oracle_weight_bytes(I, O, elem_bytes))


def slice_range(O: int, k: int, j: int):
    """Column range [c0, c1) of slice j of k (k = 0 means unsplit)."""
    c0, c1 = _i64(), _i64()
    _load().osdp_oracle_slice_range(O, k, j, ctypes.byref(c0), ctypes.byref(c1))
    return int(c0.value), int(c1.value)


def peak_staging_bytes(I: int, O: int, k: int, slots: int = 1, elem_bytes: int = 2) -> int:
    """Peak gathered-weight bytes with ``slots`` slices live (Section 3.3 law for slots=1)."""
    return int(_load().osdp_oracle_peak_staging_bytes(I, O, k, slots, elem_bytes))


def shard_len(I: int, O: int, N: int) -> int:
    return int(_load().osdp_oracle_shard_len(I, O, N))


def locate(I: int, O: int, N: int, r: int, c: int):
    """(shard, offset) of W[r, c] in the shard-major layout."""
    s, off = _i64(), _i64()
    _load().osdp_oracle_locate(I, O, N, r, c, ctypes.byref(s), ctypes.byref(off))
    return int(s.value), int(off.value)


# ------------------------------------------------------------------- layout
def shard(W, N: int):
    """Cut dense W[I x O] (bf16 bits) into N shards of ceil(I*O/N) elements."""
    W = _u16(W)
    I, O = W.shape
    L = shard_len(I, O, N)
    shards = [np.empty(L, dtype=np.uint16) for _ in range(N)]
    _load().osdp_oracle_shard(I, O, N, _ptr(W), _ptr_array(shards))
    return shards


def assemble(shards, I: int, O: int):
    """Dense W[I x O] from its shards."""
    N = len(shards)
    sh = _check_shards(shards, I, O, N)
    W = np.empty((I, O), dtype=np.uint16)
    _load().osdp_oracle_assemble(I, O, N, _ptr_array(sh), _ptr(W))
    return W


def gather_slice(shards, I: int, O: int, k: int, j: int):
    """Column slice j of k, dense row-major [I x w_j] bf16 bits."""
    N = len(shards)
    sh = _check_shards(shards, I, O, N)
    c0, c1 = slice_range(O, k, j)
    Ws = np.empty((I, c1 - c0), dtype=np.uint16)
    _load().osdp_oracle_gather_slice(I, O, N, k, j, _ptr_array(sh), _ptr(Ws))
    return Ws


# --------------------------------------------------------- definition route
def matmul_fwd(X, W):
    X, W = _u16(X), _u16(W)
    T, I = X.shape
    I2, O = W.shape
    assert I == I2
    Y = np.empty((T, O), dtype=np.float64)
    _load().osdp_oracle_matmul_fwd(T, I, O, _ptr(X), I, _ptr(W), O, _ptr(Y))
    return Y


def matmul_dx(dY, W):
    dY, W = _u16(dY), _u16(W)
    T, O = dY.shape
    I, O2 = W.shape
    assert O == O2
    dX = np.empty((T, I), dtype=np.float64)
    _load().osdp_oracle_matmul_dx(T, I, O, _ptr(dY), O, _ptr(W), O, _ptr(dX))
    return dX


def matmul_dw(X, dY):
    X, dY = _u16(X), _u16(dY)
    T, I = X.shape
    T2, O = dY.shape
    assert T == T2
    dW = np.empty((I, O), dtype=np.float64)
    _load().osdp_oracle_matmul_dw(T, I, O, _ptr(X), I, _ptr(dY), O, _ptr(dW))
    return dW


def linear(X, shards, O: int, dY=None, want=("Y", "dX", "dW")):
    """Unsplit operator from shards: dict with fp64 Y [T x O], dX [T x I], dW [I x O]."""
    X = _u16(X)
    T, I = X.shape
    N = len(shards)
    sh = _check_shards(shards, I, O, N)
    out = {}
    Y = np.empty((T, O)) if "Y" in want else None
    dX = np.empty((T, I)) if "dX" in want else None
    dW = np.empty((I, O)) if "dW" in want else None
    if (dX is not None or dW is not None):
        dY = _u16(dY, (T, O))
    rc = _load().osdp_oracle_linear(
        T, I, O, N, _ptr(X), _ptr(dY) if dY is not None else None, _ptr_array(sh),
        _ptr(Y) if Y is not None else None, _ptr(dX) if dX is not None else None,
        _ptr(dW) if dW is not None else None)
    if rc != 0:
        raise MemoryError("oracle allocation failed")
    if Y is not None:
        out["Y"] = Y
    if dX is not None:
        out["dX"] = dX
    if dW is not None:
        out["dW"] = dW
    return out


# -------------------------------------------------------------- split route
def split_fwd(X, shards, O: int, k: int):
    """Split forward: returns (Y fp64 [T x O], peak live staging bytes)."""
    X = _u16(X)
    T, I = X.shape
    N = len(shards)
    sh = _check_shards(shards, I, O, N)
    Y = np.empty((T, O), dtype=np.float64)
    peak = _i64()
    rc = _load().osdp_oracle_split_fwd(T, I, O, N, k, _ptr(X), _ptr_array(sh), _ptr(Y),
                                       ctypes.byref(peak))
    if rc != 0:
        raise MemoryError("oracle allocation failed")
    return Y, int(peak.value)


def split_bwd(X, dY, shards, O: int, k: int):
    """Split backward: returns (dX fp64 [T x I], dW shards (list of N fp64 arrays), peak bytes)."""
    X = _u16(X)
    T, I = X.shape
    dY = _u16(dY, (T, O))
    N = len(shards)
    sh = _check_shards(shards, I, O, N)
    L = shard_len(I, O, N)
    dX = np.empty((T, I), dtype=np.float64)
    dW = [np.zeros(L, dtype=np.float64) for _ in range(N)]
    peak = _i64()
    rc = _load().osdp_oracle_split_bwd(T, I, O, N, k, _ptr(X), _ptr(dY), _ptr_array(sh), _ptr(dX),
                                       _ptr_array(dW), ctypes.byref(peak))
    if rc != 0:
        raise MemoryError("oracle allocation failed")
    return dX, dW, int(peak.value)


def dense_from_f64_shards(dW_shards, I: int, O: int):
    """Dense [I x O] fp64 view of a shard-major fp64 gradient (drops the padding)."""
    flat = np.concatenate([np.asarray(s, dtype=np.float64).reshape(-1) for s in dW_shards])
    return flat[: I * O].reshape(I, O)


# ------------------------------------- split route along the reduction dimension
def row_slice_range(I: int, k: int, j: int):
    """Row range [r0, r1) of W (= column range of X) of slice j of k when the reduction dimension is split."""
    r0, r1 = _i64(), _i64()
    _load().osdp_oracle_row_slice_range(I, k, j, ctypes.byref(r0), ctypes.byref(r1))
    return int(r0.value), int(r1.value)


def gather_row_slice(shards, I: int, O: int, k: int, j: int):
    """Row slice j of k, dense row-major [w_j x O] bf16 bits."""
    N = len(shards)
    sh = _check_shards(shards, I, O, N)
    r0, r1 = row_slice_range(I, k, j)
    Ws = np.empty((r1 - r0, O), dtype=np.uint16)
    _load().osdp_oracle_gather_row_slice(I, O, N, k, j, _ptr_array(sh), _ptr(Ws))
    return Ws


def peak_staging_bytes_rows(I: int, O: int, k: int, slots: int = 1, elem_bytes: int = 2) -> int:
    return int(_load().osdp_oracle_peak_staging_bytes_rows(I, O, k, slots, elem_bytes))


def split_fwd_rows(X, shards, O: int, k: int):
    """Forward with the reduction dimension split (Section 3.3 as printed): (Y fp64, peak staging bytes)."""
    X = _u16(X)
    T, I = X.shape
    N = len(shards)
    sh = _check_shards(shards, I, O, N)
    Y = np.empty((T, O), dtype=np.float64)
    peak = _i64()
    rc = _load().osdp_oracle_split_fwd_rows(T, I, O, N, k, _ptr(X), _ptr_array(sh), _ptr(Y), ctypes.byref(peak))
    if rc != 0:
        raise MemoryError("oracle allocation failed")
    return Y, int(peak.value)


def split_bwd_rows(X, dY, shards, O: int, k: int):
    """Backward with the reduction dimension split: (dX fp64, dW shards fp64, peak staging bytes)."""
    X = _u16(X)
    T, I = X.shape
    dY = _u16(dY, (T, O))
    N = len(shards)
    sh = _check_shards(shards, I, O, N)
    L = shard_len(I, O, N)
    dX = np.empty((T, I), dtype=np.float64)
    dW = [np.zeros(L, dtype=np.float64) for _ in range(N)]
    peak = _i64()
    rc = _load().osdp_oracle_split_bwd_rows(T, I, O, N, k, _ptr(X), _ptr(dY), _ptr_array(sh), _ptr(dX),
                                            _ptr_array(dW), ctypes.byref(peak))
    if rc != 0:
        raise MemoryError("oracle allocation failed")
    return dX, dW, int(peak.value)


# ------------------------------------------------------ slices in DP or ZDP mode
def _dp_pointers(w_dp, k, zdp_mask, rows_needed, cols_needed, ld_dp):
    """ctypes array of k weight pointers; a DP slice must cover (rows - 1) * ld + cols elements."""
    keep, ptrs = [], []
    for j in range(k):
        if (zdp_mask >> j) & 1:
            ptrs.append(None)        # never looked at
            continue
        a = np.ascontiguousarray(w_dp[j], dtype=np.uint16).reshape(-1)
        need = (rows_needed[j] - 1) * ld_dp + cols_needed[j]
        if a.size < need:
            raise ValueError(f"DP slice {j} holds {a.size} elements, {need} needed")
        keep.append(a)
        ptrs.append(a.ctypes.data)
    return (ctypes.c_void_p * k)(*ptrs), keep


def _slice_shapes(I, O, k, rows):
    keff = max(k, 1)
    rng = [row_slice_range(I, k, j) if rows else slice_range(O, k, j) for j in range(keff)]
    sr = [(b - a) if rows else I for a, b in rng]
    sc = [O if rows else (b - a) for a, b in rng]
    return keff, sr, sc


def split_fwd_mixed(X, shards, O: int, k: int, zdp_mask: int, w_dp, ld_dp: int, rows: bool = False):
    """Forward with every slice in its own mode (Section 3.3, last paragraph): bit j of zdp_mask set = slice j is
    gathered from the shards, clear = slice j is read where it lies in w_dp[j] (leading dimension ld_dp).
    Returns (Y fp64, peak staging bytes)."""
    X = _u16(X)
    T, I = X.shape
    N = len(shards)
    sh = _check_shards(shards, I, O, N)
    keff, sr, sc = _slice_shapes(I, O, k, rows)
    ptrs, keep = _dp_pointers(w_dp, keff, zdp_mask, sr, sc, ld_dp)
    Y = np.empty((T, O), dtype=np.float64)
    peak = _i64()
    rc = _load().osdp_oracle_split_fwd_mixed(T, I, O, N, k, int(rows), zdp_mask, _ptr(X), _ptr_array(sh), ptrs, ld_dp,
                                             _ptr(Y), ctypes.byref(peak))
    if rc != 0:
        raise MemoryError("oracle allocation failed")
    del keep
    return Y, int(peak.value)


def split_bwd_mixed(X, dY, shards, O: int, k: int, zdp_mask: int, w_dp, ld_dp: int, rows: bool = False):
    """Backward with every slice in its own mode.  Returns (dX fp64, dW shards fp64 with NaN wherever no ZDP slice
    wrote, list of per-slice DP gradients [slice rows x ld_dp] fp64 (None for ZDP slices; NaN outside the slice's
    columns), peak staging bytes)."""
    X = _u16(X)
    T, I = X.shape
    dY = _u16(dY, (T, O))
    N = len(shards)
    sh = _check_shards(shards, I, O, N)
    L = shard_len(I, O, N)
    keff, sr, sc = _slice_shapes(I, O, k, rows)
    ptrs, keep = _dp_pointers(w_dp, keff, zdp_mask, sr, sc, ld_dp)
    dX = np.empty((T, I), dtype=np.float64)
    dW = [np.full(L, np.nan, dtype=np.float64) for _ in range(N)]
    dw_dp = [None if (zdp_mask >> j) & 1 else np.full((sr[j], ld_dp), np.nan, dtype=np.float64) for j in range(keff)]
    dptrs = (ctypes.c_void_p * keff)(*[None if a is None else a.ctypes.data for a in dw_dp])
    peak = _i64()
    rc = _load().osdp_oracle_split_bwd_mixed(T, I, O, N, k, int(rows), zdp_mask, _ptr(X), _ptr(dY), _ptr_array(sh), ptrs,
                                             ld_dp, _ptr(dX), _ptr_array(dW), dptrs, ctypes.byref(peak))
    if rc != 0:
        raise MemoryError("oracle allocation failed")
    del keep
    return dX, dW, dw_dp, int(peak.value)


# ------------------------------------------------ choice of the slice granularity
def granularity_select(table, staging_budget: int = 0, workspace_budget: int = 0, max_slowdown: float = 0.0):
    """The rule by which a granularity is picked from measured candidates (Section 4.3 leaves the choice open;
    its discussion asks for the memory footprint to be reduced as far as the time cost stays acceptable).

    ``table`` is a sequence of (peak_weight_staging bytes, workspace bytes, milliseconds); an entry with
    milliseconds <= 0 has not been measured.  A budget of 0 means no limit.  Returns the index of the chosen
    entry, or None when nothing fits: of the entries that fit both budgets, those no slower than
    (1 + max_slowdown) times the fastest are kept, and the one with the least gathered weight wins
    (then the faster, then the earlier one).
    """
    fits = []
    for i, (peak, ws, ms) in enumerate(table):
        if ms <= 0:
            continue
        if staging_budget and peak > staging_budget:
            continue
        if workspace_budget and ws > workspace_budget:
            continue
        fits.append(i)
    if not fits:
        return None
    fastest = min(table[i][2] for i in fits)
    keep = [i for i in fits if table[i][2] <= (1.0 + max_slowdown) * fastest]
    keep.sort(key=lambda i: (table[i][0], table[i][2], i))
    return keep[0]


# --------------------------------------------- cost model and plan search (Section 3)
def cost_model(ops, N: int, alpha: float, beta: float, modes, b: int):
    """Memory and time of one execution plan (Section 3.1).  ops: (M_model, M_act, M_extra, S, gamma) per operator;
    modes[i]: 0 = DP, 1 = ZDP.  Returns (M(p, b), T(p, b)) with T the time per sample, (1/b) * sum_i T_i."""
    mem, time = 0.0, 0.0
    for (m_model, m_act, m_extra, s, gamma), zdp in zip(ops, modes):
        mem = mem + ((m_model / N if zdp else m_model) + (b * m_act + m_extra))
        steps = (3.0 if zdp else 2.0) * (N - 1)
        time = time + (steps * (alpha + s / N * beta) + b * gamma)
    return mem, time / b


def plan_search(ops, N: int, alpha: float, beta: float, m_limit: float, b_max: int = 0):
    """Algorithm 1 by exhaustive enumeration: for b = 1, 2, ... every plan of {DP, ZDP}^n is costed, the fastest one
    within the memory limit is kept (the first in enumeration order among equals: operator 0 varies slowest, DP before
    ZDP), the loop ends at the first b with no feasible plan, and the best (plan, b) over all b by time per sample is
    returned (the smaller b among equals) as dict(modes, b, time_per_sample, memory), or None."""
    n = len(ops)
    best = None
    b = 1
    while b <= (b_max if b_max > 0 else 65536):
        # every plan at once, one operator after the other so that each plan's sums run left to right
        bits = (np.arange(1 << n, dtype=np.int64)[:, None] >> np.arange(n - 1, -1, -1, dtype=np.int64)[None, :]) & 1
        mem = np.zeros(1 << n)
        time = np.zeros(1 << n)
        for i, (m_model, m_act, m_extra, s, gamma) in enumerate(ops):
            rest = b * m_act + m_extra
            step = alpha + s / N * beta
            mem = mem + np.where(bits[:, i] == 1, m_model / N + rest, m_model + rest)
            time = time + np.where(bits[:, i] == 1, 3.0 * (N - 1) * step + b * gamma, 2.0 * (N - 1) * step + b * gamma)
        ok = mem <= m_limit
        if not ok.any():
            break
        time = np.where(ok, time, np.inf)
        p = int(np.argmin(time))            # numpy returns the first of equal minima
        per_sample = time[p] / b
        if best is None or per_sample < best["time_per_sample"]:
            best = dict(modes=[int(v) for v in bits[p]], b=b, time_per_sample=float(per_sample), memory=float(mem[p]))
        b += 1
    return best


# ------------------------------------------------------------ sampled entries
def _idx(a):
    return np.ascontiguousarray(a, dtype=np.int64)


def sample_y(X, shards, O: int, rows, cols):
    X = _u16(X)
    T, I = X.shape
    N = len(shards)
    sh = _check_shards(shards, I, O, N)
    rows, cols = _idx(rows), _idx(cols)
    out = np.empty(rows.size, dtype=np.float64)
    _load().osdp_oracle_sample_y(T, I, O, N, _ptr(X), _ptr_array(sh), rows.size, _ptr(rows),
                                 _ptr(cols), _ptr(out))
    return out


def sample_dx(dY, shards, I: int, rows, cols):
    dY = _u16(dY)
    T, O = dY.shape
    N = len(shards)
    sh = _check_shards(shards, I, O, N)
    rows, cols = _idx(rows), _idx(cols)
    out = np.empty(rows.size, dtype=np.float64)
    _load().osdp_oracle_sample_dx(T, I, O, N, _ptr(dY), _ptr_array(sh), rows.size, _ptr(rows),
                                  _ptr(cols), _ptr(out))
    return out


def sample_dw(X, dY, rows, cols):
    X, dY = _u16(X), _u16(dY)
    T, I = X.shape
    T2, O = dY.shape
    assert T == T2
    rows, cols = _idx(rows), _idx(cols)
    out = np.empty(rows.size, dtype=np.float64)
    _load().osdp_oracle_sample_dw(T, I, O, _ptr(X), _ptr(dY), rows.size, _ptr(rows), _ptr(cols),
                                  _ptr(out))
    return out
