"""ctypes front end of the CPU oracle (tbe_oracle.c).  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg import this package; the product
path never does.  Arrays are numpy; tables are a list with one [R_t, D_t] array per table
(float32, or uint16 holding IEEE binary16 bit patterns / numpy float16).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tbe_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

F32, F16 = 0, 1
SUM, MEAN = 0, 1
IO_F32, IO_F16, IO_BF16 = 0, 1, 2     # element type of the pooled output / upstream gradient matrix
_IO = {"f32": IO_F32, "f16": IO_F16, "bf16": IO_BF16}


def build(force: bool = False) -> str:
    """Compile tbe_oracle.c with gcc (no fast-math: fp64 semantics must stay IEEE)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fno-fast-math", "-Wall", "-Wextra",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        i64p, i32p, f32p, f64p = (ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_int32),
                                  ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_double))
        vpp = ctypes.POINTER(ctypes.c_void_p)
        L.oracle_half_to_double.restype = ctypes.c_double
        L.oracle_half_to_double.argtypes = [ctypes.c_uint16]
        L.oracle_double_to_half.restype = ctypes.c_uint16
        L.oracle_double_to_half.argtypes = [ctypes.c_double]
        L.oracle_bf16_to_double.restype = ctypes.c_double
        L.oracle_bf16_to_double.argtypes = [ctypes.c_uint16]
        L.oracle_double_to_bf16.restype = ctypes.c_uint16
        L.oracle_double_to_bf16.argtypes = [ctypes.c_double]
        L.oracle_forward_io.restype = ctypes.c_int
        L.oracle_forward_io.argtypes = [ctypes.c_int32, i64p, i32p, ctypes.c_int, vpp, i64p, i64p, ctypes.c_int32,
                                        ctypes.c_int, ctypes.c_void_p, ctypes.c_int]
        L.oracle_backward_rowwise_adagrad_io.restype = ctypes.c_int64
        L.oracle_backward_rowwise_adagrad_io.argtypes = [ctypes.c_int32, i64p, i32p, ctypes.c_int, vpp, f32p,
                                                         ctypes.c_void_p, ctypes.c_int, i64p, i64p, ctypes.c_int32,
                                                         ctypes.c_int, ctypes.c_double, ctypes.c_double, ctypes.c_double,
                                                         i64p, i64p, i64p, i64p]
        L.oracle_lookup_seq_io.restype = ctypes.c_int
        L.oracle_lookup_seq_io.argtypes = [ctypes.c_int32, i64p, i32p, ctypes.c_int, vpp, i64p, i64p, ctypes.c_void_p,
                                           ctypes.c_int]
        L.oracle_backward_seq_io.restype = ctypes.c_int64
        L.oracle_backward_seq_io.argtypes = [ctypes.c_int32, i64p, i32p, ctypes.c_int, vpp, f32p, ctypes.c_void_p,
                                             ctypes.c_int, i64p, i64p, ctypes.c_double, ctypes.c_double, ctypes.c_double]
        L.oracle_replica_mean.restype = None
        L.oracle_replica_mean.argtypes = [vpp, ctypes.c_int32, ctypes.c_int64, ctypes.c_int]
        L.oracle_forward_bag.restype = ctypes.c_int
        L.oracle_forward_bag.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_int32, i64p,
                                         ctypes.c_int64, ctypes.c_int64, ctypes.c_int, f32p]
        L.oracle_forward.restype = ctypes.c_int
        L.oracle_forward.argtypes = [ctypes.c_int32, i64p, i32p, ctypes.c_int, vpp, i64p, i64p, ctypes.c_int32,
                                     ctypes.c_int, f32p]
        L.oracle_linearize.restype = ctypes.c_int
        L.oracle_linearize.argtypes = [ctypes.c_int32, i64p, i64p, i64p, ctypes.c_int32, i64p, i64p]
        L.oracle_stable_sort.restype = None
        L.oracle_stable_sort.argtypes = [i64p, ctypes.c_int64, i64p, i64p]
        L.oracle_run_lengths.restype = ctypes.c_int64
        L.oracle_run_lengths.argtypes = [i64p, ctypes.c_int64, i64p, i64p]
        L.oracle_adagrad_row.restype = None
        L.oracle_adagrad_row.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_int32, f32p, f64p,
                                         ctypes.c_double, ctypes.c_double, ctypes.c_double]
        L.oracle_row_gradient_by_scan.restype = ctypes.c_int64
        L.oracle_row_gradient_by_scan.argtypes = [ctypes.c_int32, ctypes.c_int64, ctypes.c_int32, ctypes.c_int64,
                                                  ctypes.c_int64, f32p, i64p, i64p, ctypes.c_int32, ctypes.c_int, f64p]
        L.oracle_backward_rowwise_adagrad.restype = ctypes.c_int64
        L.oracle_backward_rowwise_adagrad.argtypes = [ctypes.c_int32, i64p, i32p, ctypes.c_int, vpp, f32p, f32p, i64p,
                                                      i64p, ctypes.c_int32, ctypes.c_int, ctypes.c_double,
                                                      ctypes.c_double, ctypes.c_double, i64p, i64p, i64p, i64p]
        _lib = L
    return _lib


# ---- marshalling helpers ---------------------------------------------------------------------
def _p(a: np.ndarray, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct))


def _i64(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a), dtype=np.int64)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a), dtype=np.int32)


def _pooling(p) -> int:
    return {"sum": SUM, "mean": MEAN, SUM: SUM, MEAN: MEAN}[p]


def _tables(tables: Sequence[np.ndarray]):
    """Returns (dtype code, rows, D, void*[T]); every table must be C-contiguous [R_t, D_t]."""
    dt = None
    rows, D, ptrs = [], [], []
    for a in tables:
        assert a.ndim == 2 and a.flags["C_CONTIGUOUS"]
        if a.dtype == np.float32:
            code = F32
        elif a.dtype in (np.float16, np.uint16):
            code = F16
        else:
            raise TypeError(a.dtype)
        assert dt is None or dt == code
        dt = code
        rows.append(a.shape[0])
        D.append(a.shape[1])
        ptrs.append(a.ctypes.data)
    arr = (ctypes.c_void_p * len(ptrs))(*ptrs)
    return dt, _i64(rows), _i32(D), arr


# ---- API ---------------------------------------------------------------------------------------
def half_to_double(bits: int) -> float:
    return lib().oracle_half_to_double(int(bits))


def double_to_half(x: float) -> int:
    return lib().oracle_double_to_half(float(x))


def bf16_to_double(bits: int) -> float:
    return lib().oracle_bf16_to_double(int(bits))


def double_to_bf16(x: float) -> int:
    return lib().oracle_double_to_bf16(float(x))


def forward(tables: Sequence[np.ndarray], indices, offsets, B: int, pooling="sum", out_dtype="f32") -> np.ndarray:
    """Pooled activations [B, sum(D)]: float32, float16, or uint16 holding bfloat16 bit patterns (out_dtype
    "f32" | "f16" | "bf16"); each value is rounded once from the fp64 sum."""
    dt, rows, D, ptrs = _tables(tables)
    indices, offsets = _i64(indices), _i64(offsets)
    assert offsets.shape[0] == len(tables) * B + 1 and offsets[-1] == indices.shape[0]
    np_dt = {"f32": np.float32, "f16": np.float16, "bf16": np.uint16}[out_dtype]
    out = np.zeros((B, int(D.sum())), dtype=np_dt)
    rc = lib().oracle_forward_io(len(tables), _p(rows, ctypes.c_int64), _p(D, ctypes.c_int32), dt, ptrs,
                                 _p(indices, ctypes.c_int64), _p(offsets, ctypes.c_int64), B, _pooling(pooling),
                                 out.ctypes.data, _IO[out_dtype])
    if rc:
        raise IndexError("id outside its table")
    return out


def forward_bag(table: np.ndarray, indices, start: int, end: int, pooling="sum") -> np.ndarray:
    """One bag of one table: float32 [D]."""
    dt, rows, D, _ = _tables([table])
    indices = _i64(indices)
    out = np.zeros(int(D[0]), dtype=np.float32)
    rc = lib().oracle_forward_bag(table.ctypes.data, dt, int(rows[0]), int(D[0]), _p(indices, ctypes.c_int64),
                                  int(start), int(end), _pooling(pooling), _p(out, ctypes.c_float))
    if rc:
        raise IndexError("id outside its table")
    return out


def linearize(rows, indices, offsets, B: int):
    """(keys[N], bag_of[N]) int64."""
    rows, indices, offsets = _i64(rows), _i64(indices), _i64(offsets)
    N = indices.shape[0]
    keys = np.zeros(N, dtype=np.int64)
    bag_of = np.zeros(N, dtype=np.int64)
    rc = lib().oracle_linearize(len(rows), _p(rows, ctypes.c_int64), _p(indices, ctypes.c_int64),
                                _p(offsets, ctypes.c_int64), B, _p(keys, ctypes.c_int64), _p(bag_of, ctypes.c_int64))
    if rc:
        raise IndexError("id outside its table")
    return keys, bag_of


def stable_sort(keys):
    """(keys_sorted[N], order[N]) int64; order is the unique stable ascending permutation."""
    keys = _i64(keys)
    N = keys.shape[0]
    ks = np.zeros(N, dtype=np.int64)
    order = np.zeros(N, dtype=np.int64)
    lib().oracle_stable_sort(_p(keys, ctypes.c_int64), N, _p(ks, ctypes.c_int64), _p(order, ctypes.c_int64))
    return ks, order


def run_lengths(keys_sorted):
    """(unique_rows[U], seg_start[U+1]) int64."""
    ks = _i64(keys_sorted)
    N = ks.shape[0]
    uniq = np.zeros(max(N, 1), dtype=np.int64)
    seg = np.zeros(N + 1, dtype=np.int64)
    U = lib().oracle_run_lengths(_p(ks, ctypes.c_int64), N, _p(uniq, ctypes.c_int64), _p(seg, ctypes.c_int64))
    return uniq[:U].copy(), seg[:U + 1].copy()


def adagrad_row(table: np.ndarray, r: int, v: np.ndarray, g, lr: float, eps: float, c: float) -> None:
    """In place: one moment-scaled row-wise AdaGrad step on row r of `table`; v is a 1-element float32 array."""
    dt, rows, D, _ = _tables([table])
    g = np.ascontiguousarray(g, dtype=np.float64)
    assert g.shape == (int(D[0]),) and v.dtype == np.float32 and v.size == 1
    lib().oracle_adagrad_row(table.ctypes.data, dt, int(r), int(D[0]), _p(v, ctypes.c_float),
                             _p(g, ctypes.c_double), float(lr), float(eps), float(c))


def row_gradient_by_scan(t: int, r: int, D_t: int, doff: int, grad_out: np.ndarray, indices, offsets, B: int,
                         pooling="sum"):
    """(g[D_t] float64, hits): the row gradient from its definition, by scanning table t's positions."""
    assert grad_out.dtype == np.float32 and grad_out.flags["C_CONTIGUOUS"] and grad_out.shape[0] == B
    indices, offsets = _i64(indices), _i64(offsets)
    g = np.zeros(D_t, dtype=np.float64)
    hits = lib().oracle_row_gradient_by_scan(int(t), int(r), int(D_t), int(doff), int(grad_out.shape[1]),
                                             _p(grad_out, ctypes.c_float), _p(indices, ctypes.c_int64),
                                             _p(offsets, ctypes.c_int64), B, _pooling(pooling), _p(g, ctypes.c_double))
    return g, int(hits)


class BackwardResult:
    __slots__ = ("U", "keys_sorted", "order", "unique_rows", "seg_start")


def backward_rowwise_adagrad(tables: List[np.ndarray], state: np.ndarray, grad_out: np.ndarray, indices, offsets,
                             B: int, pooling="sum", lr: float = 0.01, eps: float = 1e-8, c: float = 1.0,
                             want_indices: bool = True, grad_dtype: str = "f32") -> BackwardResult:
    """In place on `tables` and `state`.  Returns the exact integer by-products of the sorted formulation.
    grad_out is float32, float16, or uint16 holding bfloat16 bit patterns (grad_dtype "f32" | "f16" | "bf16")."""
    dt, rows, D, ptrs = _tables(tables)
    indices, offsets = _i64(indices), _i64(offsets)
    N = indices.shape[0]
    if state is not None:     # None: plain SGD step (backward_sgd)
        assert state.dtype == np.float32 and state.shape == (int(rows.sum()),) and state.flags["C_CONTIGUOUS"]
    want_np = {"f32": np.float32, "f16": np.float16, "bf16": np.uint16}[grad_dtype]
    assert grad_out.dtype == want_np and grad_out.shape == (B, int(D.sum())) and grad_out.flags["C_CONTIGUOUS"]
    assert offsets.shape[0] == len(tables) * B + 1 and offsets[-1] == N
    res = BackwardResult()
    n1 = max(N, 1)
    ks = np.zeros(n1, dtype=np.int64) if want_indices else None
    order = np.zeros(n1, dtype=np.int64) if want_indices else None
    uniq = np.zeros(n1, dtype=np.int64) if want_indices else None
    seg = np.zeros(n1 + 1, dtype=np.int64) if want_indices else None
    null = ctypes.POINTER(ctypes.c_int64)()

    def ptr(a):
        return _p(a, ctypes.c_int64) if a is not None else null

    U = lib().oracle_backward_rowwise_adagrad_io(len(tables), _p(rows, ctypes.c_int64), _p(D, ctypes.c_int32), dt, ptrs,
                                                 _p(state, ctypes.c_float) if state is not None
                                                 else ctypes.POINTER(ctypes.c_float)(),
                                                 grad_out.ctypes.data, _IO[grad_dtype],
                                                 _p(indices, ctypes.c_int64), _p(offsets, ctypes.c_int64), B,
                                                 _pooling(pooling), float(lr), float(eps), float(c),
                                                 ptr(ks), ptr(order), ptr(uniq), ptr(seg))
    if U < 0:
        raise IndexError("id outside its table")
    res.U = int(U)
    if want_indices:
        res.keys_sorted, res.order = ks[:N], order[:N]
        res.unique_rows, res.seg_start = uniq[:U].copy(), seg[:U + 1].copy()
    else:
        res.keys_sorted = res.order = res.unique_rows = res.seg_start = None
    return res


def backward_sgd(tables: List[np.ndarray], grad_out: np.ndarray, indices, offsets, B: int, pooling="sum",
                 lr: float = 0.01, want_indices: bool = True, grad_dtype: str = "f32") -> BackwardResult:
    """Same sparse backward with the plain SGD step w -= lr * g per unique row; in place on `tables`."""
    return backward_rowwise_adagrad(tables, None, grad_out, indices, offsets, B, pooling, lr, 0.0, 1.0, want_indices,
                                    grad_dtype)


def replica_mean(replicas: Sequence[np.ndarray]) -> None:
    """In place: every array (one per replica, same shape; float32, or float16/uint16 holding binary16) becomes the
    element-wise mean over the replicas (Algorithm 1, weight sync and moment sync)."""
    M = len(replicas)
    assert M >= 1
    first = replicas[0]
    for a in replicas:
        assert a.shape == first.shape and a.dtype == first.dtype and a.flags["C_CONTIGUOUS"]
    code = F32 if first.dtype == np.float32 else F16
    assert first.dtype in (np.float32, np.float16, np.uint16)
    ptrs = (ctypes.c_void_p * M)(*[a.ctypes.data for a in replicas])
    lib().oracle_replica_mean(ptrs, M, int(first.size), code)


_IO_NP = {"f32": np.float32, "f16": np.float16, "bf16": np.uint16}


def lookup_seq(tables: Sequence[np.ndarray], indices, table_offsets, out_dtype="f32") -> np.ndarray:
    """Non-pooled lookup.  Returns the flat output: one row-major [n_t, D_t] block per table, one after the other."""
    dt, rows, D, ptrs = _tables(tables)
    indices, table_offsets = _i64(indices), _i64(table_offsets)
    assert table_offsets.shape[0] == len(tables) + 1 and table_offsets[-1] == indices.shape[0] and table_offsets[0] == 0
    total = int(((table_offsets[1:] - table_offsets[:-1]) * D).sum())
    out = np.zeros(max(total, 1), dtype=_IO_NP[out_dtype])
    rc = lib().oracle_lookup_seq_io(len(tables), _p(rows, ctypes.c_int64), _p(D, ctypes.c_int32), dt, ptrs,
                                    _p(indices, ctypes.c_int64), _p(table_offsets, ctypes.c_int64), out.ctypes.data,
                                    _IO[out_dtype])
    if rc:
        raise IndexError("id outside its table")
    return out[:total]


def backward_seq(tables: List[np.ndarray], state: Optional[np.ndarray], grad_seq: np.ndarray, indices, table_offsets,
                 lr: float = 0.01, eps: float = 1e-8, c: float = 1.0, grad_dtype: str = "f32") -> int:
    """Backward of the non-pooled lookup, in place on `tables` and `state` (None: plain SGD).  Returns the number of
    rows updated."""
    dt, rows, D, ptrs = _tables(tables)
    indices, table_offsets = _i64(indices), _i64(table_offsets)
    assert table_offsets.shape[0] == len(tables) + 1 and table_offsets[-1] == indices.shape[0] and table_offsets[0] == 0
    total = int(((table_offsets[1:] - table_offsets[:-1]) * D).sum())
    assert grad_seq.dtype == _IO_NP[grad_dtype] and grad_seq.size >= total and grad_seq.flags["C_CONTIGUOUS"]
    if state is not None:
        assert state.dtype == np.float32 and state.shape == (int(rows.sum()),)
    U = lib().oracle_backward_seq_io(len(tables), _p(rows, ctypes.c_int64), _p(D, ctypes.c_int32), dt, ptrs,
                                     _p(state, ctypes.c_float) if state is not None else ctypes.POINTER(ctypes.c_float)(),
                                     grad_seq.ctypes.data, _IO[grad_dtype], _p(indices, ctypes.c_int64),
                                     _p(table_offsets, ctypes.c_int64), float(lr), float(eps), float(c))
    if U < 0:
        raise IndexError("id outside its table")
    return int(U)
