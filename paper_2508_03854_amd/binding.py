"""Thin ctypes binding of libtbe355.so: same names as the C ABI, argument marshalling only.

torch is used for device memory and streams.  There is no fallback: if the HIP library is missing or a
call fails, an exception is raised."""
from __future__ import annotations

import ctypes
import os
from typing import Dict, List, Optional, Sequence, Tuple

import torch  # must be imported before the library so that both share one HIP runtime

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libtbe355.so")

OK, EINVAL, ESHAPE, EDTYPE, EWORKSPACE, EINDEX, EHIP = range(7)
STATIC_SCRATCH_BYTES = 64 << 20        # TBE_STATIC_SCRATCH_BYTES
F32, F16 = 0, 1
SUM, MEAN = 0, 1
I64, I32 = 0, 1                       # tbe_index_dtype
IO_F32, IO_F16, IO_BF16 = 0, 1, 2     # tbe_io_dtype
TUNABLES = {"hot_rows_min_workgroups": 0}   # tbe_tunable
_IDX = {torch.int64: I64, torch.int32: I32}
_IO = {torch.float32: IO_F32, torch.float16: IO_F16, torch.bfloat16: IO_BF16}

# every symbol include/tbe355.h declares
EXPORTS = ["tbe_create", "tbe_destroy", "tbe_workspace_bytes", "tbe_forward", "tbe_backward_rowwise_adagrad",
           "tbe_forward_ex", "tbe_backward_rowwise_adagrad_ex", "tbe_backward_rowwise_adagrad_static", "tbe_backward_prepare",
           "tbe_backward_apply_rowwise_adagrad", "tbe_backward_apply_sgd", "tbe_backward_sgd", "tbe_replica_mean", "tbe_lookup_seq",
           "tbe_backward_seq_rowwise_adagrad", "tbe_debug_sorted", "tbe_poll_index_error", "tbe_set_tunable", "tbe_timing_enable",
           "tbe_timing_count", "tbe_timing_read", "tbe_calibration_copy", "tbe_calibration_gather", "tbe_status_string", "tbe_build_info"]


class TbeError(RuntimeError):
    def __init__(self, status: int, what: str):
        super().__init__(f"{what}: status {status} ({_status_string(status)})")
        self.status = status


_lib = None


def lib_path() -> str:
    return _LIB_PATH


def load_library():
    """Loads libtbe355.so; raises if it has not been built (python -m paper_2508_03854_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise FileNotFoundError(f"{_LIB_PATH} is missing: build it with `python paper_2508_03854_amd/build.py`")
    L = ctypes.CDLL(_LIB_PATH)
    vp, i32, i64, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float
    L.tbe_create.restype = ctypes.c_int
    L.tbe_create.argtypes = [i32, ctypes.POINTER(i64), ctypes.POINTER(i32), ctypes.c_int, ctypes.POINTER(vp)]
    L.tbe_destroy.restype = ctypes.c_int
    L.tbe_destroy.argtypes = [vp]
    L.tbe_workspace_bytes.restype = ctypes.c_int
    L.tbe_workspace_bytes.argtypes = [vp, i32, i64, ctypes.POINTER(ctypes.c_size_t)]
    L.tbe_forward.restype = ctypes.c_int
    L.tbe_forward.argtypes = [vp, vp, vp, vp, vp, i32, i64, ctypes.c_int, vp, vp]
    L.tbe_backward_rowwise_adagrad.restype = ctypes.c_int
    L.tbe_backward_rowwise_adagrad.argtypes = [vp, vp, vp, vp, i32, i64, ctypes.c_int, f32, f32, f32, vp, vp, vp,
                                               ctypes.c_size_t, vp]
    L.tbe_forward_ex.restype = ctypes.c_int
    L.tbe_forward_ex.argtypes = [vp, vp, vp, vp, vp, ctypes.c_int, i32, i64, ctypes.c_int, vp, ctypes.c_int, vp]
    L.tbe_backward_rowwise_adagrad_ex.restype = ctypes.c_int
    L.tbe_backward_rowwise_adagrad_ex.argtypes = [vp, vp, ctypes.c_int, vp, vp, ctypes.c_int, i32, i64, ctypes.c_int,
                                                  f32, f32, f32, vp, vp, vp, ctypes.c_size_t, vp]
    L.tbe_backward_rowwise_adagrad_static.restype = ctypes.c_int
    L.tbe_backward_rowwise_adagrad_static.argtypes = [vp, vp, ctypes.c_int, vp, vp, ctypes.c_int, i32, i64, ctypes.c_int,
                                                      f32, f32, f32, vp, vp, vp]
    L.tbe_backward_prepare.restype = ctypes.c_int
    L.tbe_backward_prepare.argtypes = [vp, vp, vp, ctypes.c_int, i32, i64, vp, ctypes.c_size_t, vp]
    L.tbe_backward_apply_rowwise_adagrad.restype = ctypes.c_int
    L.tbe_backward_apply_rowwise_adagrad.argtypes = [vp, vp, ctypes.c_int, vp, ctypes.c_int, i32, i64, ctypes.c_int,
                                                     f32, f32, f32, vp, vp, vp, ctypes.c_size_t, vp]
    L.tbe_backward_apply_sgd.restype = ctypes.c_int
    L.tbe_backward_apply_sgd.argtypes = [vp, vp, ctypes.c_int, vp, ctypes.c_int, i32, i64, ctypes.c_int, f32, vp, vp,
                                         ctypes.c_size_t, vp]
    L.tbe_backward_sgd.restype = ctypes.c_int
    L.tbe_backward_sgd.argtypes = [vp, vp, ctypes.c_int, vp, vp, ctypes.c_int, i32, i64, ctypes.c_int, f32, vp, vp,
                                   ctypes.c_size_t, vp]
    L.tbe_lookup_seq.restype = ctypes.c_int
    L.tbe_lookup_seq.argtypes = [vp, vp, vp, vp, ctypes.c_int, i64, vp, ctypes.c_int, i64, vp]
    L.tbe_backward_seq_rowwise_adagrad.restype = ctypes.c_int
    L.tbe_backward_seq_rowwise_adagrad.argtypes = [vp, vp, ctypes.c_int, i64, vp, vp, ctypes.c_int, i64, f32, f32, f32,
                                                   vp, vp, vp, ctypes.c_size_t, vp]
    L.tbe_replica_mean.restype = ctypes.c_int
    L.tbe_replica_mean.argtypes = [vp, ctypes.POINTER(vp), i32, ctypes.c_size_t, ctypes.c_int, vp]
    L.tbe_debug_sorted.restype = ctypes.c_int
    L.tbe_debug_sorted.argtypes = [vp, vp, i32, i64] + [ctypes.POINTER(vp)] * 5
    L.tbe_poll_index_error.restype = ctypes.c_int
    L.tbe_poll_index_error.argtypes = [vp]
    L.tbe_set_tunable.restype = ctypes.c_int
    L.tbe_set_tunable.argtypes = [vp, ctypes.c_int, i64]
    L.tbe_timing_enable.restype = ctypes.c_int
    L.tbe_timing_enable.argtypes = [vp, ctypes.c_int]
    L.tbe_timing_count.restype = ctypes.c_int
    L.tbe_timing_count.argtypes = [vp, ctypes.POINTER(i32)]
    L.tbe_timing_read.restype = ctypes.c_int
    L.tbe_timing_read.argtypes = [vp, i32, ctypes.POINTER(ctypes.c_char_p), ctypes.POINTER(f32)]
    L.tbe_calibration_copy.restype = ctypes.c_int
    L.tbe_calibration_copy.argtypes = [vp, vp, vp, ctypes.c_size_t, vp]
    L.tbe_calibration_gather.restype = ctypes.c_int
    L.tbe_calibration_gather.argtypes = [vp, vp, ctypes.c_size_t, ctypes.c_size_t, i32, i32, i64, i32, vp,
                                         ctypes.c_size_t, vp]
    L.tbe_build_info.restype = ctypes.c_char_p
    L.tbe_build_info.argtypes = []
    L.tbe_status_string.restype = ctypes.c_char_p
    L.tbe_status_string.argtypes = [ctypes.c_int]
    _lib = L
    return L


def build_info() -> str:
    """tbe_build_info(): "tbe355 gfx950 <digest of the sources the loaded library was built from>"."""
    return load_library().tbe_build_info().decode()


def _status_string(s: int) -> str:
    try:
        return load_library().tbe_status_string(int(s)).decode()
    except Exception:  # pragma: no cover
        return "?"


def _check(status: int, what: str) -> None:
    if status != OK:
        raise TbeError(status, what)


def _dev_ptr(t: Optional[torch.Tensor], dtype: torch.dtype, what: str) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError(f"{what} must be a device tensor")
    if t.dtype != dtype:
        raise TypeError(f"{what} must be {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{what} must be contiguous")
    return t.data_ptr()


def _index_dtype(indices: torch.Tensor, offsets: torch.Tensor) -> int:
    if indices.dtype != offsets.dtype or indices.dtype not in _IDX:
        raise TypeError(f"indices and offsets must both be int64 or both int32, got {indices.dtype} / {offsets.dtype}")
    return _IDX[indices.dtype]


def _stream_ptr(stream: Optional[torch.cuda.Stream]) -> int:
    s = stream if stream is not None else torch.cuda.current_stream()
    return s.cuda_stream


class TBE:
    """One table set (tbe_handle).  Methods mirror the C entry points one to one."""

    def __init__(self, rows: Sequence[int], D: Sequence[int], weight_dtype: str = "f32"):
        self._lib = load_library()
        self.rows = [int(r) for r in rows]
        self.D = [int(d) for d in D]
        self.T = len(self.rows)
        assert len(self.D) == self.T
        self.weight_dtype = weight_dtype
        self.torch_dtype = {"f32": torch.float32, "f16": torch.float16}[weight_dtype]
        self.sum_D = sum(self.D)
        self.total_rows = sum(self.rows)
        self.total_elems = sum(r * d for r, d in zip(self.rows, self.D))
        rows_a = (ctypes.c_int64 * self.T)(*self.rows)
        D_a = (ctypes.c_int32 * self.T)(*self.D)
        h = ctypes.c_void_p()
        _check(self._lib.tbe_create(self.T, rows_a, D_a, {"f32": F32, "f16": F16}[weight_dtype], ctypes.byref(h)),
               "tbe_create")
        self._h = h

    def close(self) -> None:
        if getattr(self, "_h", None):
            self._lib.tbe_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- tbe_workspace_bytes
    def workspace_bytes(self, B: int, max_nnz: int) -> int:
        n = ctypes.c_size_t()
        _check(self._lib.tbe_workspace_bytes(self._h, int(B), int(max_nnz), ctypes.byref(n)), "tbe_workspace_bytes")
        return int(n.value)

    def alloc_workspace(self, B: int, max_nnz: int, device="cuda") -> torch.Tensor:
        return torch.empty(self.workspace_bytes(B, max_nnz), dtype=torch.uint8, device=device)

    # ---- tbe_forward
    def forward(self, tables: torch.Tensor, indices: torch.Tensor, offsets: torch.Tensor, B: int, pooling: str = "sum",
                out: Optional[torch.Tensor] = None, D_offsets: Optional[torch.Tensor] = None,
                stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
        if out is None:
            out = torch.empty(B, self.sum_D, dtype=torch.float32, device=tables.device)
        if tables.numel() != self.total_elems or out.shape != (B, self.sum_D):
            raise ValueError("tables / out shape does not match the handle")
        if offsets.numel() != self.T * B + 1:
            raise ValueError("offsets must have T*B+1 entries")
        nnz = indices.numel()
        st = self._lib.tbe_forward(self._h, _dev_ptr(tables, self.torch_dtype, "tables"),
                                   _dev_ptr(D_offsets, torch.int32, "D_offsets"),
                                   _dev_ptr(indices, torch.int64, "indices"), _dev_ptr(offsets, torch.int64, "offsets"),
                                   int(B), int(nnz), {"sum": SUM, "mean": MEAN}[pooling],
                                   _dev_ptr(out, torch.float32, "out"), _stream_ptr(stream))
        _check(st, "tbe_forward")
        return out

    # ---- tbe_forward_ex
    def forward_ex(self, tables: torch.Tensor, indices: torch.Tensor, offsets: torch.Tensor, B: int,
                   pooling: str = "sum", out: Optional[torch.Tensor] = None, out_dtype: torch.dtype = torch.float32,
                   D_offsets: Optional[torch.Tensor] = None, stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
        """int64 or int32 indices/offsets (both the same); float32, float16 or bfloat16 out."""
        if out is None:
            out = torch.empty(B, self.sum_D, dtype=out_dtype, device=tables.device)
        if out.dtype not in _IO:
            raise TypeError(f"out must be float32, float16 or bfloat16, got {out.dtype}")
        if tables.numel() != self.total_elems or out.shape != (B, self.sum_D):
            raise ValueError("tables / out shape does not match the handle")
        if offsets.numel() != self.T * B + 1:
            raise ValueError("offsets must have T*B+1 entries")
        idt = _index_dtype(indices, offsets)
        st = self._lib.tbe_forward_ex(self._h, _dev_ptr(tables, self.torch_dtype, "tables"),
                                      _dev_ptr(D_offsets, torch.int32, "D_offsets"),
                                      _dev_ptr(indices, indices.dtype, "indices"),
                                      _dev_ptr(offsets, offsets.dtype, "offsets"), idt, int(B), int(indices.numel()),
                                      {"sum": SUM, "mean": MEAN}[pooling], _dev_ptr(out, out.dtype, "out"),
                                      _IO[out.dtype], _stream_ptr(stream))
        _check(st, "tbe_forward_ex")
        return out

    # ---- tbe_backward_rowwise_adagrad_ex
    def backward_rowwise_adagrad_ex(self, grad_out: torch.Tensor, indices: torch.Tensor, offsets: torch.Tensor, B: int,
                                    tables: torch.Tensor, state: torch.Tensor, workspace: torch.Tensor, *,
                                    pooling: str = "sum", lr: float, eps: float, momentum_scale: float = 1.0,
                                    stream: Optional[torch.cuda.Stream] = None) -> None:
        """int64 or int32 indices/offsets (both the same); float32, float16 or bfloat16 grad_out."""
        if tables.numel() != self.total_elems or state.numel() != self.total_rows:
            raise ValueError("tables / state shape does not match the handle")
        if grad_out.shape != (B, self.sum_D) or offsets.numel() != self.T * B + 1:
            raise ValueError("grad_out / offsets shape does not match the handle")
        if grad_out.dtype not in _IO:
            raise TypeError(f"grad_out must be float32, float16 or bfloat16, got {grad_out.dtype}")
        idt = _index_dtype(indices, offsets)
        st = self._lib.tbe_backward_rowwise_adagrad_ex(
            self._h, _dev_ptr(grad_out, grad_out.dtype, "grad_out"), _IO[grad_out.dtype],
            _dev_ptr(indices, indices.dtype, "indices"), _dev_ptr(offsets, offsets.dtype, "offsets"), idt, int(B),
            int(indices.numel()), {"sum": SUM, "mean": MEAN}[pooling], float(lr), float(eps), float(momentum_scale),
            _dev_ptr(tables, self.torch_dtype, "tables"), _dev_ptr(state, torch.float32, "state"),
            _dev_ptr(workspace, torch.uint8, "workspace"), int(workspace.numel()), _stream_ptr(stream))
        _check(st, "tbe_backward_rowwise_adagrad_ex")

    # ---- tbe_backward_rowwise_adagrad_static
    def backward_rowwise_adagrad_static(self, grad_out: torch.Tensor, indices: torch.Tensor, offsets: torch.Tensor,
                                        B: int, tables: torch.Tensor, state: torch.Tensor, *, pooling: str = "sum",
                                        lr: float, eps: float, momentum_scale: float = 1.0,
                                        stream: Optional[torch.cuda.Stream] = None) -> None:
        """The backward with the library's own fixed scratch array instead of a caller's workspace."""
        if tables.numel() != self.total_elems or state.numel() != self.total_rows:
            raise ValueError("tables / state shape does not match the handle")
        if grad_out.shape != (B, self.sum_D) or offsets.numel() != self.T * B + 1:
            raise ValueError("grad_out / offsets shape does not match the handle")
        if grad_out.dtype not in _IO:
            raise TypeError(f"grad_out must be float32, float16 or bfloat16, got {grad_out.dtype}")
        idt = _index_dtype(indices, offsets)
        st = self._lib.tbe_backward_rowwise_adagrad_static(
            self._h, _dev_ptr(grad_out, grad_out.dtype, "grad_out"), _IO[grad_out.dtype],
            _dev_ptr(indices, indices.dtype, "indices"), _dev_ptr(offsets, offsets.dtype, "offsets"), idt, int(B),
            int(indices.numel()), {"sum": SUM, "mean": MEAN}[pooling], float(lr), float(eps), float(momentum_scale),
            _dev_ptr(tables, self.torch_dtype, "tables"), _dev_ptr(state, torch.float32, "state"), _stream_ptr(stream))
        _check(st, "tbe_backward_rowwise_adagrad_static")

    # ---- tbe_backward_prepare / tbe_backward_apply_rowwise_adagrad
    def backward_prepare(self, indices: torch.Tensor, offsets: torch.Tensor, B: int, workspace: torch.Tensor,
                         stream: Optional[torch.cuda.Stream] = None) -> None:
        """Sort / dedup / segment the batch's ids into `workspace` (needs no gradient; may run on another stream)."""
        if offsets.numel() != self.T * B + 1:
            raise ValueError("offsets shape does not match the handle")
        idt = _index_dtype(indices, offsets)
        st = self._lib.tbe_backward_prepare(
            self._h, _dev_ptr(indices, indices.dtype, "indices"), _dev_ptr(offsets, offsets.dtype, "offsets"), idt,
            int(B), int(indices.numel()), _dev_ptr(workspace, torch.uint8, "workspace"), int(workspace.numel()),
            _stream_ptr(stream))
        _check(st, "tbe_backward_prepare")

    def backward_apply_rowwise_adagrad(self, grad_out: torch.Tensor, offsets: torch.Tensor, B: int, nnz: int,
                                       tables: torch.Tensor, state: torch.Tensor, workspace: torch.Tensor, *,
                                       pooling: str = "sum", lr: float, eps: float, momentum_scale: float = 1.0,
                                       stream: Optional[torch.cuda.Stream] = None) -> None:
        """Row gradients and the step from a workspace that backward_prepare filled for the same batch."""
        if tables.numel() != self.total_elems or state.numel() != self.total_rows:
            raise ValueError("tables / state shape does not match the handle")
        if grad_out.shape != (B, self.sum_D) or offsets.numel() != self.T * B + 1:
            raise ValueError("grad_out / offsets shape does not match the handle")
        if grad_out.dtype not in _IO:
            raise TypeError(f"grad_out must be float32, float16 or bfloat16, got {grad_out.dtype}")
        if offsets.dtype not in _IDX:
            raise TypeError(f"offsets must be int64 or int32, got {offsets.dtype}")
        st = self._lib.tbe_backward_apply_rowwise_adagrad(
            self._h, _dev_ptr(grad_out, grad_out.dtype, "grad_out"), _IO[grad_out.dtype],
            _dev_ptr(offsets, offsets.dtype, "offsets"), _IDX[offsets.dtype], int(B), int(nnz),
            {"sum": SUM, "mean": MEAN}[pooling], float(lr), float(eps), float(momentum_scale),
            _dev_ptr(tables, self.torch_dtype, "tables"), _dev_ptr(state, torch.float32, "state"),
            _dev_ptr(workspace, torch.uint8, "workspace"), int(workspace.numel()), _stream_ptr(stream))
        _check(st, "tbe_backward_apply_rowwise_adagrad")

    def backward_apply_sgd(self, grad_out: torch.Tensor, offsets: torch.Tensor, B: int, nnz: int, tables: torch.Tensor,
                           workspace: torch.Tensor, *, pooling: str = "sum", lr: float,
                           stream: Optional[torch.cuda.Stream] = None) -> None:
        """Row gradients and the plain SGD step from a workspace that backward_prepare filled for the same batch."""
        if tables.numel() != self.total_elems:
            raise ValueError("tables shape does not match the handle")
        if grad_out.shape != (B, self.sum_D) or offsets.numel() != self.T * B + 1:
            raise ValueError("grad_out / offsets shape does not match the handle")
        if grad_out.dtype not in _IO:
            raise TypeError(f"grad_out must be float32, float16 or bfloat16, got {grad_out.dtype}")
        if offsets.dtype not in _IDX:
            raise TypeError(f"offsets must be int64 or int32, got {offsets.dtype}")
        st = self._lib.tbe_backward_apply_sgd(
            self._h, _dev_ptr(grad_out, grad_out.dtype, "grad_out"), _IO[grad_out.dtype],
            _dev_ptr(offsets, offsets.dtype, "offsets"), _IDX[offsets.dtype], int(B), int(nnz),
            {"sum": SUM, "mean": MEAN}[pooling], float(lr), _dev_ptr(tables, self.torch_dtype, "tables"),
            _dev_ptr(workspace, torch.uint8, "workspace"), int(workspace.numel()), _stream_ptr(stream))
        _check(st, "tbe_backward_apply_sgd")

    # ---- tbe_backward_sgd
    def backward_sgd(self, grad_out: torch.Tensor, indices: torch.Tensor, offsets: torch.Tensor, B: int,
                     tables: torch.Tensor, workspace: torch.Tensor, *, pooling: str = "sum", lr: float,
                     stream: Optional[torch.cuda.Stream] = None) -> None:
        if tables.numel() != self.total_elems:
            raise ValueError("tables shape does not match the handle")
        if grad_out.shape != (B, self.sum_D) or offsets.numel() != self.T * B + 1:
            raise ValueError("grad_out / offsets shape does not match the handle")
        if grad_out.dtype not in _IO:
            raise TypeError(f"grad_out must be float32, float16 or bfloat16, got {grad_out.dtype}")
        idt = _index_dtype(indices, offsets)
        st = self._lib.tbe_backward_sgd(
            self._h, _dev_ptr(grad_out, grad_out.dtype, "grad_out"), _IO[grad_out.dtype],
            _dev_ptr(indices, indices.dtype, "indices"), _dev_ptr(offsets, offsets.dtype, "offsets"), idt, int(B),
            int(indices.numel()), {"sum": SUM, "mean": MEAN}[pooling], float(lr),
            _dev_ptr(tables, self.torch_dtype, "tables"), _dev_ptr(workspace, torch.uint8, "workspace"),
            int(workspace.numel()), _stream_ptr(stream))
        _check(st, "tbe_backward_sgd")

    # ---- tbe_backward_rowwise_adagrad
    def backward_rowwise_adagrad(self, grad_out: torch.Tensor, indices: torch.Tensor, offsets: torch.Tensor, B: int,
                                 tables: torch.Tensor, state: torch.Tensor, workspace: torch.Tensor, *,
                                 pooling: str = "sum", lr: float, eps: float, momentum_scale: float = 1.0,
                                 stream: Optional[torch.cuda.Stream] = None) -> None:
        if tables.numel() != self.total_elems or state.numel() != self.total_rows:
            raise ValueError("tables / state shape does not match the handle")
        if grad_out.shape != (B, self.sum_D) or offsets.numel() != self.T * B + 1:
            raise ValueError("grad_out / offsets shape does not match the handle")
        nnz = indices.numel()
        st = self._lib.tbe_backward_rowwise_adagrad(
            self._h, _dev_ptr(grad_out, torch.float32, "grad_out"), _dev_ptr(indices, torch.int64, "indices"),
            _dev_ptr(offsets, torch.int64, "offsets"), int(B), int(nnz), {"sum": SUM, "mean": MEAN}[pooling],
            float(lr), float(eps), float(momentum_scale), _dev_ptr(tables, self.torch_dtype, "tables"),
            _dev_ptr(state, torch.float32, "state"), _dev_ptr(workspace, torch.uint8, "workspace"),
            int(workspace.numel()), _stream_ptr(stream))
        _check(st, "tbe_backward_rowwise_adagrad")

    # ---- tbe_lookup_seq
    def lookup_seq(self, tables: torch.Tensor, indices: torch.Tensor, offsets: torch.Tensor, out: torch.Tensor,
                   stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
        """offsets: [T+1]; out: flat tensor of >= sum_t n_t * D_t elements (float32, float16 or bfloat16)."""
        if tables.numel() != self.total_elems or offsets.numel() != self.T + 1:
            raise ValueError("tables / offsets shape does not match the handle")
        if out.dtype not in _IO:
            raise TypeError(f"out must be float32, float16 or bfloat16, got {out.dtype}")
        idt = _index_dtype(indices, offsets)
        st = self._lib.tbe_lookup_seq(self._h, _dev_ptr(tables, self.torch_dtype, "tables"),
                                      _dev_ptr(indices, indices.dtype, "indices"),
                                      _dev_ptr(offsets, offsets.dtype, "offsets"), idt, int(indices.numel()),
                                      _dev_ptr(out, out.dtype, "out"), _IO[out.dtype], int(out.numel()),
                                      _stream_ptr(stream))
        _check(st, "tbe_lookup_seq")
        return out

    # ---- tbe_backward_seq_rowwise_adagrad
    def backward_seq_rowwise_adagrad(self, grad_seq: torch.Tensor, indices: torch.Tensor, offsets: torch.Tensor,
                                     tables: torch.Tensor, state: torch.Tensor, workspace: torch.Tensor, *, lr: float,
                                     eps: float, momentum_scale: float = 1.0,
                                     stream: Optional[torch.cuda.Stream] = None) -> None:
        if tables.numel() != self.total_elems or state.numel() != self.total_rows or offsets.numel() != self.T + 1:
            raise ValueError("tables / state / offsets shape does not match the handle")
        if grad_seq.dtype not in _IO:
            raise TypeError(f"grad_seq must be float32, float16 or bfloat16, got {grad_seq.dtype}")
        idt = _index_dtype(indices, offsets)
        st = self._lib.tbe_backward_seq_rowwise_adagrad(
            self._h, _dev_ptr(grad_seq, grad_seq.dtype, "grad_seq"), _IO[grad_seq.dtype], int(grad_seq.numel()),
            _dev_ptr(indices, indices.dtype, "indices"), _dev_ptr(offsets, offsets.dtype, "offsets"), idt,
            int(indices.numel()), float(lr), float(eps), float(momentum_scale),
            _dev_ptr(tables, self.torch_dtype, "tables"), _dev_ptr(state, torch.float32, "state"),
            _dev_ptr(workspace, torch.uint8, "workspace"), int(workspace.numel()), _stream_ptr(stream))
        _check(st, "tbe_backward_seq_rowwise_adagrad")

    # ---- tbe_replica_mean
    def replica_mean(self, replicas: Sequence[torch.Tensor], stream: Optional[torch.cuda.Stream] = None) -> None:
        """Every tensor (one per replica, same shape; float32 or float16) becomes the element-wise mean."""
        first = replicas[0]
        if first.dtype not in (torch.float32, torch.float16):
            raise TypeError(f"replicas must be float32 or float16, got {first.dtype}")
        for r in replicas:
            if r.dtype != first.dtype or r.numel() != first.numel():
                raise ValueError("replicas must agree in dtype and size")
        ptrs = (ctypes.c_void_p * len(replicas))(*[_dev_ptr(r, first.dtype, "replica") for r in replicas])
        st = self._lib.tbe_replica_mean(self._h, ptrs, len(replicas), first.numel(),
                                        F32 if first.dtype == torch.float32 else F16, _stream_ptr(stream))
        _check(st, "tbe_replica_mean")

    # ---- tbe_debug_sorted
    def debug_sorted(self, workspace: torch.Tensor, B: int, nnz: int) -> Dict[str, torch.Tensor]:
        """Copies the integer by-products of the last backward to host tensors (int64; synchronises)."""
        ptrs = [ctypes.c_void_p() for _ in range(5)]
        _check(self._lib.tbe_debug_sorted(self._h, workspace.data_ptr(), int(B), int(nnz),
                                          *[ctypes.byref(p) for p in ptrs]), "tbe_debug_sorted")
        base = workspace.data_ptr()
        torch.cuda.synchronize()

        def view(p: ctypes.c_void_p, n: int) -> torch.Tensor:
            off = p.value - base
            return workspace[off:off + 4 * n].view(torch.int32).cpu().to(torch.int64) & 0xFFFFFFFF

        U = int(view(ptrs[4], 1).item())
        return {"keys_sorted": view(ptrs[0], nnz), "vals_sorted": view(ptrs[1], nnz),
                "unique_rows": view(ptrs[2], U), "seg_start": view(ptrs[3], U + 1), "num_unique": U}

    def debug_sorted_device(self, workspace: torch.Tensor, B: int, nnz: int) -> Dict[str, torch.Tensor]:
        """Same by-products as device tensors (int64 copies), for checks that stay on the GPU at full size."""
        ptrs = [ctypes.c_void_p() for _ in range(5)]
        _check(self._lib.tbe_debug_sorted(self._h, workspace.data_ptr(), int(B), int(nnz),
                                          *[ctypes.byref(p) for p in ptrs]), "tbe_debug_sorted")
        base = workspace.data_ptr()

        def view(p: ctypes.c_void_p, n: int) -> torch.Tensor:
            off = p.value - base
            return workspace[off:off + 4 * n].view(torch.int32).to(torch.int64) & 0xFFFFFFFF

        U = int(view(ptrs[4], 1).item())
        return {"keys_sorted": view(ptrs[0], nnz), "vals_sorted": view(ptrs[1], nnz),
                "unique_rows": view(ptrs[2], U), "seg_start": view(ptrs[3], U + 1), "num_unique": U}

    # ---- tbe_poll_index_error
    def poll_index_error(self) -> bool:
        st = self._lib.tbe_poll_index_error(self._h)
        if st == EINDEX:
            return True
        _check(st, "tbe_poll_index_error")
        return False

    # ---- tbe_calibration_copy
    def calibration_copy(self, dst: torch.Tensor, src: torch.Tensor, stream: Optional[torch.cuda.Stream] = None) -> None:
        nbytes = src.numel() * src.element_size()
        if dst.numel() * dst.element_size() != nbytes or not (dst.is_cuda and src.is_cuda):
            raise ValueError("dst and src must be device tensors of the same byte size")
        _check(self._lib.tbe_calibration_copy(self._h, dst.data_ptr(), src.data_ptr(), nbytes, _stream_ptr(stream)),
               "tbe_calibration_copy")

    # ---- tbe_calibration_gather
    def calibration_gather(self, buf: torch.Tensor, window_bytes: int, slice_bytes: int, gathers: int, *,
                           per_xcd: bool = True, write_back: bool = False, sink: torch.Tensor,
                           stream: Optional[torch.cuda.Stream] = None) -> None:
        if not (buf.is_cuda and sink.is_cuda):
            raise ValueError("buf and sink must be device tensors")
        _check(self._lib.tbe_calibration_gather(self._h, buf.data_ptr(), buf.numel() * buf.element_size(),
                                                int(window_bytes), 1 if per_xcd else 0, int(slice_bytes), int(gathers),
                                                1 if write_back else 0, sink.data_ptr(),
                                                sink.numel() * sink.element_size(), _stream_ptr(stream)),
               "tbe_calibration_gather")

    # ---- tbe_set_tunable
    def set_tunable(self, which: str, value: int) -> None:
        _check(self._lib.tbe_set_tunable(self._h, TUNABLES[which], int(value)), "tbe_set_tunable")

    # ---- tbe_timing_*
    def timing_enable(self, on: bool = True) -> None:
        _check(self._lib.tbe_timing_enable(self._h, 1 if on else 0), "tbe_timing_enable")

    def timing_read(self) -> List[Tuple[str, float]]:
        n = ctypes.c_int32()
        _check(self._lib.tbe_timing_count(self._h, ctypes.byref(n)), "tbe_timing_count")
        out = []
        for i in range(n.value):
            name = ctypes.c_char_p()
            ms = ctypes.c_float()
            _check(self._lib.tbe_timing_read(self._h, i, ctypes.byref(name), ctypes.byref(ms)), "tbe_timing_read")
            out.append((name.value.decode(), float(ms.value)))
        return out
