"""ctypes binding of libeasyquant.so: same names as the C ABI, argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence

import torch

EQ_F16, EQ_BF16 = 0, 1
EQ_SYMMETRIC, EQ_ASYMMETRIC = 0, 1
EQ_STAT_ROW, EQ_STAT_GROUP, EQ_STAT_MATRIX = 0, 1, 2
EQ_SELECT_BEST, EQ_SELECT_LAST = 0, 1
EQ_S_OUTLIER_OVERFLOW, EQ_S_NONFINITE = 1, 2
EQ_STATIC_SCRATCH_BYTES = 32 * 1024 * 1024

_HERE = os.path.dirname(os.path.abspath(__file__))


def lib_path() -> str:
    return os.path.join(_HERE, "libeasyquant.so")


class EasyQuantError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"{what}: {eq_strerror(code)} ({code})")
        self.code = code


class _CParams(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("bits", C.c_int32), ("group_size", C.c_int32), ("mode", C.c_int32),
                ("stat_scope", C.c_int32), ("n_sigma", C.c_float), ("iters", C.c_int32), ("lr", C.c_float),
                ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float), ("select", C.c_int32)]


class _CQMatrix(C.Structure):
    _fields_ = [("codes", C.c_void_p), ("scales", C.c_void_p), ("zero_points", C.c_void_p),
                ("out_row_ptr", C.c_void_p), ("out_col", C.c_void_p), ("out_val", C.c_void_p),
                ("out_capacity", C.c_int64), ("status", C.c_void_p)]


_lib: Optional[C.CDLL] = None


def lib() -> C.CDLL:
    """The loaded library; raises if it has not been built (there is no fallback path)."""
    global _lib
    if _lib is None:
        path = lib_path()
        if not os.path.exists(path):
            raise ImportError(f"{path} is missing: build it with `python -m paper_2403_02775_amd.build` "
                              "(hipcc, gfx950); this package has no CPU fallback")
        L = C.CDLL(path)
        L.eq_quantize_matrix.restype = C.c_int
        L.eq_quantize_matrix.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_int64, C.POINTER(_CParams),
                                         C.POINTER(_CQMatrix), C.c_void_p, C.c_size_t, C.c_void_p]
        L.eq_quantize_matrix_noalloc.restype = C.c_int
        L.eq_quantize_matrix_noalloc.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_int64, C.POINTER(_CParams),
                                                 C.POINTER(_CQMatrix), C.c_void_p]
        L.eq_quantize_batch.restype = C.c_int
        L.eq_quantize_batch.argtypes = [C.c_int32, C.POINTER(C.c_void_p), C.POINTER(C.c_int64), C.POINTER(C.c_int64),
                                        C.POINTER(C.c_int64), C.POINTER(_CParams), C.POINTER(_CQMatrix), C.c_void_p,
                                        C.c_size_t, C.c_void_p]
        L.eq_dequantize.restype = C.c_int
        L.eq_dequantize.argtypes = [C.POINTER(_CQMatrix), C.c_int64, C.c_int64, C.POINTER(_CParams), C.c_void_p,
                                    C.c_int64, C.c_void_p]
        L.eq_dequant_matvec.restype = C.c_int
        L.eq_dequant_matvec.argtypes = [C.POINTER(_CQMatrix), C.c_int64, C.c_int64, C.POINTER(_CParams), C.c_void_p,
                                        C.c_void_p, C.c_void_p]
        L.eq_workspace_bytes.restype = C.c_size_t
        L.eq_workspace_bytes.argtypes = [C.c_int32, C.POINTER(C.c_int64), C.POINTER(C.c_int64), C.POINTER(C.c_int64),
                                         C.POINTER(_CParams)]
        L.eq_code_words_per_row.restype = C.c_int64
        L.eq_code_words_per_row.argtypes = [C.c_int64, C.c_int32]
        L.eq_outlier_capacity_bound.restype = C.c_int64
        L.eq_outlier_capacity_bound.argtypes = [C.c_int64, C.c_int64, C.c_float]
        L.eq_default_params.restype = None
        L.eq_default_params.argtypes = [C.POINTER(_CParams)]
        L.eq_strerror.restype = C.c_char_p
        L.eq_strerror.argtypes = [C.c_int]
        L.eq_last_hip_error.restype = C.c_int
        L.eq_last_hip_error.argtypes = []
        # hooks for the library's own tests and measurements (csrc/eq_testing.h; not part of the C ABI)
        L.eq_test_div_f64.restype = C.c_double
        L.eq_test_div_f64.argtypes = [C.c_double, C.c_double]
        L.eq_test_div_f32.restype = C.c_float
        L.eq_test_div_f32.argtypes = [C.c_float, C.c_float]
        L.eq_test_set_override.restype = C.c_int
        L.eq_test_set_override.argtypes = [C.c_int, C.c_int64]
        L.eq_test_plan_items.restype = C.c_int64
        L.eq_test_plan_items.argtypes = [C.c_int32, C.POINTER(C.c_int64), C.POINTER(C.c_int64), C.POINTER(C.c_int64),
                                         C.POINTER(_CParams), C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.c_int64]
        L.eq_test_plan_sort_segments.restype = C.c_int64
        L.eq_test_plan_sort_segments.argtypes = [C.c_int32, C.POINTER(C.c_int64), C.POINTER(C.c_int64), C.POINTER(C.c_int64),
                                                 C.POINTER(_CParams), C.POINTER(C.c_int64), C.c_int64, C.POINTER(C.c_int64)]
        L.eq_profile_enable.restype = C.c_int
        L.eq_profile_enable.argtypes = [C.c_int]
        L.eq_profile_read.restype = C.c_int
        L.eq_profile_read.argtypes = [C.POINTER(C.c_double), C.POINTER(C.c_int32)]
        _lib = L
    return _lib


@dataclass
class Params:
    """Mirror of `eq_params` (defaults = eq_default_params: the paper's BLOOM setting)."""
    dtype: int = EQ_F16
    bits: int = 4
    group_size: int = 0
    mode: int = EQ_SYMMETRIC
    stat_scope: int = EQ_STAT_ROW
    n_sigma: float = 3.0
    iters: int = 100
    lr: float = 1e-3
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    select: int = EQ_SELECT_BEST

    def c(self) -> _CParams:
        return _CParams(self.dtype, self.bits, self.group_size, self.mode, self.stat_scope, self.n_sigma, self.iters,
                        self.lr, self.beta1, self.beta2, self.eps, self.select)


@dataclass
class QMatrix:
    """Mirror of `eq_qmatrix`: device tensors owned by the caller."""
    codes: torch.Tensor        # int32  [rows, words_per_row]
    scales: torch.Tensor       # float32 [rows, units_per_row]
    zero_points: torch.Tensor  # uint8  [rows, units_per_row]
    out_row_ptr: torch.Tensor  # int32  [rows + 1]   (bit pattern of uint32)
    out_col: torch.Tensor      # int32  [capacity]
    out_val: torch.Tensor      # int16  [capacity]   (raw 16-bit patterns)
    status: torch.Tensor       # int32  [1]

    @property
    def capacity(self) -> int:
        return int(self.out_col.numel())

    def c(self) -> _CQMatrix:
        cap = self.capacity
        return _CQMatrix(self.codes.data_ptr(), self.scales.data_ptr(), self.zero_points.data_ptr(),
                         self.out_row_ptr.data_ptr(), self.out_col.data_ptr() if cap else None,
                         self.out_val.data_ptr() if cap else None, cap, self.status.data_ptr())


def eq_strerror(code: int) -> str:
    return lib().eq_strerror(int(code)).decode()


def eq_profile_enable(on: bool) -> None:
    lib().eq_profile_enable(1 if on else 0)


def eq_profile_read():
    """(summed main-kernel milliseconds, number of launches) since the last read."""
    ms, n = C.c_double(0.0), C.c_int32(0)
    rc = lib().eq_profile_read(C.byref(ms), C.byref(n))
    if rc != 0:
        raise EasyQuantError(rc, "eq_profile_read")
    return ms.value, n.value


def eq_code_words_per_row(cols: int, bits: int) -> int:
    return int(lib().eq_code_words_per_row(cols, bits))


def eq_outlier_capacity_bound(rows: int, cols: int, n_sigma: float) -> int:
    return int(lib().eq_outlier_capacity_bound(rows, cols, n_sigma))


def eq_workspace_bytes(rows: Sequence[int], cols: Sequence[int], capacities: Sequence[int], p: Params) -> int:
    n = len(rows)
    A = C.c_int64 * max(n, 1)
    cp = p.c()
    return int(lib().eq_workspace_bytes(n, A(*rows), A(*cols), A(*capacities), C.byref(cp)))


def alloc_outputs(rows: int, cols: int, p: Params, capacity: int, device) -> QMatrix:
    """Allocates the output tensors of one matrix (device memory comes from PyTorch)."""
    upr = 1 if p.group_size == 0 else cols // p.group_size
    wpr = (cols * p.bits + 31) // 32
    return QMatrix(
        codes=torch.empty((rows, wpr), dtype=torch.int32, device=device),
        scales=torch.empty((rows, upr), dtype=torch.float32, device=device),
        zero_points=torch.empty((rows, upr), dtype=torch.uint8, device=device),
        out_row_ptr=torch.empty(rows + 1, dtype=torch.int32, device=device),
        out_col=torch.empty(capacity, dtype=torch.int32, device=device),
        out_val=torch.empty(capacity, dtype=torch.int16, device=device),
        status=torch.empty(1, dtype=torch.int32, device=device),
    )


def _stream_ptr(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def _ld(W: torch.Tensor) -> int:
    """Row stride in elements (a matrix with at most one row, or no columns, has no meaningful stride)."""
    rows, cols = W.shape
    return int(cols) if rows <= 1 or cols == 0 else int(W.stride(0))


def _check_w(W: torch.Tensor, p: Params):
    want = torch.float16 if p.dtype == EQ_F16 else torch.bfloat16
    if W.dtype != want or W.dim() != 2 or W.stride(1) != 1 or not W.is_cuda:
        raise ValueError("W must be a 2-D CUDA tensor of the dtype named in the parameters, unit stride along columns")


def eq_quantize_matrix(W: torch.Tensor, p: Params, out: QMatrix, workspace: torch.Tensor, stream=None) -> None:
    _check_w(W, p)
    rows, cols = W.shape
    cp, cq = p.c(), out.c()
    rc = lib().eq_quantize_matrix(W.data_ptr(), rows, cols, _ld(W),
                                  C.byref(cp), C.byref(cq), workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                  _stream_ptr(stream))
    if rc != 0:
        raise EasyQuantError(rc, "eq_quantize_matrix")


def eq_quantize_matrix_noalloc(W: torch.Tensor, p: Params, out: QMatrix, stream=None) -> None:
    """eq_quantize_matrix without a workspace argument (the library's built-in scratch array)."""
    _check_w(W, p)
    rows, cols = W.shape
    cp, cq = p.c(), out.c()
    rc = lib().eq_quantize_matrix_noalloc(W.data_ptr(), rows, cols, _ld(W), C.byref(cp), C.byref(cq), _stream_ptr(stream))
    if rc != 0:
        raise EasyQuantError(rc, "eq_quantize_matrix_noalloc")


def eq_quantize_batch(Ws: List[torch.Tensor], p: Params, outs: List[QMatrix], workspace: torch.Tensor, stream=None) -> None:
    n = len(Ws)
    for W in Ws:
        _check_w(W, p)
    PA, IA, QA = C.c_void_p * max(n, 1), C.c_int64 * max(n, 1), _CQMatrix * max(n, 1)
    rows = [int(W.shape[0]) for W in Ws]
    cols = [int(W.shape[1]) for W in Ws]
    lds = [_ld(W) for W in Ws]
    cp = p.c()
    rc = lib().eq_quantize_batch(n, PA(*[W.data_ptr() for W in Ws]), IA(*rows), IA(*cols), IA(*lds), C.byref(cp),
                                 QA(*[o.c() for o in outs]), workspace.data_ptr(),
                                 workspace.numel() * workspace.element_size(), _stream_ptr(stream))
    if rc != 0:
        raise EasyQuantError(rc, "eq_quantize_batch")


def eq_dequant_matvec(q: QMatrix, rows: int, cols: int, p: Params, x: torch.Tensor, y: torch.Tensor, stream=None) -> None:
    """y (rows, float32) = dequantized matrix times x (cols, the matrix's 16-bit type), fused."""
    want = torch.float16 if p.dtype == EQ_F16 else torch.bfloat16
    if x.dtype != want or x.dim() != 1 or not x.is_contiguous() or x.numel() != cols:
        raise ValueError("x must be a contiguous vector of cols elements in the matrix's 16-bit type")
    if y.dtype != torch.float32 or y.dim() != 1 or not y.is_contiguous() or y.numel() != rows:
        raise ValueError("y must be a contiguous float32 vector of rows elements")
    cp, cq = p.c(), q.c()
    rc = lib().eq_dequant_matvec(C.byref(cq), rows, cols, C.byref(cp), x.data_ptr(), y.data_ptr(), _stream_ptr(stream))
    if rc != 0:
        raise EasyQuantError(rc, "eq_dequant_matvec")


def eq_dequantize(q: QMatrix, rows: int, cols: int, p: Params, W_out: torch.Tensor, stream=None) -> None:
    _check_w(W_out, p)
    cp, cq = p.c(), q.c()
    rc = lib().eq_dequantize(C.byref(cq), rows, cols, C.byref(cp), W_out.data_ptr(),
                             _ld(W_out), _stream_ptr(stream))
    if rc != 0:
        raise EasyQuantError(rc, "eq_dequantize")


# ---- hooks for tests and measurements (csrc/eq_testing.h; not part of the C ABI) ----------------
(OVR_UNITS_PER_ITEM, OVR_FORCE_GENERAL, OVR_RTN_THREADS, OVR_CHANNEL_KERNEL, OVR_MATVEC_ARITHMETIC, OVR_MATVEC_LOOKUP,
 OVR_SORTED_ROWS, OVR_SORT_CHUNK_ROWS, OVR_CLASS_STREAMS) = range(9)
OVR_COUNT = 9


class override:
    """`with override(OVR_FORCE_GENERAL, 1): ...` sets a kernel-selection override of the library
    for the duration of the block (process-wide; results do not depend on it)."""

    def __init__(self, which: int, value: int):
        self.which, self.value = which, int(value)

    def __enter__(self):
        set_override(self.which, self.value)
        return self

    def __exit__(self, *exc):
        set_override(self.which, 0)
        return False


def set_override(which: int, value: int) -> None:
    rc = lib().eq_test_set_override(which, int(value))
    if rc != 0:
        raise EasyQuantError(rc, "eq_test_set_override")


def plan_items(rows: Sequence[int], cols: Sequence[int], capacities: Sequence[int], p: Params):
    """The work items eq_quantize_batch would launch for these shapes, in launch order (host only,
    no GPU): a list of (matrix, first row, rows, stride, step, launch index).  The workgroup takes
    rows [first, first + rows): all of them when stride == 0, else the `step` rows at first,
    first + stride, first + 2 stride, ..."""
    n = len(rows)
    A = C.c_int64 * max(n, 1)
    cp = p.c()
    args = (n, A(*rows), A(*cols), A(*capacities), C.byref(cp))
    cnt = int(lib().eq_test_plan_items(*args, None, None, 0))
    if cnt < 0:
        raise EasyQuantError(cnt, "eq_test_plan_items")
    items = (C.c_int32 * (5 * max(cnt, 1)))()
    launch = (C.c_int32 * max(cnt, 1))()
    lib().eq_test_plan_items(*args, items, launch, cnt)
    return [tuple(items[5 * i:5 * i + 5]) + (launch[i],) for i in range(cnt)]


def plan_sort_segments(rows: Sequence[int], cols: Sequence[int], capacities: Sequence[int], p: Params):
    """The chunks of the sorted evaluation of rows with one range each for these shapes (host only, no
    GPU): (list of (chunk, matrix, first row, rows, first group, first row in chunk, byte offset of the
    first record), bytes of the record region)."""
    n = len(rows)
    A = C.c_int64 * max(n, 1)
    cp = p.c()
    args = (n, A(*rows), A(*cols), A(*capacities), C.byref(cp))
    region = C.c_int64(0)
    cnt = int(lib().eq_test_plan_sort_segments(*args, None, 0, C.byref(region)))
    if cnt < 0:
        raise EasyQuantError(cnt, "eq_test_plan_sort_segments")
    segs = (C.c_int64 * (7 * max(cnt, 1)))()
    lib().eq_test_plan_sort_segments(*args, segs, cnt, C.byref(region))
    return [tuple(segs[7 * i:7 * i + 7]) for i in range(cnt)], int(region.value)

