"""ctypes binding of the C ABI declared in include/grim_bcr.h.

Argument marshalling only.  Host arrays are NumPy; device buffers are anything
with a ``data_ptr()`` (torch tensors) or a raw integer address.  There is no
CPU fallback: if libgrim_bcr.so is missing, importing a function that needs it
raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np

F32, F16, BF16 = 0, 1, 2
_DT_CODE = {"f32": F32, "f16": F16, "bf16": BF16, F32: F32, F16: F16, BF16: BF16}
_DT_NUMPY = {F32: np.float32, F16: np.float16, BF16: np.uint16}
STATUS_NAMES = ["GRIM_OK", "GRIM_ERR_NULL", "GRIM_ERR_SHAPE", "GRIM_ERR_INDEX", "GRIM_ERR_DTYPE",
                "GRIM_ERR_ALLOC", "GRIM_ERR_DEVICE", "GRIM_ERR_UNSUPPORTED"]

_HERE = os.path.dirname(os.path.abspath(__file__))
_lib = None


class GrimError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = int(status)
        name = STATUS_NAMES[status] if 0 <= status < len(STATUS_NAMES) else str(status)
        super().__init__(f"{where}: {name}")
        self.name = name


class Options(ctypes.Structure):
    _fields_ = [("no_reorder", ctypes.c_int32), ("host_only", ctypes.c_int32),
                ("chunk_rows", ctypes.c_int32), ("reserved", ctypes.c_int32 * 5)]


class View(ctypes.Structure):
    _fields_ = [("M", ctypes.c_int64), ("K", ctypes.c_int64), ("BR", ctypes.c_int32), ("BC", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("reordered", ctypes.c_int32),
                ("nbr", ctypes.c_int64), ("nbc", ctypes.c_int64), ("nb", ctypes.c_int64), ("nnz", ctypes.c_int64),
                ("strip_order", ctypes.c_void_p), ("row_ptr", ctypes.c_void_p), ("row_idx", ctypes.c_void_p),
                ("col_ptr", ctypes.c_void_p), ("col_idx", ctypes.c_void_p), ("blk_ptr", ctypes.c_void_p),
                ("weights", ctypes.c_void_p),
                ("dev_bytes_canonical", ctypes.c_int64), ("dev_bytes_mma", ctypes.c_int64),
                ("dev_bytes_gemv", ctypes.c_int64)]


class BcrcView(ctypes.Structure):
    _fields_ = [("M", ctypes.c_int64), ("K", ctypes.c_int64), ("ngroups", ctypes.c_int64), ("nnz", ctypes.c_int64),
                ("ncols", ctypes.c_int64), ("dtype", ctypes.c_int32),
                ("reorder", ctypes.c_void_p), ("row_offset", ctypes.c_void_p), ("occurrence", ctypes.c_void_p),
                ("column_stride", ctypes.c_void_p), ("compact_column", ctypes.c_void_p), ("weights", ctypes.c_void_p)]


EXPORTS = ["grim_bcr_pack", "grim_bcr_unpack", "grim_bcr_arrays", "grim_bcr_spmm", "grim_bcr_spmm_tuned",
           "grim_bcr_spmv", "grim_bcr_group_create", "grim_bcr_spmv_batched", "grim_bcr_group_free",
           "grim_bcr_free", "grim_status_str", "grim_bcr_spmm_kernel_name",
           "grim_bcr_export_bcrc", "grim_bcrc_arrays", "grim_bcrc_free", "grim_lstm_cell", "grim_bcr_lstm_step", "grim_gru_cell", "grim_bcr_gru_step",
           "grim_bcr_conv2d", "grim_bcr_conv2d_act", "grim_bcr_unpack_layout", "grim_bcr_rnn_step_launches",
           "grim_bcr_rnn_sequence_supported", "grim_bcr_lstm_sequence", "grim_bcr_gru_sequence",
           "grim_bcr_lstm_sequence_noalloc", "grim_bcr_rnn_sequence_batch_supported", "grim_bcr_lstm_sequence_batch",
           "grim_bcr_gru_sequence_batch", "grim_bcr_conv_plan_create", "grim_bcr_conv_plan_free", "grim_bcr_conv2d_plan", "grim_bcr_conv2d_kernel_name"]


def lib_path() -> str:
    """The in-tree library; GRIM_BCR_LIB names another build of it (the sanitizer build of the host code)."""
    return os.environ.get("GRIM_BCR_LIB") or os.path.join(_HERE, "libgrim_bcr.so")


def load_library():
    """Load libgrim_bcr.so (built in-tree by paper_2108_11033_amd/build.py)."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: run `python paper_2108_11033_amd/build.py` "
                          "(there is no CPU fallback)")
    # PyTorch ships its own HIP runtime (same SONAME as the system one).  Two HIP runtimes in
    # one process cannot both own the GPU, so let torch's be loaded first; the library's
    # dependency then binds to it.  Without torch the system runtime is used.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = ctypes.CDLL(path)
    i64, i32, p = ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p
    lib.grim_bcr_pack.argtypes = [p, i32, i64, i64, i64, i32, i32, p, p, p, p, p, ctypes.POINTER(p)]
    lib.grim_bcr_unpack.argtypes = [p, p, i64]
    lib.grim_bcr_unpack_layout.argtypes = [p, i32, p, i64]
    lib.grim_bcr_arrays.argtypes = [p, ctypes.POINTER(View)]
    lib.grim_bcr_spmm.argtypes = [p, p, i64, i64, p, i64, p]
    lib.grim_bcr_spmm_tuned.argtypes = [p, p, i64, i64, p, i64, i32, i32, i32, p]
    lib.grim_bcr_spmv.argtypes = [p, p, i32, i64, p, i64, p]
    lib.grim_bcr_group_create.argtypes = [ctypes.POINTER(p), i32, ctypes.POINTER(p)]
    lib.grim_bcr_spmv_batched.argtypes = [p, p, i64, i32, i64, p, i64, i64, p]
    lib.grim_bcr_group_free.argtypes = [p]
    lib.grim_bcr_free.argtypes = [p]
    lib.grim_status_str.argtypes = [i32]
    lib.grim_bcr_export_bcrc.argtypes = [p, ctypes.POINTER(p)]
    lib.grim_bcrc_arrays.argtypes = [p, ctypes.POINTER(BcrcView)]
    lib.grim_bcrc_free.argtypes = [p]
    lib.grim_bcr_conv2d.argtypes = [p, p, i32, i32, i32, i32, i32, p, i64, p]
    lib.grim_bcr_conv2d_act.argtypes = [p, p, i32, i32, i32, i32, i32, p, i32, p, i32, i64, p]
    lib.grim_lstm_cell.argtypes = [p, i64, p, p, i64, p, i32, i64, p, i64, i64, i32, p]
    lib.grim_bcr_lstm_step.argtypes = [p, p, i32, i64, p, i64, p, p, i64, p, i64, p, i64, p]
    lib.grim_gru_cell.argtypes = [p, i64, p, i64, p, p, p, i64, p, i32, i64, i64, i32, p]
    lib.grim_bcr_gru_step.argtypes = [p, p, p, i64, p, i64, i32, p, i64, p, i64, p, p, p, i64, p, i64, p]
    lib.grim_bcr_spmm_kernel_name.argtypes = [p, p, i64, i64, i32, i32, i32]
    lib.grim_bcr_rnn_step_launches.argtypes = [p, p, i32]
    lib.grim_bcr_rnn_sequence_supported.argtypes = [p, p]
    lib.grim_bcr_lstm_sequence.argtypes = [p, p, i64, i32, p, p, p, p, i64, p, i64, p, ctypes.c_uint32, p]
    lib.grim_bcr_conv_plan_create.argtypes = [p, i32, i32, i32, i32, i32, i32, ctypes.POINTER(p)]
    lib.grim_bcr_conv_plan_free.argtypes = [p]
    lib.grim_bcr_conv2d_kernel_name.argtypes = [p, i32, i32, i32, i32, i32, i32, i32]
    lib.grim_bcr_conv2d_plan.argtypes = [p, p, i32, i64, p, i32, p, i32, i64, i64, p]
    lib.grim_bcr_lstm_sequence_noalloc.argtypes = [p, p, i64, i32, p, p, p, p, i64, p, i64, p, ctypes.c_uint32, p]
    lib.grim_bcr_gru_sequence.argtypes = [p, p, p, i64, i32, p, p, p, p, p, i64, p, i64, p, ctypes.c_uint32, p]
    lib.grim_bcr_rnn_sequence_batch_supported.argtypes = [p, p, i32]
    lib.grim_bcr_lstm_sequence_batch.argtypes = [p, p, i64, i32, i32, p, p, p, p, i64, p, i64, p, ctypes.c_uint32, p]
    lib.grim_bcr_gru_sequence_batch.argtypes = [p, p, p, i64, i32, i32, p, p, p, p, p, i64, p, i64, p, ctypes.c_uint32, p]
    for name in EXPORTS:
        getattr(lib, name).restype = i32
    lib.grim_status_str.restype = ctypes.c_char_p
    lib.grim_bcr_spmm_kernel_name.restype = ctypes.c_char_p
    lib.grim_bcr_conv2d_kernel_name.restype = ctypes.c_char_p
    lib.grim_bcr_free.restype = None
    lib.grim_bcrc_free.restype = None
    lib.grim_bcr_group_free.restype = None
    lib.grim_bcr_conv_plan_free.restype = None
    _lib = lib
    return lib


def _check(status: int, where: str):
    if status != 0:
        raise GrimError(status, where)


def _addr(buf) -> Optional[int]:
    if buf is None:
        return None
    if isinstance(buf, int):
        return buf
    if hasattr(buf, "data_ptr"):
        return int(buf.data_ptr())
    raise TypeError("device buffer must be an int address or expose data_ptr()")


def _np_ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _stream(stream) -> Optional[int]:
    if stream is None:
        return None
    if isinstance(stream, int):
        return stream or None
    return int(stream.cuda_stream) or None


class BcrMatrix:
    """Owner of a packed matrix handle (grim_bcr_matrix*)."""

    def __init__(self, handle: int, lib):
        self._h = ctypes.c_void_p(handle)
        self._lib = lib

    @property
    def handle(self) -> ctypes.c_void_p:
        if not self._h:
            raise ValueError("matrix already freed")
        return self._h

    def view(self) -> View:
        v = View()
        _check(self._lib.grim_bcr_arrays(self.handle, ctypes.byref(v)), "grim_bcr_arrays")
        return v

    def arrays(self) -> dict:
        """Copies of the canonical compact arrays as NumPy arrays."""
        v = self.view()

        def take(addr, count, dtype):
            if count == 0 or not addr:
                return np.zeros(0, dtype=dtype)
            n = count * np.dtype(dtype).itemsize
            return np.frombuffer(ctypes.string_at(addr, n), dtype=dtype).copy()

        row_ptr = take(v.row_ptr, v.nb + 1, np.int32)
        col_ptr = take(v.col_ptr, v.nb + 1, np.int32)
        return {
            "strip_order": take(v.strip_order, v.nbr, np.int32),
            "row_ptr": row_ptr,
            "row_idx": take(v.row_idx, int(row_ptr[-1]), np.uint16),
            "col_ptr": col_ptr,
            "col_idx": take(v.col_idx, int(col_ptr[-1]), np.uint16),
            "blk_ptr": take(v.blk_ptr, v.nb + 1, np.int64),
            "weights": take(v.weights, v.nnz, _DT_NUMPY[v.dtype]),
        }

    def unpack(self) -> np.ndarray:
        v = self.view()
        out = np.empty((v.M, v.K), dtype=_DT_NUMPY[v.dtype])
        _check(self._lib.grim_bcr_unpack(self.handle, _np_ptr(out), v.K), "grim_bcr_unpack")
        return out

    def unpack_layout(self, layout: int) -> np.ndarray:
        """The masked dense matrix decoded from a kernel layout (1 staged SpMM, 2 row-gathering SpMM, 3 SpMV)."""
        v = self.view()
        out = np.empty((v.M, v.K), dtype=_DT_NUMPY[v.dtype])
        _check(self._lib.grim_bcr_unpack_layout(self.handle, layout, _np_ptr(out), v.K), "grim_bcr_unpack_layout")
        return out

    def free(self):
        if self._h:
            self._lib.grim_bcr_free(self._h)
            self._h = ctypes.c_void_p(None)

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


class BcrGroup:
    def __init__(self, handle: int, lib, mats: Sequence[BcrMatrix]):
        self._h = ctypes.c_void_p(handle)
        self._lib = lib
        self._mats = list(mats)     # keep the matrices alive

    @property
    def handle(self):
        return self._h

    @property
    def count(self) -> int:
        return len(self._mats)

    def free(self):
        if self._h:
            self._lib.grim_bcr_group_free(self._h)
            self._h = ctypes.c_void_p(None)

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def pack(W: np.ndarray, dtype, BR: int, BC: int, row_ptr, row_idx, col_ptr, col_idx, *,
         no_reorder: bool = False, host_only: bool = False, chunk_rows: int = 0) -> BcrMatrix:
    """grim_bcr_pack.  ``W`` is a C-contiguous M x K NumPy array in the storage
    type (uint16 bit patterns for bf16)."""
    lib = load_library()
    dt = _DT_CODE[dtype]
    W = np.ascontiguousarray(W)
    if W.dtype != _DT_NUMPY[dt]:
        raise TypeError(f"W must be {_DT_NUMPY[dt]} for dtype {dtype}")
    M, K = W.shape
    row_ptr = np.ascontiguousarray(row_ptr, dtype=np.int32)
    col_ptr = np.ascontiguousarray(col_ptr, dtype=np.int32)
    row_idx = np.ascontiguousarray(row_idx, dtype=np.uint16)
    col_idx = np.ascontiguousarray(col_idx, dtype=np.uint16)
    opt = Options(int(no_reorder), int(host_only), int(chunk_rows))
    out = ctypes.c_void_p()
    st = lib.grim_bcr_pack(_np_ptr(W), dt, M, K, K, BR, BC,
                           _np_ptr(row_ptr), _np_ptr(row_idx), _np_ptr(col_ptr), _np_ptr(col_idx),
                           ctypes.byref(opt), ctypes.byref(out))
    _check(st, "grim_bcr_pack")
    return BcrMatrix(out.value, lib)


def spmm(A: BcrMatrix, X, N: int, ldx: int, Y, ldy: int, stream=None, *,
         tile_n: int = 0, strips_per_wg: int = 0, kernel: int = 0):
    """grim_bcr_spmm / grim_bcr_spmm_tuned: enqueue Y = W_bcr * X."""
    lib = A._lib
    if tile_n or strips_per_wg or kernel:
        st = lib.grim_bcr_spmm_tuned(A.handle, _addr(X), N, ldx, _addr(Y), ldy, tile_n, strips_per_wg,
                                     kernel, _stream(stream))
        _check(st, "grim_bcr_spmm_tuned")
    else:
        _check(lib.grim_bcr_spmm(A.handle, _addr(X), N, ldx, _addr(Y), ldy, _stream(stream)), "grim_bcr_spmm")


def conv2d(A: BcrMatrix, F, Cin: int, H: int, W: int, kh: int, kw: int, Y, ldy: int, stream=None):
    """grim_bcr_conv2d: enqueue the stride-1 "same" convolution of feature map F with the packed filter matrix."""
    _check(A._lib.grim_bcr_conv2d(A.handle, _addr(F), Cin, H, W, kh, kw, _addr(Y), ldy, _stream(stream)), "grim_bcr_conv2d")


def conv2d_act(A: BcrMatrix, F, Cin: int, H: int, W: int, kh: int, kw: int, bias, relu: bool, out, out_dtype, ldo: int,
               stream=None):
    """grim_bcr_conv2d_act: the convolution with bias, rectifier and output rounding in its epilogue."""
    _check(A._lib.grim_bcr_conv2d_act(A.handle, _addr(F), Cin, H, W, kh, kw, _addr(bias), int(bool(relu)), _addr(out),
                                      _DT_CODE[out_dtype], ldo, _stream(stream)), "grim_bcr_conv2d_act")


def rnn_step_launches(A: BcrMatrix, Ah: Optional[BcrMatrix], batch: int) -> int:
    """grim_bcr_rnn_step_launches: kernels per LSTM step of A (Ah None) or GRU step of (A, Ah)."""
    return int(A._lib.grim_bcr_rnn_step_launches(A.handle, Ah.handle if Ah is not None else None, batch))


class ConvPlan:
    """grim_bcr_conv_plan: a packed filter matrix bound to one layer geometry (and a stride); freed with the object.
    Keeps the matrix alive."""

    def __init__(self, A: "BcrMatrix", Cin: int, H: int, W: int, kh: int, kw: int, stride: int = 1):
        self._lib = A._lib
        self.A = A
        self.geometry = (Cin, H, W, kh, kw, stride)
        self.out_hw = ((H + stride - 1) // stride, (W + stride - 1) // stride)
        h = ctypes.c_void_p()
        _check(self._lib.grim_bcr_conv_plan_create(A.handle, Cin, H, W, kh, kw, stride, ctypes.byref(h)),
               "grim_bcr_conv_plan_create")
        self.handle = h

    def __del__(self):
        h, self.handle = getattr(self, "handle", None), None
        if h:
            self._lib.grim_bcr_conv_plan_free(h)


def conv2d_kernel_name(A: "BcrMatrix", Cin: int, H: int, W: int, kh: int, kw: int, batch: int = 1, stride: int = 1) -> str:
    """grim_bcr_conv2d_kernel_name: the kernel a convolution of this geometry runs on."""
    return A._lib.grim_bcr_conv2d_kernel_name(A.handle, Cin, H, W, kh, kw, batch, stride).decode()


def conv2d_plan(plan: ConvPlan, F, batch: int, f_image_stride: int, bias, relu: bool, out, out_dtype, ldo: int,
                out_image_stride: int, stream=None):
    """grim_bcr_conv2d_plan: the planned convolution layer on `batch` images."""
    _check(plan._lib.grim_bcr_conv2d_plan(plan.handle, _addr(F), batch, f_image_stride, _addr(bias), 1 if relu else 0,
                                          _addr(out), _DT_CODE[out_dtype], ldo, out_image_stride, _stream(stream)),
           "grim_bcr_conv2d_plan")


def lstm_cell(gates, ldg: int, bias, c, ldc: int, h, dtype, ldh: int, h32, ldh32: int, H: int, batch: int, stream=None):
    """grim_lstm_cell: enqueue the elementwise part of an LSTM step (c updated in place, h written)."""
    lib = load_library()
    _check(lib.grim_lstm_cell(_addr(gates), ldg, _addr(bias), _addr(c), ldc, _addr(h), _DT_CODE[dtype], ldh,
                              _addr(h32), ldh32, H, batch, _stream(stream)), "grim_lstm_cell")


def lstm_step(A: BcrMatrix, xh, batch: int, ldx: int, gates, ldg: int, bias, c, ldc: int, h, ldh: int,
              h32=None, ldh32: int = 0, stream=None):
    """grim_bcr_lstm_step: gate product of [W_ih | W_hh] with [x; h], then the cell."""
    _check(A._lib.grim_bcr_lstm_step(A.handle, _addr(xh), batch, ldx, _addr(gates), ldg, _addr(bias), _addr(c), ldc,
                                     _addr(h), ldh, _addr(h32), ldh32, _stream(stream)), "grim_bcr_lstm_step")


def rnn_sequence_supported(A: BcrMatrix, Ah: Optional[BcrMatrix] = None, batch: int = 1) -> bool:
    """grim_bcr_rnn_sequence_batch_supported: can the whole-sequence kernel run this LSTM (Ah None) / GRU layer
    on `batch` sequences side by side?"""
    return bool(A._lib.grim_bcr_rnn_sequence_batch_supported(A.handle, Ah.handle if Ah is not None else None, batch))


def lstm_sequence_batch(A: BcrMatrix, xs, ldxs: int, T: int, batch: int, bias, h0, c, hs, ldhs: int, hs32, ldhs32: int,
                        status, max_polls: int = 0, stream=None):
    """grim_bcr_lstm_sequence_batch: T LSTM steps of `batch` sequences in one launch (row t * batch + b)."""
    _check(A._lib.grim_bcr_lstm_sequence_batch(A.handle, _addr(xs), ldxs, T, batch, _addr(bias), _addr(h0), _addr(c),
                                               _addr(hs), ldhs, _addr(hs32), ldhs32, _addr(status), max_polls,
                                               _stream(stream)), "grim_bcr_lstm_sequence_batch")


def gru_sequence_batch(Ai: BcrMatrix, Ah: BcrMatrix, xs, ldxs: int, T: int, batch: int, bias_i, bias_h, h0, h32, hs,
                       ldhs: int, hs32, ldhs32: int, status, max_polls: int = 0, stream=None):
    """grim_bcr_gru_sequence_batch: T GRU steps of `batch` sequences in one launch (row t * batch + b)."""
    _check(Ai._lib.grim_bcr_gru_sequence_batch(Ai.handle, Ah.handle, _addr(xs), ldxs, T, batch, _addr(bias_i), _addr(bias_h),
                                               _addr(h0), _addr(h32), _addr(hs), ldhs, _addr(hs32), ldhs32, _addr(status),
                                               max_polls, _stream(stream)), "grim_bcr_gru_sequence_batch")


def lstm_sequence(A: BcrMatrix, xs, ldxs: int, T: int, bias, h0, c, hs, ldhs: int, hs32, ldhs32: int, status,
                  max_polls: int = 0, stream=None):
    """grim_bcr_lstm_sequence: T LSTM steps in one launch; `status` is a device int32 (0 done, 1 gave up)."""
    _check(A._lib.grim_bcr_lstm_sequence(A.handle, _addr(xs), ldxs, T, _addr(bias), _addr(h0), _addr(c), _addr(hs), ldhs,
                                         _addr(hs32), ldhs32, _addr(status), max_polls, _stream(stream)),
           "grim_bcr_lstm_sequence")


def lstm_sequence_noalloc(A: BcrMatrix, xs, ldxs: int, T: int, bias, h0, c, hs, ldhs: int, hs32, ldhs32: int, status,
                          max_polls: int = 0, stream=None):
    """grim_bcr_lstm_sequence_noalloc: the same sequence with the exchange words in the library's static device array."""
    _check(A._lib.grim_bcr_lstm_sequence_noalloc(A.handle, _addr(xs), ldxs, T, _addr(bias), _addr(h0), _addr(c), _addr(hs),
                                                 ldhs, _addr(hs32), ldhs32, _addr(status), max_polls, _stream(stream)),
           "grim_bcr_lstm_sequence_noalloc")


def gru_sequence(Ai: BcrMatrix, Ah: BcrMatrix, xs, ldxs: int, T: int, bias_i, bias_h, h0, h32, hs, ldhs: int, hs32,
                 ldhs32: int, status, max_polls: int = 0, stream=None):
    """grim_bcr_gru_sequence: T GRU steps in one launch; `status` is a device int32 (0 done, 1 gave up)."""
    _check(Ai._lib.grim_bcr_gru_sequence(Ai.handle, Ah.handle, _addr(xs), ldxs, T, _addr(bias_i), _addr(bias_h), _addr(h0),
                                         _addr(h32), _addr(hs), ldhs, _addr(hs32), ldhs32, _addr(status), max_polls,
                                         _stream(stream)), "grim_bcr_gru_sequence")


def gru_cell(gi, ldgi: int, gh, ldgh: int, bias_i, bias_h, h32, ldh32: int, h, dtype, ldh: int, H: int, batch: int,
             stream=None):
    """grim_gru_cell: enqueue the elementwise part of a GRU step (fp32 state updated in place, h written)."""
    lib = load_library()
    _check(lib.grim_gru_cell(_addr(gi), ldgi, _addr(gh), ldgh, _addr(bias_i), _addr(bias_h), _addr(h32), ldh32,
                             _addr(h), _DT_CODE[dtype], ldh, H, batch, _stream(stream)), "grim_gru_cell")


def gru_step(Ai: BcrMatrix, Ah: BcrMatrix, x, ldx: int, hin, ldhin: int, batch: int, gi, ldgi: int, gh, ldgh: int,
             bias_i, bias_h, h32, ldh32: int, hout, ldhout: int, stream=None):
    """grim_bcr_gru_step: the products W_i x and W_h h, then the cell."""
    _check(Ai._lib.grim_bcr_gru_step(Ai.handle, Ah.handle, _addr(x), ldx, _addr(hin), ldhin, batch, _addr(gi), ldgi,
                                     _addr(gh), ldgh, _addr(bias_i), _addr(bias_h), _addr(h32), ldh32, _addr(hout),
                                     ldhout, _stream(stream)), "grim_bcr_gru_step")


def export_bcrc(A: BcrMatrix) -> dict:
    """grim_bcr_export_bcrc: copies of the paper's six BCRC arrays (plus sizes) as NumPy arrays."""
    lib = A._lib
    h = ctypes.c_void_p()
    _check(lib.grim_bcr_export_bcrc(A.handle, ctypes.byref(h)), "grim_bcr_export_bcrc")
    try:
        v = BcrcView()
        _check(lib.grim_bcrc_arrays(h, ctypes.byref(v)), "grim_bcrc_arrays")

        def arr(ptr, n, dt):
            if n == 0:
                return np.zeros(0, dtype=dt)
            return np.ctypeslib.as_array(ctypes.cast(ptr, ctypes.POINTER(ctypes.c_uint8)), shape=(n * np.dtype(dt).itemsize,)).view(dt).copy()
        wdt = np.float32 if v.dtype == F32 else np.uint16
        return {"M": v.M, "K": v.K, "ngroups": v.ngroups, "nnz": v.nnz,
                "reorder": arr(v.reorder, v.M, np.int32), "row_offset": arr(v.row_offset, v.M + 1, np.int64),
                "occurrence": arr(v.occurrence, v.ngroups + 1, np.int32),
                "column_stride": arr(v.column_stride, v.ngroups + 1, np.int64),
                "compact_column": arr(v.compact_column, v.ncols, np.int32),
                "weights": arr(v.weights, v.nnz, wdt)}
    finally:
        lib.grim_bcrc_free(h)


def spmm_kernel_name(A: BcrMatrix, X, N: int, ldx: int, *, tile_n: int = 0, strips_per_wg: int = 0, kernel: int = 0) -> str:
    """grim_bcr_spmm_kernel_name: the kernel family the same spmm call would launch."""
    return A._lib.grim_bcr_spmm_kernel_name(A.handle, _addr(X), N, ldx, tile_n, strips_per_wg, kernel).decode()


def spmv(A: BcrMatrix, x, batch: int, ldx: int, y, ldy: int, stream=None):
    """grim_bcr_spmv: enqueue y = W_bcr * x for 1..8 right-hand sides."""
    _check(A._lib.grim_bcr_spmv(A.handle, _addr(x), batch, ldx, _addr(y), ldy, _stream(stream)), "grim_bcr_spmv")


def group(mats: Sequence[BcrMatrix]) -> BcrGroup:
    lib = load_library()
    arr = (ctypes.c_void_p * len(mats))(*[m.handle for m in mats])
    out = ctypes.c_void_p()
    _check(lib.grim_bcr_group_create(arr, len(mats), ctypes.byref(out)), "grim_bcr_group_create")
    return BcrGroup(out.value, lib, mats)


def spmv_batched(G: BcrGroup, x, x_stride: int, batch: int, ldx: int, y, y_stride: int, ldy: int, stream=None):
    """grim_bcr_spmv_batched: all products of the group in one launch."""
    st = G._lib.grim_bcr_spmv_batched(G.handle, _addr(x), x_stride, batch, ldx, _addr(y), y_stride, ldy,
                                      _stream(stream))
    _check(st, "grim_bcr_spmv_batched")
