"""ctypes binding for libmacko.so: same names as the C ABI, argument marshalling only."""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libmacko.so")
_lib = None

EXPORTED_SYMBOLS = [
    "macko_encode", "macko_encode_device", "macko_wrap_device", "macko_encode_ex", "macko_encode_device_ex",
    "macko_wrap_device_ex", "macko_storage_by_code_width", "macko_get_report",
    "macko_device_bytes", "macko_bind_device", "macko_host_buffers", "macko_fetch_device",
    "macko_decode", "macko_encode_fp8", "macko_encode_device_fp8", "macko_wrap_device_fp8", "macko_host_values_fp8", "macko_decode_fp8", "macko_check_device", "macko_columns_device", "macko_decode_device", "macko_spmv", "macko_dense_gemv", "macko_spmv_group", "macko_spmv_many", "macko_spmv_chain", "macko_spmv_chain_static", "macko_chain_status", "macko_dense_gemv_group", "macko_spmm", "macko_destroy", "macko_status_string",
    "macko_last_hip_error", "macko_set_tuning", "macko_get_tuning",
]


MACKO_E_CORRUPT = -7
MACKO_E_WAIT_EXPIRED = -8
MAX_CHAIN_PHASES = 8
MAX_CHAIN_PRODUCTS = 16
CHAIN_WORKSPACE_BYTES = 8192


class MackoError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = status_string(status)
        if status == -6:
            msg += f" (hipError {load_library().macko_last_hip_error()})"
        super().__init__(f"{where}: {msg} [{status}]")


class _CReport(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int64) for n in (
        "rows", "cols", "nnz", "pad_nnz", "alloc_nnz", "padding_entries", "empty_rows",
        "max_row_entries", "values_bytes", "deltas_bytes", "rowptr_bytes", "total_bytes",
        "dense_bytes")] + [(n, ctypes.c_double) for n in (
            "density", "effd", "effd_best", "effd_expected", "effd_worst")] + [
        ("b_val", ctypes.c_int32), ("b_delta", ctypes.c_int32)]


@dataclass
class Report:
    rows: int
    cols: int
    nnz: int
    pad_nnz: int
    alloc_nnz: int
    padding_entries: int
    empty_rows: int
    max_row_entries: int
    values_bytes: int
    deltas_bytes: int
    rowptr_bytes: int
    total_bytes: int
    dense_bytes: int
    density: float
    effd: float
    effd_best: float
    effd_expected: float
    effd_worst: float
    b_val: int
    b_delta: int

    @classmethod
    def _from_c(cls, c: _CReport) -> "Report":
        return cls(**{name: getattr(c, name) for name, _ in _CReport._fields_})


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libmacko.so.  There is no fallback: a missing library is an error."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_2511_13061_amd.build` "
            "(or __graft_entry__.build()); there is no CPU fallback")
    # PyTorch ships its own copy of the HIP runtime.  When it is going to be used in this process it has
    # to be loaded before this library, so that both bind to the same runtime: the other order leaves
    # the process without a visible device (hipErrorNoDevice from the first call that touches the GPU).
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i64, ci = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
    i64p = ctypes.POINTER(i64)
    rp = ctypes.POINTER(_CReport)
    hp = ctypes.POINTER(vp)
    lib.macko_encode.argtypes = [vp, i64, i64, i64, hp, rp]
    lib.macko_encode_device.argtypes = [vp, i64, i64, i64, vp, hp, rp]
    lib.macko_wrap_device.argtypes = [i64, i64, i64, vp, vp, vp, hp]
    lib.macko_encode_ex.argtypes = [vp, i64, i64, i64, ci, hp, rp]
    lib.macko_encode_device_ex.argtypes = [vp, i64, i64, i64, ci, vp, hp, rp]
    lib.macko_wrap_device_ex.argtypes = [i64, i64, i64, ci, vp, vp, vp, hp]
    lib.macko_storage_by_code_width.argtypes = [vp, i64, i64, i64, i64p, ctypes.POINTER(ci)]
    lib.macko_get_report.argtypes = [vp, rp]
    lib.macko_device_bytes.argtypes = [vp, i64p, i64p, i64p]
    lib.macko_bind_device.argtypes = [vp, vp, vp, vp, vp]
    lib.macko_host_buffers.argtypes = [vp, hp, hp, hp]
    lib.macko_fetch_device.argtypes = [vp, vp, vp, vp]
    lib.macko_decode.argtypes = [vp, vp, i64]
    lib.macko_columns_device.argtypes = [vp, vp, vp]
    lib.macko_encode_fp8.argtypes = [vp, i64, i64, i64, hp, rp]
    lib.macko_host_values_fp8.argtypes = [vp, hp]
    lib.macko_encode_device_fp8.argtypes = [vp, i64, i64, i64, vp, hp, rp]
    lib.macko_wrap_device_fp8.argtypes = [i64, i64, i64, vp, vp, vp, hp]
    lib.macko_decode_fp8.argtypes = [vp, vp, i64]
    lib.macko_check_device.argtypes = [vp, vp, i64p]
    lib.macko_decode_device.argtypes = [vp, vp, i64, vp]
    lib.macko_spmv.argtypes = [vp, vp, vp, vp]
    lib.macko_dense_gemv.argtypes = [vp, i64, i64, i64, vp, vp, vp]
    vpp = ctypes.POINTER(vp)
    lib.macko_spmv_group.argtypes = [ci, vpp, vpp, vpp, vp]
    lib.macko_spmv_many.argtypes = [i64, vpp, vpp, vpp, vp]
    lib.macko_spmv_chain.argtypes = [ci, ctypes.POINTER(ci), vpp, vpp, vpp, vp, i64, vp]
    lib.macko_spmv_chain_static.argtypes = [ci, ctypes.POINTER(ci), vpp, vpp, vpp, vp]
    lib.macko_chain_status.argtypes = [vp, vp, ctypes.POINTER(ci)]
    lib.macko_dense_gemv_group.argtypes = [ci, vpp, i64p, i64p, i64p, vpp, vpp, vp]
    lib.macko_spmm.argtypes = [vp, ci, vp, i64, vp, i64, vp]
    lib.macko_destroy.argtypes = [vp]
    lib.macko_destroy.restype = None
    lib.macko_status_string.argtypes = [ci]
    lib.macko_status_string.restype = ctypes.c_char_p
    lib.macko_last_hip_error.argtypes = []
    lib.macko_set_tuning.argtypes = [ctypes.c_char_p, i64]
    lib.macko_get_tuning.argtypes = [ctypes.c_char_p, i64p]
    for name in EXPORTED_SYMBOLS:
        fn = getattr(lib, name)
        if name not in ("macko_destroy", "macko_status_string"):
            fn.restype = ci
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load_library().macko_status_string(int(status)).decode()


def _check(status: int, where: str) -> None:
    if status != 0:
        raise MackoError(status, where)


def set_tuning(name: str, value: int) -> None:
    _check(load_library().macko_set_tuning(name.encode(), int(value)), f"macko_set_tuning({name})")


def get_tuning(name: str) -> int:
    v = ctypes.c_int64(0)
    _check(load_library().macko_get_tuning(name.encode(), ctypes.byref(v)), f"macko_get_tuning({name})")
    return int(v.value)


def _host_u16_matrix(dense) -> np.ndarray:
    a = np.asarray(dense)
    if a.dtype == np.float16:
        a = a.view(np.uint16)
    if a.dtype != np.uint16 or a.ndim != 2:
        raise TypeError("dense must be a 2-D float16 / uint16 array")
    if a.size and (a.strides[1] != 2 or a.strides[0] % 2 != 0 or a.strides[0] < 2 * a.shape[1]):
        a = np.ascontiguousarray(a)
    return a


def _stream_ptr(stream) -> int:
    if stream is None:
        import torch
        return int(torch.cuda.current_stream().cuda_stream)
    if isinstance(stream, int):
        return stream
    return int(stream.cuda_stream)


def _dev_ptr(t) -> int:
    return int(t.data_ptr())


class MackoMatrix:
    """Owner of a macko_handle_t (and of the torch tensors bound to it)."""

    def __init__(self, handle: int, report: Optional[Report]):
        self._h = ctypes.c_void_p(handle)
        self.report = report
        self._keep = []          # torch tensors that back the device arrays

    # -- lifetime ---------------------------------------------------------
    def destroy(self) -> None:
        if self._h:
            load_library().macko_destroy(self._h)
            self._h = ctypes.c_void_p(None)
            self._keep = []

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    @property
    def rows(self) -> int:
        return self.get_report().rows

    @property
    def cols(self) -> int:
        return self.get_report().cols

    # -- C ABI calls ------------------------------------------------------
    def get_report(self) -> Report:
        c = _CReport()
        _check(load_library().macko_get_report(self._h, ctypes.byref(c)), "macko_get_report")
        return Report._from_c(c)

    def device_bytes(self):
        a, b, c = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64()
        _check(load_library().macko_device_bytes(self._h, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c)),
               "macko_device_bytes")
        return int(a.value), int(b.value), int(c.value)

    def bind_device(self, values_dev, deltas_dev, rowptr_dev, stream=None) -> None:
        """values_dev / deltas_dev / rowptr_dev: torch uint8 CUDA tensors of at
        least device_bytes() bytes."""
        _check(load_library().macko_bind_device(self._h, _dev_ptr(values_dev), _dev_ptr(deltas_dev),
                                                _dev_ptr(rowptr_dev), _stream_ptr(stream)),
               "macko_bind_device")
        self._keep = [values_dev, deltas_dev, rowptr_dev]

    def to_device(self, device="cuda", stream=None) -> "MackoMatrix":
        """Allocate torch device memory for the three arrays and bind it."""
        import torch
        vb, db, rb = self.device_bytes()
        bufs = [torch.empty(max(n, 16), dtype=torch.uint8, device=device) for n in (vb, db, rb)]
        self.bind_device(*bufs, stream=stream)
        return self

    def device_buffers(self):
        return list(self._keep)

    def host_buffers(self):
        """Copies of the host arrays as numpy (values u16, or u8 for 8-bit values; deltas u8, row_ptr u32)."""
        v, d, r = ctypes.c_void_p(), ctypes.c_void_p(), ctypes.c_void_p()
        rep = self.get_report()
        if rep.b_val == 8:
            _check(load_library().macko_host_buffers(self._h, None, ctypes.byref(d), ctypes.byref(r)),
                   "macko_host_buffers")
            _check(load_library().macko_host_values_fp8(self._h, ctypes.byref(v)), "macko_host_values_fp8")
        else:
            _check(load_library().macko_host_buffers(self._h, ctypes.byref(v), ctypes.byref(d), ctypes.byref(r)),
                   "macko_host_buffers")
        def grab(ptr, nbytes, dtype):
            if nbytes == 0:
                return np.zeros(0, dtype=dtype)
            raw = (ctypes.c_uint8 * nbytes).from_address(ptr.value)
            return np.frombuffer(raw, dtype=dtype).copy()
        return (grab(v, rep.values_bytes, np.uint8 if rep.b_val == 8 else np.uint16),
                grab(d, rep.deltas_bytes, np.uint8), grab(r, rep.rowptr_bytes, np.uint32))

    def fetch_device(self):
        """Device arrays copied back to numpy (values u16, deltas u8, row_ptr u32)."""
        vb, db, rb = self.device_bytes()
        v = np.zeros(vb, dtype=np.uint8) if self.get_report().b_val == 8 else np.zeros(vb // 2, dtype=np.uint16)
        d = np.zeros(db, dtype=np.uint8)
        r = np.zeros(rb // 4, dtype=np.uint32)
        _check(load_library().macko_fetch_device(self._h, v.ctypes.data, d.ctypes.data, r.ctypes.data),
               "macko_fetch_device")
        return v, d, r

    def decode(self) -> np.ndarray:
        rep = self.get_report()
        if rep.b_val == 8:
            out = np.empty((rep.rows, rep.cols), dtype=np.uint8)
            _check(load_library().macko_decode_fp8(self._h, out.ctypes.data, rep.cols), "macko_decode_fp8")
            return out
        out = np.empty((rep.rows, rep.cols), dtype=np.uint16)
        _check(load_library().macko_decode(self._h, out.ctypes.data, rep.cols), "macko_decode")
        return out

    def check_device(self, stream=None):
        """macko_check_device: None if the bound arrays are a consistent encoding, else the first bad row."""
        bad = ctypes.c_int64(-1)
        st = load_library().macko_check_device(self._h, _stream_ptr(stream), ctypes.byref(bad))
        if st == MACKO_E_CORRUPT:
            return int(bad.value)
        _check(st, "macko_check_device")
        return None

    def columns_device(self, cols_dev=None, stream=None):
        """macko_columns_device: int32 column index of every stored entry (torch CUDA tensor [alloc_nnz])."""
        import torch
        rep = self.get_report()
        if cols_dev is None:
            cols_dev = torch.full((max(int(rep.alloc_nnz), 1),), -1, dtype=torch.int32, device="cuda")
        _check(load_library().macko_columns_device(self._h, _dev_ptr(cols_dev), _stream_ptr(stream)),
               "macko_columns_device")
        return cols_dev

    def decode_device(self, dense_dev=None, stream=None):
        """macko_decode_device: the dense matrix back, as a torch CUDA tensor [rows, cols] (float16, or
        uint8 bit patterns for a matrix with 8-bit values)."""
        import torch
        if dense_dev is None:
            dt = torch.uint8 if self.get_report().b_val == 8 else torch.float16
            dense_dev = torch.empty((self.rows, self.cols), dtype=dt, device="cuda")
        if dense_dev.dim() != 2 or (dense_dev.shape[1] > 1 and dense_dev.stride(1) != 1):
            raise ValueError("dense_dev must be a row-major [rows, >= cols] tensor")
        ld = dense_dev.stride(0) if dense_dev.shape[0] > 1 else max(dense_dev.shape[1], 1)
        _check(load_library().macko_decode_device(self._h, _dev_ptr(dense_dev), ld, _stream_ptr(stream)),
               "macko_decode_device")
        return dense_dev

    def spmv(self, x_dev, y_dev=None, stream=None):
        """y = W x.  x_dev: torch float16 CUDA tensor [cols]; returns y_dev [rows]."""
        import torch
        if y_dev is None:
            y_dev = torch.empty(self.rows, dtype=torch.float16, device=x_dev.device)
        _check(load_library().macko_spmv(self._h, _dev_ptr(x_dev), _dev_ptr(y_dev), _stream_ptr(stream)),
               "macko_spmv")
        return y_dev

    def spmm(self, X_dev, Y_dev=None, stream=None):
        """Y[b] = W X[b] for a torch float16 CUDA matrix X_dev [batch, cols]; returns [batch, rows]."""
        import torch
        if X_dev.dim() != 2 or X_dev.stride(1) != 1:
            raise ValueError("X_dev must be a row-major [batch, cols] tensor")
        batch = X_dev.shape[0]
        if Y_dev is None:
            Y_dev = torch.empty((batch, self.rows), dtype=torch.float16, device=X_dev.device)
        _check(load_library().macko_spmm(self._h, batch, _dev_ptr(X_dev), X_dev.stride(0) if batch > 1 else max(X_dev.shape[1], 1),
                                         _dev_ptr(Y_dev), Y_dev.stride(0) if batch > 1 else max(Y_dev.shape[1], 1),
                                         _stream_ptr(stream)), "macko_spmm")
        return Y_dev

    def spmv_raw(self, x_ptr: int, y_ptr: int, stream_ptr: int) -> int:
        """Unchecked call for timing loops; returns the status."""
        return load_library().macko_spmv(self._h, x_ptr, y_ptr, stream_ptr)


def encode(dense, b_delta: int = 4) -> MackoMatrix:
    """macko_encode / macko_encode_ex on a host fp16 matrix (numpy float16 or uint16 bits)."""
    a = _host_u16_matrix(dense)
    h = ctypes.c_void_p()
    rep = _CReport()
    ld = a.strides[0] // 2 if a.size else a.shape[1]      # numpy reports zero strides for empty arrays
    if b_delta == 4:
        _check(load_library().macko_encode(a.ctypes.data, a.shape[0], a.shape[1], ld,
                                           ctypes.byref(h), ctypes.byref(rep)), "macko_encode")
    else:
        _check(load_library().macko_encode_ex(a.ctypes.data, a.shape[0], a.shape[1], ld, int(b_delta),
                                              ctypes.byref(h), ctypes.byref(rep)), "macko_encode_ex")
    return MackoMatrix(h.value, Report._from_c(rep))


def storage_by_code_width(dense):
    """macko_storage_by_code_width: ({1: bytes, 2: bytes, 4: bytes, 8: bytes}, best width) for a host fp16 matrix."""
    a = _host_u16_matrix(dense)
    ld = a.strides[0] // 2 if a.size else a.shape[1]
    out = (ctypes.c_int64 * 4)()
    best = ctypes.c_int(0)
    _check(load_library().macko_storage_by_code_width(a.ctypes.data, a.shape[0], a.shape[1], ld, out,
                                                      ctypes.byref(best)), "macko_storage_by_code_width")
    return {1: out[0], 2: out[1], 4: out[2], 8: out[3]}, best.value


def encode_fp8(dense) -> MackoMatrix:
    """macko_encode_fp8 on a host matrix of 8-bit values (numpy uint8, OCP E4M3 bit patterns)."""
    a = np.asarray(dense)
    if a.dtype != np.uint8 or a.ndim != 2:
        raise TypeError("dense must be a 2-D uint8 array of E4M3 bit patterns")
    if a.size and a.strides[1] != 1:
        a = np.ascontiguousarray(a)
    h = ctypes.c_void_p()
    rep = _CReport()
    ld = a.strides[0] if a.size else a.shape[1]
    _check(load_library().macko_encode_fp8(a.ctypes.data, a.shape[0], a.shape[1], ld,
                                           ctypes.byref(h), ctypes.byref(rep)), "macko_encode_fp8")
    return MackoMatrix(h.value, Report._from_c(rep))


def encode_device_fp8(dense_dev, stream=None) -> MackoMatrix:
    """macko_encode_device_fp8 on a torch uint8 CUDA matrix of E4M3 bit patterns (row-major)."""
    if dense_dev.dim() != 2 or (dense_dev.shape[1] > 1 and dense_dev.stride(1) != 1):
        raise ValueError("dense_dev must be a row-major 2-D tensor")
    if dense_dev.element_size() != 1:
        raise TypeError("dense_dev must hold one byte per element")
    h = ctypes.c_void_p()
    rep = _CReport()
    ld = dense_dev.stride(0) if dense_dev.shape[0] > 1 else max(dense_dev.shape[1], 1)
    _check(load_library().macko_encode_device_fp8(_dev_ptr(dense_dev), dense_dev.shape[0], dense_dev.shape[1], ld,
                                                  _stream_ptr(stream), ctypes.byref(h), ctypes.byref(rep)),
           "macko_encode_device_fp8")
    return MackoMatrix(h.value, Report._from_c(rep))


def encode_device(dense_dev, stream=None, b_delta: int = 4) -> MackoMatrix:
    """macko_encode_device / macko_encode_device_ex on a torch float16 CUDA matrix (row-major)."""
    if dense_dev.dim() != 2 or dense_dev.stride(1) != 1:
        raise ValueError("dense_dev must be a row-major 2-D tensor")
    h = ctypes.c_void_p()
    rep = _CReport()
    if b_delta == 4:
        _check(load_library().macko_encode_device(_dev_ptr(dense_dev), dense_dev.shape[0], dense_dev.shape[1],
                                                  dense_dev.stride(0), _stream_ptr(stream), ctypes.byref(h),
                                                  ctypes.byref(rep)), "macko_encode_device")
    else:
        _check(load_library().macko_encode_device_ex(_dev_ptr(dense_dev), dense_dev.shape[0], dense_dev.shape[1],
                                                     dense_dev.stride(0), int(b_delta), _stream_ptr(stream),
                                                     ctypes.byref(h), ctypes.byref(rep)), "macko_encode_device_ex")
    return MackoMatrix(h.value, Report._from_c(rep))


def wrap_device(rows: int, cols: int, pad_nnz: int, values_dev, deltas_dev, rowptr_dev,
                b_delta: int = 4) -> MackoMatrix:
    """macko_wrap_device / macko_wrap_device_ex: adopt device arrays that already hold an encoding."""
    h = ctypes.c_void_p()
    if b_delta == 4:
        _check(load_library().macko_wrap_device(rows, cols, pad_nnz, _dev_ptr(values_dev), _dev_ptr(deltas_dev),
                                                _dev_ptr(rowptr_dev), ctypes.byref(h)), "macko_wrap_device")
    else:
        _check(load_library().macko_wrap_device_ex(rows, cols, pad_nnz, int(b_delta), _dev_ptr(values_dev),
                                                   _dev_ptr(deltas_dev), _dev_ptr(rowptr_dev), ctypes.byref(h)),
               "macko_wrap_device_ex")
    m = MackoMatrix(h.value, None)
    m._keep = [values_dev, deltas_dev, rowptr_dev]
    return m


def wrap_device_fp8(rows: int, cols: int, pad_nnz: int, values_dev, deltas_dev, rowptr_dev) -> MackoMatrix:
    """macko_wrap_device_fp8: adopt device arrays that hold an encoding with 8-bit values."""
    h = ctypes.c_void_p()
    _check(load_library().macko_wrap_device_fp8(rows, cols, pad_nnz, _dev_ptr(values_dev), _dev_ptr(deltas_dev),
                                                _dev_ptr(rowptr_dev), ctypes.byref(h)), "macko_wrap_device_fp8")
    m = MackoMatrix(h.value, None)
    m._keep = [values_dev, deltas_dev, rowptr_dev]
    return m


def dense_gemv(W_dev, x_dev, y_dev=None, stream=None):
    """macko_dense_gemv: y = W x for a row-major fp16 CUDA matrix."""
    import torch
    if W_dev.dim() != 2 or W_dev.stride(1) != 1:
        raise ValueError("W_dev must be a row-major 2-D tensor")
    if y_dev is None:
        y_dev = torch.empty(W_dev.shape[0], dtype=torch.float16, device=W_dev.device)
    _check(load_library().macko_dense_gemv(_dev_ptr(W_dev), W_dev.shape[0], W_dev.shape[1], W_dev.stride(0),
                                           _dev_ptr(x_dev), _dev_ptr(y_dev), _stream_ptr(stream)),
           "macko_dense_gemv")
    return y_dev


class SpmvGroup:
    """Pre-marshalled arguments of macko_spmv_group for a fixed set of products."""

    def __init__(self, matrices, xs, ys):
        n = len(matrices)
        self.n = n
        self._keep = (list(matrices), list(xs), list(ys))
        VP = ctypes.c_void_p * n
        self._h = VP(*[m._h.value for m in matrices])
        self._x = VP(*[_dev_ptr(x) for x in xs])
        self._y = VP(*[_dev_ptr(y) for y in ys])

    def launch_raw(self, stream_ptr: int) -> int:
        return load_library().macko_spmv_group(self.n, self._h, self._x, self._y, stream_ptr)

    def launch(self, stream=None) -> None:
        _check(self.launch_raw(_stream_ptr(stream)), "macko_spmv_group")


class SpmvMany:
    """Pre-marshalled arguments of macko_spmv_many: any number of independent products."""

    def __init__(self, matrices, xs, ys):
        n = len(matrices)
        self.n = n
        self._keep = (list(matrices), list(xs), list(ys))
        VP = ctypes.c_void_p * max(n, 1)
        self._h = VP(*[m._h.value for m in matrices])
        self._x = VP(*[_dev_ptr(x) for x in xs])
        self._y = VP(*[_dev_ptr(y) for y in ys])

    def launch_raw(self, stream_ptr: int) -> int:
        return load_library().macko_spmv_many(self.n, self._h, self._x, self._y, stream_ptr)

    def launch(self, stream=None) -> None:
        _check(self.launch_raw(_stream_ptr(stream)), "macko_spmv_many")


class SpmvChain:
    """Pre-marshalled arguments of macko_spmv_chain: `phases` is a list of phases, each a list of
    (matrix, x, y); phase p + 1 runs after phase p inside one launch.  `workspace` is a zeroed uint8
    device tensor of CHAIN_WORKSPACE_BYTES, 256-byte aligned (chain_workspace() makes one)."""

    def __init__(self, phases, workspace=None):
        """workspace None: macko_spmv_chain_static (the library's own scratch, nothing to provide)."""
        flat = [item for ph in phases for item in ph]
        n = len(flat)
        self.n_phases = len(phases)
        self._keep = (flat, workspace)
        self._sizes = (ctypes.c_int * max(self.n_phases, 1))(*[len(ph) for ph in phases])
        VP = ctypes.c_void_p * max(n, 1)
        self._h = VP(*[m._h.value for m, _, _ in flat])
        self._x = VP(*[_dev_ptr(x) for _, x, _ in flat])
        self._y = VP(*[_dev_ptr(y) for _, _, y in flat])
        self._ws = _dev_ptr(workspace) if workspace is not None else None
        self._ws_bytes = int(workspace.numel() * workspace.element_size()) if workspace is not None else 0

    def launch_raw(self, stream_ptr: int) -> int:
        if self._ws is None:
            return load_library().macko_spmv_chain_static(self.n_phases, self._sizes, self._h, self._x, self._y,
                                                          stream_ptr)
        return load_library().macko_spmv_chain(self.n_phases, self._sizes, self._h, self._x, self._y, self._ws,
                                               self._ws_bytes, stream_ptr)

    def launch(self, stream=None) -> None:
        _check(self.launch_raw(_stream_ptr(stream)), "macko_spmv_chain")

    def status(self, stream=None):
        """macko_chain_status for this chain's workspace: (status, failed_phase)."""
        return chain_status(self._keep[1], stream)


def chain_workspace(device="cuda"):
    """A zeroed workspace for macko_spmv_chain (torch allocations are 256-byte aligned or better)."""
    import torch
    return torch.zeros(CHAIN_WORKSPACE_BYTES, dtype=torch.uint8, device=device)


def chain_status(workspace, stream=None):
    """macko_chain_status: (0, -1) or (MACKO_E_WAIT_EXPIRED, phase whose inputs were not ready)."""
    phase = ctypes.c_int(-1)
    ws = _dev_ptr(workspace) if workspace is not None else None
    st = load_library().macko_chain_status(ws, _stream_ptr(stream), ctypes.byref(phase))
    if st not in (0, MACKO_E_WAIT_EXPIRED):
        _check(st, "macko_chain_status")
    return st, phase.value


class GemvGroup:
    """Pre-marshalled arguments of macko_dense_gemv_group."""

    def __init__(self, Ws, xs, ys):
        n = len(Ws)
        self.n = n
        self._keep = (list(Ws), list(xs), list(ys))
        VP = ctypes.c_void_p * n
        I64 = ctypes.c_int64 * n
        self._W = VP(*[_dev_ptr(W) for W in Ws])
        self._rows = I64(*[W.shape[0] for W in Ws])
        self._cols = I64(*[W.shape[1] for W in Ws])
        self._ld = I64(*[W.stride(0) for W in Ws])
        self._x = VP(*[_dev_ptr(x) for x in xs])
        self._y = VP(*[_dev_ptr(y) for y in ys])

    def launch_raw(self, stream_ptr: int) -> int:
        return load_library().macko_dense_gemv_group(self.n, self._W, self._rows, self._cols, self._ld,
                                                     self._x, self._y, stream_ptr)

    def launch(self, stream=None) -> None:
        _check(self.launch_raw(_stream_ptr(stream)), "macko_dense_gemv_group")


def spmv_group(matrices, xs, ys=None, stream=None):
    """macko_spmv_group: independent products y_i = W_i x_i in one launch."""
    import torch
    if ys is None:
        ys = [torch.empty(m.rows, dtype=torch.float16, device=x.device) for m, x in zip(matrices, xs)]
    SpmvGroup(matrices, xs, ys).launch(stream)
    return ys


def dense_gemv_group(Ws, xs, ys=None, stream=None):
    """macko_dense_gemv_group."""
    import torch
    if ys is None:
        ys = [torch.empty(W.shape[0], dtype=torch.float16, device=W.device) for W in Ws]
    GemvGroup(Ws, xs, ys).launch(stream)
    return ys
