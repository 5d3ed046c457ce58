"""CPU oracle for the MACKO format and its matrix-vector product.

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the
CPU-baseline leg of the benchmark.  The GPU library never imports or links it,
and it imports nothing from the GPU library.

``macko_oracle.c`` holds the arithmetic (encoder, decoder, fp64 products);
this module marshals numpy arrays to it.  ``closed_forms`` holds the paper's
storage formulas (eqs. 2, 4-10).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

from . import closed_forms  # noqa: F401  (re-export)

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "macko_oracle.c")
_LIB = os.path.join(_HERE, "libmacko_oracle.so")
# The mutation tests point this at a deliberately broken copy of the source to
# show that the pins notice; nothing else sets it.
if os.environ.get("MACKO_ORACLE_SRC"):
    _SRC = os.environ["MACKO_ORACLE_SRC"]
    _LIB = os.path.splitext(_SRC)[0] + ".so"
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc.  Building the checker is not using it."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-fvisibility=hidden", "-o", tmp, _SRC, "-lm"]
        )
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build()
    lib = ctypes.CDLL(_LIB)
    P = ctypes.POINTER
    u16p, u8p, u32p = P(ctypes.c_uint16), P(ctypes.c_uint8), P(ctypes.c_uint32)
    i32p, i64p, f64p = P(ctypes.c_int32), P(ctypes.c_int64), P(ctypes.c_double)
    i64, ci = ctypes.c_int64, ctypes.c_int
    lib.oracle_half_to_double_array.argtypes = [u16p, f64p, i64]
    lib.oracle_half_to_double_array.restype = None
    lib.oracle_double_to_half_array.argtypes = [f64p, u16p, i64]
    lib.oracle_double_to_half_array.restype = None
    lib.oracle_alloc_granule.argtypes = [ci]
    lib.oracle_alloc_granule.restype = i64
    lib.oracle_count_entries.argtypes = [u16p, i64, i64, i64, ci, i64p]
    lib.oracle_count_entries.restype = i64
    lib.oracle_encode.argtypes = [u16p, i64, i64, i64, ci, u16p, u8p, u32p, i64]
    lib.oracle_encode.restype = i64
    lib.oracle_decode.argtypes = [u16p, u8p, u32p, i64, i64, ci, u16p, i64]
    lib.oracle_decode.restype = i64
    lib.oracle_unpack.argtypes = [u8p, u32p, i64, ci, i32p, i32p]
    lib.oracle_unpack.restype = None
    lib.oracle_check.argtypes = [u16p, u8p, u32p, i64, i64, ci, i64]
    lib.oracle_check.restype = ci
    lib.oracle_spmv.argtypes = [u16p, u8p, u32p, i64, i64, ci, u16p, f64p, f64p]
    lib.oracle_spmv.restype = None
    lib.oracle_dense_matvec.argtypes = [u16p, i64, i64, i64, u16p, f64p, f64p]
    lib.oracle_dense_matvec.restype = None
    lib.oracle_fp8_to_double_array.argtypes = [u8p, f64p, i64]
    lib.oracle_fp8_to_double_array.restype = None
    lib.oracle_count_entries8.argtypes = [u8p, i64, i64, i64, ci, i64p]
    lib.oracle_count_entries8.restype = i64
    lib.oracle_encode8.argtypes = [u8p, i64, i64, i64, ci, u8p, u8p, u32p, i64]
    lib.oracle_encode8.restype = i64
    lib.oracle_decode8.argtypes = [u8p, u8p, u32p, i64, i64, ci, u8p, i64]
    lib.oracle_decode8.restype = i64
    lib.oracle_spmv8.argtypes = [u8p, u8p, u32p, i64, i64, ci, u16p, f64p, f64p]
    lib.oracle_spmv8.restype = None
    lib.oracle_dense_matvec8.argtypes = [u8p, i64, i64, i64, u16p, f64p, f64p]
    lib.oracle_dense_matvec8.restype = None
    lib.oracle_max_threads.argtypes = []
    lib.oracle_max_threads.restype = ci
    lib.oracle_set_threads.argtypes = [ci]
    lib.oracle_set_threads.restype = None
    _lib = lib
    return lib


def _p(a: np.ndarray, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct))


def _as_u16_matrix(dense) -> np.ndarray:
    a = np.asarray(dense)
    if a.dtype == np.float16:
        a = a.view(np.uint16)
    if a.dtype != np.uint16:
        raise TypeError("dense must be float16 or uint16 (fp16 bit patterns)")
    if a.ndim != 2:
        raise ValueError("dense must be 2-D")
    return np.ascontiguousarray(a)


def _as_u16_vector(x) -> np.ndarray:
    a = np.asarray(x)
    if a.dtype == np.float16:
        a = a.view(np.uint16)
    if a.dtype != np.uint16 or a.ndim != 1:
        raise TypeError("vector must be 1-D float16 or uint16")
    return np.ascontiguousarray(a)


@dataclass
class Encoded:
    """The three arrays of Section 4.1 plus the counts of the storage report."""
    rows: int
    cols: int
    b_delta: int
    nnz: int
    pad_nnz: int
    alloc_nnz: int
    values: np.ndarray     # uint16[alloc_nnz], fp16 bits (uint8[alloc_nnz], E4M3 bits, when b_val == 8)
    deltas: np.ndarray     # uint8[alloc_nnz * b_delta / 8], packed codes (delta - 1)
    row_ptr: np.ndarray    # uint32[rows + 1], entry indices
    b_val: int = 16        # bits per value

    @property
    def padding_entries(self) -> int:
        return self.pad_nnz - self.nnz

    @property
    def values_bytes(self) -> int:
        return self.alloc_nnz * self.b_val // 8

    @property
    def deltas_bytes(self) -> int:
        return self.alloc_nnz * self.b_delta // 8

    @property
    def rowptr_bytes(self) -> int:
        return 4 * (self.rows + 1)

    @property
    def total_bytes(self) -> int:
        return self.values_bytes + self.deltas_bytes + self.rowptr_bytes

    @property
    def dense_bytes(self) -> int:
        return self.rows * self.cols * self.b_val // 8

    @property
    def effd(self) -> float:
        """Eq. 2: storage over the dense footprint R*C*b_val."""
        return self.total_bytes / self.dense_bytes if self.dense_bytes else 0.0


def half_to_double(h) -> np.ndarray:
    a = np.ascontiguousarray(np.asarray(h).view(np.uint16) if np.asarray(h).dtype == np.float16 else h,
                             dtype=np.uint16)
    out = np.empty(a.shape, dtype=np.float64)
    _load().oracle_half_to_double_array(_p(a, ctypes.c_uint16), _p(out, ctypes.c_double), a.size)
    return out


def double_to_half(v) -> np.ndarray:
    a = np.ascontiguousarray(v, dtype=np.float64)
    out = np.empty(a.shape, dtype=np.uint16)
    _load().oracle_double_to_half_array(_p(a, ctypes.c_double), _p(out, ctypes.c_uint16), a.size)
    return out


def alloc_granule(b_delta: int = 4) -> int:
    return int(_load().oracle_alloc_granule(b_delta))


def encode(dense, b_delta: int = 4) -> Encoded:
    """Dense fp16 matrix -> MACKO buffers (Section 4.1, tail padding of 4.5)."""
    lib = _load()
    W = _as_u16_matrix(dense)
    R, C = W.shape
    nnz = ctypes.c_int64(0)
    pad_nnz = lib.oracle_count_entries(_p(W, ctypes.c_uint16), R, C, C, b_delta, ctypes.byref(nnz))
    if pad_nnz < 0:
        raise ValueError("bad arguments to the oracle encoder")
    g = alloc_granule(b_delta)
    alloc = (pad_nnz + g - 1) // g * g
    values = np.empty(alloc, dtype=np.uint16)
    deltas = np.empty(alloc * b_delta // 8, dtype=np.uint8)
    row_ptr = np.empty(R + 1, dtype=np.uint32)
    got = lib.oracle_encode(_p(W, ctypes.c_uint16), R, C, C, b_delta, _p(values, ctypes.c_uint16),
                            _p(deltas, ctypes.c_uint8), _p(row_ptr, ctypes.c_uint32), alloc)
    if got == -2:
        raise OverflowError("entry index does not fit the 32-bit row pointers")
    if got != pad_nnz:
        raise RuntimeError("oracle encoder: count and fill disagree")
    return Encoded(R, C, b_delta, int(nnz.value), int(pad_nnz), int(alloc), values, deltas, row_ptr)


def decode(enc: Encoded) -> np.ndarray:
    """MACKO buffers -> dense fp16 bit matrix (the format is lossless)."""
    out = np.empty((enc.rows, enc.cols), dtype=np.uint16)
    rc = _load().oracle_decode(_p(enc.values, ctypes.c_uint16), _p(enc.deltas, ctypes.c_uint8),
                               _p(enc.row_ptr, ctypes.c_uint32), enc.rows, enc.cols, enc.b_delta,
                               _p(out, ctypes.c_uint16), enc.cols)
    if rc != 0:
        raise ValueError(f"row {-rc - 1} decodes past the last column")
    return out


def unpack(enc: Encoded):
    """Per-entry (delta, column) of the stored entries, as int32 arrays."""
    d = np.zeros(enc.alloc_nnz, dtype=np.int32)
    c = np.zeros(enc.alloc_nnz, dtype=np.int32)
    _load().oracle_unpack(_p(enc.deltas, ctypes.c_uint8), _p(enc.row_ptr, ctypes.c_uint32), enc.rows,
                          enc.b_delta, _p(d, ctypes.c_int32), _p(c, ctypes.c_int32))
    return d[: enc.pad_nnz], c[: enc.pad_nnz]


def check(enc: Encoded) -> int:
    """0 if every structural invariant of a canonical encoding holds."""
    return int(_load().oracle_check(_p(enc.values, ctypes.c_uint16), _p(enc.deltas, ctypes.c_uint8),
                                    _p(enc.row_ptr, ctypes.c_uint32), enc.rows, enc.cols, enc.b_delta,
                                    enc.alloc_nnz))


def spmv(enc: Encoded, x):
    """(y64, abs64): the product from the format buffers in fp64, and
    sum_j |w_ij x_j| per row."""
    xv = _as_u16_vector(x)
    if xv.size != enc.cols:
        raise ValueError("x has the wrong length")
    y = np.empty(enc.rows, dtype=np.float64)
    s = np.empty(enc.rows, dtype=np.float64)
    _load().oracle_spmv(_p(enc.values, ctypes.c_uint16), _p(enc.deltas, ctypes.c_uint8),
                        _p(enc.row_ptr, ctypes.c_uint32), enc.rows, enc.cols, enc.b_delta,
                        _p(xv, ctypes.c_uint16), _p(y, ctypes.c_double), _p(s, ctypes.c_double))
    return y, s


def dense_matvec(dense, x):
    """(y64, abs64): y_i = sum_j W_ij x_j by definition, fp64."""
    W = _as_u16_matrix(dense)
    xv = _as_u16_vector(x)
    if xv.size != W.shape[1]:
        raise ValueError("x has the wrong length")
    y = np.empty(W.shape[0], dtype=np.float64)
    s = np.empty(W.shape[0], dtype=np.float64)
    _load().oracle_dense_matvec(_p(W, ctypes.c_uint16), W.shape[0], W.shape[1], W.shape[1],
                                _p(xv, ctypes.c_uint16), _p(y, ctypes.c_double), _p(s, ctypes.c_double))
    return y, s


# ---- 8-bit values (OCP E4M3 bit patterns, one byte per element) ----------------

def _as_u8_matrix(dense) -> np.ndarray:
    a = np.asarray(dense)
    if a.dtype != np.uint8 or a.ndim != 2:
        raise TypeError("dense must be a 2-D uint8 array of E4M3 bit patterns")
    return np.ascontiguousarray(a)


def fp8_to_double(b) -> np.ndarray:
    a = np.ascontiguousarray(b, dtype=np.uint8)
    out = np.empty(a.shape, dtype=np.float64)
    _load().oracle_fp8_to_double_array(_p(a, ctypes.c_uint8), _p(out, ctypes.c_double), a.size)
    return out


def encode8(dense, b_delta: int = 4) -> Encoded:
    """Dense matrix of 8-bit values -> MACKO buffers with one byte per stored value."""
    lib = _load()
    W = _as_u8_matrix(dense)
    R, C = W.shape
    nnz = ctypes.c_int64(0)
    pad_nnz = lib.oracle_count_entries8(_p(W, ctypes.c_uint8), R, C, C, b_delta, ctypes.byref(nnz))
    if pad_nnz < 0:
        raise ValueError("bad arguments")
    g = alloc_granule(b_delta)
    alloc = (pad_nnz + g - 1) // g * g
    values = np.zeros(max(alloc, 1), dtype=np.uint8)[:alloc]
    deltas = np.zeros(max(alloc * b_delta // 8, 1), dtype=np.uint8)[: alloc * b_delta // 8]
    row_ptr = np.zeros(R + 1, dtype=np.uint32)
    got = lib.oracle_encode8(_p(W, ctypes.c_uint8), R, C, C, b_delta, _p(values, ctypes.c_uint8),
                             _p(deltas, ctypes.c_uint8), _p(row_ptr, ctypes.c_uint32), alloc)
    if got == -2:
        raise OverflowError("entry index does not fit the 32-bit row pointers")
    if got != pad_nnz:
        raise RuntimeError("oracle encoder: count and fill disagree")
    return Encoded(R, C, b_delta, int(nnz.value), int(pad_nnz), int(alloc), values, deltas, row_ptr, 8)


def decode8(enc: Encoded) -> np.ndarray:
    out = np.empty((enc.rows, enc.cols), dtype=np.uint8)
    rc = _load().oracle_decode8(_p(enc.values, ctypes.c_uint8), _p(enc.deltas, ctypes.c_uint8),
                                _p(enc.row_ptr, ctypes.c_uint32), enc.rows, enc.cols, enc.b_delta,
                                _p(out, ctypes.c_uint8), enc.cols)
    if rc != 0:
        raise ValueError(f"row {-rc - 1} decodes past the last column")
    return out


def spmv8(enc: Encoded, x):
    """(y64, abs64) from the format buffers with 8-bit values."""
    xv = _as_u16_vector(x)
    if xv.size != enc.cols or enc.b_val != 8:
        raise ValueError("x has the wrong length or the encoding does not hold 8-bit values")
    y = np.empty(enc.rows, dtype=np.float64)
    s = np.empty(enc.rows, dtype=np.float64)
    _load().oracle_spmv8(_p(enc.values, ctypes.c_uint8), _p(enc.deltas, ctypes.c_uint8),
                         _p(enc.row_ptr, ctypes.c_uint32), enc.rows, enc.cols, enc.b_delta,
                         _p(xv, ctypes.c_uint16), _p(y, ctypes.c_double), _p(s, ctypes.c_double))
    return y, s


def dense_matvec8(dense, x):
    """(y64, abs64): y_i = sum_j W_ij x_j by definition, 8-bit W, fp16 x, fp64 arithmetic."""
    W = _as_u8_matrix(dense)
    xv = _as_u16_vector(x)
    if xv.size != W.shape[1]:
        raise ValueError("x has the wrong length")
    y = np.empty(W.shape[0], dtype=np.float64)
    s = np.empty(W.shape[0], dtype=np.float64)
    _load().oracle_dense_matvec8(_p(W, ctypes.c_uint8), W.shape[0], W.shape[1], W.shape[1],
                                 _p(xv, ctypes.c_uint16), _p(y, ctypes.c_double), _p(s, ctypes.c_double))
    return y, s


def max_threads() -> int:
    return int(_load().oracle_max_threads())


def set_threads(n: int) -> None:
    _load().oracle_set_threads(int(n))
