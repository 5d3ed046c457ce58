"""Seeded synthetic inputs with the shapes and sparsity structure of the
paper's pruned-LLM workloads (Section 5.1, Appendix D).

This package only draws inputs.  It contains none of the format's or the
product's arithmetic, and it is the one module that both the CPU oracle's
tests and the GPU library's tests may share.

Matrices and vectors are returned as ``numpy.uint16`` arrays holding fp16 bit
patterns (view them with ``.view(numpy.float16)``).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

BASE_SEED = 251113061

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gen.c")
_LIB = os.path.join(_HERE, "libmacko_workloads.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile gen.c with gcc (host only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-fvisibility=hidden", "-o", tmp, _SRC, "-lm"]
        )
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        u16p = ctypes.POINTER(ctypes.c_uint16)
        i64 = ctypes.c_int64
        u64 = ctypes.c_uint64
        dbl = ctypes.c_double
        lib.wl_normal_f16.argtypes = [u16p, i64, dbl, u64, u64, ctypes.c_int]
        lib.wl_normal_f16.restype = None
        lib.wl_rows_exact.argtypes = [u16p, i64, i64, i64, ctypes.POINTER(i64), dbl, u64, u64, i64]
        lib.wl_rows_exact.restype = None
        lib.wl_bernoulli.argtypes = [u16p, i64, i64, i64, dbl, dbl, u64, u64, i64]
        lib.wl_bernoulli.restype = None
        lib.wl_uniforms.argtypes = [ctypes.POINTER(dbl), i64, u64, u64]
        lib.wl_uniforms.restype = None
        _lib = lib
    return _lib


def _u16p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16))


# --------------------------------------------------------------------------
# primitives
# --------------------------------------------------------------------------

def normal_f16(n: int, sigma: float, seed: int, stream: int, nonzero: bool = False) -> np.ndarray:
    """n draws of N(0, sigma) rounded to fp16 (round to nearest even)."""
    out = np.empty(int(n), dtype=np.uint16)
    _load().wl_normal_f16(_u16p(out), int(n), float(sigma), seed, stream, int(nonzero))
    return out


def rows_exact(rows: int, cols: int, keep, sigma: float, seed: int, stream: int) -> np.ndarray:
    """rows x cols matrix; row r keeps exactly keep[r] uniformly random
    positions with N(0, sigma) fp16 values that are never +-0."""
    keep = np.ascontiguousarray(np.broadcast_to(np.asarray(keep, dtype=np.int64), (rows,)))
    out = np.empty((rows, cols), dtype=np.uint16)
    _load().wl_rows_exact(_u16p(out), rows, cols, cols,
                          keep.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)),
                          float(sigma), seed, stream, 0)
    return out


def bernoulli(rows: int, cols: int, density: float, sigma: float, seed: int, stream: int) -> np.ndarray:
    """rows x cols matrix; each cell kept independently with probability
    ``density`` (the assumption behind the expected-case formula, eq. 10)."""
    out = np.empty((rows, cols), dtype=np.uint16)
    _load().wl_bernoulli(_u16p(out), rows, cols, cols, float(density), float(sigma), seed, stream, 0)
    return out


def uniforms(n: int, seed: int, stream: int) -> np.ndarray:
    out = np.empty(int(n), dtype=np.float64)
    _load().wl_uniforms(out.ctypes.data_as(ctypes.POINTER(ctypes.c_double)), int(n), seed, stream)
    return out


def x_vector(cols: int, seed: int = BASE_SEED, stream: int = 0) -> np.ndarray:
    """Activation vector: N(0,1) rounded to fp16."""
    return normal_f16(cols, 1.0, seed, 0x7800_0000 + stream)


# --------------------------------------------------------------------------
# the five workload families
# --------------------------------------------------------------------------

@dataclass
class Case:
    name: str
    W: np.ndarray      # uint16 [rows, cols], fp16 bits
    x: np.ndarray      # uint16 [cols], fp16 bits
    note: str = ""

    @property
    def rows(self) -> int:
        return self.W.shape[0]

    @property
    def cols(self) -> int:
        return self.W.shape[1]


def half_row_matrix(rows: int, cols: int, stream: int, sparsity: float = 0.5, sigma: float = 0.02,
                    seed: int = BASE_SEED) -> np.ndarray:
    """Exactly round((1-sparsity)*cols) kept cells in every row (the structure a
    per-output pruner such as Wanda produces)."""
    keep = int(round((1.0 - sparsity) * cols))
    return rows_exact(rows, cols, keep, sigma, seed, stream)


def config1(seed: int = BASE_SEED) -> Case:
    """512 x 512, exactly 50 % per row, N(0, 0.02)."""
    return Case("c1_512x512_s50", half_row_matrix(512, 512, 100, seed=seed), x_vector(512, seed, 100))


LLAMA2_7B_SHAPES = [("qkvo", 4096, 4096), ("gate_up", 11008, 4096), ("down", 4096, 11008)]
LLAMA2_7B_LAYER = [("qkvo", 4), ("gate_up", 2), ("down", 1)]
LLAMA2_13B_SHAPES = [("qkvo", 5120, 5120), ("gate_up", 13824, 5120), ("down", 5120, 13824)]
LLAMA2_13B_LAYER = [("qkvo", 4), ("gate_up", 2), ("down", 1)]


def config2(seed: int = BASE_SEED):
    """The three Llama2-7B linear-layer shapes at exactly 50 % per row."""
    for i, (tag, r, c) in enumerate(LLAMA2_7B_SHAPES):
        yield Case(f"c2_{tag}_{r}x{c}_s50", half_row_matrix(r, c, 200 + i, seed=seed),
                   x_vector(c, seed, 200 + i))


SWEEP_SPARSITIES = [0, 25, 30, 40, 50, 60, 70, 80, 90]


def config3(sparsity_pct: int, rows: int = 36864, cols: int = 12288, seed: int = BASE_SEED) -> Case:
    """Sparsity sweep matrix (the paper's Figure 1 shape): iid Bernoulli mask."""
    d = 1.0 - sparsity_pct / 100.0
    W = bernoulli(rows, cols, d, 0.02, seed, 300 + sparsity_pct)
    return Case(f"c3_{rows}x{cols}_s{sparsity_pct}", W, x_vector(cols, seed, 300))


def config4(rows: int = 8192, cols: int = 8192, seed: int = BASE_SEED) -> Case:
    """Adversarial stress.  Even rows: non-zeros at columns 16, 33, 50, ... so
    that every gap (including the first) is 17 and each non-zero costs one
    padding entry.  Odd rows: row sparsity ~ U(0.10, 0.99), that many
    uniformly placed non-zeros.  Values N(0,1)."""
    u = uniforms(rows, seed, 400)
    spars = 0.10 + 0.89 * u
    keep = np.rint((1.0 - spars) * cols).astype(np.int64)
    keep[0::2] = 0
    W = rows_exact(rows, cols, keep, 1.0, seed, 401)
    pos = np.arange(16, cols, 17)
    vals = normal_f16(((rows + 1) // 2) * pos.size, 1.0, seed, 402, nonzero=True).reshape(-1, pos.size)
    W[0::2, :][:, pos] = vals
    return Case(f"c4_adversarial_{rows}x{cols}", W, x_vector(cols, seed, 400),
                note="even rows gap-17 pattern, odd rows skewed density")


def config4b(rows: int = 8192, cols: int = 8192, seed: int = BASE_SEED) -> Case:
    """Worst-case padding at exactly 50 %: every row repeats
    [16 zeros][16 non-zeros] (the pattern behind eq. 9)."""
    vals = normal_f16(rows * cols, 1.0, seed, 410, nonzero=True).reshape(rows, cols)
    colmask = (np.arange(cols) % 32) >= 16
    W = np.where(colmask[None, :], vals, np.uint16(0)).astype(np.uint16)
    return Case(f"c4b_worstcase_{rows}x{cols}", W, x_vector(cols, seed, 410))


def config5_layer(seed: int = BASE_SEED):
    """One Llama2-13B-shaped decoder layer's three distinct shapes at 50 %."""
    for i, (tag, r, c) in enumerate(LLAMA2_13B_SHAPES):
        yield Case(f"c5_{tag}_{r}x{c}_s50", half_row_matrix(r, c, 500 + i, seed=seed),
                   x_vector(c, seed, 500 + i))


# Appendix D of the paper: the matrix shapes (rows, cols) its runtime sweep uses.
APPENDIX_D_SHAPES = [
    (4096, 4096), (8192, 8192), (8192, 29568), (32000, 5120), (32000, 8192), (28672, 8192), (5120, 5120),
    (5120, 13824), (3584, 20480), (4096, 11008), (13824, 5120), (18944, 3584), (14336, 4096), (4096, 14336),
    (8192, 28672), (11008, 4096), (32000, 4096), (20480, 3584), (3584, 18944), (21504, 7168), (7168, 7168),
    (28672, 7168), (7168, 28672), (27648, 9216), (9216, 9216), (36864, 9216), (9216, 36864), (36864, 12288),
    (12288, 12288), (49152, 12288), (12288, 49152),
]


def appendix_d_case(rows: int, cols: int, sparsity_pct: int = 50, seed: int = BASE_SEED) -> Case:
    """One shape of the Appendix-D list with exactly (1 - s) * cols kept per row."""
    W = half_row_matrix(rows, cols, 7000 + (rows * 31 + cols) % 997, sparsity=sparsity_pct / 100.0, seed=seed)
    return Case(f"appD_{rows}x{cols}_s{sparsity_pct}", W, x_vector(cols, seed, 7000))


def fp8_values_of(W16: np.ndarray, scale: float = 32.0) -> np.ndarray:
    """The same matrix with 8-bit values: every fp16 element times `scale`, rounded to the OCP E4M3
    format by the framework's own conversion (torch.float8_e4m3fn), as uint8 bit patterns.  With the
    default scale a N(0, 0.02) matrix becomes N(0, 0.64), which E4M3 holds with its full 3-bit
    fraction.  Elements that round to zero become zeros (about 0.1 % of the kept ones)."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(W16).view(np.float16)).to(torch.float32) * scale
    return t.to(torch.float8_e4m3fn).view(torch.uint8).numpy().copy()


def fp8_case(rows: int, cols: int, sparsity_pct: int = 50, seed: int = BASE_SEED) -> Case:
    """A matrix of 8-bit values with about (1 - s) * cols kept per row, and an fp16 x."""
    c = appendix_d_case(rows, cols, sparsity_pct, seed)
    return Case(f"fp8_{rows}x{cols}_s{sparsity_pct}", fp8_values_of(c.W), c.x)
