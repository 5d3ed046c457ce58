"""Storage closed forms of the paper (oracle side; test infrastructure only).

Effective density is storage divided by the dense footprint R*C*b_val (eq. 2).
All functions take the density d = nnz / (R*C) (Section 3.1; Appendix A prints
the reciprocal, which is a typo) and return effective density, ignoring row
pointers and constant terms as Section 3.2 does.
"""
from __future__ import annotations


def effd_csr(d: float, index_bits: int, b_val: int = 16) -> float:
    """Eqs. 4 and 5: one index_bits-wide column index per non-zero."""
    return d * (index_bits + b_val) / b_val


def effd_tiled_csl(d: float, n_tiles: int, rows: int, cols: int, b_val: int = 16) -> float:
    """Eq. 6: 16-bit in-tile index per non-zero plus a 32-bit offset per tile."""
    return d * (16 + b_val) / b_val + 32.0 * n_tiles / (rows * cols)


def effd_bitmask(d: float, b_val: int = 16) -> float:
    """Eq. 7: one mask bit per cell plus the non-zero values."""
    return d + 1.0 / b_val


def effd_macko_best(d: float, b_val: int = 16, b_delta: int = 4) -> float:
    """Eq. 8: no gap exceeds 2^b_delta, so no padding."""
    return d * (b_val + b_delta) / b_val


def effd_macko_worst(d: float, b_val: int = 16, b_delta: int = 4) -> float:
    """Eq. 9: all zeros sit in runs of exactly 2^b_delta, each run costs one entry."""
    return (d + (1.0 - d) / 2 ** b_delta) * (b_val + b_delta) / b_val


def padding_per_nonzero_expected(d: float, b_delta: int = 4) -> float:
    """z / (1 - z) with z = (1-d)^(2^b_delta): expected padding entries per
    non-zero under an iid Bernoulli(d) mask (text before eq. 10)."""
    if d >= 1.0 or d <= 0.0:      # no zeros to bridge / no non-zeros to bridge to
        return 0.0
    z = (1.0 - d) ** (2 ** b_delta)
    return z / (1.0 - z)


def effd_macko_expected(d: float, b_val: int = 16, b_delta: int = 4) -> float:
    """Eq. 10."""
    return d * (1.0 + padding_per_nonzero_expected(d, b_delta)) * (b_val + b_delta) / b_val


def storage_bytes(alloc_nnz: int, rows: int, b_val: int = 16, b_delta: int = 4) -> int:
    """Exact byte count of the three arrays of Section 4.1 (row pointers
    included): alloc_nnz values and codes plus R+1 32-bit pointers."""
    return alloc_nnz * b_val // 8 + alloc_nnz * b_delta // 8 + 4 * (rows + 1)
