"""Pins for the oracle's products and number conversions (CPU only)."""
import numpy as np
import pytest

import oracle
import workloads as wl


def f16bits(a):
    return np.asarray(a, dtype=np.float16).view(np.uint16)


# ------------------------------------------------------------ fp16 <-> fp64

def test_half_to_double_matches_numpy_on_every_bit_pattern():
    allbits = np.arange(65536, dtype=np.uint16)
    mine = oracle.half_to_double(allbits)
    ref = allbits.view(np.float16).astype(np.float64)
    assert np.array_equal(np.isnan(mine), np.isnan(ref))
    ok = ~np.isnan(ref)
    assert np.array_equal(mine[ok], ref[ok])
    assert np.array_equal(np.signbit(mine[ok]), np.signbit(ref[ok]))


def test_double_to_half_rounds_to_nearest_even_like_numpy():
    rng = np.random.default_rng(0)
    allh = np.arange(65536, dtype=np.uint16).view(np.float16).astype(np.float64)
    finite = allh[np.isfinite(allh)]
    srt = np.sort(finite)
    mids = (srt[:-1] + srt[1:]) / 2                  # exact ties between neighbours
    vals = np.concatenate([
        finite, mids, np.nextafter(mids, np.inf), np.nextafter(mids, -np.inf),
        rng.standard_normal(20000) * 10.0 ** rng.integers(-9, 6, 20000),
        [65504.0, 65519.99, 65520.0, 65536.0, 1e9, -1e9, 2.0 ** -25, 2.0 ** -24, 3 * 2.0 ** -26, 0.0, -0.0],
    ])
    with np.errstate(over="ignore"):
        ref = vals.astype(np.float16).view(np.uint16)
    assert np.array_equal(oracle.double_to_half(vals), ref)


# ------------------------------------------------------------ product vs library routine

@pytest.mark.parametrize("shape,density", [((64, 96), 0.5), ((33, 1000), 0.1), ((200, 517), 0.9), ((5, 4000), 0.01)])
def test_products_match_numpy_fp64_matmul(shape, density):
    W = wl.bernoulli(shape[0], shape[1], density, 0.02, 21, 6000)
    x = wl.x_vector(shape[1], 21, 6000)
    Wd = W.view(np.float16).astype(np.float64)
    xd = x.view(np.float16).astype(np.float64)
    ref = Wd @ xd
    ref_abs = np.abs(Wd) @ np.abs(xd)
    y_dense, s_dense = oracle.dense_matvec(W, x)
    y_fmt, s_fmt = oracle.spmv(oracle.encode(W), x)
    scale = ref_abs + 1e-300
    assert np.max(np.abs(y_dense - ref) / scale) < 1e-13
    assert np.max(np.abs(y_fmt - ref) / scale) < 1e-13
    assert np.allclose(s_dense, ref_abs, rtol=1e-12, atol=0)
    assert np.allclose(s_fmt, ref_abs, rtol=1e-12, atol=0)


def test_identity_zero_and_ones():
    n = 300
    x = wl.x_vector(n, 3, 1)
    eye = np.zeros((n, n), dtype=np.float16)
    np.fill_diagonal(eye, 1.0)
    y, s = oracle.spmv(oracle.encode(eye), x)          # needs padding: first deltas up to 300
    xd = x.view(np.float16).astype(np.float64)
    assert np.array_equal(y, xd) and np.array_equal(s, np.abs(xd))
    y0, s0 = oracle.spmv(oracle.encode(np.zeros((7, n), dtype=np.float16)), x)
    assert not y0.any() and not s0.any()
    W = wl.bernoulli(40, n, 0.3, 1.0, 9, 2)
    ones = f16bits(np.ones(n))
    y1, _ = oracle.spmv(oracle.encode(W), ones)
    assert np.allclose(y1, W.view(np.float16).astype(np.float64).sum(axis=1), rtol=1e-13, atol=1e-13)


def test_single_entry_rows_pick_the_right_column():
    C = 777
    cols = [0, 1, 15, 16, 17, 255, 256, 776]
    W = np.zeros((len(cols), C), dtype=np.float16)
    for r, c in enumerate(cols):
        W[r, c] = 2.0
    x = f16bits(np.arange(C) % 1000)                    # x[c] = c exactly (c < 2048)
    y, _ = oracle.spmv(oracle.encode(W), x)
    assert y.tolist() == [2.0 * c for c in cols]


def test_padding_entries_never_change_the_product():
    W = wl.bernoulli(60, 900, 0.04, 0.02, 13, 3)
    x = wl.x_vector(900, 13, 3)
    ys = []
    for b in (1, 2, 4, 8):
        enc = oracle.encode(W, b_delta=b)
        ys.append(oracle.spmv(enc, x)[0])
    assert oracle.encode(W, 2).padding_entries > oracle.encode(W, 4).padding_entries > 0
    for y in ys[1:]:
        assert np.array_equal(y, ys[0])                # same order of non-zero terms, pads add exact zeros


def test_transposed_operand_would_be_caught():
    # guards the row/column convention: W is rows x cols and y has `rows` entries
    W = wl.bernoulli(20, 50, 0.5, 1.0, 1, 4)
    x = wl.x_vector(50, 1, 4)
    y, _ = oracle.spmv(oracle.encode(W), x)
    assert y.shape == (20,)
    ref = W.view(np.float16).astype(np.float64) @ x.view(np.float16).astype(np.float64)
    assert np.allclose(y, ref, rtol=1e-12, atol=1e-15)
