"""Pins of the oracle's 8-bit-value functions (CPU only).

The paper leaves 8-bit values to future work and does not define them; the reading taken is the
OCP E4M3 format.  What pins the oracle: the published bit patterns of that format
(tests/golden/fp8_e4m3_pins.txt), the framework's own E4M3 conversion on all 256 patterns, the
already pinned 16-bit encoder for the coordinates (same mask, same codes), the worked example of
Section 4.1 carried over to 8-bit values, exact round trip, and numpy's fp64 matmul for the products.
"""
import os

import numpy as np
import pytest
import torch

import oracle
import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "fp8_e4m3_pins.txt")


def test_published_bit_patterns():
    for line in open(GOLDEN):
        line = line.split("#")[0].split()
        if not line:
            continue
        code, want = int(line[0], 16), float(line[1])
        got = oracle.fp8_to_double(np.array([code], dtype=np.uint8))[0]
        if np.isnan(want):
            assert np.isnan(got), hex(code)
        else:
            assert got == want and np.signbit(got) == np.signbit(want), hex(code)


def test_all_256_patterns_against_the_framework_conversion_and_the_format_structure():
    codes = np.arange(256, dtype=np.uint8)
    got = oracle.fp8_to_double(codes)
    ref = torch.from_numpy(codes).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    assert np.array_equal(np.isnan(got), np.isnan(ref)) and np.isnan(got).sum() == 2
    ok = ~np.isnan(ref)
    assert np.array_equal(got[ok], ref[ok]) and np.array_equal(np.signbit(got[ok]), np.signbit(ref[ok]))
    # structure: strictly increasing over the positive patterns, mirrored by the sign bit, 8 values per binade
    pos = got[:0x7F]
    assert (np.diff(pos) > 0).all()
    assert np.array_equal(got[0x80:0xFF], -pos)
    for e in range(1, 15):
        binade = got[8 * e: 8 * e + 8]
        assert binade[0] == 2.0 ** (e - 7) and np.allclose(np.diff(binade), 2.0 ** (e - 10), rtol=0, atol=0)


def _random_fp8(rows, cols, density, seed):
    rng = np.random.default_rng(seed)
    W = rng.integers(0, 256, size=(rows, cols), dtype=np.uint8)
    W[(W & 0x7F) == 0x7F] = 0x3A                      # no NaNs in product tests
    W[rng.random((rows, cols)) >= density] = 0
    return W


@pytest.mark.parametrize("b_delta", [1, 2, 4, 8])
@pytest.mark.parametrize("density", [0.03, 0.5, 1.0])
def test_coordinates_equal_those_of_the_pinned_16_bit_encoder(b_delta, density):
    """Same mask, same codes, same row pointers: the value width does not touch the coordinates."""
    W8 = _random_fp8(37, 700, density, 11)
    W8[5] = 0
    W8[9, 3] = 0x80                                   # -0 is a zero
    W16 = np.where((W8 & 0x7F) != 0, np.uint16(0x3C00), np.uint16(0))
    e8, e16 = oracle.encode8(W8, b_delta), oracle.encode(W16, b_delta)
    assert (e8.nnz, e8.pad_nnz, e8.alloc_nnz) == (e16.nnz, e16.pad_nnz, e16.alloc_nnz)
    assert np.array_equal(e8.row_ptr, e16.row_ptr) and np.array_equal(e8.deltas, e16.deltas)
    # values: the element at the decoded (row, column) for real entries, +0 for padding entries and the tail
    _, cols = oracle.unpack(e16)
    rows = np.repeat(np.arange(37), np.diff(e16.row_ptr.astype(np.int64)))
    is_pad = e16.values[: e16.pad_nnz] == 0
    assert np.array_equal(e8.values[: e8.pad_nnz][~is_pad], W8[rows[~is_pad], cols[~is_pad]])
    assert (e8.values[: e8.pad_nnz][is_pad] == 0).all() and (e8.values[e8.pad_nnz:] == 0).all()
    assert e8.values_bytes == e8.alloc_nnz and e8.dense_bytes == 37 * 700
    assert e8.total_bytes == oracle.closed_forms.storage_bytes(e8.alloc_nnz, 37, 8, b_delta)


def test_worked_example_of_section_4_1_with_8_bit_values():
    # values 1, 2, 3, 4 at 1-based columns 2, 5, 12, 13, 2-bit deltas: one zero at column 9
    one, two, three, four = 0x38, 0x40, 0x44, 0x48
    assert list(oracle.fp8_to_double(np.array([one, two, three, four], dtype=np.uint8))) == [1.0, 2.0, 3.0, 4.0]
    row = np.zeros((1, 13), dtype=np.uint8)
    row[0, [1, 4, 11, 12]] = [one, two, three, four]
    enc = oracle.encode8(row, 2)
    assert list(enc.values[: enc.pad_nnz]) == [one, two, 0, three, four]
    d, c = oracle.unpack(enc)
    assert list(d) == [2, 3, 4, 3, 1] and list(c + 1) == [2, 5, 9, 12, 13]


@pytest.mark.parametrize("b_delta", [1, 2, 4, 8])
def test_round_trip_is_exact(b_delta):
    W = _random_fp8(61, 900, 0.2, 12)
    W[0] = 0
    W[60, 899] = 0xFF                                  # NaN patterns are values like any other
    W[7, 5] = 0x80
    back = oracle.decode8(oracle.encode8(W, b_delta))
    canon = np.where((W & 0x7F) == 0, np.uint8(0), W)
    assert np.array_equal(back, canon)


@pytest.mark.parametrize("density", [0.05, 0.5, 1.0])
def test_products_match_numpy_fp64_matmul(density):
    W = _random_fp8(53, 640, density, 13)
    x = wl.x_vector(640, 13, 1)
    Wf = torch.from_numpy(W).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    xf = x.view(np.float16).astype(np.float64)
    want, mag = Wf @ xf, np.abs(Wf) @ np.abs(xf)
    yd, sd = oracle.dense_matvec8(W, x)
    assert np.allclose(yd, want, rtol=1e-12, atol=1e-12) and np.allclose(sd, mag, rtol=1e-12)
    for b in (2, 4):
        ys, ss = oracle.spmv8(oracle.encode8(W, b), x)
        assert np.allclose(ys, want, rtol=1e-12, atol=1e-12) and np.allclose(ss, mag, rtol=1e-12)


def test_single_entry_rows_pick_the_right_column_and_value():
    W = np.zeros((8, 300), dtype=np.uint8)
    cols = [0, 1, 15, 16, 17, 150, 298, 299]
    for r, c in enumerate(cols):
        W[r, c] = 0x38 + r                             # 1, 1.125, 1.25, ...
    x = np.arange(300, dtype=np.float16).view(np.uint16)   # x_j = j, exact in fp16
    y, _ = oracle.spmv8(oracle.encode8(W, 4), x)
    assert list(y) == [(1 + r / 8) * c for r, c in enumerate(cols)]


def test_generator_of_8_bit_matrices():
    c = wl.fp8_case(64, 512, 50)
    assert c.W.dtype == np.uint8 and c.W.shape == (64, 512)
    kept = ((c.W & 0x7F) != 0).sum(axis=1)
    assert (kept <= 256).all() and kept.mean() > 250          # a few values round to zero
    assert ((c.W & 0x7F) != 0x7F).all()                        # no NaNs
    vals = oracle.fp8_to_double(c.W[(c.W & 0x7F) != 0])
    assert 0.4 < vals.std() < 0.9                              # N(0, 0.64)
