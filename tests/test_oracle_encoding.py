"""Pins for the oracle's encoder / decoder (CPU only).

Each test fixes the oracle against something other than itself: the paper's
worked example, its closed forms (eqs. 8-10), exact round trips through an
independent numpy decode, and brute force over every mask of a short row.
"""
import itertools
import math
import os

import numpy as np
import pytest

import oracle
from oracle import closed_forms as cf
import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def f16(a):
    return np.asarray(a, dtype=np.float16).view(np.uint16)


def row_from(cols_0based, values, C):
    W = np.zeros((1, C), dtype=np.float16)
    W[0, list(cols_0based)] = values
    return W.view(np.uint16)


def numpy_codes(enc):
    """Independent unpacking of the packed codes (little-endian bit fields)."""
    bits = np.unpackbits(enc.deltas, bitorder="little")
    b = enc.b_delta
    fields = bits[: enc.alloc_nnz * b].reshape(-1, b)
    return (fields * (1 << np.arange(b))).sum(axis=1)


def numpy_decode(enc):
    """Independent decode: columns are cumulative sums of (code+1) minus one."""
    delta = numpy_codes(enc) + 1
    out = np.zeros((enc.rows, enc.cols), dtype=np.uint16)
    for r in range(enc.rows):
        a, b = int(enc.row_ptr[r]), int(enc.row_ptr[r + 1])
        cols = np.cumsum(delta[a:b]) - 1
        assert cols.size == 0 or cols[-1] < enc.cols
        out[r, cols] = enc.values[a:b]
    return out


def padding_from_mask(mask_row, D):
    """Padding entries a row needs, from the mask alone: a gap g between
    consecutive stored columns (first one measured from -1) needs
    ceil(g / D) - 1 intermediate entries."""
    cols = np.flatnonzero(mask_row)
    if cols.size == 0:
        return 0
    gaps = np.diff(np.concatenate(([-1], cols)))
    return int(((gaps + D - 1) // D - 1).sum())


def read_golden(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                k, *v = line.split()
                out[k] = v
    return out


# ---------------------------------------------------------------- worked example

def test_worked_example_section_4_1():
    g = read_golden("worked_example_section_4_1.txt")
    b = int(g["b_delta"][0])
    cols = [int(c) - 1 for c in g["columns_1based"]]
    vals = [float(v) for v in g["values"]]
    enc = oracle.encode(row_from(cols, vals, 16), b_delta=b)
    delta, col = oracle.unpack(enc)
    assert enc.values[: enc.pad_nnz].view(np.float16).tolist() == [float(v) for v in g["expected_values"]]
    assert delta.tolist() == [int(v) for v in g["expected_deltas"]]
    assert enc.nnz == 4 and enc.pad_nnz == 5
    # the inserted zero sits at 1-based column 9
    assert col[2] + 1 == int(g["padding_column_1based"][0])
    assert enc.row_ptr.tolist() == [0, 5]
    assert oracle.check(enc) == 0


def test_worked_example_with_4_bit_deltas_needs_no_padding():
    enc = oracle.encode(row_from([1, 4, 11, 12], [1, 2, 3, 4], 16), b_delta=4)
    delta, _ = oracle.unpack(enc)
    assert delta.tolist() == [2, 3, 7, 1]
    assert enc.padding_entries == 0
    assert enc.values[:4].view(np.float16).tolist() == [1, 2, 3, 4]


# ---------------------------------------------------------------- bit layout

def test_code_is_delta_minus_one_and_nibbles_are_little_endian():
    # non-zeros at columns 0, 2, 5, 21 -> deltas 1, 2, 3, 16 -> codes 0, 1, 2, 15
    enc = oracle.encode(row_from([0, 2, 5, 21], [1, 1, 1, 1], 32), b_delta=4)
    assert enc.alloc_nnz == 32 and enc.deltas.size == 16 and enc.values.size == 32
    assert enc.deltas[0] == (0 | (1 << 4)) and enc.deltas[1] == (2 | (15 << 4))
    assert not enc.deltas[2:].any() and not enc.values[4:].any()


@pytest.mark.parametrize("b", [1, 2, 4, 8])
def test_tail_alignment_both_arrays_multiple_of_16_bytes(b):
    rng = np.random.default_rng(b)
    W = (rng.random((7, 133)) < 0.4) * rng.standard_normal((7, 133))
    enc = oracle.encode(W.astype(np.float16), b_delta=b)
    assert enc.values_bytes % 16 == 0 and enc.deltas_bytes % 16 == 0
    assert enc.alloc_nnz - enc.pad_nnz < 128 // b
    assert enc.total_bytes == cf.storage_bytes(enc.alloc_nnz, enc.rows, 16, b)
    assert enc.values.nbytes == enc.values_bytes and enc.deltas.nbytes == enc.deltas_bytes
    assert enc.row_ptr.nbytes == 4 * (enc.rows + 1) and enc.row_ptr.dtype == np.uint32
    assert oracle.check(enc) == 0


# ---------------------------------------------------------------- round trips

@pytest.mark.parametrize("b", [1, 2, 4, 8])
@pytest.mark.parametrize("density", [0.02, 0.1, 0.5, 0.9, 1.0])
def test_round_trip_is_exact(b, density):
    W = wl.bernoulli(37, 301, density, 0.02, 7, 1000 + b)
    enc = oracle.encode(W, b_delta=b)
    assert oracle.check(enc) == 0
    assert np.array_equal(oracle.decode(enc), W)
    assert np.array_equal(numpy_decode(enc), W)
    assert enc.nnz == int(np.count_nonzero(W))
    # encode(decode(F)) == F
    again = oracle.encode(oracle.decode(enc), b_delta=b)
    for name in ("values", "deltas", "row_ptr"):
        assert np.array_equal(getattr(again, name), getattr(enc, name))


def test_special_values_and_negative_zero():
    W = np.zeros((3, 40), dtype=np.uint16)
    W[0, 3] = 0x8000          # -0: a zero, dropped
    W[0, 5] = 0x0001          # smallest subnormal: kept
    W[0, 39] = 0x7C00         # +inf: kept, and needs padding (gap 34)
    W[1, 0] = 0xFE00          # a NaN: kept
    W[2, 17] = 0x8001         # negative subnormal, first delta 18 > 16
    enc = oracle.encode(W, b_delta=4)
    canon = W.copy()
    canon[0, 3] = 0
    assert np.array_equal(oracle.decode(enc), canon)
    assert enc.nnz == 4
    assert enc.row_ptr.tolist() == [0, 4, 5, 7]   # row 0: 5, pad 21, pad 37, 39; row 2: pad 15, 17
    delta, col = oracle.unpack(enc)
    assert col.tolist() == [5, 21, 37, 39, 0, 15, 17]
    assert delta.tolist() == [6, 16, 16, 2, 1, 16, 2]


def test_empty_rows_empty_matrix_and_trailing_zeros():
    W = np.zeros((4, 50), dtype=np.uint16)
    W[1, 2] = f16([1.5])[0]
    enc = oracle.encode(W)
    assert enc.row_ptr.tolist() == [0, 0, 1, 1, 1]     # nothing stored after the last non-zero
    assert enc.pad_nnz == 1 and enc.alloc_nnz == 32
    empty = oracle.encode(np.zeros((5, 9), dtype=np.uint16))
    assert empty.pad_nnz == 0 and empty.alloc_nnz == 0 and empty.values.size == 0
    assert empty.row_ptr.tolist() == [0] * 6
    assert oracle.check(empty) == 0
    none = oracle.encode(np.zeros((0, 9), dtype=np.uint16))
    assert none.row_ptr.tolist() == [0] and none.total_bytes == 4


# ---------------------------------------------------------------- padding counts

@pytest.mark.parametrize("b", [2, 4])
def test_padding_equals_gap_formula(b):
    D = 1 << b
    for density in (0.03, 0.1, 0.3, 0.7):
        W = wl.bernoulli(64, 777, density, 1.0, 11, 2000 + b)
        enc = oracle.encode(W, b_delta=b)
        per_row = np.diff(enc.row_ptr.astype(np.int64)) - np.count_nonzero(W, axis=1)
        want = [padding_from_mask(W[r] != 0, D) for r in range(W.shape[0])]
        assert per_row.tolist() == want


def test_best_case_no_padding_iff_all_gaps_fit():
    # gaps of exactly 16 everywhere: no padding, effd hits eq. 8 up to row pointers and tail
    C = 16 * 64
    W = np.zeros((32, C), dtype=np.float16)
    W[:, 15::16] = 1.0
    enc = oracle.encode(W)
    assert enc.padding_entries == 0
    d = enc.nnz / (32 * C)
    assert abs(2.5 * enc.pad_nnz / enc.dense_bytes - cf.effd_macko_best(d)) < 1e-12
    # one gap of 17 anywhere -> exactly one padding entry
    W2 = W.copy()
    W2[5, 15] = 0
    W2[5, 16] = 1.0     # first gap 17, next gap 15
    assert oracle.encode(W2).padding_entries == 1


def test_worst_case_pattern_hits_eq_9_exactly():
    case = wl.config4b(rows=64, cols=1024)
    enc = oracle.encode(case.W)
    R, C = case.W.shape
    d = enc.nnz / (R * C)
    assert d == 0.5
    assert enc.padding_entries == R * C * (1 - d) / 16
    measured = 2.5 * enc.pad_nnz / enc.dense_bytes        # values + deltas only, as in eq. 9
    assert abs(measured - cf.effd_macko_worst(d)) < 1e-12
    assert abs(cf.effd_macko_worst(0.5) - 0.6640625) < 1e-15


@pytest.mark.parametrize("seed", range(4))
def test_worst_case_bound_holds_for_any_input(seed):
    rng = np.random.default_rng(seed)
    dens = rng.choice([0.01, 0.05, 0.2, 0.6])
    W = wl.bernoulli(50, 500, float(dens), 1.0, 100 + seed, 3000)
    enc = oracle.encode(W)
    R, C = W.shape
    per_row_pad = np.diff(enc.row_ptr.astype(np.int64)) - np.count_nonzero(W, axis=1)
    for r in range(R):
        nz = np.flatnonzero(W[r])
        zeros_before_last = 0 if nz.size == 0 else int(nz[-1] + 1 - nz.size)
        assert per_row_pad[r] <= zeros_before_last // 16
    d = enc.nnz / (R * C)
    assert 2.5 * enc.pad_nnz / enc.dense_bytes <= cf.effd_macko_worst(d) + 1e-12


@pytest.mark.parametrize("sparsity", [0.5, 0.7, 0.8, 0.9, 0.95])
def test_expected_case_matches_eq_10_on_bernoulli_masks(sparsity):
    d = 1 - sparsity
    R, C = 512, 8192
    W = wl.bernoulli(R, C, d, 0.02, 5, 4000 + int(sparsity * 100))
    enc = oracle.encode(W)
    expected_pad = enc.nnz * cf.padding_per_nonzero_expected(d)
    # iid model on an infinite row; finite rows add O(1) per row and sampling noise
    tol = 5 * math.sqrt(max(expected_pad, 1.0)) + 2 * R + 0.02 * expected_pad
    assert abs(enc.padding_entries - expected_pad) <= tol
    measured = 2.5 * enc.pad_nnz / enc.dense_bytes
    assert abs(measured - cf.effd_macko_expected(d)) <= 0.02 * cf.effd_macko_expected(d)


def test_adversarial_rows_of_config4_cost_one_pad_per_nonzero():
    case = wl.config4(rows=64, cols=1024)
    enc = oracle.encode(case.W)
    nnz_row = np.count_nonzero(case.W, axis=1)
    ent_row = np.diff(enc.row_ptr.astype(np.int64))
    assert np.array_equal(ent_row[0::2], 2 * nnz_row[0::2])
    assert (nnz_row[0::2] == len(range(16, 1024, 17))).all()


# ---------------------------------------------------------------- brute force

def _min_entries_bruteforce(mask, D):
    """Fewest stored columns S containing every non-zero such that consecutive
    stored columns (starting from -1) are at most D apart: dynamic programme
    over 'last stored column'."""
    nz = [i for i, m in enumerate(mask) if m]
    if not nz:
        return 0
    last = nz[-1]
    INF = 10 ** 9
    best = {-1: 0}
    for c in range(last + 1):
        cands = [best[p] for p in best if c - p <= D and not any(mask[q] for q in range(p + 1, c))]
        best[c] = min(cands) + 1 if cands else INF
    return best[last]


def test_brute_force_all_masks_of_a_12_wide_row_with_2_bit_deltas():
    C, b, D = 12, 2, 4
    masks = np.array(list(itertools.product([0, 1], repeat=C)), dtype=np.uint16)
    W = masks * f16([1.0])[0]
    enc = oracle.encode(W, b_delta=b)
    assert np.array_equal(oracle.decode(enc), W)
    entries = np.diff(enc.row_ptr.astype(np.int64))
    delta, col = oracle.unpack(enc)
    for r in range(masks.shape[0]):
        want = _min_entries_bruteforce(masks[r].tolist(), D)
        assert entries[r] == want == int(masks[r].sum()) + padding_from_mask(masks[r], D)
        a, e = int(enc.row_ptr[r]), int(enc.row_ptr[r + 1])
        # padding entries sit exactly D after the previously stored column
        pads = [k for k in range(a, e) if enc.values[k] == 0]
        assert all(delta[k] == D for k in pads)


# ---------------------------------------------------------------- the checker itself

def test_check_rejects_planted_mistakes():
    W = wl.bernoulli(8, 200, 0.05, 1.0, 3, 5000)
    good = oracle.encode(W)
    assert good.padding_entries > 0 and oracle.check(good) == 0

    def mutated(**kw):
        import copy
        m = copy.deepcopy(good)
        for k, v in kw.items():
            setattr(m, k, v)
        return m

    k_pad = int(np.flatnonzero(good.values[: good.pad_nnz] == 0)[0])
    d = good.deltas.copy()
    d[k_pad >> 1] &= 0xF0 if (k_pad & 1) == 0 else 0x0F        # padding code no longer 15
    assert oracle.check(mutated(deltas=d)) in (4, 5)
    rp = good.row_ptr.copy(); rp[3], rp[4] = rp[4], rp[3]
    if rp[3] != rp[4]:
        assert oracle.check(mutated(row_ptr=rp)) == 2
    v = good.values.copy(); v[-1] = 1
    if good.alloc_nnz > good.pad_nnz:
        assert oracle.check(mutated(values=v)) == 7
    d2 = good.deltas.copy(); d2[0] |= 0xFF; d2[1] |= 0xFF; d2[2:40] |= 0xFF
    assert oracle.check(mutated(deltas=d2)) in (4, 5)


def test_check_names_every_kind_of_planted_mistake():
    """Each return code of the checker provoked on its own: the mistake is planted in a copy of a good
    encoding, every other invariant left intact, so exactly that code must come back."""
    import copy
    W = wl.bernoulli(8, 200, 0.05, 1.0, 3, 5000)
    W[5, :] = 0
    W[5, 3] = 0x3C00
    W[5, 60] = 0x4000                       # row 5: entries at columns 3, then padding up to 60
    good = oracle.encode(W)
    assert oracle.check(good) == 0 and good.alloc_nnz > good.pad_nnz

    def with_(**kw):
        m = copy.deepcopy(good)
        for k, v in kw.items():
            setattr(m, k, v)
        return m

    # 1: the first row pointer is not 0
    rp = good.row_ptr.copy(); rp[0] = 1
    assert oracle.check(with_(row_ptr=rp)) == 1
    # 2: a row pointer decreases
    rp = good.row_ptr.copy(); rp[4] = rp[3] - 1 if rp[3] > 0 else rp[3]; rp[3] = max(rp[3], 1); rp[4] = rp[3] - 1
    assert oracle.check(with_(row_ptr=rp)) == 2
    # 3: more entries than the arrays hold
    rp = good.row_ptr.copy(); rp[-1] = good.alloc_nnz + 1
    assert oracle.check(with_(row_ptr=rp)) == 3
    # 8: the arrays are longer than pad_nnz rounded up to 32 entries
    longer = with_(alloc_nnz=good.alloc_nnz + 32,
                   values=np.concatenate([good.values, np.zeros(32, np.uint16)]),
                   deltas=np.concatenate([good.deltas, np.zeros(16, np.uint8)]))
    assert oracle.check(longer) == 8
    # 4: an entry decodes to a column beyond the last (the last entry of a row pushed out by a larger code)
    k_last = int(good.row_ptr[1]) - 1
    d = good.deltas.copy()
    d[k_last >> 1] |= 0xF0 if (k_last & 1) else 0x0F
    last_col = oracle.unpack(good)[1][k_last]
    if last_col + 15 >= good.cols:
        assert oracle.check(with_(deltas=d)) == 4
    # 5: a zero value whose code is not 15, and a -0 stored as a padding value
    k_pad = int(np.flatnonzero(good.values[: good.pad_nnz] == 0)[0])
    d = good.deltas.copy()
    d[k_pad >> 1] &= 0xF0 if (k_pad & 1) == 0 else 0x0F
    assert oracle.check(with_(deltas=d)) in (4, 5)
    v = good.values.copy(); v[k_pad] = 0x8000
    assert oracle.check(with_(values=v)) == 5
    # 6: a row that ends in a padding entry (row 5 cut off after its first padding entry)
    a5 = int(good.row_ptr[5])
    assert good.values[a5] != 0 and good.values[a5 + 1] == 0
    rows6 = oracle.encode(W[:6])
    cut = copy.deepcopy(rows6)
    cut.row_ptr = rows6.row_ptr.copy(); cut.row_ptr[6] = a5 + 2          # entries: column 3, one padding entry
    cut.pad_nnz = a5 + 2
    cut.alloc_nnz = (cut.pad_nnz + 31) // 32 * 32
    cut.values = rows6.values[: cut.alloc_nnz].copy(); cut.values[cut.pad_nnz:] = 0
    cut.deltas = rows6.deltas[: cut.alloc_nnz // 2].copy()
    for k in range(cut.pad_nnz, cut.alloc_nnz):
        cut.deltas[k >> 1] &= 0x0F if (k & 1) else 0xF0
    assert oracle.check(cut) == 6
    # 7: something in the tail
    v = good.values.copy(); v[-1] = 1
    assert oracle.check(with_(values=v)) == 7
    d = good.deltas.copy(); d[-1] |= 0x10
    assert oracle.check(with_(deltas=d)) == 7
