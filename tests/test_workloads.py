"""The seeded input generators: determinism and the stated structure (CPU only)."""
import numpy as np

import workloads as wl


def test_deterministic_and_seed_sensitive():
    a = wl.half_row_matrix(64, 256, 1)
    b = wl.half_row_matrix(64, 256, 1)
    c = wl.half_row_matrix(64, 256, 2)
    assert np.array_equal(a, b) and not np.array_equal(a, c)
    assert np.array_equal(wl.x_vector(100), wl.x_vector(100))


def test_exact_half_per_row_no_signed_zero_and_scale():
    case = wl.config1()
    W = case.W
    assert W.shape == (512, 512) and case.x.shape == (512,)
    assert (np.count_nonzero(W & 0x7FFF, axis=1) == 256).all()
    assert not (W == 0x8000).any()
    vals = W.view(np.float16)[W != 0].astype(np.float64)
    assert abs(vals.std() - 0.02) < 0.0005 and abs(vals.mean()) < 0.0005
    xs = case.x.view(np.float16).astype(np.float64)
    assert 0.85 < xs.std() < 1.15
    # positions are spread: every column is used by some row, usage near 50 %
    use = (W != 0).mean(axis=0)
    assert 0.35 < use.min() and use.max() < 0.65


def test_bernoulli_density():
    W = wl.bernoulli(256, 4096, 0.3, 0.02, wl.BASE_SEED, 9)
    assert abs((W != 0).mean() - 0.3) < 0.005
    assert (wl.bernoulli(4, 64, 1.0, 0.02, 1, 1) != 0).all()


def test_config4_structure():
    case = wl.config4(rows=128, cols=2048)
    W = case.W
    even = W[0::2] != 0
    cols = np.flatnonzero(even[0])
    assert (even == even[0]).all() and cols[0] == 16 and (np.diff(cols) == 17).all()
    nnz_odd = np.count_nonzero(W[1::2], axis=1)
    assert nnz_odd.min() >= int(0.01 * 2048) - 1 and nnz_odd.max() <= int(0.90 * 2048) + 1
    assert nnz_odd.std() > 200          # skewed, not constant


def test_config4b_is_exactly_half_dense():
    case = wl.config4b(rows=16, cols=256)
    assert (case.W != 0).mean() == 0.5
    assert not (case.W[:, :16] != 0).any() and (case.W[:, 16:32] != 0).all()
