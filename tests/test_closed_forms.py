"""The paper's storage formulas against the numbers it prints (CPU only)."""
import os

import numpy as np

from oracle import closed_forms as cf

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "closed_form_pins.txt")


def pins():
    out = {}
    with open(GOLDEN) as f:
        for line in f:
            line = line.split("#")[0].split()
            if line:
                out[line[0]] = float(line[1])
    return out


def test_effd_at_half_density_and_theoretical_speedup():
    p = pins()
    assert cf.effd_macko_best(0.5) == p["best_effd_at_d0.5"]
    assert abs(1.0 / cf.effd_macko_expected(0.5) - p["theoretical_speedup_at_s50"]) < 1e-3
    # the abstract's 1.5x memory reduction is the same number rounded down
    assert 1.5 <= 1.0 / cf.effd_macko_expected(0.5) < 1.65
    assert p["memory_reduction_at_s50"] == 1.5


def test_bitmask_crossover_is_at_density_0_23():
    p = pins()
    d = p["bitmask_crossover_density"]
    assert cf.effd_macko_expected(d) < cf.effd_bitmask(d)
    assert cf.effd_macko_expected(d + 0.01) > cf.effd_bitmask(d + 0.01)


def test_eight_bit_quantisation_equivalents():
    p = pins()
    assert abs(cf.effd_macko_expected(1 - p["q8_equivalent_sparsity_macko"]) - 0.5) < 2e-3
    assert abs(cf.effd_csr(1 - p["q8_equivalent_sparsity_csr"], 32) - 0.5) < 0.02
    # and CSR at 60 % sparsity is nowhere near it
    assert cf.effd_csr(0.4, 32) > 1.0


def test_one_bit_deltas_beat_dense_from_7_percent_sparsity():
    p = pins()
    s = p["bdelta1_breakeven_sparsity"]
    assert cf.effd_macko_expected(1 - s, b_delta=1) < 1.0
    assert cf.effd_macko_expected(1 - (s - 0.02), b_delta=1) > 1.0


def test_ordering_and_limits():
    for d in np.linspace(0.01, 1.0, 50):
        assert cf.effd_macko_best(d) <= cf.effd_macko_expected(d) + 1e-15
        assert cf.effd_macko_expected(d) <= cf.effd_macko_worst(d) + 1e-12
        assert cf.effd_macko_best(d) < cf.effd_csr(d, 16) < cf.effd_csr(d, 32)
    assert cf.effd_macko_best(1.0) == 1.25 == cf.effd_macko_expected(1.0) == cf.effd_macko_worst(1.0)
    # padding noticeable only below 20 % density, dominant below 4 % (text after eq. 10)
    assert cf.padding_per_nonzero_expected(0.2) < 0.03
    assert cf.padding_per_nonzero_expected(0.04) > 1.0
    assert cf.effd_tiled_csl(0.5, 0, 1, 1) == cf.effd_csr(0.5, 16)
    # matching the dense footprint: d * 20/16 = 1 at density 0.8
    assert abs(cf.effd_macko_best(0.8) - 1.0) < 1e-15


def test_storage_bytes():
    assert cf.storage_bytes(64, 3) == 128 + 32 + 16
    assert cf.storage_bytes(64, 3, 16, 2) == 128 + 16 + 16
