"""Pins for the compute-intensity closed forms (Eq. 1, Eq. 2) against the values the paper prints."""
import json
import os

import pytest

GOLD = os.path.join(os.path.dirname(__file__), "golden", "roofline_fig5.json")
A100_TC_PEAK = 312e12   # the paper's test bed (Sec. 6): A100 fp16 tensor-core peak
A100_HBM = 2.0e12       # memory roof that reproduces the printed figures


def test_eq1_eq2_closed_forms(oracle_mod):
    assert oracle_mod.ci_dense(1024, 768) == pytest.approx(1024 * 768 / 1792)
    assert oracle_mod.ci_dense(10 ** 9, 16) == pytest.approx(16, rel=1e-6)      # "strict upper bound of 16"
    assert oracle_mod.ci_sparse_load(4096, 16, 0.0) == oracle_mod.ci_dense(4096, 16)
    assert oracle_mod.ci_sparse_load(10 ** 9, 8, 0.4) == pytest.approx(8 / 0.6, rel=1e-6)
    # from bytes: 2MNK flop over 2(MK(1-b) + KN) bytes
    M, K, N, b = 300, 70, 9, 0.25
    assert oracle_mod.ci_sparse_load(M, N, b) == pytest.approx(2 * M * N * K / (2 * (M * K * (1 - b) + K * N)))


def test_printed_roofline_percentages(oracle_mod):
    g = json.load(open(GOLD))
    M = g["M"]
    for i, N in enumerate(g["N"]):
        dense = 100 * oracle_mod.roof_fraction(oracle_mod.ci_dense(M, N), A100_HBM, A100_TC_PEAK)
        sparse = 100 * oracle_mod.roof_fraction(oracle_mod.ci_sparse_load(M, N, 0.4), A100_HBM, A100_TC_PEAK)
        assert sparse == pytest.approx(g["sparse40_percent_of_tc_peak"][i], abs=0.1)
        if N != 64:  # the dense N=64 figure is printed as 40.1; Eq. 1 gives 41.0 (see the fixture's note)
            assert dense == pytest.approx(g["dense_percent_of_tc_peak"][i], abs=0.1)
        else:
            assert dense == pytest.approx(41.0, abs=0.1)
        assert sparse / dense == pytest.approx((M + N) / (0.6 * M + N), rel=1e-9)
