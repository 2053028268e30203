"""Pins for the oracle's SpMM definition C = W . X (Sec. 2.2; zeros are not skipped, Sec. 6.2)."""
from fractions import Fraction

import numpy as np

import fls_workloads as wl


def _f64(bits):
    return bits.view(np.float16).astype(np.float64)


def test_tiny_cases_vs_exact_rational_product(oracle_mod):
    # brute force with exact rationals: any wrong index, transposed operand or dropped term shows
    g = np.random.Generator(np.random.Philox(3))
    for (M, K, N) in [(3, 5, 2), (1, 7, 1), (4, 2, 3)]:
        W = (g.standard_normal((M, K)) * 0.5).astype(np.float16).view(np.uint16)
        X = g.standard_normal((N, K)).astype(np.float16).view(np.uint16)
        W[g.random((M, K)) < 0.4] = 0
        C = oracle_mod.ref_spmm_f64(W, X)
        assert C.shape == (N, M)
        for m in range(M):
            for n in range(N):
                exact = sum(Fraction(float(_f64(W)[m, k])) * Fraction(float(_f64(X)[n, k])) for k in range(K))
                assert abs(Fraction(float(C[n, m])) - exact) <= abs(exact) * Fraction(1, 2 ** 50) + Fraction(1, 2 ** 80)


def test_small_integers_are_exact(oracle_mod):
    g = np.random.Generator(np.random.Philox(4))
    M, K, N = 37, 129, 5
    Wi = g.integers(-8, 9, size=(M, K))
    Xi = g.integers(-8, 9, size=(N, K))
    Wi[g.random((M, K)) < 0.7] = 0
    W = Wi.astype(np.float16).view(np.uint16)
    X = Xi.astype(np.float16).view(np.uint16)
    C = oracle_mod.ref_spmm_f64(W, X)
    assert np.array_equal(C, (Xi @ Wi.T).astype(np.float64))


def test_identity_x_returns_columns_of_w(oracle_mod):
    W, _ = wl.make_inputs(wl.CONFIGS["C1"])
    W = W[:200, :64]
    X = np.zeros((64, 64), dtype=np.uint16)
    X[np.arange(64), np.arange(64)] = 0x3C00  # 1.0
    C = oracle_mod.ref_spmm_f64(W, X)
    assert np.array_equal(C, _f64(W).T)
    # a column selector with a scale: column 5 of W times -2, column 63 times 0.5
    X = np.zeros((2, 64), dtype=np.uint16)
    X[0, 5] = 0xC000
    X[1, 63] = 0x3800
    C = oracle_mod.ref_spmm_f64(W, X)
    assert np.array_equal(C[0], -2.0 * _f64(W)[:, 5]) and np.array_equal(C[1], 0.5 * _f64(W)[:, 63])


def test_masked_and_dense_vs_library_matmul(oracle_mod):
    cfg = wl.CONFIGS["C1"]
    W32 = wl.make_w32(cfg)[:384, :512]
    X = wl.gen_x(9, 512, 77)
    for W in (wl.dense_bits(W32), wl.prune_uniform(W32, 0.8, 1), wl.prune_magnitude(W32, 0.9),
              np.zeros_like(wl.dense_bits(W32))):
        C = oracle_mod.ref_spmm_f64(W, X)
        ref = _f64(X) @ _f64(W).T
        assert np.abs(C - ref).max() <= 1e-13 * max(1.0, np.abs(ref).max())
    assert np.count_nonzero(oracle_mod.ref_spmm_f64(np.zeros((8, 16), np.uint16), X[:, :16])) == 0


def test_linearity_and_row_subset(oracle_mod):
    W, X = wl.make_inputs(wl.CONFIGS["C1"])
    W = W[:256, :256]
    X1 = (np.arange(3 * 256).reshape(3, 256) % 7 - 3).astype(np.float16).view(np.uint16)
    X2 = (np.arange(3 * 256).reshape(3, 256) % 5 - 2).astype(np.float16).view(np.uint16)
    X12 = (_f64(X1) + _f64(X2)).astype(np.float16).view(np.uint16)  # exact: small integers
    C1, C2, C12 = (oracle_mod.ref_spmm_f64(W, x) for x in (X1, X2, X12))
    assert np.abs(C12 - (C1 + C2)).max() <= 1e-12
    part = oracle_mod.ref_spmm_f64(W, X1, rows=(100, 164))
    assert np.array_equal(part[:, 100:164], C1[:, 100:164])
    assert np.count_nonzero(part[:, :100]) == 0 and np.count_nonzero(part[:, 164:]) == 0


def test_spmm_of_decompressed_blob_equals_spmm_of_w(oracle_mod):
    # compress -> decompress -> product is the product of the masked matrix, for either word order
    W, X = wl.make_inputs(wl.CONFIGS["C1"])
    W = W[:256, :128]
    X = X[:, :128]
    ref = oracle_mod.ref_spmm_f64(W, X)
    for policy in (0, 1):
        Wd = oracle_mod.ref_decompress(oracle_mod.ref_compress(W, policy=policy), 256, 128)
        assert np.array_equal(oracle_mod.ref_spmm_f64(Wd, X), ref)
