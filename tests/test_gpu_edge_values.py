"""Value edge cases through fls_spmm and fls_dense_gemm: fp16 subnormal weights, stored -0.0 entries, and
Inf / NaN in X against zero and non-zero weights.

The method multiplies the rebuilt dense tiles, zeros included (Sec. 6.2: no computation is skipped), so the
result is that of a dense GEMM on the masked matrix in IEEE arithmetic: 0 * Inf is NaN, a subnormal weight
contributes its exact product, -0.0 is an ordinary stored entry.  Cases are built so that every partial sum is
exact in fp32 (products of fp16 values with powers of two, sums below 2^24 units): the fp16 output then equals
the oracle's fp64 result rounded once, bit for bit, whatever the order of the additions.
"""
import numpy as np
import pytest

import fls_workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def fls():
    import torch

    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2309_10285_amd as f

    f.lib()
    return f


def _both(fls, Wbits, Xbits):
    import torch

    M, K = Wbits.shape
    N = Xbits.shape[0]
    W = torch.from_numpy(Wbits.view(np.float16)).cuda()
    X = torch.from_numpy(Xbits.view(np.float16)).cuda()
    blob, _ = fls.fls_compress(W)
    fls.ensure_workspace(M, K, N)
    C = torch.full((N, M), 7.0, dtype=torch.float16, device="cuda")
    D = torch.full((N, M), 7.0, dtype=torch.float16, device="cuda")
    fls.fls_spmm(blob, X, C, M, K, N)
    fls.fls_dense_gemm(W, X, D, M, K, N)
    torch.cuda.synchronize()
    fls.fls_forget(blob)
    return C.cpu().numpy().view(np.uint16), D.cpu().numpy().view(np.uint16)


# widths: one column block per wave, two, the 64-column pass, a 64-column pass followed by a 16-column rest
WIDTHS = [8, 32, 64, 80]


@pytest.mark.parametrize("N", WIDTHS)
def test_subnormal_and_negative_zero_weights_bit_exact(fls, oracle_mod, N):
    g = np.random.Generator(np.random.Philox(601))
    M, K = 640, 1024  # five bands x 32 K tiles: bands are cut between workgroups
    # weights: fp16 subnormals j * 2^-24 (j = 1..1023), either sign, -0.0, and a few smallest normals
    mag = g.integers(1, 1024, size=(M, K)).astype(np.uint16)
    sign = (g.integers(0, 2, size=(M, K)).astype(np.uint16)) << 15
    W = mag | sign
    W[g.random((M, K)) < 0.05] = 0x8000          # stored -0.0
    W[g.random((M, K)) < 0.02] = 0x0400          # 2^-14, the smallest normal
    W[g.random((M, K)) < 0.8] = 0                # pruned
    W[128:256] = np.where(W[128:256] != 0, 0x8000, 0).astype(np.uint16)  # a band whose stored entries are all -0.0
    # X: signed powers of two 2^0 .. 2^3 (exact products; a row's sum stays far below 2^24 units of 2^-24)
    e = g.integers(0, 4, size=(N, K))
    X = ((15 + e) << 10).astype(np.uint16) | (g.integers(0, 2, size=(N, K)).astype(np.uint16) << 15)
    ref = oracle_mod.ref_spmm_f64(W, X)
    assert np.abs(ref).max() * 2.0**24 < 2.0**24  # every partial sum is an integer below 2^24 in units of 2^-24
    want = oracle_mod.double_to_half(ref)
    C, D = _both(fls, W, X)
    assert np.count_nonzero(want & 0x7FFF) > 0.7 * want.size  # the case is not trivially zero
    assert np.array_equal(C, want), "fls_spmm"
    assert np.array_equal(D, want), "fls_dense_gemm"
    assert not C[:, 128:256].any()  # the all -0.0 band: +0 + (-0) = +0, bit pattern 0x0000


@pytest.mark.parametrize("N", WIDTHS)
def test_inf_and_nan_in_x_meet_zero_and_nonzero_weights(fls, oracle_mod, N):
    """Rows of X (one k each) holding +Inf, -Inf and NaN in some columns.  Against a pruned (zero) weight the
    product is NaN, against a stored weight it is +-Inf: the positions of NaN, +Inf and -Inf in C must be the
    oracle's, and the finite elements must agree to the usual tolerance."""
    g = np.random.Generator(np.random.Philox(602))
    M, K = 512, 2048
    W = wl.prune_uniform(wl.gen_weights_f32(M, K, 603), 0.8, 604)
    W[:, 1000] = wl.dense_bits(wl.gen_weights_f32(M, 1, 605))[:, 0]  # a column of W without zeros
    W[0:128, 64:96] = 0                                               # an empty tile under a special row of X
    X = wl.gen_x(N, K, 606)
    cols = np.arange(N)
    X[cols[cols % 5 == 0], 70] = 0x7C00    # +Inf at k = 70 (meets the empty tile in band 0, mixed tiles elsewhere)
    X[cols[cols % 5 == 1], 1000] = 0xFC00  # -Inf at k = 1000, where every weight is stored: -+Inf, never NaN
    X[cols[cols % 5 == 2], 1999] = 0x7E00  # NaN
    X[cols[cols % 5 == 3], 5] = 0x7C00     # +Inf and -Inf in the same column of X: NaN unless both weights are 0...
    X[cols[cols % 5 == 3], 2040] = 0xFC00
    ref = oracle_mod.ref_spmm_f64(W, X)
    assert np.isnan(ref).any() and np.isinf(ref).any() and np.isfinite(ref).any()
    C, D = _both(fls, W, X)
    finite = np.isfinite(ref)
    scale = float(np.abs(ref[finite]).max())
    for name, got in (("fls_spmm", C), ("fls_dense_gemm", D)):
        got = got.view(np.float16).astype(np.float64)
        assert np.array_equal(np.isnan(got), np.isnan(ref)), name
        assert np.array_equal(np.isposinf(got), np.isposinf(ref)), name
        assert np.array_equal(np.isneginf(got), np.isneginf(ref)), name
        assert float(np.abs(got[finite] - ref[finite]).max()) / scale <= 2e-3, name
