"""Closed forms of the paper's compute-intensity model (Sec. 3.2, Eq. 1 and Eq. 2).  Test infrastructure."""


def ci_dense(M, N):
    """Eq. 1: 2MNK FLOP over 2(MK + KN) bytes of fp16 reads = MN / (M + N) FLOP per byte."""
    return M * N / (M + N)


def ci_sparse_load(M, N, beta):
    """Eq. 2: weights loaded at density (1 - beta); index bytes ignored, as the paper's footnote says."""
    return M * N / (M * (1.0 - beta) + N)


def roof_fraction(ci, bandwidth_bytes_per_s, peak_flops):
    """Memory-roof performance as a fraction of the matrix-core peak (Fig. 5's vertical axis)."""
    return min(1.0, ci * bandwidth_bytes_per_s / peak_flops)
