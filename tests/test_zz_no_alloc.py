"""fls_spmm_noalloc (the entry point for callers that cannot allocate: static device scratch, statistics passed
in) against fls_spmm, through the C ABI: two calls in a row on the same GPU, the second with a smaller input, both
on shapes whose row bands are cut between workgroups (the hand-over through the scratch is what differs)."""
import ctypes

import numpy as np
import pytest

import fls_workloads as wl

pytestmark = pytest.mark.gpu

TOL = 2e-3


def test_noalloc_entry_point_matches_fls_spmm_twice_in_a_row(oracle_mod):
    import torch

    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2309_10285_amd as fls

    L = fls.lib()
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    # first a larger call (12 bands x 128 K tiles over all CUs, N = 32), then a smaller one (5 bands, N = 8)
    for M, K, N, beta, seed in ((1536, 4096, 32, 0.8, 901), (640, 1024, 8, 0.7, 911)):
        W = wl.prune_uniform(wl.gen_weights_f32(M, K, seed), beta, seed + 1)
        Xb = wl.gen_x(N, K, seed + 2)
        Wd = torch.from_numpy(W.view(np.float16)).cuda()
        X = torch.from_numpy(Xb.view(np.float16)).cuda()
        blob, stats = fls.fls_compress(Wd)
        st = fls.FlsStats(**{k: stats[k] for k, _ in fls.FlsStats._fields_})
        # the existing entry point, on a registered workspace
        fls.ensure_workspace(M, K, N)
        want = torch.full((N, M), float("nan"), dtype=torch.float16, device="cuda")
        fls.fls_spmm(blob, X, want, M, K, N)
        torch.cuda.synchronize()
        # the new one, through the raw C ABI; outputs allocated before the call
        got = torch.full((N, M), float("nan"), dtype=torch.float16, device="cuda")
        rc = L.fls_spmm_noalloc(ctypes.c_void_p(blob.data_ptr()), ctypes.byref(st), ctypes.c_void_p(X.data_ptr()),
                                ctypes.c_void_p(got.data_ptr()), M, K, N, stream)
        assert rc == fls.OK
        torch.cuda.synchronize()
        fls.fls_check_workspace()
        got_h, want_h = got.cpu().numpy(), want.cpu().numpy()
        assert not np.isnan(got_h).any()
        ref = oracle_mod.ref_spmm_f64(W, Xb)
        scale = float(np.abs(ref).max())
        assert float(np.abs(got_h.astype(np.float64) - ref).max()) / scale <= TOL
        # against the existing entry point: the same kernels, so at most the last fp32 bit of a sum may differ
        assert float(np.abs(got_h.astype(np.float64) - want_h.astype(np.float64)).max()) / scale <= TOL
        # beyond the static array's limit: a clear error, nothing launched
        wide = torch.zeros((64, M), dtype=torch.float16, device="cuda")
        Xw = torch.zeros((64, K), dtype=torch.float16, device="cuda")
        assert L.fls_spmm_noalloc(ctypes.c_void_p(blob.data_ptr()), ctypes.byref(st), ctypes.c_void_p(Xw.data_ptr()),
                                  ctypes.c_void_p(wide.data_ptr()), M, K, 64, stream) == fls.ESCRATCH
        # statistics of another shape: rejected on the host
        bad = fls.FlsStats(**{k: stats[k] for k, _ in fls.FlsStats._fields_})
        bad.M = M + 128
        assert L.fls_spmm_noalloc(ctypes.c_void_p(blob.data_ptr()), ctypes.byref(bad), ctypes.c_void_p(X.data_ptr()),
                                  ctypes.c_void_p(got.data_ptr()), M, K, N, stream) == fls.EFORMAT
        fls.fls_forget(blob)


def test_noalloc_entry_point_reads_format_version_2(oracle_mod):
    """The same entry point on a version-2 blob (the statistics name the version): split bands, N = 16."""
    import torch

    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2309_10285_amd as fls

    L = fls.lib()
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    M, K, N = 1280, 2048, 16
    W = wl.prune_uniform(wl.gen_weights_f32(M, K, 921), 0.8, 922)
    Xb = wl.gen_x(N, K, 923)
    X = torch.from_numpy(Xb.view(np.float16)).cuda()
    blob, stats = fls.fls_compress_v2(torch.from_numpy(W.view(np.float16)).cuda())
    assert stats["format_version"] == 2
    st = fls.FlsStats(**{k: stats[k] for k, _ in fls.FlsStats._fields_})
    got = torch.full((N, M), float("nan"), dtype=torch.float16, device="cuda")
    rc = L.fls_spmm_noalloc(ctypes.c_void_p(blob.data_ptr()), ctypes.byref(st), ctypes.c_void_p(X.data_ptr()),
                            ctypes.c_void_p(got.data_ptr()), M, K, N, stream)
    assert rc == fls.OK
    torch.cuda.synchronize()
    fls.fls_check_workspace()
    got_h = got.cpu().numpy()
    assert not np.isnan(got_h).any()
    ref = oracle_mod.ref_spmm_f64(W, Xb)
    assert float(np.abs(got_h.astype(np.float64) - ref).max()) / float(np.abs(ref).max()) <= TOL
