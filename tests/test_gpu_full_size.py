"""Full-size parity: the named configurations, the 12288 x 12288 sweep shape and the four MatMuls of an
OPT-30B-shaped decoder layer, each in the launch configuration bench.py times, with the WHOLE of C (every row
band) against the oracle's fp64 triple loop, and the compressed buffers byte for byte.

A wrong result of this kernel family is typically confined to one row band (a window of TileOffsets read one
entry off, a partial sum handed over too early), so nothing here samples bands.
"""
import numpy as np
import pytest

import fls_workloads as wl

pytestmark = pytest.mark.gpu

TOL = 2e-3


@pytest.fixture(scope="module")
def fls():
    import torch

    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2309_10285_amd as f

    f.lib()  # raises if the HIP library was not built: there is no fallback
    return f


def _whole_c_err(C_gpu, ref):
    """max |C - C_ref| / max |C_ref| over the whole matrix, plus the per-band worst (for the message)."""
    assert not np.isnan(C_gpu).any()
    scale = max(float(np.abs(ref).max()), 1e-30)
    diff = np.abs(C_gpu.astype(np.float64) - ref)
    per_band = diff.reshape(diff.shape[0], -1, 128).max(axis=(0, 2)) / scale
    return float(per_band.max()), int(per_band.argmax())


def _spmm(fls, Wbits, Xbits):
    import torch

    M, K = Wbits.shape
    N = Xbits.shape[0]
    blob, st = fls.fls_compress(torch.from_numpy(Wbits.view(np.float16)).cuda())
    X = torch.from_numpy(Xbits.view(np.float16)).cuda()
    C = torch.full((N, M), float("nan"), dtype=torch.float16, device="cuda")
    fls.ensure_workspace(M, K, N)
    fls.fls_spmm(blob, X, C, M, K, N)
    torch.cuda.synchronize()
    fls.fls_check_workspace()
    out = C.cpu().numpy()
    blob_host = blob.cpu().numpy()
    fls.fls_forget(blob)
    return blob_host, st, out


def _dense(fls, Wbits, Xbits):
    import torch

    M, K = Wbits.shape
    N = Xbits.shape[0]
    W = torch.from_numpy(Wbits.view(np.float16)).cuda()
    X = torch.from_numpy(Xbits.view(np.float16)).cuda()
    C = torch.full((N, M), float("nan"), dtype=torch.float16, device="cuda")
    fls.ensure_workspace(M, K, N)
    fls.fls_dense_gemm(W, X, C, M, K, N)
    torch.cuda.synchronize()
    return C.cpu().numpy()


@pytest.mark.parametrize("name", ["C2", "C3", "C4", "S1"])
def test_named_configuration_whole_c_and_blob(fls, oracle_mod, name):
    """C2 (N = 16, one band per workgroup), C4 (N = 64: the 64-column pass), C3 and S1 (N = 32 on long bands: the
    64-column pass with one 32-column block multiplied): blob byte-exact against the oracle's compressor, every
    element of C against the oracle."""
    cfg = wl.CONFIGS[name]
    W, X = wl.make_inputs(cfg)
    blob, st, C = _spmm(fls, W, X)
    ref_blob = oracle_mod.ref_compress(W)
    assert st["bytes_total"] == ref_blob.size and st["nnz"] == int(np.count_nonzero(W))
    assert np.array_equal(blob, ref_blob)
    del ref_blob, blob
    err, band = _whole_c_err(C, oracle_mod.ref_spmm_f64(W, X))
    assert err <= TOL, (name, "worst band", band)


def test_c3_in_the_narrow_kernel_whole_c(fls, oracle_mod):
    """C3 through fls_spmm_noalloc, which keeps to the narrow kernel (two column blocks per wave, one band per
    workgroup) where fls_spmm takes the 64-column pass: every element of C against the oracle."""
    import torch

    cfg = wl.CONFIGS["C3"]
    W, X = wl.make_inputs(cfg)
    blob, st = fls.fls_compress(torch.from_numpy(W.view(np.float16)).cuda())
    Xd = torch.from_numpy(X.view(np.float16)).cuda()
    C = torch.full((cfg.N, cfg.M), float("nan"), dtype=torch.float16, device="cuda")
    fls.fls_spmm_noalloc(blob, st, Xd, C, cfg.M, cfg.K, cfg.N)
    torch.cuda.synchronize()
    fls.fls_check_workspace()
    err, band = _whole_c_err(C.cpu().numpy(), oracle_mod.ref_spmm_f64(W, X))
    assert err <= TOL, ("worst band", band)


@pytest.fixture(scope="module")
def sweep_w32():
    return wl.gen_weights_f32(wl.SWEEP_M, wl.SWEEP_K, wl.SWEEP_SEED)


# one point per kernel path of the sweep: 96 bands cut between all workgroups with the hand-over through
# memory (N = 8, N = 32 at 60 %), the 64-column pass with K slices (N = 64), two such passes (N = 128), the
# row-skewed mask at 50 %, whose densest tiles need the ten-round register ring of the 64-column pass, and
# 32 columns at 90 %, which take the 64-column pass with one column block
SWEEP_POINTS = [("uniform", 0.8, 8), ("uniform", 0.6, 32), ("uniform", 0.9, 64), ("uniform", 0.7, 128),
                ("row_skewed", 0.5, 64), ("row_skewed", 0.5, 16), ("uniform", 0.9, 256), ("uniform", 0.9, 32)]


@pytest.mark.parametrize("mask,beta,N", SWEEP_POINTS, ids=[f"{m}-{int(b * 100)}-N{n}" for m, b, n in SWEEP_POINTS])
def test_sweep_shape_whole_c(fls, oracle_mod, sweep_w32, mask, beta, N):
    prune = wl.prune_uniform if mask == "uniform" else wl.prune_row_skewed
    W = prune(sweep_w32, beta, wl.SWEEP_SEED + 1)
    X = wl.gen_x(N, wl.SWEEP_K, wl.SWEEP_SEED + 2)
    blob, st, C = _spmm(fls, W, X)
    assert st["nnz"] == int(np.count_nonzero(W))
    if mask == "row_skewed":
        assert st["max_tile_words"] > 2048  # the case this point is here for
    err, band = _whole_c_err(C, oracle_mod.ref_spmm_f64(W, X))
    assert err <= TOL, ("worst band", band)


@pytest.mark.parametrize("N", [16, 64])
def test_sweep_shape_dense_pair_whole_c(fls, oracle_mod, sweep_w32, N):
    W = wl.dense_bits(sweep_w32)
    X = wl.gen_x(N, wl.SWEEP_K, wl.SWEEP_SEED + 2)
    err, band = _whole_c_err(_dense(fls, W, X), oracle_mod.ref_spmm_f64(W, X))
    assert err <= TOL, ("worst band", band)


LAYER = wl.decoder_layer(7168, 28672, 16, 0.8)


@pytest.mark.parametrize("cfg", LAYER, ids=[c.what.replace(" ", "-") for c in LAYER])
def test_decoder_layer_matmul_whole_c(fls, oracle_mod, cfg):
    """The four weight MatMuls of one OPT-30B-shaped decoder layer at N = 16 (168, 56, 224 and 56 row bands: three
    of them cut bands between workgroups)."""
    W, X = wl.make_inputs(cfg)
    blob, st, C = _spmm(fls, W, X)
    assert np.array_equal(blob, oracle_mod.ref_compress(W))
    err, band = _whole_c_err(C, oracle_mod.ref_spmm_f64(W, X))
    assert err <= TOL, (cfg.what, "worst band", band)


def test_latency_breakdown_builds_run_and_the_unablated_one_is_right(fls, oracle_mod):
    """The latency-breakdown tool (the method of the paper's Fig. 11): its build with nothing erased
    (-DFLS_ABLATE=0) must give the oracle's result, and a build with the on-chip stages erased must run to its
    end (its results are wrong by design).  Both are compiled beforehand by __graft_entry__.build(); narrow and
    64-column pass."""
    import os

    import torch

    from paper_2309_10285_amd import latency_breakdown as lb

    libs = {m: os.path.join(lb.PREBUILT_DIR, f"libfls_ablate{m}.so") for m in lb.PREBUILT_MASKS}
    for path in libs.values():
        assert os.path.exists(path), f"{path} is missing: run __graft_entry__.build()"
    M, K = 1536, 4096  # 12 bands: cut between workgroups in both passes
    W = wl.prune_uniform(wl.gen_weights_f32(M, K, 701), 0.8, 702)
    blob, _ = fls.fls_compress(torch.from_numpy(W.view(np.float16)).cuda())
    for N in (16, 64):
        Xb = wl.gen_x(N, K, 703 + N)
        X = torch.from_numpy(Xb.view(np.float16)).cuda()
        ws = torch.empty(fls.fls_workspace_bytes(M, K, N), dtype=torch.uint8, device="cuda")
        C = torch.full((N, M), float("nan"), dtype=torch.float16, device="cuda")
        assert lb.run_once(libs[0], blob, X, C, M, K, N, ws) == 0
        err, band = _whole_c_err(C.cpu().numpy(), oracle_mod.ref_spmm_f64(W, Xb))
        assert err <= TOL, (N, band)
        assert lb.run_once(libs[lb.PREBUILT_MASKS[1]], blob, X, C, M, K, N, ws) == 0
    fls.fls_forget(blob)
