"""Randomly drawn shapes, widths, sparsities and masks (seeded): fls_spmm and fls_dense_gemm through the C ABI
against the oracle, every element of C.  The fixed cases of test_gpu_parity.py were chosen by thought; these
are not, which is the point: a wrong answer for a shape nobody thought of shows up here."""
import numpy as np
import pytest

import fls_workloads as wl

pytestmark = pytest.mark.gpu

TOL = 2e-3


def _draw(seed, count):
    g = np.random.Generator(np.random.Philox(seed))
    out = []
    for i in range(count):
        M = 128 * int(g.integers(1, 65))
        K = 32 * int(g.integers(1, 257))
        N = int(g.integers(1, 257))
        beta = float(g.choice([0.0, 0.3, 0.5, 0.6, 0.7, 0.8, 0.9, 0.95, 0.99, 1.0]))
        mask = str(g.choice(["uniform", "uniform", "magnitude", "row_skewed"]))
        out.append((i, M, K, N, beta, mask))
    return out


CASES = _draw(20240917, 30)


@pytest.mark.parametrize("i,M,K,N,beta,mask", CASES, ids=[f"{c[1]}x{c[2]}-N{c[3]}-{int(c[4] * 100)}-{c[5]}" for c in CASES])
def test_random_shape_matches_oracle(oracle_mod, i, M, K, N, beta, mask):
    import torch

    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2309_10285_amd as fls

    fls.lib()
    W32 = wl.gen_weights_f32(M, K, 1000 + i)
    if beta >= 1.0:
        W = np.zeros((M, K), dtype=np.uint16)
    elif beta <= 0.0:
        W = wl.dense_bits(W32)
    elif mask == "magnitude":
        W = wl.prune_magnitude(W32, beta)
    elif mask == "row_skewed":
        W = wl.prune_row_skewed(W32, beta, 2000 + i)
    else:
        W = wl.prune_uniform(W32, beta, 2000 + i)
    X = wl.gen_x(N, K, 3000 + i)
    Wd = torch.from_numpy(W.view(np.float16)).cuda()
    Xd = torch.from_numpy(X.view(np.float16)).cuda()
    blob, st = fls.fls_compress(Wd)
    assert st["nnz"] == int(np.count_nonzero(W))
    fls.ensure_workspace(M, K, N)
    C = torch.full((N, M), float("nan"), dtype=torch.float16, device="cuda")
    D = torch.full((N, M), float("nan"), dtype=torch.float16, device="cuda")
    fls.fls_spmm(blob, Xd, C, M, K, N)
    fls.fls_dense_gemm(Wd, Xd, D, M, K, N)
    torch.cuda.synchronize()
    C, D = C.cpu().numpy(), D.cpu().numpy()
    assert not np.isnan(C).any() and not np.isnan(D).any()
    ref = oracle_mod.ref_spmm_f64(W, X)  # the whole of C
    scale = max(float(np.abs(ref).max()), 1e-30)
    for got in (C, D):
        assert float(np.abs(got.astype(np.float64) - ref).max()) / scale <= TOL
    if beta >= 1.0:
        assert not C.any() and not D.any()
    fls.fls_forget(blob)
    fls.fls_check_workspace()


def test_random_call_sequence_on_one_workspace(oracle_mod):
    """Eight matrices of different shapes, widths and sparsities; 2000 calls drawn at random among them (sparse and
    dense), back to back on one registered workspace, most of them without waiting in between.  Each matrix's first
    result is checked against the oracle in full; every later result must repeat it to within fp16
    rounding.  Calls of different shapes reuse the same flags, partial-sum slots and repacked-X area, so anything
    one call leaves behind, or reads before it is there, shows up as a wrong band in another."""
    import torch

    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2309_10285_amd as fls

    fls.lib()
    g = np.random.Generator(np.random.Philox(777))
    items = []
    for i in range(8):
        M = 128 * int(g.integers(8, 200))
        K = 32 * int(g.integers(8, 400))
        N = int(g.integers(1, 257))
        beta = float(g.choice([0.5, 0.7, 0.8, 0.9, 0.95]))
        W = wl.prune_uniform(wl.gen_weights_f32(M, K, 5000 + i), beta, 6000 + i)
        X = wl.gen_x(N, K, 7000 + i)
        Wd = torch.from_numpy(W.view(np.float16)).cuda()
        Xd = torch.from_numpy(X.view(np.float16)).cuda()
        blob, _ = fls.fls_compress(Wd)
        items.append(dict(M=M, K=K, N=N, W=W, X=X, Wd=Wd, Xd=Xd, blob=blob.clone()))
    fls.fls_forget()
    fls.ensure_workspace(128 * 200, 32 * 400, 256)
    for it in items:  # first results, against the oracle
        M, K, N = it["M"], it["K"], it["N"]
        for kind in ("spmm", "dense"):
            C = torch.full((N, M), float("nan"), dtype=torch.float16, device="cuda")
            if kind == "spmm":
                fls.fls_spmm(it["blob"], it["Xd"], C, M, K, N)
            else:
                fls.fls_dense_gemm(it["Wd"], it["Xd"], C, M, K, N)
            torch.cuda.synchronize()
            got = C.cpu().numpy()
            assert not np.isnan(got).any()
            ref = oracle_mod.ref_spmm_f64(it["W"], it["X"])  # the whole of C
            scale = max(float(np.abs(ref).max()), 1e-30)
            assert float(np.abs(got.astype(np.float64) - ref).max()) / scale <= TOL, kind
            it[kind] = C.float()
            it[kind + "_scale"] = max(float(C.float().abs().max()), 1e-30)
    worst = torch.zeros((), device="cuda")
    for step in range(2000):
        it = items[int(g.integers(0, len(items)))]
        kind = "spmm" if g.random() < 0.8 else "dense"
        M, K, N = it["M"], it["K"], it["N"]
        C = torch.full((N, M), float("nan"), dtype=torch.float16, device="cuda")
        if kind == "spmm":
            fls.fls_spmm(it["blob"], it["Xd"], C, M, K, N)
        else:
            fls.fls_dense_gemm(it["Wd"], it["Xd"], C, M, K, N)
        err = torch.nan_to_num((C.float() - it[kind]).abs(), nan=float("inf")).max() / it[kind + "_scale"]
        worst = torch.maximum(worst, err)
        if g.random() < 0.2:
            torch.cuda.synchronize()
    assert float(worst) <= TOL
    fls.fls_check_workspace()
    assert int(fls._ws_tensor[:512 * 4].cpu().numpy().view(np.uint32).max()) == 0  # every flag is down again
    fls.fls_forget()
