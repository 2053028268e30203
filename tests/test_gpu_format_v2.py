"""Format version 2 (four entries share a word of locations, 3 bytes per nonzero) on the GPU: the compressor bit for bit
against the oracle's, and fls_spmm on version-2 blobs against the oracle's fp64 triple loop (whole C)."""
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

    f.lib()
    return f


def _dev(bits):
    import torch

    return torch.from_numpy(bits.view(np.float16)).cuda()


def _cases():
    out = []
    for name, M, K, beta, mask in [
        ("one-tile", 128, 32, 0.8, "uniform"),
        ("ragged-7x9-tiles", 896, 288, 0.7, "uniform"),
        ("C1", 1024, 1024, 0.8, "uniform"),
        ("magnitude-90", 1536, 2048, 0.9, "magnitude"),
        ("half-dense", 640, 512, 0.5, "uniform"),
        ("dense-0pct", 384, 256, 0.0, "uniform"),
        ("row-skewed", 2048, 1024, 0.8, "row_skewed"),
        # sparse enough for many gaps of more than 63 locations (bridge entries), and for empty tiles
        ("uniform-99", 1024, 512, 0.99, "uniform"),
        ("uniform-99.9", 512, 1024, 0.999, "uniform"),
        ("long-share-kt2", 128 * 700, 64, 0.8, "uniform"),
    ]:
        W32 = wl.gen_weights_f32(M, K, 4000 + len(out))
        if mask == "uniform":
            W = wl.prune_uniform(W32, beta, 7) if beta > 0 else wl.dense_bits(W32)
        elif mask == "magnitude":
            W = wl.prune_magnitude(W32, beta)
        else:
            W = wl.prune_row_skewed(W32, beta, 7)
        out.append((name, W))
    return out


CASES = _cases()


@pytest.mark.parametrize("name,W", CASES, ids=[c[0] for c in CASES])
def test_compress_v2_bit_exact(fls, oracle_mod, name, W):
    blob, st = fls.fls_compress_v2(_dev(W))
    ref = oracle_mod.ref_compress_v2(W)
    got = blob.cpu().numpy()
    assert got.size == ref.size == st["bytes_total"]
    assert np.array_equal(got, ref)
    info = oracle_mod.ref_inspect_v2(ref)
    assert st["format_version"] == 2 and st["nnz"] == info["nnz"] == int(np.count_nonzero(W))
    assert st["max_tile_words"] == info["max_tile_words"]
    assert fls.fls_inspect(got[:64].tobytes())["bytes_total"] == ref.size


def test_compress_v2_special_values_and_edge_tiles(fls, oracle_mod):
    g = np.random.Generator(np.random.Philox(8))
    M, K = 384, 128
    bits = g.integers(0, 65536, size=(M, K), dtype=np.uint32).astype(np.uint16)  # NaN, Inf, -0, subnormals
    W = np.where(g.random((M, K)) < 0.3, bits, np.uint16(0))
    W[:128, :32] = 0                               # an empty tile
    W[128:256, 32:64] = bits[128:256, 32:64] | 1   # a full tile
    W[256, 0] = 0x8000                             # -0.0 at the first location
    W[383, 127] = 0x7E01                           # NaN payload at the last location
    W[0:128, 64:96] = 0
    W[127, 95] = 0x3C00                            # a tile whose only element is its last location: 16 bridges
    blob, st = fls.fls_compress_v2(_dev(W))
    assert np.array_equal(blob.cpu().numpy(), oracle_mod.ref_compress_v2(W))
    assert np.array_equal(oracle_mod.ref_decompress_v2(blob.cpu().numpy(), M, K), W)
    Z = np.zeros((256, 64), dtype=np.uint16)
    blob, st = fls.fls_compress_v2(_dev(Z))
    assert st["nnz"] == 0 and np.array_equal(blob.cpu().numpy(), oracle_mod.ref_compress_v2(Z))


def _spmm_v2(fls, W, X):
    import torch

    M, K = W.shape
    N = X.shape[0]
    blob, st = fls.fls_compress_v2(_dev(W))
    Xd = torch.from_numpy(X.view(np.float16)).cuda()
    C = torch.full((N, M), float("nan"), dtype=torch.float16, device="cuda")
    fls.ensure_workspace(M, K, N)
    fls.fls_spmm(blob, Xd, C, M, K, N)
    torch.cuda.synchronize()
    fls.fls_check_workspace()
    fls.fls_forget(blob)
    return st, C.cpu().numpy()


@pytest.mark.parametrize("name,W", CASES, ids=[c[0] for c in CASES])
@pytest.mark.parametrize("N", [1, 16, 17, 32, 100])
def test_spmm_on_v2_blobs_matches_oracle(fls, oracle_mod, name, W, N):
    M, K = W.shape
    X = wl.gen_x(N, K, 199 + N)
    _, C = _spmm_v2(fls, W, X)
    ref = oracle_mod.ref_spmm_f64(W, X)
    assert np.isfinite(C).all()
    assert float(np.abs(C.astype(np.float64) - ref).max()) / max(float(np.abs(ref).max()), 1e-30) <= TOL


def test_spmm_v2_small_integers_exact_and_identity(fls, oracle_mod):
    g = np.random.Generator(np.random.Philox(4))
    M, K, N = 512, 640, 24
    Wi = g.integers(-3, 4, size=(M, K))
    Wi[g.random((M, K)) < 0.8] = 0
    Xi = g.integers(-2, 3, size=(N, K))
    W = Wi.astype(np.float16).view(np.uint16)
    X = Xi.astype(np.float16).view(np.uint16)
    _, C = _spmm_v2(fls, W, X)
    assert np.array_equal(C.astype(np.float64), oracle_mod.ref_spmm_f64(W, X))
    # identity X returns the columns of W bit for bit (so every value sits at its own location)
    W2 = CASES[2][1][:, :32].copy()
    X2 = np.zeros((32, 32), dtype=np.uint16)
    X2[np.arange(32), np.arange(32)] = 0x3C00
    _, C2 = _spmm_v2(fls, W2, X2)
    assert np.array_equal(C2.view(np.uint16), W2.T)


@pytest.mark.parametrize("name", ["C2", "C3", "C4"])
def test_named_configuration_v2_whole_c_and_blob(fls, oracle_mod, name):
    cfg = wl.CONFIGS[name]
    W, X = wl.make_inputs(cfg)
    import torch

    blob, st = fls.fls_compress_v2(_dev(W))
    ref_blob = oracle_mod.ref_compress_v2(W)
    assert np.array_equal(blob.cpu().numpy(), ref_blob)
    assert 2.99 < st["bytes_nonzeros"] / st["nnz"] < 3.02  # three bytes per kept weight
    del blob, ref_blob
    _, C = _spmm_v2(fls, W, X)
    ref = oracle_mod.ref_spmm_f64(W, X)
    assert not np.isnan(C).any()
    assert float(np.abs(C.astype(np.float64) - ref).max()) / float(np.abs(ref).max()) <= TOL


@pytest.mark.parametrize("N", [16, 64])
def test_v2_blob_replaced_in_place_by_a_denser_one(fls, oracle_mod, N):
    """The kernel variant is picked for a sparse blob, then a denser version-2 blob of the same shape is copied
    over it without fls_forget: its tiles have more groups than the ring stages, and the rest goes through the
    slow path (N = 16) or the whole grid takes the plain tile-by-tile path (N = 64)."""
    import torch

    M, K = 1024, 2048
    W32 = wl.gen_weights_f32(M, K, 41)
    sparse, dense = wl.prune_uniform(W32, 0.9, 42), wl.prune_uniform(W32, 0.45, 43)
    X = wl.gen_x(N, K, 44)
    Xd = torch.from_numpy(X.view(np.float16)).cuda()
    blob_s, _ = fls.fls_compress_v2(_dev(sparse))
    blob_d, _ = fls.fls_compress_v2(_dev(dense))
    blob_s, blob_d = blob_s.clone(), blob_d.clone()
    place = torch.zeros(max(blob_s.numel(), blob_d.numel()), dtype=torch.uint8, device="cuda")
    fls.ensure_workspace(M, K, N)
    fls.fls_forget(place)
    place[:blob_s.numel()].copy_(blob_s)
    C = torch.full((N, M), float("nan"), dtype=torch.float16, device="cuda")
    fls.fls_spmm(place, Xd, C, M, K, N)
    place[:blob_d.numel()].copy_(blob_d)
    fls.fls_spmm(place, Xd, C, M, K, N)
    torch.cuda.synchronize()
    ref = oracle_mod.ref_spmm_f64(dense, X)
    assert float(np.abs(C.cpu().numpy().astype(np.float64) - ref).max()) / float(np.abs(ref).max()) <= TOL
    fls.fls_forget(place)
