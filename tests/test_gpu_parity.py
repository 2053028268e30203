"""GPU parity tests: the HIP path, called through the C ABI, against the CPU oracle on the same seeded inputs.

Bars: compressed buffers bit-exact; C within max|C - C_ref| / max|C_ref| <= 2e-3 after fp16 output
rounding (products exact, fp32 accumulation, one fp16 rounding; the bound is the task's stated tolerance).
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


def _dev_w(bits):
    import torch

    return torch.from_numpy(bits.view(np.float16)).cuda()


def _rel_err(C_gpu, C_ref):
    scale = max(float(np.abs(C_ref).max()), 1e-30)
    return float(np.abs(C_gpu.astype(np.float64) - C_ref).max()) / scale


def _run_spmm(fls, Wbits, Xbits, N):
    import torch

    M, K = Wbits.shape
    blob, st = fls.fls_compress(_dev_w(Wbits))
    X = torch.from_numpy(Xbits.view(np.float16)).cuda()
    C = torch.full((N, M), float("nan"), dtype=torch.float16, device="cuda")
    fls.ensure_workspace(M, K, N)
    fls.fls_spmm(blob, X, C, M, K, N)
    torch.cuda.synchronize()
    return blob, st, C.cpu().numpy()


def _run_dense(fls, Wbits, Xbits, N):
    import torch

    M, K = Wbits.shape
    X = torch.from_numpy(Xbits.view(np.float16)).cuda()
    C = torch.full((N, M), float("nan"), dtype=torch.float16, device="cuda")
    fls.ensure_workspace(M, K, N)
    fls.fls_dense_gemm(_dev_w(Wbits), X, C, M, K, N)
    torch.cuda.synchronize()
    return C.cpu().numpy()


def _cases():
    g = np.random.Generator(np.random.Philox(2024))
    out = []
    # (name, M, K, beta, mask)
    for name, M, K, beta, mask in [
        ("one-tile", 128, 32, 0.8, "uniform"),
        ("one-band", 128, 1024, 0.8, "uniform"),
        ("ragged-7x9-tiles", 896, 288, 0.7, "uniform"),
        ("C1", 1024, 1024, 0.8, "uniform"),
        ("magnitude-90", 1536, 2048, 0.9, "magnitude"),
        ("half-dense", 640, 512, 0.5, "uniform"),
        ("dense-0pct", 384, 256, 0.0, "uniform"),
        ("row-skewed", 2048, 1024, 0.8, "row_skewed"),
        ("many-bands-short-k", 8192, 64, 0.8, "uniform"),
        # shares of a workgroup that span many bands (slot turns, whole bands inside one wave)
        ("long-share-kt1", 128 * 2304, 32, 0.8, "uniform"),
        ("long-share-kt2", 128 * 1500, 64, 0.8, "uniform"),
        ("long-share-kt3", 128 * 1111, 96, 0.7, "uniform"),
        # longest tile between 512 and 768 words, and between 1024 and 1536: the three- and six-round rings
        ("uniform-87", 1024, 1024, 0.87, "uniform"),
        ("uniform-68", 768, 1024, 0.68, "uniform"),
        # longest tile between 2048 and 2560 words: the ten-round ring of the 64-column pass
        ("uniform-45", 512, 1024, 0.45, "uniform"),
    ]:
        W32 = wl.gen_weights_f32(M, K, int(g.integers(1 << 30)))
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
def test_compress_bit_exact(fls, oracle_mod, name, W):
    blob, st = fls.fls_compress(_dev_w(W))
    ref = oracle_mod.ref_compress(W)
    got = blob.cpu().numpy()
    assert got.size == ref.size == st["bytes_total"]
    assert np.array_equal(got, ref)
    info = oracle_mod.ref_inspect(ref)
    assert st["nnz"] == info["nnz"] == int(np.count_nonzero(W))
    assert st["max_tile_words"] == info["max_tile_words"] and st["num_tiles"] == info["num_tiles"]
    assert fls.fls_inspect(got[:64].tobytes())["bytes_total"] == ref.size


def test_compress_special_values_and_edge_tiles(fls, oracle_mod):
    g = np.random.Generator(np.random.Philox(8))
    M, K = 384, 128
    bits = g.integers(0, 65536, size=(M, K), dtype=np.uint32).astype(np.uint16)  # NaN, Inf, -0, subnormals
    W = np.where(g.random((M, K)) < 0.3, bits, np.uint16(0))
    W[:128, :32] = 0                      # an empty tile
    W[128:256, 32:64] = bits[128:256, 32:64] | 1   # a full tile
    W[256, 0] = 0x8000                    # -0.0 at the first location
    W[383, 127] = 0x7E01                  # NaN payload at the last location
    blob, st = fls.fls_compress(_dev_w(W))
    ref = oracle_mod.ref_compress(W)
    assert np.array_equal(blob.cpu().numpy(), ref)
    assert np.array_equal(oracle_mod.ref_decompress(blob.cpu().numpy(), M, K), W)
    # all-zero matrix
    Z = np.zeros((256, 64), dtype=np.uint16)
    blob, st = fls.fls_compress(_dev_w(Z))
    assert st["nnz"] == 0 and np.array_equal(blob.cpu().numpy(), oracle_mod.ref_compress(Z))


@pytest.mark.parametrize("name,W", CASES, ids=[c[0] for c in CASES])
@pytest.mark.parametrize("N", [1, 8, 16, 17, 32, 64])
def test_spmm_matches_oracle(fls, oracle_mod, name, W, N):
    M, K = W.shape
    X = wl.gen_x(N, K, 99 + N)
    _, _, C = _run_spmm(fls, W, X, N)
    ref = oracle_mod.ref_spmm_f64(W, X)
    assert np.isfinite(C).all()
    assert _rel_err(C, ref) <= TOL


@pytest.mark.parametrize("N", [33, 48, 80, 96, 100, 128, 256])
def test_spmm_wide_n(fls, oracle_mod, N):
    # column groups of 64 in one launch, the last one partly empty (33, 48: a single group; 80, 96, 100: two)
    W = CASES[3][1]
    M, K = W.shape
    X = wl.gen_x(N, K, 5)
    _, _, C = _run_spmm(fls, W, X, N)
    assert _rel_err(C, oracle_mod.ref_spmm_f64(W, X)) <= TOL


@pytest.mark.parametrize("fmt", [1, 2])
@pytest.mark.parametrize("M,K,beta,N", [(512, 12288, 0.9, 32), (640, 16384, 0.8, 17), (640, 12288, 0.85, 24),
                                        (512, 12288, 0.8, 96), (384, 12288, 0.6, 32), (640, 32768, 0.9, 32),
                                        (256, 40960, 0.8, 20), (256, 12288, 0.45, 32), (384, 6144, 0.8, 32)])
def test_17_to_32_columns_on_long_bands(fls, oracle_mod, M, K, beta, N, fmt):
    """Calls (or the rest of a call) of 17 - 32 columns on bands of at least 384 K tiles take the 64-column pass
    with only its first 32-column block multiplied, whatever the density of the tiles (90 ... 45 %: the rings of two
    to ten rounds) - in format version 2 only sparse tiles on bands of at least 1024 K tiles (the shapes with
    K = 32768 and 40960) - and the narrow kernel otherwise (K = 6144).  Five bands: the second workgroup of a K slice
    has three waves without a band.  N = 96: two groups of 64 columns in one launch, the second half empty.  Whole C against the oracle.
    """
    import torch

    W = wl.prune_uniform(wl.gen_weights_f32(M, K, 1300 + N), beta, 1301 + N)
    Xb = wl.gen_x(N, K, 1302 + N)
    blob, st = (fls.fls_compress_v2 if fmt == 2 else fls.fls_compress)(_dev_w(W))
    X = torch.from_numpy(Xb.view(np.float16)).cuda()
    C = torch.full((N, M), float("nan"), dtype=torch.float16, device="cuda")
    fls.ensure_workspace(M, K, N)
    fls.fls_spmm(blob, X, C, M, K, N)
    fls.fls_spmm(blob, X, C, M, K, N)  # the second call finds the header remembered
    torch.cuda.synchronize()
    fls.fls_check_workspace()
    fls.fls_forget(blob)
    out = C.cpu().numpy()
    assert np.isfinite(out).all()
    assert _rel_err(out, oracle_mod.ref_spmm_f64(W, Xb)) <= TOL


@pytest.mark.parametrize("N", [384, 512, 1000, 4096])
def test_spmm_and_dense_non_skinny_n(fls, oracle_mod, N):
    """N beyond the skinny range (Sec. 6.2, non-skinny shapes): groups of 64 columns in one launch, a ragged last
    one for N = 1000 (40 of its 64 columns exist); byte offsets into X and C reach tens of MB."""
    W = CASES[4][1]  # 1536 x 2048, 90 % magnitude-pruned: bands cut between workgroups, K slices
    M, K = W.shape
    X = wl.gen_x(N, K, 700 + N)
    ref = oracle_mod.ref_spmm_f64(W, X)
    _, _, C = _run_spmm(fls, W, X, N)
    assert _rel_err(C, ref) <= TOL
    assert _rel_err(_run_dense(fls, W, X, N), ref) <= TOL


def test_spmm_small_integers_exact(fls, oracle_mod):
    # every partial sum is an integer below 2^24: fp32 accumulation in any order is exact, and so is fp16 output
    g = np.random.Generator(np.random.Philox(4))
    M, K, N = 512, 640, 24
    Wi = g.integers(-3, 4, size=(M, K))
    Wi[g.random((M, K)) < 0.8] = 0
    Xi = g.integers(-2, 3, size=(N, K))
    W = Wi.astype(np.float16).view(np.uint16)
    X = Xi.astype(np.float16).view(np.uint16)
    _, _, C = _run_spmm(fls, W, X, N)
    ref = oracle_mod.ref_spmm_f64(W, X)
    assert np.abs(ref).max() < 2048
    assert np.array_equal(C.astype(np.float64), ref)
    assert np.array_equal(_run_dense(fls, W, X, N).astype(np.float64), ref)


def test_spmm_identity_x_returns_columns(fls):
    W = CASES[3][1][:, :64].copy()
    M, K = W.shape
    X = np.zeros((64, 64), dtype=np.uint16)
    X[np.arange(64), np.arange(64)] = 0x3C00
    _, _, C = _run_spmm(fls, W, X, 64)
    assert np.array_equal(C.view(np.uint16), W.T)  # bit exact, incl. zeros


def test_spmm_zero_matrix_and_repeat_calls(fls, oracle_mod):
    import torch

    Z = np.zeros((256, 128), dtype=np.uint16)
    X = wl.gen_x(16, 128, 1)
    _, _, C = _run_spmm(fls, Z, X, 16)
    assert np.count_nonzero(C) == 0
    # the workspace must come back clean: repeated calls give the same answer
    W = CASES[3][1]
    M, K = W.shape
    X = wl.gen_x(16, K, 2)
    ref = oracle_mod.ref_spmm_f64(W, X)
    blob, _ = fls.fls_compress(_dev_w(W))
    Xd = torch.from_numpy(X.view(np.float16)).cuda()
    fls.ensure_workspace(M, K, 16)
    for _ in range(5):
        C = torch.zeros((16, M), dtype=torch.float16, device="cuda")
        fls.fls_spmm(blob, Xd, C, M, K, 16)
        torch.cuda.synchronize()
        assert _rel_err(C.cpu().numpy(), ref) <= TOL


def test_spmm_order_invariance(fls, oracle_mod):
    """Sec. 4.3.3: reordering a tile's words changes global-memory order only; the kernel result stays."""
    import torch

    W = CASES[3][1]
    M, K = W.shape
    N = 16
    X = wl.gen_x(N, K, 3)
    ref = oracle_mod.ref_spmm_f64(W, X)
    blob = oracle_mod.ref_compress(W, policy=1)      # an oracle-made blob in the other word order
    blob[20:24] = 0                                  # keep the header's policy field within what the library takes
    bd = torch.from_numpy(blob).cuda()
    Xd = torch.from_numpy(X.view(np.float16)).cuda()
    C = torch.zeros((N, M), dtype=torch.float16, device="cuda")
    fls.ensure_workspace(M, K, N)
    fls.fls_spmm(bd, Xd, C, M, K, N)
    torch.cuda.synchronize()
    assert _rel_err(C.cpu().numpy(), ref) <= TOL


@pytest.mark.parametrize("name,W", CASES[:6] + CASES[9:12], ids=[c[0] for c in CASES[:6] + CASES[9:12]])
@pytest.mark.parametrize("N", [8, 16, 40, 64, 256])
def test_dense_gemm_matches_oracle(fls, oracle_mod, name, W, N):
    M, K = W.shape
    X = wl.gen_x(N, K, 17 + N)
    C = _run_dense(fls, W, X, N)
    assert _rel_err(C, oracle_mod.ref_spmm_f64(W, X)) <= TOL


def test_error_codes_on_device(fls):
    import torch

    W = _dev_w(CASES[0][1])
    small = torch.empty(1024, dtype=torch.uint8, device="cuda")
    with pytest.raises(fls.FlsError) as e:
        fls.fls_compress(W, out=small)
    assert e.value.code == fls.ECAPACITY
    blob, _ = fls.fls_compress(W)
    X = torch.zeros((8, 32), dtype=torch.float16, device="cuda")
    C = torch.zeros((8, 128), dtype=torch.float16, device="cuda")
    fls.ensure_workspace(256, 32, 8)
    bad = blob.clone()
    bad[0] = 0
    rc = fls.lib().fls_spmm(bad.data_ptr(), X.data_ptr(), C.data_ptr(), 128, 32, 8, None)
    assert rc == fls.EFORMAT
    rc = fls.lib().fls_spmm(blob.data_ptr(), X.data_ptr(), C.data_ptr(), 256, 32, 8, None)
    assert rc == fls.EFORMAT  # header says 128 rows
    rc = fls.lib().fls_spmm(blob.data_ptr() + 2, X.data_ptr(), C.data_ptr(), 128, 32, 8, None)
    assert rc == fls.EALIGN


def test_spmm_wide_n_split_bands(fls, oracle_mod):
    # few bands, long K: every band is cut between workgroups, so the 64-column pass hands 32 KB partial sums over
    W = wl.prune_uniform(wl.gen_weights_f32(384, 8192, 11), 0.9, 12)
    for N in (64, 72):
        X = wl.gen_x(N, 8192, 13)
        _, _, C = _run_spmm(fls, W, X, N)
        assert _rel_err(C, oracle_mod.ref_spmm_f64(W, X)) <= TOL


def test_back_to_back_shapes_share_one_workspace(fls, oracle_mod):
    """Calls of different shapes and widths, alternating, on one registered workspace: flags raised by a launch are lowered by it,
    nothing is cleared in between, and the kernels' error word (a hand-over wait that gave up) stays 0."""
    import torch

    work = []
    for (name, W), N in zip([CASES[3], CASES[4], CASES[7], CASES[1]], [16, 64, 32, 80]):
        M, K = W.shape
        X = wl.gen_x(N, K, 21 + N)
        work.append((W, X, N, oracle_mod.ref_spmm_f64(W, X)))
    fls.ensure_workspace(2048, 2048, 256)  # large enough for all of them
    ws = fls._ws_tensor
    blobs = [fls.fls_compress(_dev_w(W))[0] for W, _, _, _ in work]
    for rep in range(3):
        for (W, X, N, ref), blob in zip(work, blobs):
            M, K = W.shape
            Xd = torch.from_numpy(X.view(np.float16)).cuda()
            C = torch.full((N, M), float("nan"), dtype=torch.float16, device="cuda")
            fls.fls_spmm(blob, Xd, C, M, K, N)
            D = torch.full((N, M), float("nan"), dtype=torch.float16, device="cuda")
            fls.fls_dense_gemm(_dev_w(W), Xd, D, M, K, N)
            torch.cuda.synchronize()
            assert _rel_err(C.cpu().numpy(), ref) <= TOL
            assert _rel_err(D.cpu().numpy(), ref) <= TOL
    assert fls._ws_tensor is ws  # still the same registration
    fls.fls_check_workspace()  # raises if a hand-over wait gave up


def test_very_long_k(fls, oracle_mod):
    """One row band with K = 2^21 (65536 K tiles, every workgroup inside the same band, byte offsets into X beyond
    2^27): the blob against the oracle's, C for a narrow and a 64-column call."""
    M, K = 128, 1 << 21
    W = wl.prune_uniform(wl.gen_weights_f32(M, K, 31), 0.95, 32)
    ref_blob = oracle_mod.ref_compress(W)
    for N in (8, 64):
        X = wl.gen_x(N, K, 33 + N)
        blob, st, C = _run_spmm(fls, W, X, N)
        if N == 8:
            assert np.array_equal(blob.cpu().numpy(), ref_blob)
        assert _rel_err(C, oracle_mod.ref_spmm_f64(W, X)) <= TOL
    assert _rel_err(_run_dense(fls, W, X[:16], 16), oracle_mod.ref_spmm_f64(W, X[:16])) <= TOL


@pytest.mark.parametrize("M,K,N", [(1024, 2048, 16), (1024, 2048, 64), (1024, 2048, 100), (256, 12288, 32)])
def test_blob_replaced_in_place_behind_the_librarys_back(fls, oracle_mod, M, K, N):
    """A sparse blob is used at an address, then the bytes of a denser blob of the same shape are copied over it
    without fls_forget: the kernel variant is still picked for the sparse one (a ring too short for the new tiles),
    and the results must be right all the same, in the 32-column passes, in the 64-column pass and (32 columns on
    bands of 384 K tiles) in that pass with one column block.  Then the other way round (a ring longer than needed)."""
    import torch

    W32 = wl.gen_weights_f32(M, K, 41)
    sparse, dense = wl.prune_uniform(W32, 0.9, 42), wl.prune_uniform(W32, 0.45, 43)
    X = wl.gen_x(N, K, 44)
    Xd = torch.from_numpy(X.view(np.float16)).cuda()
    blob_s, st_s = fls.fls_compress(_dev_w(sparse))
    blob_d, st_d = fls.fls_compress(_dev_w(dense))
    assert st_s["max_tile_words"] <= 1024 and st_d["max_tile_words"] > 2048
    blob_s, blob_d = blob_s.clone(), blob_d.clone()
    place = torch.zeros(max(blob_s.numel(), blob_d.numel()), dtype=torch.uint8, device="cuda")
    fls.ensure_workspace(M, K, N)
    for first, second, W_second in ((blob_s, blob_d, dense), (blob_d, blob_s, sparse)):
        fls.fls_forget(place)
        place[:first.numel()].copy_(first)
        C = torch.full((N, M), float("nan"), dtype=torch.float16, device="cuda")
        fls.fls_spmm(place, Xd, C, M, K, N)  # the header of `first` is remembered for this address from here on
        place[:second.numel()].copy_(second)
        fls.fls_spmm(place, Xd, C, M, K, N)
        torch.cuda.synchronize()
        assert _rel_err(C.cpu().numpy(), oracle_mod.ref_spmm_f64(W_second, X)) <= TOL
    fls.fls_forget(place)


def test_calls_recorded_in_a_graph_replay_right(fls, oracle_mod):
    """fls_spmm (32-column pass with bands cut between workgroups, 64-column pass) and fls_dense_gemm recorded
    into one HIP graph: every replay, with new contents in X and eager calls in between, must match the oracle -
    nothing in a launch's arguments may go stale (the hand-over flags are lowered by the launch that raised them)."""
    import torch

    M, K = 384, 8192  # 3 bands over all CUs: every band's sum crosses workgroups
    W = wl.prune_uniform(wl.gen_weights_f32(M, K, 51), 0.85, 52)
    blob, _ = fls.fls_compress(_dev_w(W))
    Wd = _dev_w(W)
    fls.ensure_workspace(M, K, 80)
    Xs = {N: wl.gen_x(N, K, 53 + N) for N in (16, 80)}
    Xd = {N: torch.from_numpy(Xs[N].view(np.float16)).cuda() for N in Xs}
    Cs = {N: torch.zeros((N, M), dtype=torch.float16, device="cuda") for N in Xs}
    D = torch.zeros((16, M), dtype=torch.float16, device="cuda")
    for N in Xs:  # ordinary calls first: headers read, kernel attributes set
        fls.fls_spmm(blob, Xd[N], Cs[N], M, K, N)
    fls.fls_dense_gemm(Wd, Xd[16], D, M, K, 16)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for N in Xs:
            fls.fls_spmm(blob, Xd[N], Cs[N], M, K, N)
        fls.fls_dense_gemm(Wd, Xd[16], D, M, K, 16)
    for rep in range(4):
        for N in Xs:
            Xs[N] = wl.gen_x(N, K, 60 + 7 * rep + N)
            Xd[N].copy_(torch.from_numpy(Xs[N].view(np.float16)))
            Cs[N].fill_(float("nan"))
        D.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        for N in Xs:
            assert _rel_err(Cs[N].cpu().numpy(), oracle_mod.ref_spmm_f64(W, Xs[N])) <= TOL, (rep, N)
        assert _rel_err(D.cpu().numpy(), oracle_mod.ref_spmm_f64(W, Xs[16])) <= TOL, rep
        # eager work on the same workspace between replays
        E = torch.full((16, M), float("nan"), dtype=torch.float16, device="cuda")
        fls.fls_spmm(blob, Xd[16], E, M, K, 16)
        torch.cuda.synchronize()
        assert torch.equal(E, Cs[16])
    fls.fls_check_workspace()  # raises if a hand-over wait gave up
    assert int(fls._ws_tensor[:512 * 4].cpu().numpy().view(np.uint32).max()) == 0  # every flag is down again


def test_check_workspace_reports_a_hand_over_that_gave_up(fls, oracle_mod):
    """The error word a kernel would set after its bounded wait is planted from the host (no kernel is made to
    wait): fls_check_workspace reports it once, clears the control area, and the next calls run clean."""
    import torch

    name, W = CASES[1]
    M, K = W.shape
    X = wl.gen_x(16, K, 71)
    fls.ensure_workspace(M, K, 16)
    fls.fls_check_workspace()
    ws32 = fls._ws_tensor[:4 << 20].view(torch.int32)
    ws32[512] = 1  # the error word
    ws32[3] = 1    # and a flag left up, as the launch that gave up would leave it
    torch.cuda.synchronize()
    with pytest.raises(fls.FlsError) as e:
        fls.fls_check_workspace()
    assert e.value.code == fls.EHANDOVER
    fls.fls_check_workspace()
    assert int(ws32[:513].abs().max()) == 0
    _, _, C = _run_spmm(fls, W, X, 16)
    assert _rel_err(C, oracle_mod.ref_spmm_f64(W, X)) <= TOL
    fls.fls_check_workspace()


def test_piece_boundary_at_the_edge_of_the_offset_window(fls, oracle_mod):
    """Waves with more than 64 tiles whose run crosses into the next row band exactly at the last entry of their
    window of TileOffsets: the load side looks past the end of the piece and moves the window on, and the next
    piece starts one tile before the new window.  With 256 CUs that takes at least 129 000 tiles; this shape
    (258 bands x 500 K tiles) has four such waves, in bands 65, 81, 194 and 210 (a first version read the wrong
    offset there).  The whole of C is checked against the oracle."""
    import torch

    M, K, N = 258 * 128, 500 * 32, 16
    W = wl.prune_uniform(wl.gen_weights_f32(M, K, 81), 0.9, 82)
    X = wl.gen_x(N, K, 83)
    blob, st = fls.fls_compress(_dev_w(W))
    assert st["nnz"] == int(np.count_nonzero(W))
    Xd = torch.from_numpy(X.view(np.float16)).cuda()
    C = torch.full((N, M), float("nan"), dtype=torch.float16, device="cuda")
    fls.ensure_workspace(M, K, N)
    fls.fls_spmm(blob, Xd, C, M, K, N)
    torch.cuda.synchronize()
    C = C.cpu().numpy()
    assert not np.isnan(C).any()
    ref = oracle_mod.ref_spmm_f64(W, X)
    scale = float(np.abs(ref).max())
    per_band = np.abs(C.astype(np.float64) - ref).reshape(N, M // 128, 128).max(axis=(0, 2)) / scale
    assert per_band.max() <= TOL, ("worst band", int(per_band.argmax()))
    fls.fls_forget(blob)


def test_split_bands_after_wide_passes_many_repeats(fls, oracle_mod):
    """222 columns on a matrix whose bands are cut between workgroups, as two calls on one workspace: 192 columns
    through the 64-column pass (three groups in one launch), then 30 columns through the narrow kernel, whose
    partial-sum slots lie where the pass's partial results were a moment ago.  A hand-over that raised its flag
    before its partial sum had left the XCD's L2 gave a wrong band about once in a thousand such sequences; the
    first result is checked against the oracle in full, then 3000 more rounds must repeat it to within fp16
    rounding (inside a workgroup the waves' sums are added in the order they finish, so the last bit may differ; a
    wrong band is off by tens of percent)."""
    import torch

    M, K, N, NW = 24960, 9216, 222, 192
    W = wl.prune_uniform(wl.gen_weights_f32(M, K, 91), 0.9, 92)
    X = wl.gen_x(N, K, 93)
    blob, st = fls.fls_compress(_dev_w(W))
    Xd = torch.from_numpy(X.view(np.float16)).cuda()
    fls.ensure_workspace(M, K, N)

    def both(C):
        fls.fls_spmm(blob, Xd[:NW], C[:NW], M, K, NW)
        fls.fls_spmm(blob, Xd[NW:], C[NW:], M, K, N - NW)

    first = torch.full((N, M), float("nan"), dtype=torch.float16, device="cuda")
    both(first)
    torch.cuda.synchronize()
    got = first.cpu().numpy()
    assert not np.isnan(got).any()
    ref = oracle_mod.ref_spmm_f64(W, X)  # the whole of C: every later round is compared with this first result
    assert float(np.abs(got.astype(np.float64) - ref).max()) / float(np.abs(ref).max()) <= TOL
    del ref
    C = torch.empty_like(first)
    ref32 = first.float()
    scale = float(ref32.abs().max())
    worst = torch.zeros((), device="cuda")
    for rep in range(3000):
        C.fill_(float("nan"))
        both(C)
        worst = torch.maximum(worst, torch.nan_to_num((C.float() - ref32).abs(), nan=float("inf")).max())
    assert float(worst) / scale <= TOL
    fls.fls_check_workspace()
    fls.fls_forget(blob)


@pytest.mark.parametrize("N", [16, 32])
def test_offsets_past_the_end_of_nonzeros_are_clamped(fls, oracle_mod, N):
    """A blob whose last TileOffsets entries point past the end of NonZeros (a truncated or damaged file).  The
    passes of up to 32 columns take no offset to lie beyond the word count in the blob's header, so the last tile
    keeps its own words and the result is that of the intact blob.  (The 64-column pass trusts TileOffsets: a
    clamp there cost 5 - 14 % of its time.)  The buffer has room behind the blob, filled with words (1.0 at
    location 0) that would change C if they were read: every load of this test stays inside it."""
    import torch

    M, K = 512, 2048
    W = wl.prune_uniform(wl.gen_weights_f32(M, K, 1400), 0.8, 1401)
    X = wl.gen_x(N, K, 1402)
    blob, st = fls.fls_compress(_dev_w(W))
    Xd = torch.from_numpy(X.view(np.float16)).cuda()
    fls.ensure_workspace(M, K, N)
    good = torch.full((N, M), float("nan"), dtype=torch.float16, device="cuda")
    fls.fls_spmm(blob, Xd, good, M, K, N)
    torch.cuda.synchronize()
    ref = oracle_mod.ref_spmm_f64(W, X)
    assert float(np.abs(good.cpu().numpy().astype(np.float64) - ref).max()) / float(np.abs(ref).max()) <= TOL
    host = blob.cpu().numpy().view(np.uint32).copy()
    tiles = (M // 128) * (K // 32)
    n_off = st["bytes_offsets"] // 4
    assert host[16 + tiles] == st["bytes_nonzeros"] // 4
    host[16 + tiles: 16 + n_off] += 2000  # the last tile's end, and the guard entries behind it
    slack = np.full(16384, (0x3C00 << 16) | 0, dtype=np.uint32)
    damaged = torch.from_numpy(np.concatenate([host, slack]).view(np.uint8)).cuda()
    for call in ("spmm", "stats"):
        C = torch.full((N, M), float("nan"), dtype=torch.float16, device="cuda")
        if call == "spmm":
            fls.fls_spmm(damaged, Xd, C, M, K, N)
        else:
            fls.fls_spmm_stats(damaged, st, Xd, C, M, K, N)
        torch.cuda.synchronize()
        # (not bit for bit: with 32 columns the waves' sums are added in the order they finish; a slack word read
        # would add about 1 to an element of size 0.4)
        assert float((C.float() - good.float()).abs().max()) <= TOL * float(good.float().abs().max()), call
    fls.fls_forget()


@pytest.mark.parametrize("M,K,N", [(7168, 4096, 16), (12288, 6144, 32)])
def test_two_matrices_taking_turns_on_the_same_partial_sum_slots(fls, oracle_mod, M, K, N):
    """Two different matrices of one shape, multiplied in turns: both calls use the same grid, so workgroup q of
    either stores its partial sum at the same address and the band's owner reads it from there (56 bands cut
    evenly over 224 workgroups; 96 bands cut wherever the shares fall).  An owner that was served a slot's
    contents of the call before - from a cache on its side - would return the other matrix's band.  First
    results against the oracle over the whole of C, then 1000 more calls of each."""
    import torch

    items = []
    for i in range(2):
        W = wl.prune_uniform(wl.gen_weights_f32(M, K, 1300 + i), 0.8, 1310 + i)
        X = wl.gen_x(N, K, 1320 + i)
        blob, _ = fls.fls_compress(_dev_w(W))
        items.append(dict(W=W, X=X, blob=blob.clone(), Xd=torch.from_numpy(X.view(np.float16)).cuda()))
    fls.ensure_workspace(M, K, N)
    for it in items:
        C = torch.full((N, M), float("nan"), dtype=torch.float16, device="cuda")
        fls.fls_spmm(it["blob"], it["Xd"], C, M, K, N)
        torch.cuda.synchronize()
        got = C.cpu().numpy()
        assert not np.isnan(got).any()
        ref = oracle_mod.ref_spmm_f64(it["W"], it["X"])
        assert float(np.abs(got.astype(np.float64) - ref).max()) / float(np.abs(ref).max()) <= TOL
        it["first"] = C.float()
        it["scale"] = float(C.float().abs().max())
    worst = torch.zeros((), device="cuda")
    C = torch.empty((N, M), dtype=torch.float16, device="cuda")
    for rep in range(2000):
        it = items[rep & 1]
        C.fill_(float("nan"))
        fls.fls_spmm(it["blob"], it["Xd"], C, M, K, N)
        worst = torch.maximum(worst, torch.nan_to_num((C.float() - it["first"]).abs(), nan=float("inf")).max() / it["scale"])
    assert float(worst) <= TOL
    fls.fls_check_workspace()
    fls.fls_forget()


@pytest.mark.parametrize("N", [16, 100])
def test_spmm_with_caller_passed_stats_is_recordable_at_first_sight(fls, oracle_mod, N):
    """fls_spmm_stats takes the blob's statistics from the caller: no header read-back, nothing remembered.  A
    call on a blob address the library has never seen can therefore be recorded straight into a HIP graph
    (fls_spmm would have to copy the header back and wait); every replay must match the oracle."""
    import torch

    W = CASES[4][1]  # 1536 x 2048: bands cut between workgroups
    M, K = W.shape
    blob0, stats = fls.fls_compress(_dev_w(W))
    blob = blob0.clone()  # an address the library knows nothing about
    fls.fls_forget()
    fls.ensure_workspace(M, K, N)
    X = wl.gen_x(N, K, 880 + N)
    Xd = torch.from_numpy(X.view(np.float16)).cuda()
    C = torch.full((N, M), float("nan"), dtype=torch.float16, device="cuda")
    # eager first (sets kernel attributes), on yet another unseen address
    fls.fls_spmm_stats(blob0.clone(), stats, Xd, C, M, K, N)
    torch.cuda.synchronize()
    ref = oracle_mod.ref_spmm_f64(W, X)
    assert _rel_err(C.cpu().numpy(), ref) <= TOL
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        fls.fls_spmm_stats(blob, stats, Xd, C, M, K, N)
    for rep in range(3):
        X = wl.gen_x(N, K, 890 + 3 * rep + N)
        Xd.copy_(torch.from_numpy(X.view(np.float16)))
        C.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        assert _rel_err(C.cpu().numpy(), oracle_mod.ref_spmm_f64(W, X)) <= TOL, rep
    # statistics of another shape are refused on the host
    bad = dict(stats)
    bad["K"] = K + 32
    with pytest.raises(fls.FlsError) as e:
        fls.fls_spmm_stats(blob, bad, Xd, C, M, K, N)
    assert e.value.code == fls.EFORMAT
    fls.fls_check_workspace()
