"""Host-side checks of the C ABI that need no GPU: the library loads, exports what include/fls.h
declares, and rejects bad arguments before anything is launched."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def fls():
    import paper_2309_10285_amd as f
    from paper_2309_10285_amd import _build

    if not os.path.exists(f.LIB_PATH):
        _build.build()
    return f


def test_every_declared_symbol_is_exported(fls):
    hdr = open(os.path.join(ROOT, "include", "fls.h")).read()
    declared = set(re.findall(r"\b(fls_[a-z0-9_]+)\s*\(", hdr))
    assert declared == set(fls.EXPORTS)
    L = fls.lib()
    for name in declared:
        assert getattr(L, name) is not None


def test_sizes_and_bounds(fls):
    # closed forms: header + offsets (round_up(tiles + 4, 16) u32) + 4 B per element
    assert fls.fls_compress_bound(128, 32) == 64 + 4 * 16 + 4 * 4096
    assert fls.fls_compress_bound(1024, 1024) == 64 + 4 * 272 + 4 * 1024 * 1024
    # 4 MiB control area + [512 workgroups][column blocks][128 x 16] fp32
    assert fls.fls_workspace_bytes(1024, 1024, 8) == (4 << 20) + 512 * 1 * 2048 * 4
    # from 17 columns on: the 64-column pass's [4 x 512 bands x slices][4 column blocks][128 x 16] fp32
    assert fls.fls_workspace_bytes(1024, 1024, 17) == (4 << 20) + 4 * 512 * 4 * 2048 * 4
    assert fls.fls_workspace_bytes(1024, 1024, 256) == (4 << 20) + 4 * 512 * 4 * 2048 * 4 + 1024 * 256 * 2
    assert fls.fls_workspace_bytes(1000, 1024, 8) == 0 and fls.fls_workspace_bytes(1024, 1024, 8193) == 0
    assert fls.TILE_M == 128 and fls.TILE_K == 32


def test_argument_errors_need_no_device(fls):
    L = fls.lib()
    sz = ctypes.c_size_t(0)
    assert L.fls_compress_bound(100, 32, ctypes.byref(sz)) == fls.EINVAL
    assert L.fls_compress_bound(128, 33, ctypes.byref(sz)) == fls.EINVAL
    assert L.fls_compress_bound(128, 32, None) == fls.EINVAL
    assert L.fls_spmm(None, None, None, 128, 32, 8, None) == fls.EINVAL
    assert L.fls_spmm(16, 16, 16, 128, 32, 0, None) == fls.EINVAL
    assert L.fls_spmm(16, 16, 16, 128, 32, 8193, None) == fls.EINVAL
    assert L.fls_spmm(16, 16, 16, 127, 32, 8, None) == fls.EINVAL
    # X (K x N fp16) and C are addressed with 32-bit byte offsets: 2 K N and 2 M N must stay below 2^31
    assert L.fls_spmm(16, 16, 16, 128, 1 << 23, 256, None) == fls.EINVAL
    assert L.fls_dense_gemm(16, 16, 16, 128 << 16, 32, 256, None) == fls.EINVAL
    assert L.fls_spmm(16, 8, 16, 128, 32, 8, None) == fls.EALIGN
    assert L.fls_spmm(16, 16, 16, 128, 32, 8, None) == fls.EWORKSPACE   # nothing registered
    assert L.fls_dense_gemm(16, 16, 16, 128, 32, 8, None) == fls.EWORKSPACE
    assert L.fls_check_workspace(None) == fls.EWORKSPACE
    assert L.fls_dense_gemm(None, 16, 16, 128, 32, 8, None) == fls.EINVAL
    assert L.fls_compress(None, 128, 32, 16, 1 << 20, 0, None, None) == fls.EINVAL
    assert L.fls_compress(16, 128, 32, 16, 1 << 20, 7, None, None) == fls.EINVAL
    assert L.fls_compress(16, 128, 32, 24, 1 << 20, 0, None, None) == fls.EALIGN
    st = fls.FlsStats()
    assert L.fls_compress(16, 128, 32, 16, 100, 0, ctypes.byref(st), None) == fls.ECAPACITY
    assert st.bytes_total == fls.fls_compress_bound(128, 32)  # a size that is certainly enough
    assert L.fls_set_workspace(None, 64, None) == fls.EINVAL
    assert L.fls_set_workspace(8, 64, None) == fls.EALIGN
    for code in (0, -1, -2, -3, -4, -5, -6, -99):
        assert len(fls.strerror(code)) > 1


def test_inspect_validates_headers(fls, oracle_mod):
    import numpy as np
    import fls_workloads as wl

    W, _ = wl.make_inputs(wl.CONFIGS["C1"])
    blob = oracle_mod.ref_compress(W[:256, :128])
    st = fls.fls_inspect(blob[:64].tobytes())
    info = oracle_mod.ref_inspect(blob)
    for k in ("M", "K", "nnz", "num_tiles", "max_tile_words", "bytes_total", "bytes_offsets", "bytes_nonzeros"):
        assert st[k] == info[k]
    for off, val in ((0, 0), (4, 2), (8, 64), (12, 64), (16, 8)):
        bad = blob[:64].copy()
        bad[off] = val
        with pytest.raises(fls.FlsError) as e:
            fls.fls_inspect(bad.tobytes())
        assert e.value.code == fls.EFORMAT


def test_measurement_probe_library_loads(fls):
    """libfls_probe.so (the plain streaming read bench.py uses as its empirical ceiling) is built beside the
    library, exports its one entry point and rejects bad arguments before any launch."""
    from paper_2309_10285_amd import stream_probe

    L = stream_probe.lib()
    assert L.fls_probe_stream_read(None, 1024, 8, 8, 16, None) == -1
    assert L.fls_probe_stream_read(16, 1024, 8, 5, 16, None) == -1   # unroll not offered
    assert L.fls_probe_stream_read(16, 1024, 0, 8, 16, None) == -1   # empty grid
