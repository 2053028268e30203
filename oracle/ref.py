"""ctypes front end of ``fls_oracle.c``: reference Tiled-CSL compressor / decompressor and the
fp64 definition of the SpMM.  TEST INFRASTRUCTURE ONLY (see the header of the C file).

Array conventions (numpy):
  W  uint16 [M, K]   fp16 bit patterns, row-major            (Alg. 3 addressing)
  X  uint16 [N, K]   fp16 bit patterns == column-major K x N (ld = K)
  C  float64 [N, M]  == column-major M x N (ld = M)
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fls_oracle.c")
_SRC_V2 = os.path.join(_HERE, "fls_oracle_v2.c")  # format version 2 (groups of four entries, 6-bit location distances)
_LIB = os.path.join(_HERE, "libfls_oracle.so")
_lib = None

# geometry this build's HIP library uses (the oracle itself is parametric)
TILE_M = 128
TILE_K = 32
PAD_WORDS = 4


def build_oracle(force=False):
    """Compile the C oracle with gcc (plain -O2, OpenMP for the row loop)."""
    newest = max(os.path.getmtime(_SRC), os.path.getmtime(_SRC_V2))
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < newest:
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-o", _LIB, _SRC, _SRC_V2, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build_oracle()
        lib = ctypes.CDLL(_LIB)
        u8p, u16p, f64p, u64p = (ctypes.POINTER(t) for t in
                                 (ctypes.c_uint8, ctypes.c_uint16, ctypes.c_double, ctypes.c_uint64))
        i64, u32, sz = ctypes.c_int64, ctypes.c_uint32, ctypes.c_size_t
        lib.flso_half_to_double_array.argtypes = [u16p, f64p, sz]
        lib.flso_half_to_double_array.restype = None
        lib.flso_double_to_half_array.argtypes = [f64p, u16p, sz]
        lib.flso_double_to_half_array.restype = None
        lib.flso_compress.argtypes = [u16p, i64, i64, u32, u32, u32, u32, u32, u32, u8p, sz]
        lib.flso_compress.restype = sz
        lib.flso_compress_bound.argtypes = [i64, i64, u32, u32, u32]
        lib.flso_compress_bound.restype = sz
        lib.flso_inspect.argtypes = [u8p, sz, u64p]
        lib.flso_inspect.restype = ctypes.c_int
        lib.flso_decompress.argtypes = [u8p, sz, u16p, i64, i64]
        lib.flso_decompress.restype = ctypes.c_int
        lib.flso_spmm_f64_rows.argtypes = [u16p, u16p, f64p, i64, i64, i64, i64, i64]
        lib.flso_spmm_f64_rows.restype = None
        lib.flso2_compress.argtypes = [u16p, i64, i64, u32, u32, u8p, sz]
        lib.flso2_compress.restype = sz
        lib.flso2_compress_bound.argtypes = [i64, i64, u32, u32]
        lib.flso2_compress_bound.restype = sz
        lib.flso2_inspect.argtypes = [u8p, sz, u64p]
        lib.flso2_inspect.restype = ctypes.c_int
        lib.flso2_decompress.argtypes = [u8p, sz, u16p, i64, i64]
        lib.flso2_decompress.restype = ctypes.c_int
        lib.flso_threads.argtypes = []
        lib.flso_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def _ptr(a, ctype):
    return a.ctypes.data_as(ctypes.POINTER(ctype))


def half_to_double(bits):
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    out = np.empty(bits.shape, dtype=np.float64)
    _load().flso_half_to_double_array(_ptr(bits, ctypes.c_uint16), _ptr(out, ctypes.c_double), bits.size)
    return out


def double_to_half(vals):
    vals = np.ascontiguousarray(vals, dtype=np.float64)
    out = np.empty(vals.shape, dtype=np.uint16)
    _load().flso_double_to_half_array(_ptr(vals, ctypes.c_double), _ptr(out, ctypes.c_uint16), vals.size)
    return out


def ref_compress_bound(M, K, tile_m=TILE_M, tile_k=TILE_K, pad=PAD_WORDS):
    return int(_load().flso_compress_bound(M, K, tile_m, tile_k, pad))


def ref_compress(W, tile_m=TILE_M, tile_k=TILE_K, pad=PAD_WORDS, policy=0, banks=32, group=32):
    """Dense masked W (uint16 [M, K]) -> blob (uint8 array).  Sec. 4.3.1 + Alg. 3."""
    W = np.ascontiguousarray(W, dtype=np.uint16)
    M, K = W.shape
    lib = _load()
    need = lib.flso_compress(_ptr(W, ctypes.c_uint16), M, K, tile_m, tile_k, pad, policy, banks, group,
                             None, 0)
    if need == 0:
        raise ValueError("unsupported geometry for the oracle compressor")
    out = np.zeros(need, dtype=np.uint8)
    got = lib.flso_compress(_ptr(W, ctypes.c_uint16), M, K, tile_m, tile_k, pad, policy, banks, group,
                            _ptr(out, ctypes.c_uint8), need)
    assert got == need
    return out


_FIELDS = ("magic", "version", "tile_m", "tile_k", "pad_words", "order_policy", "max_tile_words",
           "reserved", "M", "K", "nnz", "total_words")


def ref_inspect(blob):
    blob = np.ascontiguousarray(blob, dtype=np.uint8)
    out = np.zeros(12, dtype=np.uint64)
    rc = _load().flso_inspect(_ptr(blob, ctypes.c_uint8), blob.size, _ptr(out, ctypes.c_uint64))
    d = {k: int(v) for k, v in zip(_FIELDS, out)}
    d["rc"] = rc
    if rc == 0:
        d["num_tiles"] = (d["M"] // d["tile_m"]) * (d["K"] // d["tile_k"])
        d["n_off"] = (d["num_tiles"] + 4 + 15) // 16 * 16
        d["bytes_header"] = 64
        d["bytes_offsets"] = 4 * d["n_off"]
        d["bytes_nonzeros"] = 4 * d["total_words"]
        d["bytes_total"] = 64 + d["bytes_offsets"] + d["bytes_nonzeros"]
    return d


def ref_decompress(blob, M, K):
    blob = np.ascontiguousarray(blob, dtype=np.uint8)
    W = np.empty((M, K), dtype=np.uint16)
    rc = _load().flso_decompress(_ptr(blob, ctypes.c_uint8), blob.size, _ptr(W, ctypes.c_uint16), M, K)
    if rc != 0:
        raise ValueError(f"malformed blob (oracle code {rc})")
    return W


def ref_compress_v2(W, tile_m=TILE_M, tile_k=TILE_K):
    """Dense masked W (uint16 [M, K]) -> format-version-2 blob (uint8 array): groups of four entries, first location in full, then 6-bit distances."""
    W = np.ascontiguousarray(W, dtype=np.uint16)
    M, K = W.shape
    lib = _load()
    need = lib.flso2_compress(_ptr(W, ctypes.c_uint16), M, K, tile_m, tile_k, None, 0)
    if need == 0:
        raise ValueError("unsupported geometry for the oracle compressor")
    out = np.zeros(need, dtype=np.uint8)
    got = lib.flso2_compress(_ptr(W, ctypes.c_uint16), M, K, tile_m, tile_k, _ptr(out, ctypes.c_uint8), need)
    assert got == need
    return out


def ref_compress_bound_v2(M, K, tile_m=TILE_M, tile_k=TILE_K):
    return int(_load().flso2_compress_bound(M, K, tile_m, tile_k))


def ref_inspect_v2(blob):
    blob = np.ascontiguousarray(blob, dtype=np.uint8)
    out = np.zeros(12, dtype=np.uint64)
    rc = _load().flso2_inspect(_ptr(blob, ctypes.c_uint8), blob.size, _ptr(out, ctypes.c_uint64))
    d = {k: int(v) for k, v in zip(_FIELDS, out)}
    d["rc"] = rc
    if rc == 0:
        d["num_tiles"] = (d["M"] // d["tile_m"]) * (d["K"] // d["tile_k"])
        d["n_off"] = (d["num_tiles"] + 4 + 15) // 16 * 16
        d["bytes_header"] = 64
        d["bytes_offsets"] = 4 * d["n_off"]
        d["bytes_nonzeros"] = 4 * d["total_words"]
        d["bytes_total"] = 64 + d["bytes_offsets"] + d["bytes_nonzeros"]
    return d


def ref_decompress_v2(blob, M, K):
    blob = np.ascontiguousarray(blob, dtype=np.uint8)
    W = np.empty((M, K), dtype=np.uint16)
    rc = _load().flso2_decompress(_ptr(blob, ctypes.c_uint8), blob.size, _ptr(W, ctypes.c_uint16), M, K)
    if rc != 0:
        raise ValueError(f"malformed version-2 blob (oracle code {rc})")
    return W


def ref_spmm_f64(W, X, rows=None):
    """C = W . X by the definition, in fp64 (Sec. 2.2).  W uint16 [M,K], X uint16 [N,K] -> float64 [N,M].

    rows=(m0, m1) computes only those rows of W (other entries of the result are 0).
    """
    W = np.ascontiguousarray(W, dtype=np.uint16)
    X = np.ascontiguousarray(X, dtype=np.uint16)
    M, K = W.shape
    N, K2 = X.shape
    assert K == K2
    m0, m1 = (0, M) if rows is None else rows
    C = np.zeros((N, M), dtype=np.float64)
    _load().flso_spmm_f64_rows(_ptr(W, ctypes.c_uint16), _ptr(X, ctypes.c_uint16), _ptr(C, ctypes.c_double),
                               M, K, N, m0, m1)
    return C


def ref_threads():
    return int(_load().flso_threads())
