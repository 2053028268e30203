"""Python binding of libfls (argument marshalling only; every step of the path runs in the HIP kernels).

Function names and argument order follow include/fls.h.  Tensors are torch tensors on the GPU,
used for device memory and streams only:
  W  dense : float16 [M, K] contiguous            (row-major M x K)
  X        : float16 [N, K] contiguous            (== column-major K x N, ld = K)
  C        : float16 [N, M] contiguous            (== column-major M x N, ld = M)
  blob     : uint8 1-D
There is no CPU fallback: without the built library, or without a GPU, calls raise.
"""
import ctypes
import os

TILE_M = 128
TILE_K = 32
MAX_N = 8192
ORDER_LOCATION = 0
ORDER_BANK = 1

OK, EINVAL, EALIGN, ECAPACITY, EFORMAT, EWORKSPACE, EHIP, EHANDOVER, ESCRATCH = 0, -1, -2, -3, -4, -5, -6, -7, -8
NOALLOC_MAX_N = 32

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfls.so")
_lib = None
_ws_tensor = None  # keeps the registered workspace alive

EXPORTS = ("fls_compress_bound", "fls_compress", "fls_compress_bound_v2", "fls_compress_v2", "fls_inspect", "fls_workspace_bytes", "fls_set_workspace",
           "fls_check_workspace", "fls_spmm", "fls_spmm_stats", "fls_spmm_noalloc", "fls_forget", "fls_dense_gemm", "fls_strerror")


class FlsStats(ctypes.Structure):
    _fields_ = [("format_version", ctypes.c_uint32), ("tile_m", ctypes.c_uint32), ("tile_k", ctypes.c_uint32),
                ("order_policy", ctypes.c_uint32), ("M", ctypes.c_uint64), ("K", ctypes.c_uint64),
                ("nnz", ctypes.c_uint64), ("num_tiles", ctypes.c_uint64), ("max_tile_words", ctypes.c_uint64),
                ("bytes_total", ctypes.c_uint64), ("bytes_header", ctypes.c_uint64),
                ("bytes_offsets", ctypes.c_uint64), ("bytes_nonzeros", ctypes.c_uint64)]

    def as_dict(self):
        return {k: int(getattr(self, k)) for k, _ in self._fields_}


class FlsError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        super().__init__(f"{where}: {strerror(code)} ({code})")


def lib():
    """The loaded C-ABI library; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with paper_2309_10285_amd._build.build()")
        L = ctypes.CDLL(LIB_PATH)
        vp, i64, sz, ci = ctypes.c_void_p, ctypes.c_int64, ctypes.c_size_t, ctypes.c_int
        L.fls_compress_bound.argtypes = [i64, i64, ctypes.POINTER(sz)]
        L.fls_compress_bound.restype = ci
        L.fls_compress.argtypes = [vp, i64, i64, vp, sz, ci, ctypes.POINTER(FlsStats), vp]
        L.fls_compress.restype = ci
        L.fls_compress_bound_v2.argtypes = [i64, i64, ctypes.POINTER(sz)]
        L.fls_compress_bound_v2.restype = ci
        L.fls_compress_v2.argtypes = [vp, i64, i64, vp, sz, ctypes.POINTER(FlsStats), vp]
        L.fls_compress_v2.restype = ci
        L.fls_inspect.argtypes = [vp, ctypes.POINTER(FlsStats)]
        L.fls_inspect.restype = ci
        L.fls_workspace_bytes.argtypes = [i64, i64, i64]
        L.fls_workspace_bytes.restype = sz
        L.fls_set_workspace.argtypes = [vp, sz, vp]
        L.fls_set_workspace.restype = ci
        L.fls_check_workspace.argtypes = [vp]
        L.fls_check_workspace.restype = ci
        L.fls_spmm.argtypes = [vp, vp, vp, i64, i64, i64, vp]
        L.fls_spmm.restype = ci
        L.fls_spmm_stats.argtypes = [vp, ctypes.POINTER(FlsStats), vp, vp, i64, i64, i64, vp]
        L.fls_spmm_stats.restype = ci
        L.fls_spmm_noalloc.argtypes = [vp, ctypes.POINTER(FlsStats), vp, vp, i64, i64, i64, vp]
        L.fls_spmm_noalloc.restype = ci
        L.fls_forget.argtypes = [vp]
        L.fls_forget.restype = None
        L.fls_dense_gemm.argtypes = [vp, vp, vp, i64, i64, i64, vp]
        L.fls_dense_gemm.restype = ci
        L.fls_strerror.argtypes = [ci]
        L.fls_strerror.restype = ctypes.c_char_p
        _lib = L
    return _lib


def strerror(code):
    return lib().fls_strerror(code).decode()


def _stream():
    import torch

    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(rc, where):
    if rc != OK:
        raise FlsError(rc, where)


def fls_compress_bound(M, K):
    out = ctypes.c_size_t(0)
    _check(lib().fls_compress_bound(M, K, ctypes.byref(out)), "fls_compress_bound")
    return out.value


def fls_inspect(header_bytes):
    """header_bytes: the first 64 bytes of a blob, on the host (bytes / bytearray / numpy uint8)."""
    buf = (ctypes.c_uint8 * 64).from_buffer_copy(bytes(header_bytes)[:64])
    st = FlsStats()
    _check(lib().fls_inspect(ctypes.cast(buf, ctypes.c_void_p), ctypes.byref(st)), "fls_inspect")
    return st.as_dict()


def fls_workspace_bytes(M, K, N):
    return int(lib().fls_workspace_bytes(M, K, N))


def fls_set_workspace(ws):
    """ws: uint8 CUDA tensor (caller-owned device memory); kept referenced until replaced."""
    global _ws_tensor
    _check(lib().fls_set_workspace(ctypes.c_void_p(ws.data_ptr()), ws.numel() * ws.element_size(), _stream()),
           "fls_set_workspace")
    _ws_tensor = ws


def ensure_workspace(M, K, N):
    """Registers a (torch-allocated) workspace large enough for this shape if the current one is not."""
    import torch

    need = fls_workspace_bytes(M, K, N)
    if need == 0:
        raise FlsError(EINVAL, "fls_workspace_bytes")
    if _ws_tensor is None or _ws_tensor.numel() < need:
        fls_set_workspace(torch.empty(need, dtype=torch.uint8, device="cuda"))


def fls_compress(W, out=None, order_policy=ORDER_LOCATION):
    """W: float16 [M, K] CUDA tensor.  Returns (blob uint8 CUDA tensor trimmed to its size, stats dict)."""
    import torch

    assert W.is_cuda and W.dtype == torch.float16 and W.is_contiguous() and W.dim() == 2
    M, K = W.shape
    if out is None:
        out = torch.empty(fls_compress_bound(M, K), dtype=torch.uint8, device=W.device)
    st = FlsStats()
    rc = lib().fls_compress(ctypes.c_void_p(W.data_ptr()), M, K, ctypes.c_void_p(out.data_ptr()), out.numel(),
                            order_policy, ctypes.byref(st), _stream())
    _check(rc, "fls_compress")
    return out[:st.bytes_total], st.as_dict()


def fls_compress_bound_v2(M, K):
    out = ctypes.c_size_t(0)
    _check(lib().fls_compress_bound_v2(M, K, ctypes.byref(out)), "fls_compress_bound_v2")
    return out.value


def fls_compress_v2(W, out=None):
    """fls_compress for format version 2 (four entries share a word of locations, 3 bytes per nonzero)."""
    import torch

    assert W.is_cuda and W.dtype == torch.float16 and W.is_contiguous() and W.dim() == 2
    M, K = W.shape
    if out is None:
        out = torch.empty(fls_compress_bound_v2(M, K), dtype=torch.uint8, device=W.device)
    st = FlsStats()
    rc = lib().fls_compress_v2(ctypes.c_void_p(W.data_ptr()), M, K, ctypes.c_void_p(out.data_ptr()), out.numel(),
                               ctypes.byref(st), _stream())
    _check(rc, "fls_compress_v2")
    return out[:st.bytes_total], st.as_dict()


def fls_spmm(blob, X, C, M, K, N):
    import torch

    assert blob.is_cuda and blob.dtype == torch.uint8 and blob.is_contiguous()
    assert X.is_cuda and X.dtype == torch.float16 and X.is_contiguous() and tuple(X.shape) == (N, K)
    assert C.is_cuda and C.dtype == torch.float16 and C.is_contiguous() and tuple(C.shape) == (N, M)
    _check(lib().fls_spmm(ctypes.c_void_p(blob.data_ptr()), ctypes.c_void_p(X.data_ptr()),
                          ctypes.c_void_p(C.data_ptr()), M, K, N, _stream()), "fls_spmm")
    return C


def fls_spmm_stats(blob, stats, X, C, M, K, N):
    """fls_spmm with the blob's statistics passed in (the dict fls_compress / fls_compress_v2 / fls_inspect returned):
    no header read-back, nothing remembered about the blob."""
    import torch

    assert blob.is_cuda and blob.dtype == torch.uint8 and blob.is_contiguous()
    assert X.is_cuda and X.dtype == torch.float16 and X.is_contiguous() and tuple(X.shape) == (N, K)
    assert C.is_cuda and C.dtype == torch.float16 and C.is_contiguous() and tuple(C.shape) == (N, M)
    st = FlsStats(**{k: stats[k] for k, _ in FlsStats._fields_})
    _check(lib().fls_spmm_stats(ctypes.c_void_p(blob.data_ptr()), ctypes.byref(st), ctypes.c_void_p(X.data_ptr()),
                                ctypes.c_void_p(C.data_ptr()), M, K, N, _stream()), "fls_spmm_stats")
    return C


def fls_spmm_noalloc(blob, stats, X, C, M, K, N):
    """fls_spmm on the library's static scratch (no workspace, no header read-back); stats: the dict fls_compress
    or fls_inspect returned for this blob."""
    import torch

    assert blob.is_cuda and blob.dtype == torch.uint8 and blob.is_contiguous()
    assert X.is_cuda and X.dtype == torch.float16 and X.is_contiguous() and tuple(X.shape) == (N, K)
    assert C.is_cuda and C.dtype == torch.float16 and C.is_contiguous() and tuple(C.shape) == (N, M)
    st = FlsStats(**{k: stats[k] for k, _ in FlsStats._fields_})
    _check(lib().fls_spmm_noalloc(ctypes.c_void_p(blob.data_ptr()), ctypes.byref(st), ctypes.c_void_p(X.data_ptr()),
                                  ctypes.c_void_p(C.data_ptr()), M, K, N, _stream()), "fls_spmm_noalloc")
    return C


def prepare_spmm(blob, X, C, M, K, N):
    """Checks and marshals the arguments of fls_spmm once; returns a callable that enqueues the call on the stream
    that was current when it was prepared.  For tight loops: a Python-side check per call costs as much time as
    the kernel runs."""
    import torch

    assert blob.is_cuda and blob.dtype == torch.uint8 and blob.is_contiguous()
    assert X.is_cuda and X.dtype == torch.float16 and X.is_contiguous() and tuple(X.shape) == (N, K)
    assert C.is_cuda and C.dtype == torch.float16 and C.is_contiguous() and tuple(C.shape) == (N, M)
    f = lib().fls_spmm
    args = (ctypes.c_void_p(blob.data_ptr()), ctypes.c_void_p(X.data_ptr()), ctypes.c_void_p(C.data_ptr()),
            M, K, N, _stream())
    keep = (blob, X, C)  # the tensors stay alive as long as the callable does

    def call(_keep=keep):
        rc = f(*args)
        if rc != OK:
            _check(rc, "fls_spmm")

    return call


def prepare_spmm_noalloc(blob, stats, X, C, M, K, N):
    """As prepare_spmm, for fls_spmm_noalloc (stats: the dict fls_compress or fls_inspect returned for this blob)."""
    import torch

    assert blob.is_cuda and blob.dtype == torch.uint8 and blob.is_contiguous()
    assert X.is_cuda and X.dtype == torch.float16 and X.is_contiguous() and tuple(X.shape) == (N, K)
    assert C.is_cuda and C.dtype == torch.float16 and C.is_contiguous() and tuple(C.shape) == (N, M)
    f = lib().fls_spmm_noalloc
    st = FlsStats(**{k: stats[k] for k, _ in FlsStats._fields_})
    args = (ctypes.c_void_p(blob.data_ptr()), ctypes.byref(st), ctypes.c_void_p(X.data_ptr()),
            ctypes.c_void_p(C.data_ptr()), M, K, N, _stream())
    keep = (blob, X, C, st)

    def call(_keep=keep):
        rc = f(*args)
        if rc != OK:
            _check(rc, "fls_spmm_noalloc")

    return call


def prepare_dense_gemm(W, X, C, M, K, N):
    """As prepare_spmm, for fls_dense_gemm."""
    import torch

    assert W.is_cuda and W.dtype == torch.float16 and W.is_contiguous() and tuple(W.shape) == (M, K)
    assert X.is_cuda and X.dtype == torch.float16 and X.is_contiguous() and tuple(X.shape) == (N, K)
    assert C.is_cuda and C.dtype == torch.float16 and C.is_contiguous() and tuple(C.shape) == (N, M)
    f = lib().fls_dense_gemm
    args = (ctypes.c_void_p(W.data_ptr()), ctypes.c_void_p(X.data_ptr()), ctypes.c_void_p(C.data_ptr()),
            M, K, N, _stream())
    keep = (W, X, C)

    def call(_keep=keep):
        rc = f(*args)
        if rc != OK:
            _check(rc, "fls_dense_gemm")

    return call


def fls_check_workspace():
    """Waits for the current stream; raises FlsError(EHANDOVER) if a kernel gave up on a split-K hand-over."""
    _check(lib().fls_check_workspace(_stream()), "fls_check_workspace")


def fls_forget(blob=None):
    lib().fls_forget(ctypes.c_void_p(blob.data_ptr()) if blob is not None else None)


def fls_dense_gemm(W, X, C, M, K, N):
    import torch

    assert W.is_cuda and W.dtype == torch.float16 and W.is_contiguous() and tuple(W.shape) == (M, K)
    assert X.is_cuda and X.dtype == torch.float16 and X.is_contiguous() and tuple(X.shape) == (N, K)
    assert C.is_cuda and C.dtype == torch.float16 and C.is_contiguous() and tuple(C.shape) == (N, M)
    _check(lib().fls_dense_gemm(ctypes.c_void_p(W.data_ptr()), ctypes.c_void_p(X.data_ptr()),
                                ctypes.c_void_p(C.data_ptr()), M, K, N, _stream()), "fls_dense_gemm")
    return C
