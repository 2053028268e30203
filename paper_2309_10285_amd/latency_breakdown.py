"""Latency breakdown of fls_spmm by erasing operations (the method of the paper's Fig. 11, Sec. 6.2.1).

Builds copies of libfls.so with -DFLS_ABLATE=<mask> (see csrc/fls_spmm.hip: 1 no split-K hand-over,
2 no MFMA, 4 no extract, 8 no re-zeroing, 16 no LDS fragment reads, 32 no global loads of the words,
256 no loads of X in the 64-column pass, which has no hand-over and ignores bit 1),
times each on one benchmark configuration and prints one JSON line per build.  Results of the ablated
builds are wrong by design; only their times mean something.  The builds go to a scratch folder
(default: a temporary directory), never into the package.

    python -m paper_2309_10285_amd.latency_breakdown --config C2 [--keep DIR] [--steps 200]
    python -m paper_2309_10285_amd.latency_breakdown --build-only --keep DIR     (no GPU needed)
    python -m paper_2309_10285_amd.latency_breakdown --prebuilt DIR              (time what --build-only made)
"""
import argparse
import ctypes
import json
import os
import subprocess
import sys
import tempfile

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from paper_2309_10285_amd import _build  # noqa: E402

# name -> FLS_ABLATE mask
VARIANTS = [
    ("full kernel", 0),
    ("no split-K hand-over / C store", 1),
    ("no hand-over, no MFMA", 1 | 2),
    ("no hand-over, no extract", 1 | 4),
    ("no hand-over, no re-zeroing", 1 | 8),
    ("no hand-over, no fragment reads", 1 | 16),
    ("no hand-over, no global loads of W", 1 | 32),
    ("global loads only (W and X)", 1 | 2 | 4 | 8 | 16),
    ("LDS + MFMA work only (no W loads)", 1 | 32),
    ("loop skeleton and X loads only", 1 | 2 | 4 | 8 | 16 | 32),
    ("no hand-over, no X loads (64-column pass)", 1 | 256),
    ("loop skeleton only (64-column pass)", 1 | 2 | 4 | 8 | 16 | 32 | 256),
]


# the sources that know FLS_ABLATE; the other objects of a variant are the library's own
ABLATED_SOURCES = ("fls_spmm.hip", "fls_spmm_wide.hip")
# builds that __graft_entry__.build() keeps beside the library for the GPU test of this tool
PREBUILT_DIR = os.path.join(os.path.dirname(os.path.abspath(__file__)), "ablate_builds")
PREBUILT_MASKS = (0, 1 | 2 | 4 | 8 | 16)


def build_variant(mask, folder):
    """libfls_ablate<mask>.so in `folder`: the two kernel sources compiled with -DFLS_ABLATE=<mask>, linked with
    the library's other objects (built by _build.build(); built here if missing)."""
    os.makedirs(folder, exist_ok=True)
    lib = os.path.join(folder, f"libfls_ablate{mask}.so")
    others = [os.path.join(_build.CSRC, s.replace(".hip", ".o")) for s in _build.SOURCES if s not in ABLATED_SOURCES]
    if not all(os.path.exists(o) for o in others):
        _build.build()
    objs, procs = [], []
    for src in ABLATED_SOURCES:
        obj = os.path.join(folder, f"a{mask}_{src.replace('.hip', '.o')}")
        objs.append(obj)
        cmd = ["hipcc", *_build.HIPCC_FLAGS, f"-DFLS_ABLATE={mask}", "-c", os.path.join(_build.CSRC, src), "-o", obj]
        procs.append(subprocess.Popen(cmd, stdout=subprocess.DEVNULL, stderr=subprocess.PIPE, text=True))
    for p in procs:
        _, err = p.communicate()
        if p.returncode != 0:
            raise RuntimeError(err)
    subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *objs, *others], check=True)
    for o in objs:
        os.remove(o)
    return lib


def _bind(lib_path):
    L = ctypes.CDLL(lib_path)
    vp, i64 = ctypes.c_void_p, ctypes.c_int64
    L.fls_spmm.argtypes = [vp, vp, vp, i64, i64, i64, vp]
    L.fls_set_workspace.argtypes = [vp, ctypes.c_size_t, vp]
    L.fls_check_workspace.argtypes = [vp]
    return L


def run_once(lib_path, blob, X, C, M, K, N, ws):
    """One fls_spmm call through the build at lib_path (its own workspace registration), waited for.
    Returns the error code of the call, or of the workspace check after it."""
    import torch

    L = _bind(lib_path)
    vp = ctypes.c_void_p
    stream = vp(torch.cuda.current_stream().cuda_stream)
    rc = L.fls_set_workspace(vp(ws.data_ptr()), ws.numel(), stream)
    if rc == 0:
        rc = L.fls_spmm(vp(blob.data_ptr()), vp(X.data_ptr()), vp(C.data_ptr()), M, K, N, stream)
    torch.cuda.synchronize()
    return rc if rc != 0 else L.fls_check_workspace(stream)


def time_variant(lib_path, blobs, X, C, M, K, N, ws, steps, warmup, stats=None):
    """Microseconds per call of fls_spmm through the build at lib_path; with `stats` (the blob's statistics, a ctypes
    fls_stats) of fls_spmm_noalloc instead, the entry point that keeps to the narrow kernel for any shape."""
    import torch

    L = _bind(lib_path)
    vp = ctypes.c_void_p
    stream = vp(torch.cuda.current_stream().cuda_stream)
    assert L.fls_set_workspace(vp(ws.data_ptr()), ws.numel(), stream) == 0
    calls = [vp(b.data_ptr()) for b in blobs]
    x, c = vp(X.data_ptr()), vp(C.data_ptr())
    if stats is not None:
        L.fls_spmm_noalloc.argtypes = [vp, vp, vp, vp, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, vp]
        st = ctypes.byref(stats)

        def one(i):
            return L.fls_spmm_noalloc(calls[i % len(calls)], st, x, c, M, K, N, stream)
    else:
        def one(i):
            return L.fls_spmm(calls[i % len(calls)], x, c, M, K, N, stream)
    # untimed launches for 50 ms first: after an idle period (input generation, the build before) the chip's
    # clocks take some hundred launches to come up, which the first variant timed would otherwise pay for
    import time
    t_end = time.perf_counter() + 0.05
    i = 0
    while time.perf_counter() < t_end:
        for _ in range(32):
            assert one(i) == 0
            i += 1
        torch.cuda.synchronize()
    for i in range(warmup):
        assert one(i) == 0
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(steps):
        one(i)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps * 1e3


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="C2")
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--keep", default="", help="folder for the builds (kept); default: a temporary directory")
    ap.add_argument("--build-only", action="store_true")
    ap.add_argument("--prebuilt", default="", help="folder with builds made by --build-only")
    ap.add_argument("--entry", choices=("spmm", "noalloc"), default="spmm",
                    help="noalloc: time fls_spmm_noalloc (N <= 32), which keeps to the narrow kernel on shapes where "
                         "fls_spmm takes the 64-column pass for 17 - 32 columns")
    args = ap.parse_args()

    tmp = None
    folder = args.prebuilt or args.keep
    if not folder:
        tmp = tempfile.TemporaryDirectory()
        folder = tmp.name
    os.makedirs(folder, exist_ok=True)
    libs = {}
    for name, mask in VARIANTS:
        if mask in libs:
            continue
        path = os.path.join(folder, f"libfls_ablate{mask}.so")
        libs[mask] = path if args.prebuilt else build_variant(mask, folder)
    if args.build_only:
        print(json.dumps({"built": sorted(libs.values())}))
        return

    import numpy as np
    import torch

    import fls_workloads as wl
    import paper_2309_10285_amd as fls

    cfg = wl.CONFIGS[args.config]
    M, K, N = cfg.M, cfg.K, cfg.N
    Wb, Xb = wl.make_inputs(cfg)
    X = torch.from_numpy(Xb.view(np.float16)).cuda()
    blob0, st = fls.fls_compress(torch.from_numpy(Wb.view(np.float16)).cuda())
    blob0 = blob0.clone()
    n_copies = max(2, -(-(1 << 30) // st["bytes_total"]))
    blobs = [blob0] + [blob0.clone() for _ in range(n_copies - 1)]
    C = torch.empty((N, M), dtype=torch.float16, device="cuda")
    ws = torch.empty(fls.fls_workspace_bytes(M, K, N), dtype=torch.uint8, device="cuda")
    alg = st["bytes_total"] + 2 * K * N + 2 * M * N
    stats = None
    if args.entry == "noalloc":
        stats = fls.FlsStats(**{k: st[k] for k, _ in fls.FlsStats._fields_})
    for name, mask in VARIANTS:
        us = time_variant(libs[mask], blobs, X, C, M, K, N, ws, args.steps, args.warmup, stats)
        print(json.dumps({"config": args.config, "variant": name, "FLS_ABLATE": mask, "entry": args.entry, "us": round(us, 2),
                          "GBps_on_algorithmic_bytes": round(alg / us / 1e3, 1)}), flush=True)
    if tmp:
        tmp.cleanup()


if __name__ == "__main__":
    main()
