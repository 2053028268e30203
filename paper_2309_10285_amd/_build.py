"""Builds libfls.so (the HIP kernels + C ABI) in-tree with hipcc for gfx950."""
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB = os.path.join(_HERE, "libfls.so")
SOURCES = ["fls_api.hip", "fls_spmm.hip", "fls_spmm_wide.hip", "fls_dense.hip", "fls_compress.hip"]
# measurement code (a plain streaming read: bench.py's empirical ceiling), a library of its own, not part of the C ABI
PROBE_SOURCE = "fls_stream_probe.hip"
PROBE_LIB = os.path.join(_HERE, "libfls_probe.so")
HEADERS = ["fls_device.h", "fls_launch.h", "fls_tile.h", os.path.join("..", "..", "include", "fls.h")]

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-munsafe-fp-atomics",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def build(force=True, verbose=False):
    """Compile every source to an object (in parallel) and link the shared library."""
    objs, procs = [], []
    probe_cmd = ["hipcc", *HIPCC_FLAGS, "-shared", "-o", PROBE_LIB, os.path.join(CSRC, PROBE_SOURCE)]
    probe = subprocess.Popen(probe_cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    for src in SOURCES:
        obj = os.path.join(CSRC, src.replace(".hip", ".o"))
        objs.append(obj)
        cmd = ["hipcc", *HIPCC_FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
        procs.append((cmd, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    for cmd, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            raise RuntimeError("hipcc failed: " + " ".join(cmd) + "\n" + out)
        if verbose and out.strip():
            print(out)
    out, _ = probe.communicate()
    if probe.returncode != 0:
        raise RuntimeError("hipcc failed: " + " ".join(probe_cmd) + "\n" + out)
    link = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    r = subprocess.run(link, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stdout)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
