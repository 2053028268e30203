"""Benchmark of the Load-as-Sparse / Compute-as-Dense SpMM hot path on one MI355X.

One "step" = one fls_spmm call over the headline workload, the OPT-175B-shaped FFN down-projection
(W 12288 x 49152 fp16, magnitude-pruned to 90 %, X 49152 x 64: the largest named configuration),
inputs resident in HBM.  Steps rotate over several copies of the compressed matrix so that no step
finds its weights in the 256 MB Infinity Cache.  Prints ONE JSON line: metric/value (dense-equivalent
TFLOP/s), the roofline object (algorithmic bytes per call / measured time of a call against the larger of
the HBM and the MFMA lower bound), the empirical ceiling of a plain streaming read of the same blob, the
own dense GEMM on the unpruned matrix, the CPU oracle timed on the host cores over the whole workload, and
the parity of the whole of C against that oracle; the other named configurations (C2, C3) follow under
"other_configs" with the same objects.  Exits non-zero if any C is off the oracle by more than 2e-3.

The oracle is imported by the cpu_baseline / parity leg of the bench line and by the parity checks of
--sweep and --layer; nothing that is timed touches it.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth
MIN_ROTATION_BYTES = 1 << 30

PARITY_TOL = 2e-3
HEADLINE = "C4"         # the largest named configuration that fits one GPU (604 M weights, 77 GFLOP per call)
OTHERS = ("C2", "C3")   # reported beside it in the same JSON line

# HBM traffic per call.  It cannot be read inside this process: it comes from separate rocprofv3 --pmc runs
# of this script (FETCH_SIZE, then WRITE_SIZE, scaled by a copy kernel of known size), whose summaries are
# under profiles/; the line carries the figure together with the file it was copied from, or null.
MEASURED_TRAFFIC = {
    "C2": (169.90e6, "profiles/spmm_C2_hbm_traffic.md (separate rocprofv3 --pmc runs, not this run)"),
    "C4": (335.87e6, "profiles/spmm_C4_hbm_traffic.md (separate rocprofv3 --pmc runs, not this run; both kernels of the call)"),
}


def _time_loop(calls, steps, warmup):
    """calls: prepared zero-argument launches (one per rotated copy of the weights), issued round-robin.
    Returns (GPU ms per step from events on the launch stream, host ms per step spent issuing)."""
    import torch

    n = len(calls)
    # one call per copy first: fls_spmm reads a blob's header back (and waits) the first time it sees its address
    for c in calls:
        c()
    torch.cuda.synchronize()
    # the GPU's clocks settle only after some tens of milliseconds of work: run untimed launches for that long
    # first, whatever the warm-up count asked for is
    t_end = time.perf_counter() + 0.03
    i = 0
    while time.perf_counter() < t_end:
        calls[i % n]()
        i += 1
        if i % 64 == 0:
            torch.cuda.synchronize()
    for i in range(warmup):
        calls[i % n]()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    t0 = time.perf_counter()
    for i in range(steps):
        calls[i % n]()
    host_ms = (time.perf_counter() - t0) * 1e3
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps, host_ms / steps


def run_sweep(args):
    """The sparsity x mask x N sweep on the 12288 x 12288 matrix: one JSON line per point (not the bench line)."""
    import torch

    import fls_workloads as wl
    import oracle
    import paper_2309_10285_amd as fls

    fls.lib()
    M, K = wl.SWEEP_M, wl.SWEEP_K
    W32 = wl.gen_weights_f32(M, K, wl.SWEEP_SEED)
    out = open(args.out, "w") if args.out else None

    def emit(rec):
        line = json.dumps(rec)
        print(line, flush=True)
        if out:
            out.write(line + "\n")
            out.flush()

    Xs = {N: wl.gen_x(N, K, wl.SWEEP_SEED + 2) for N in wl.SWEEP_NS}
    Xd = {N: torch.from_numpy(Xs[N].view(np.float16)).cuda() for N in wl.SWEEP_NS}
    fls.ensure_workspace(M, K, max(wl.SWEEP_NS))
    Wd = torch.from_numpy(wl.dense_bits(W32).view(np.float16)).cuda()
    dense = [Wd, Wd.clone(), Wd.clone(), Wd.clone()]
    dense_ms = {}
    for N in wl.SWEEP_NS:
        D = torch.empty((N, M), dtype=torch.float16, device="cuda")
        dense_ms[N], _ = _time_loop([fls.prepare_dense_gemm(w, Xd[N], D, M, K, N) for w in dense], args.steps, args.warmup)
        V = torch.empty((N, M), dtype=torch.float16, device="cuda")
        vms, _ = _time_loop([lambda w=w, x=Xd[N], v=V: torch.matmul(x, w.t(), out=v) for w in dense], args.steps, args.warmup)
        emit({"point": f"dense-N{N}", "N": N, "us": round(dense_ms[N] * 1e3, 2),
              "GBps": round((2 * M * K + 2 * K * N + 2 * M * N) / dense_ms[N] / 1e6, 1),
              "vendor_gemm_us": round(vms * 1e3, 2)})
    del dense, Wd
    worst = 0.0
    for mask in wl.SWEEP_MASKS:
        for beta in wl.SWEEP_BETAS:
            cfg = wl.sweep_config(beta, mask, 8)
            Wb = (wl.prune_uniform if mask == "uniform" else wl.prune_row_skewed)(W32, beta, wl.SWEEP_SEED + 1)
            W = torch.from_numpy(Wb.view(np.float16)).cuda()
            blob0, st = (fls.fls_compress_v2 if args.format == 2 else fls.fls_compress)(W)
            blob0 = blob0.clone()
            del W
            n_copies = max(2, -(-MIN_ROTATION_BYTES // st["bytes_total"]))
            blobs = [blob0] + [blob0.clone() for _ in range(n_copies - 1)]
            for N in wl.SWEEP_NS:
                C = torch.empty((N, M), dtype=torch.float16, device="cuda")
                ms, _ = _time_loop([fls.prepare_spmm(b, Xd[N], C, M, K, N) for b in blobs], args.steps, args.warmup)
                ref = oracle.ref_spmm_f64(Wb, Xs[N])  # the whole of C
                err = float(np.abs(C.cpu().numpy().astype(np.float64) - ref).max() / np.abs(ref).max())
                alg = st["bytes_total"] + 2 * K * N + 2 * M * N
                emit({"point": f"{mask}-{int(round(beta * 100))}-N{N}", "mask": mask, "sparsity": beta, "N": N,
                      "format": args.format, "nnz": st["nnz"], "max_tile_words": st["max_tile_words"], "us": round(ms * 1e3, 2),
                      "TFLOPs": round(2.0 * M * K * N / ms / 1e9, 1), "GBps": round(alg / ms / 1e6, 1),
                      "hbm_frac": round(alg / ms / 1e6 / HBM_PEAK_GBS, 4), "speedup_vs_dense": round(dense_ms[N] / ms, 3),
                      "max_rel_err_whole_c": err, "parity_ok": err <= 2e-3})
                worst = max(worst, err)
            # the copies' memory goes back to torch's allocator and will hold other blobs: the library must
            # not keep the headers it remembers for these addresses
            for b in blobs:
                fls.fls_forget(b)
            del blobs, blob0
    if worst > 2e-3:
        raise SystemExit(f"sweep: a point is off the oracle by {worst:.3g} (tolerance 2e-3)")


def run_crossover(args):
    """The study of non-skinny shapes (Sec. 6.2): the 12288 x 12288 matrix at 70 / 80 / 90 % sparsity for N from 64 to
    8192, fls_spmm against the own dense GEMM and the vendor library's, to find where loading sparse and computing
    dense stops paying.  One JSON line per point (not the bench line).  C is checked against the oracle on all
    columns up to N = 512 and on 256 sampled columns beyond."""
    import torch

    import fls_workloads as wl
    import oracle
    import paper_2309_10285_amd as fls

    fls.lib()
    M, K = wl.SWEEP_M, wl.SWEEP_K
    Ns = (64, 128, 256, 512, 1024, 2048, 4096, 8192)
    W32 = wl.gen_weights_f32(M, K, wl.SWEEP_SEED)
    out = open(args.out, "w") if args.out else None

    def emit(rec):
        line = json.dumps(rec)
        print(line, flush=True)
        if out:
            out.write(line + "\n")
            out.flush()

    def steps_for(N):  # a call takes up to some milliseconds here
        return max(10, min(args.steps, 40000 // N))

    Xs = {N: wl.gen_x(N, K, wl.SWEEP_SEED + 2) for N in Ns}
    Xd = {N: torch.from_numpy(Xs[N].view(np.float16)).cuda() for N in Ns}
    fls.ensure_workspace(M, K, max(Ns))
    Wd = torch.from_numpy(wl.dense_bits(W32).view(np.float16)).cuda()
    dense = [Wd, Wd.clone(), Wd.clone(), Wd.clone()]
    dense_ms, vendor_ms = {}, {}
    for N in Ns:
        D = torch.empty((N, M), dtype=torch.float16, device="cuda")
        dense_ms[N], _ = _time_loop([fls.prepare_dense_gemm(w, Xd[N], D, M, K, N) for w in dense], steps_for(N), 5)
        vendor_ms[N], _ = _time_loop([lambda w=w, x=Xd[N], v=D: torch.matmul(x, w.t(), out=v) for w in dense], steps_for(N), 5)
        emit({"point": f"dense-N{N}", "N": N, "own_dense_us": round(dense_ms[N] * 1e3, 1),
              "vendor_gemm_us": round(vendor_ms[N] * 1e3, 1),
              "vendor_TFLOPs": round(2.0 * M * K * N / vendor_ms[N] / 1e9, 1)})
        del D
    del dense, Wd
    worst = 0.0
    g = np.random.Generator(np.random.Philox(99))
    for beta in (0.7, 0.8, 0.9):
        Wb = wl.prune_uniform(W32, beta, wl.SWEEP_SEED + 1)
        blob0, st = fls.fls_compress(torch.from_numpy(Wb.view(np.float16)).cuda())
        blob0 = blob0.clone()
        n_copies = max(2, -(-MIN_ROTATION_BYTES // st["bytes_total"]))
        blobs = [blob0] + [blob0.clone() for _ in range(n_copies - 1)]
        for N in Ns:
            C = torch.empty((N, M), dtype=torch.float16, device="cuda")
            ms, _ = _time_loop([fls.prepare_spmm(b, Xd[N], C, M, K, N) for b in blobs], steps_for(N), 5)
            cols = np.arange(N) if N <= 512 else np.sort(g.choice(N, size=256, replace=False))
            ref = oracle.ref_spmm_f64(Wb, np.ascontiguousarray(Xs[N][cols]))
            err = float(np.abs(C.cpu().numpy()[cols].astype(np.float64) - ref).max() / np.abs(ref).max())
            worst = max(worst, err)
            emit({"point": f"uniform-{int(round(beta * 100))}-N{N}", "sparsity": beta, "N": N, "us": round(ms * 1e3, 1),
                  "TFLOPs": round(2.0 * M * K * N / ms / 1e9, 1), "speedup_vs_own_dense": round(dense_ms[N] / ms, 3),
                  "speedup_vs_vendor_gemm": round(vendor_ms[N] / ms, 3), "columns_checked": int(cols.size),
                  "max_rel_err": err, "parity_ok": err <= PARITY_TOL})
            del C
        for b in blobs:
            fls.fls_forget(b)
        del blobs, blob0
    if worst > PARITY_TOL:
        raise SystemExit(f"crossover: a point is off the oracle by {worst:.3g} (tolerance {PARITY_TOL})")


def _run_layer_on_stream(args, torch, wl, fls, side):
    N, beta = args.layer_n, 0.8
    mats = wl.decoder_layer(7168, 28672, N, beta)
    fls.ensure_workspace(max(c.M for c in mats), max(c.K for c in mats), N)
    copies = 3
    sparse, dense, recs = [], [], []
    for cfg in mats:
        W32 = wl.make_w32(cfg)
        Wb, Xb = wl.make_inputs(cfg, W32)
        X = torch.from_numpy(Xb.view(np.float16)).cuda()
        blob0, st = fls.fls_compress(torch.from_numpy(Wb.view(np.float16)).cuda())
        blobs = [blob0.clone() for _ in range(copies)]
        del blob0
        Wd = torch.from_numpy(wl.dense_bits(W32).view(np.float16)).cuda()
        Wds = [Wd] + [Wd.clone() for _ in range(copies - 1)]
        C = torch.empty((N, cfg.M), dtype=torch.float16, device="cuda")
        D = torch.empty((N, cfg.M), dtype=torch.float16, device="cuda")
        sparse.append([fls.prepare_spmm(b, X, C, cfg.M, cfg.K, N) for b in blobs])
        dense.append([fls.prepare_dense_gemm(w, X, D, cfg.M, cfg.K, N) for w in Wds])
        ms, _ = _time_loop(sparse[-1], args.steps, args.warmup)
        dms, _ = _time_loop(dense[-1], args.steps, args.warmup)
        err = None
        if not args.no_cpu_baseline:
            import oracle

            ref = oracle.ref_spmm_f64(Wb, Xb)  # the whole of C
            err = float(np.abs(C.cpu().numpy().astype(np.float64) - ref).max() / np.abs(ref).max())
        alg = st["bytes_total"] + 2 * cfg.K * N + 2 * cfg.M * N
        recs.append({"matmul": cfg.what, "M": cfg.M, "K": cfg.K, "nnz": st["nnz"], "alone_us": round(ms * 1e3, 2),
                     "alone_GBps": round(alg / ms / 1e6, 1), "dense_alone_us": round(dms * 1e3, 2),
                     "algorithmic_bytes": alg, "max_rel_err_whole_c": err})

    def layer_calls(table):
        return [lambda c=c, table=table: [calls[c]() for calls in table] for c in range(copies)]

    def graph_of(table):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            for c in range(copies):
                for calls in table:
                    calls[c]()
        return g

    layer_steps = max(50, args.steps // 4)
    out = {"mode": "decoder layer", "model": "OPT-30B-shaped (hidden 7168, FFN 28672)", "N": N, "sparsity": beta,
           "weight_copies_rotated": copies, "layers_timed": layer_steps, "matmuls": recs}
    for name, table in (("spmm", sparse), ("dense", dense)):
        ms, _ = _time_loop(layer_calls(table), layer_steps, max(10, args.warmup // 4))
        out[f"{name}_layer_us_eager"] = round(ms * 1e3, 2)
        g = graph_of(table)
        gms, _ = _time_loop([g.replay], max(20, layer_steps // copies), 5)
        out[f"{name}_layer_us_graph"] = round(gms * 1e3 / copies, 2)
    alg = sum(r["algorithmic_bytes"] for r in recs)
    out["spmm_layer_GBps_graph"] = round(alg / out["spmm_layer_us_graph"] / 1e3, 1)
    out["spmm_layer_hbm_frac_graph"] = round(alg / out["spmm_layer_us_graph"] / 1e3 / HBM_PEAK_GBS, 4)
    out["sum_of_alone_us"] = round(sum(r["alone_us"] for r in recs), 2)
    out["layer_speedup_vs_dense_graph"] = round(out["dense_layer_us_graph"] / out["spmm_layer_us_graph"], 3)
    return out


def run_layer(args):
    """The four weight MatMuls of one OPT-30B-shaped decoder layer (hidden 7168, FFN 28672) back to back on one
    stream, as eager calls and as one HIP graph, against the same four dense GEMMs.  One JSON line (not the bench
    line).  The layers in a timed sequence rotate over copies of the weights (more than 1 GB in total)."""
    import torch

    import fls_workloads as wl
    import paper_2309_10285_amd as fls

    fls.lib()
    # a stream of its own: the null stream cannot be captured into a graph, and prepared calls stay bound to the
    # stream that was current when they were prepared
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        out = _run_layer_on_stream(args, torch, wl, fls, side)
    print(json.dumps(out), flush=True)


MFMA_F16_PEAK_TFLOPS = 2500.0  # MI355X published dense fp16 matrix rate


def _pass32_rule(max_tile_words, KT, bands, cus=256):
    """The library's rule (wide32_pays in csrc/fls_launch.h, format version 1) for giving a call of 17 - 32 columns to
    the 64-column pass, restated for the kernel label of the bench line only."""
    if max_tile_words > 2560:
        return False
    if KT >= 384:
        return True
    if KT < 288 or max_tile_words <= 512:
        return False
    body = 8 if max_tile_words <= 1024 else 4
    units = (bands + 3) // 4
    S = max(1, min(cus // units if units < cus else 1, max(1, KT // (2 * body))))
    bodies = KT // body
    return -(-bodies // S) * S * 10 <= bodies * 11


def measure_config(name, args, with_dense, with_cpu):
    """Times fls_spmm on one named configuration (inputs resident in HBM, weights rotated over more than 1 GB of
    copies), the streaming-read ceiling over the same blobs, optionally the dense pair; checks the whole of C
    against the oracle (that pass is also the cpu_baseline).  Returns a dict of results."""
    import torch

    import fls_workloads as wl
    import paper_2309_10285_amd as fls
    from paper_2309_10285_amd import stream_probe

    cfg = wl.CONFIGS[name]
    M, K, N = cfg.M, cfg.K, cfg.N
    t_gen = time.perf_counter()
    W32 = wl.make_w32(cfg)
    Wb, Xb = wl.make_inputs(cfg, W32)
    if args.x_values != "workload":  # same shapes, same instruction stream: only the operand values differ
        Xb = np.full_like(Xb, 0x3C00 if args.x_values == "ones" else 0)
    t_gen = time.perf_counter() - t_gen

    X = torch.from_numpy(Xb.view(np.float16)).cuda()
    W = torch.from_numpy(Wb.view(np.float16)).cuda()
    blob0, st = fls.fls_compress(W)
    blob0 = blob0.clone()  # trimmed copy; the bound-sized buffer is released
    del W
    n_copies = max(2, -(-MIN_ROTATION_BYTES // st["bytes_total"]))
    blobs = [blob0] + [blob0.clone() for _ in range(n_copies - 1)]
    fls.ensure_workspace(M, K, N)
    C = torch.empty((N, M), dtype=torch.float16, device="cuda")

    if args.entry == "noalloc":  # the entry point on the library's static scratch: always the narrow kernel, N <= 32
        calls = [fls.prepare_spmm_noalloc(b, st, X, C, M, K, N) for b in blobs]
    else:
        calls = [fls.prepare_spmm(b, X, C, M, K, N) for b in blobs]
    ms, host_ms = _time_loop(calls, args.steps, args.warmup)
    flops = 2.0 * M * K * N
    alg_bytes = st["bytes_total"] + 2 * K * N + 2 * M * N  # blob + X + C
    tflops = flops / (ms * 1e-3) / 1e12
    gbs = alg_bytes / (ms * 1e-3) / 1e9
    C_host = C.cpu().numpy()
    fls.fls_check_workspace()

    # which roof: the larger of the two lower bounds on the time of a call
    t_hbm_us = alg_bytes / (HBM_PEAK_GBS * 1e3)
    t_mfma_us = flops / (MFMA_F16_PEAK_TFLOPS * 1e6)
    # which kernels the call runs (a label; the library decides): the 64-column pass for more than 32 columns, and for
    # 17 - 32 columns on sparse tiles and long bands (the rule of wide32_pays in csrc/fls_launch.h)
    pass32 = 16 < N <= 32 and args.entry != "noalloc" and _pass32_rule(st["max_tile_words"], K // 32, M // 128)
    narrow = (N <= 32 and not pass32) or st["max_tile_words"] > 2560
    kernels = "fls::spmm_kernel" if narrow else "fls::spmm_wide_kernel + fls::wide_reduce_kernel"
    traffic = MEASURED_TRAFFIC.get(name)
    res = {
        "name": name, "cfg": cfg, "st": st, "n_copies": n_copies, "ms": ms, "host_ms": host_ms, "tflops": tflops,
        "gbs": gbs, "alg_bytes": alg_bytes, "t_gen": t_gen,
        "roofline": {"bound": "hbm" if t_hbm_us >= t_mfma_us else "mfma",
                     "achieved": round(gbs, 1) if t_hbm_us >= t_mfma_us else round(tflops, 1),
                     "peak": HBM_PEAK_GBS if t_hbm_us >= t_mfma_us else MFMA_F16_PEAK_TFLOPS,
                     "unit": "GB/s" if t_hbm_us >= t_mfma_us else "TFLOP/s",
                     "frac": round(max(t_hbm_us, t_mfma_us) / (ms * 1e3), 4),
                     "traffic": traffic[0] if traffic else None,
                     "traffic_source": traffic[1] if traffic else None,
                     "kernel": kernels, "algorithmic_bytes_per_launch": alg_bytes,
                     "avg_launch_us": round(ms * 1e3, 3),
                     "roof_us": {"hbm_8TBps": round(t_hbm_us, 2), "mfma_f16_2.5PFLOPs": round(t_mfma_us, 2)}},
    }

    # the same matrix in format version 2 (four entries share a word of locations, 3 bytes per nonzero), timed the same way and
    # stated against its own bytes
    if args.v2:
        W2 = torch.from_numpy(Wb.view(np.float16)).cuda()
        b2, st2 = fls.fls_compress_v2(W2)
        b2 = b2.clone()
        del W2
        blobs2 = [b2] + [b2.clone() for _ in range(max(2, -(-MIN_ROTATION_BYTES // st2["bytes_total"])) - 1)]
        C2 = torch.empty((N, M), dtype=torch.float16, device="cuda")
        if args.entry == "noalloc":
            calls2 = [fls.prepare_spmm_noalloc(b, st2, X, C2, M, K, N) for b in blobs2]
        else:
            calls2 = [fls.prepare_spmm(b, X, C2, M, K, N) for b in blobs2]
        ms2, _ = _time_loop(calls2, args.steps, args.warmup)
        alg2 = st2["bytes_total"] + 2 * K * N + 2 * M * N
        res["format_v2"] = {"blob_bytes": st2["bytes_total"], "bytes_per_nnz": round(st2["bytes_nonzeros"] / max(st2["nnz"], 1), 3),
                            "ms_per_step": round(ms2, 5), "achieved_GBps_on_its_bytes": round(alg2 / ms2 / 1e6, 1),
                            "hbm_frac_on_its_bytes": round(alg2 / ms2 / 1e6 / HBM_PEAK_GBS, 4),
                            "speedup_vs_v1": round(ms / ms2, 3), "_C": C2.cpu().numpy()}
        for b in blobs2:
            fls.fls_forget(b)
        del blobs2, b2, C2

    # the empirical ceiling: a plain streaming read of the same blobs (no LDS, no MFMA, nothing stored), with as
    # many workgroups as the kernel uses when it runs one per band, and with one per CU
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    bands = M // fls.TILE_M
    grids = sorted({cus, bands * (cus // bands) if bands <= cus else cus})
    probe_steps = max(20, min(args.steps, 400))
    ceiling = {"what": "plain 16 B non-temporal read of the blob, 8 waves per workgroup, 2 x 8 loads in flight per lane",
               "bytes": st["bytes_total"]}
    best = 0.0
    for g in grids:
        rate, us = stream_probe.stream_read_gbps(blobs, g, unroll=8, steps=probe_steps, warmup=20)
        ceiling[f"grid_{g}"] = {"GBps": round(rate, 1), "us": round(us, 2)}
        best = max(best, rate)
    ceiling["GBps"] = round(best, 1)
    ceiling["kernel_vs_ceiling"] = round(gbs / best, 4)
    res["stream_ceiling"] = ceiling

    if with_dense:
        Wd = torch.from_numpy(wl.dense_bits(W32).view(np.float16)).cuda()
        n_d = max(2, -(-MIN_ROTATION_BYTES // (2 * M * K)))
        dense = [Wd] + [Wd.clone() for _ in range(n_d - 1)]
        D = torch.empty((N, M), dtype=torch.float16, device="cuda")
        dms, _ = _time_loop([fls.prepare_dense_gemm(w, X, D, M, K, N) for w in dense], args.steps, args.warmup)
        dbytes = 2 * M * K + 2 * K * N + 2 * M * N
        res["dense_gemm"] = {"ms_per_step": round(dms, 5), "TFLOPs": round(flops / (dms * 1e-3) / 1e12, 2),
                             "achieved_GBps": round(dbytes / (dms * 1e-3) / 1e9, 1),
                             "hbm_frac": round(dbytes / (dms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                             "spmm_speedup": round(dms / ms, 3), "copies_rotated": n_d}
        # context only: the vendor library's GEMM on the same operands and layouts (the paper's dense baseline is
        # the vendor library, Sec. 6.1), through torch.matmul (rocBLAS / hipBLASLt); C[N, M] = X[N, K] . W[M, K]^T
        V = torch.empty((N, M), dtype=torch.float16, device="cuda")
        vms, _ = _time_loop([lambda w=w: torch.matmul(X, w.t(), out=V) for w in dense], args.steps, args.warmup)
        res["vendor_gemm"] = {"library": "torch.matmul (rocBLAS / hipBLASLt)", "ms_per_step": round(vms, 5),
                              "achieved_GBps": round(dbytes / (vms * 1e-3) / 1e9, 1), "spmm_speedup": round(vms / ms, 3)}
        del dense, Wd, D, V
    del W32

    if with_cpu:
        import oracle  # the cpu_baseline leg is the only part of the bench line that touches the oracle

        # the oracle over the whole workload (every row of C), timed; repeated while it is short, up to about
        # ten seconds of CPU work
        t0 = time.perf_counter()
        ref = oracle.ref_spmm_f64(Wb, Xb)
        dt = time.perf_counter() - t0
        reps = int(max(1, min(50, 10.0 // max(dt, 1e-3))))
        if reps > 1:
            t0 = time.perf_counter()
            for _ in range(reps):
                ref = oracle.ref_spmm_f64(Wb, Xb)
            dt = (time.perf_counter() - t0) / reps
        scale = max(float(np.abs(ref).max()), 1e-30)
        err = float(np.abs(C_host.astype(np.float64) - ref).max()) / scale
        res["cpu_baseline"] = {"value": round(flops / dt / 1e12, 5), "unit": "TFLOP/s",
                               "cores": oracle.ref_threads(), "kind": "oracle",
                               "sample": f"the whole workload: W ({M}x{K}) x X ({K}x{N}), fp64 triple loop, zeros not "
                                         f"skipped, {dt:.3f} s per pass, mean of {reps} passes"}
        res["parity"] = {"max_rel_err_vs_oracle": err, "rows_checked": M, "tolerance": PARITY_TOL,
                         "ok": bool(err <= PARITY_TOL)}
        if "format_v2" in res:
            err2 = float(np.abs(res["format_v2"]["_C"].astype(np.float64) - ref).max()) / scale
            res["format_v2"]["max_rel_err_vs_oracle"] = err2
            res["parity"]["ok"] = bool(res["parity"]["ok"] and err2 <= PARITY_TOL)
    if "format_v2" in res:
        res["format_v2"].pop("_C")
    for b in blobs:
        fls.fls_forget(b)
    return res


def _workload_text(cfg, st):
    return (f"{cfg.name}: {cfg.what}; W {cfg.M}x{cfg.K} fp16 N(0,0.02) {cfg.mask}-pruned to "
            f"{int(cfg.beta * 100)} % sparsity, X {cfg.K}x{cfg.N} fp16 N(0,1)")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # a step is 30 - 90 us: the defaults keep the GPU busy long enough (tens of ms) for its clocks to settle
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--config", default=HEADLINE,
                    help=f"C1..C4, L1, L2 (OPT-175B-sized), S1 (C4 with 32 columns); default {HEADLINE}, the largest named single-GPU configuration")
    ap.add_argument("--no-others", action="store_true",
                    help="leave out the other named configurations (C2, C3) that the default run reports beside the headline")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--format", type=int, choices=(1, 2), default=1,
                    help="--sweep only: the blob format of the sweep's sparse points (1: the paper's word; 2: three bytes per nonzero)")
    ap.add_argument("--no-v2", dest="v2", action="store_false",
                    help="leave out the run of the same matrix in format version 2 (3 bytes per nonzero)")
    ap.add_argument("--no-dense", action="store_true")
    ap.add_argument("--sweep", action="store_true",
                    help="instead of the bench line: the 12288 x 12288 sweep (sparsity x mask x N, each with its dense pair)")
    ap.add_argument("--crossover", action="store_true",
                    help="instead of the bench line: the non-skinny study, N = 64 ... 8192 on the 12288 x 12288 matrix "
                         "against the own and the vendor's dense GEMM")
    ap.add_argument("--out", default="", help="with --sweep / --crossover: also write the lines to this file")
    ap.add_argument("--layer", action="store_true",
                    help="instead of the bench line: the four MatMuls of one OPT-30B-shaped decoder layer back to back, "
                         "eager and as a HIP graph")
    ap.add_argument("--layer-n", type=int, default=16, help="with --layer: the batch size N")
    ap.add_argument("--entry", choices=("spmm", "noalloc"), default="spmm",
                    help="the entry point that is timed: fls_spmm, or fls_spmm_noalloc (N <= 32; it keeps to the narrow "
                         "kernel and clears its flags with a small kernel of its own before every call; the line is marked)")
    ap.add_argument("--x-values", choices=("workload", "zeros", "ones"), default="workload",
                    help="a study, not the benchmark: X of the workload's shape filled with zeros or ones (how much of a "
                         "call's time depends on the operand values, i.e. on power; the line is marked)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run a plain 1 GiB device copy three times (the known-size kernel the HBM counters "
                         "of a rocprofv3 --pmc run are scaled by)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build is a one-GPU kernel path (no sharding, no collectives); run with --gpus 1")

    if args.sweep:
        run_sweep(args)
        return
    if args.layer:
        run_layer(args)
        return
    if args.crossover:
        run_crossover(args)
        return

    import torch

    import paper_2309_10285_amd as fls

    fls.lib()
    assert torch.cuda.is_available(), "bench.py needs a GPU"

    r = measure_config(args.config, args, with_dense=not args.no_dense, with_cpu=not args.no_cpu_baseline)
    cfg, st = r["cfg"], r["st"]
    out = {
        "metric": f"SpMM dense-equivalent TFLOP/s (2*M*K*N / latency), {cfg.what}, {int(cfg.beta * 100)} % sparsity, N={cfg.N}",
        "value": round(r["tflops"], 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(r["ms"], 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "data": "synthetic",
        "config": {"workload": _workload_text(cfg, st),
                   "M": cfg.M, "K": cfg.K, "N": cfg.N, "sparsity": cfg.beta, "nnz": st["nnz"], "blob_bytes": st["bytes_total"],
                   "blob_copies_rotated": r["n_copies"], "seed": cfg.seed},
        "achieved_GBps": round(r["gbs"], 1), "hbm_frac": round(r["gbs"] / HBM_PEAK_GBS, 4),
        "host_ms_per_step": round(r["host_ms"], 5),
        "roofline": r["roofline"], "stream_ceiling": r["stream_ceiling"],
    }
    for key in ("format_v2", "dense_gemm", "vendor_gemm", "cpu_baseline", "parity"):
        if key in r:
            out[key] = r[key]
    if args.entry != "spmm":
        out["config"]["entry"] = "fls_spmm_noalloc"
    if args.x_values != "workload":
        out["data"] = f"synthetic; NOT the workload's X: X filled with {args.x_values} (operand-value study)"
        out["config"]["x_values"] = args.x_values
    gen_s = r["t_gen"]
    failed = [args.config] if "parity" in r and not r["parity"]["ok"] else []

    if args.calibration_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").fill_(1.0)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    if args.config == HEADLINE and not args.no_others:
        # the other named configurations, each with its own roofline, ceiling, dense pair and parity
        others = {}
        for name in OTHERS:
            o = measure_config(name, args, with_dense=not args.no_dense, with_cpu=not args.no_cpu_baseline)
            rec = {"workload": _workload_text(o["cfg"], o["st"]), "ms_per_step": round(o["ms"], 5),
                   "TFLOPs": round(o["tflops"], 2), "achieved_GBps": round(o["gbs"], 1), "roofline": o["roofline"],
                   "stream_ceiling": o["stream_ceiling"], "nnz": o["st"]["nnz"], "blob_bytes": o["st"]["bytes_total"]}
            for key in ("format_v2", "dense_gemm", "vendor_gemm", "parity"):
                if key in o:
                    rec[key] = o[key]
            if "parity" in o and not o["parity"]["ok"]:
                failed.append(name)
            gen_s += o["t_gen"]
            others[name] = rec
        out["other_configs"] = others
    out["input_generation_s"] = round(gen_s, 2)
    print(json.dumps(out))
    if failed:
        sys.exit(f"bench.py: C is off the oracle by more than {PARITY_TOL} on {', '.join(failed)}")


if __name__ == "__main__":
    main()
