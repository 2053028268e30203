"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP library's tests / bench.

This module holds no arithmetic of the method (no compression, no products): only random
weights, pruning masks and activations with the shapes and statistics of the paper's kernel
benchmark (Sec. 6.1: the four MatMuls of OPT-30B/66B/175B, batch 8..64, 70/80/90 % sparsity),
standing in for the pruned OPT checkpoints, which are not available here.

Conventions: W is returned as uint16 fp16 bit patterns [M, K] (row-major); X as uint16 [N, K]
(column-major K x N).  Pruned entries are +0 (0x0000) by selection, never by multiplying with a
mask (which would create -0.0).
"""
from dataclasses import dataclass

import numpy as np

_ROWS_PER_CHUNK = 1024


def _rng(seed):
    return np.random.Generator(np.random.Philox(int(seed)))


def gen_weights_f32(M, K, seed, sigma=0.02):
    """i.i.d. N(0, sigma) fp32 weights, generated in row chunks (deterministic for a given seed)."""
    g = _rng(seed)
    W = np.empty((M, K), dtype=np.float32)
    for r in range(0, M, _ROWS_PER_CHUNK):
        n = min(_ROWS_PER_CHUNK, M - r)
        W[r:r + n] = g.standard_normal((n, K), dtype=np.float32) * np.float32(sigma)
    return W


def _to_bits(W32, keep):
    bits = W32.astype(np.float16).view(np.uint16)
    return np.where(keep, bits, np.uint16(0))


def prune_uniform(W32, beta, seed):
    """Each entry kept independently with probability 1 - beta ("random sparsity", Sec. 6.1)."""
    g = _rng(seed)
    keep = np.empty(W32.shape, dtype=bool)
    for r in range(0, W32.shape[0], _ROWS_PER_CHUNK):
        n = min(_ROWS_PER_CHUNK, W32.shape[0] - r)
        keep[r:r + n] = g.random((n, W32.shape[1]), dtype=np.float32) >= np.float32(beta)
    return _to_bits(W32, keep)


def prune_magnitude(W32, beta):
    """Magnitude pruning (Sec. 3.1): the ceil(beta*M*K) entries of smallest |w| (ranked in fp32) are removed."""
    n_drop = int(np.ceil(beta * W32.size))
    if n_drop <= 0:
        return _to_bits(W32, np.ones(W32.shape, dtype=bool))
    a = np.abs(W32).ravel()
    thr = np.partition(a, n_drop - 1)[n_drop - 1]
    keep = np.abs(W32) > thr
    return _to_bits(W32, keep)


def prune_row_skewed(W32, beta, seed):
    """Row-skewed mask: row i has density min(1, (1-beta) * b_i * 7/2), b_i ~ Beta(2,5) (mean 2/7)."""
    g = _rng(seed)
    M, K = W32.shape
    b = g.beta(2.0, 5.0, size=M)
    dens = np.minimum(1.0, (1.0 - beta) * b * 3.5).astype(np.float32)
    keep = np.empty(W32.shape, dtype=bool)
    for r in range(0, M, _ROWS_PER_CHUNK):
        n = min(_ROWS_PER_CHUNK, M - r)
        keep[r:r + n] = g.random((n, K), dtype=np.float32) < dens[r:r + n, None]
    return _to_bits(W32, keep)


def gen_x(N, K, seed):
    """Activations N(0,1) in fp16, as uint16 [N, K]."""
    return _rng(seed).standard_normal((N, K), dtype=np.float32).astype(np.float16).view(np.uint16)


def dense_bits(W32):
    """The unpruned matrix in fp16 (for the dense GEMM pair of each sparse point)."""
    return W32.astype(np.float16).view(np.uint16)


@dataclass(frozen=True)
class Config:
    name: str
    M: int
    K: int
    N: int
    beta: float
    mask: str  # "uniform" | "magnitude" | "row_skewed"
    seed: int
    what: str


CONFIGS = {
    "C1": Config("C1", 1024, 1024, 8, 0.80, "uniform", 0x5EED0001, "tiny correctness case"),
    "C2": Config("C2", 28672, 7168, 16, 0.80, "magnitude", 0x5EED0002, "OPT-30B-shaped FFN up-projection"),
    "C3": Config("C3", 27648, 9216, 32, 0.70, "magnitude", 0x5EED0003, "OPT-66B-shaped fused QKV"),
    "C4": Config("C4", 12288, 49152, 64, 0.90, "magnitude", 0x5EED0004, "OPT-175B-shaped FFN down-projection"),
    # beyond the five named configurations: the largest MatMul of the paper's kernel benchmark (Sec. 6.1), where a
    # call is long enough for the fixed cost of a launch not to matter
    "L1": Config("L1", 49152, 12288, 16, 0.80, "magnitude", 0x5EED0006, "OPT-175B-shaped FFN up-projection"),
    "L2": Config("L2", 49152, 12288, 8, 0.70, "magnitude", 0x5EED0007, "OPT-175B-shaped FFN up-projection"),
    # C4's matrix with 32 columns: 90 % sparsity in the passes of up to 32 columns, where the on-chip work per
    # tile, not the stream, is the ceiling (the point the two format versions are compared on with counters)
    "S1": Config("S1", 12288, 49152, 32, 0.90, "magnitude", 0x5EED0004, "OPT-175B-shaped FFN down-projection, 32 columns"),
}


def decoder_layer(hidden, ffn, N, beta, seed=0x5EED0010):
    """The four weight MatMuls of one OPT decoder layer (Sec. 2.1 / Fig. 2 of the paper): fused QKV projection,
    attention output projection, the two feed-forward layers.  Each has its own seeded weights and activations."""
    shapes = [("QKV projection", 3 * hidden, hidden), ("attention output projection", hidden, hidden),
              ("FFN up-projection", ffn, hidden), ("FFN down-projection", hidden, ffn)]
    return [Config(f"layer-{i}", M, K, N, beta, "magnitude", seed + 16 * i, what) for i, (what, M, K) in enumerate(shapes)]


SWEEP_M = 12288
SWEEP_K = 12288
SWEEP_BETAS = (0.5, 0.6, 0.7, 0.8, 0.9)
SWEEP_NS = (8, 16, 32, 64, 128, 256)
SWEEP_MASKS = ("uniform", "row_skewed")
SWEEP_SEED = 0x5EED0005


def make_w32(cfg):
    return gen_weights_f32(cfg.M, cfg.K, cfg.seed)


def make_inputs(cfg, W32=None):
    """(W bits [M,K], X bits [N,K]) of a named configuration."""
    if W32 is None:
        W32 = make_w32(cfg)
    if cfg.mask == "uniform":
        W = prune_uniform(W32, cfg.beta, cfg.seed + 1)
    elif cfg.mask == "magnitude":
        W = prune_magnitude(W32, cfg.beta)
    elif cfg.mask == "row_skewed":
        W = prune_row_skewed(W32, cfg.beta, cfg.seed + 1)
    else:
        raise ValueError(cfg.mask)
    X = gen_x(cfg.N, cfg.K, cfg.seed + 2)
    return W, X


def sweep_config(beta, mask, N):
    return Config(f"C5-{mask}-{int(round(beta * 100))}-N{N}", SWEEP_M, SWEEP_K, N, beta, mask, SWEEP_SEED,
                  "OPT-175B-shaped attention output projection sweep point")
