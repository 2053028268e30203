"""Pins for the oracle's Tiled-CSL compressor / decompressor (Sec. 4.3.1, 4.3.2, Alg. 3).

What fixes the expected values: a tile encoded by hand (tests/golden), an independent decoder
written in this file from the format rules, closed-form sizes, and the bit-exact round trip.
"""
import json
import os

import numpy as np
import pytest

import fls_workloads as wl

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _split(blob):
    hdr = blob[:64]
    u32 = hdr[:32].view(np.uint32)
    u64 = hdr[32:64].view(np.uint64)
    h = dict(magic=int(u32[0]), version=int(u32[1]), tile_m=int(u32[2]), tile_k=int(u32[3]), pad=int(u32[4]),
             policy=int(u32[5]), max_tile_words=int(u32[6]), reserved=int(u32[7]), M=int(u64[0]), K=int(u64[1]),
             nnz=int(u64[2]), total_words=int(u64[3]))
    tiles = (h["M"] // h["tile_m"]) * (h["K"] // h["tile_k"])
    n_off = (tiles + 4 + 15) // 16 * 16
    offs = blob[64:64 + 4 * n_off].view(np.uint32)
    words = blob[64 + 4 * n_off:].view(np.uint32)
    return h, tiles, offs, words


def _independent_decode(blob):
    """Decoder written from the format rules only (does not call the oracle)."""
    h, tiles, offs, words = _split(blob)
    tm, tk = h["tile_m"], h["tile_k"]
    W = np.zeros((h["M"], h["K"]), dtype=np.uint16)
    tiles_k = h["K"] // tk
    seen = 0
    for t in range(tiles):
        i, j = divmod(t, tiles_k)
        for w in words[offs[t]:offs[t + 1]].tolist():
            loc, bits = w & 0xFFFF, w >> 16
            if loc == tm * tk:
                assert bits == 0
                continue
            chunk, rem = divmod(loc, tm * 8)
            x, e = divmod(rem, 8)
            y = chunk * 8 + e
            assert W[i * tm + x, j * tk + y] == 0
            W[i * tm + x, j * tk + y] = bits
            seen += 1
    assert seen == h["nnz"]
    return W


def test_hand_encoded_tile(oracle_mod):
    g = json.load(open(os.path.join(GOLD, "tiled_csl_hand_tile.json")))
    geo = g["geometry"]
    W = np.array([[int(v, 16) for v in row] for row in g["W_rows_hex"]], dtype=np.uint16)
    blob = oracle_mod.ref_compress(W, tile_m=geo["tile_m"], tile_k=geo["tile_k"], pad=geo["pad_words"])
    h, tiles, offs, words = _split(blob)
    assert blob.size == g["bytes_total"]
    assert h["magic"] == int.from_bytes(b"FLS1", "little") and h["version"] == 1
    assert (h["tile_m"], h["tile_k"], h["pad"], h["policy"]) == (2, 16, 4, 0)
    assert (h["M"], h["K"], h["nnz"], h["total_words"], h["max_tile_words"]) == (2, 16, 7, 8, 8)
    assert offs.tolist() == g["tile_offsets"]
    assert [f"{w:08X}" for w in words.tolist()] == g["nonzeros_hex"]
    assert np.array_equal(oracle_mod.ref_decompress(blob, 2, 16), W)


def test_tile_walk_is_band_major(oracle_mod):
    # one nonzero per tile, value = tile id + 1: Alg. 3 walks row band i outer, K tile j inner
    tm, tk, M, K = 2, 8, 6, 32
    W = np.zeros((M, K), dtype=np.uint16)
    for i in range(M // tm):
        for j in range(K // tk):
            W[i * tm + 1, j * tk + 3] = i * (K // tk) + j + 1
    blob = oracle_mod.ref_compress(W, tile_m=tm, tile_k=tk, pad=1)
    h, tiles, offs, words = _split(blob)
    assert tiles == 12 and offs[:13].tolist() == list(range(13))
    assert (words >> 16).tolist() == list(range(1, 13))
    assert set((words & 0xFFFF).tolist()) == {1 * 8 + 3}


@pytest.mark.parametrize("tm,tk,pad", [(128, 32, 4), (64, 64, 4), (128, 64, 1), (16, 8, 8)])
@pytest.mark.parametrize("policy", [0, 1])
def test_round_trip_bit_exact_and_sizes(oracle_mod, tm, tk, pad, policy):
    g = np.random.Generator(np.random.Philox(5))
    M, K = 3 * tm, 4 * tk
    bits = g.integers(0, 65536, size=(M, K), dtype=np.uint32).astype(np.uint16)  # any pattern: NaN, Inf, -0, subnormal
    keep = g.random((M, K)) < 0.3
    W = np.where(keep, bits, np.uint16(0))
    W[:tm, :tk] = 0                                    # an empty tile
    W[tm:2 * tm, tk:2 * tk] = bits[tm:2 * tm, tk:2 * tk] | 1  # a completely full tile
    W[2 * tm, 0] = 0x8000                              # -0.0 at the first location of a tile
    W[3 * tm - 1, tk - 1] = 0x7E01                     # NaN payload at the last location of a tile
    blob = oracle_mod.ref_compress(W, tile_m=tm, tile_k=tk, pad=pad, policy=policy)
    h, tiles, offs, words = _split(blob)
    nnz_tile = np.array([[np.count_nonzero(W[i * tm:(i + 1) * tm, j * tk:(j + 1) * tk]) for j in range(K // tk)]
                         for i in range(M // tm)]).ravel()
    padded = (nnz_tile + pad - 1) // pad * pad
    assert h["nnz"] == int(np.count_nonzero(W)) == int(nnz_tile.sum())
    assert h["total_words"] == int(padded.sum()) == words.size
    assert h["max_tile_words"] == int(padded.max())
    assert offs[:tiles + 1].tolist() == np.concatenate([[0], np.cumsum(padded)]).tolist()
    assert (offs[tiles:] == h["total_words"]).all() and offs.size % 16 == 0 and offs.size >= tiles + 4
    assert blob.size == 64 + 4 * offs.size + 4 * int(padded.sum())
    assert blob.size <= oracle_mod.ref_compress_bound(M, K, tm, tk, pad)
    loc = words & 0xFFFF
    assert ((loc < tm * tk) | ((loc == tm * tk) & (words >> 16 == 0))).all()
    assert np.array_equal(_independent_decode(blob), W)
    assert np.array_equal(oracle_mod.ref_decompress(blob, M, K), W)
    info = oracle_mod.ref_inspect(blob)
    assert info["rc"] == 0 and info["bytes_total"] == blob.size and info["nnz"] == h["nnz"]


def test_policy0_is_ascending_location(oracle_mod):
    W, _ = wl.make_inputs(wl.CONFIGS["C1"])
    blob = oracle_mod.ref_compress(W[:256, :128])
    h, tiles, offs, words = _split(blob)
    for t in range(tiles):
        loc = (words[offs[t]:offs[t + 1]] & 0xFFFF).astype(np.int64)
        real = loc[loc < 128 * 32]
        assert (np.diff(real) > 0).all()
        assert (loc[real.size:] == 128 * 32).all() and loc.size - real.size < 4


def test_full_density_hits_the_bound(oracle_mod):
    W = np.full((128, 64), 0x3C00, dtype=np.uint16)
    blob = oracle_mod.ref_compress(W)
    assert blob.size == oracle_mod.ref_compress_bound(128, 64) == 64 + 4 * 16 + 4 * 128 * 64


@pytest.mark.parametrize("banks,group", [(32, 32), (64, 64), (32, 64)])
def test_bank_aware_order_invariants(oracle_mod, banks, group):
    """Sec. 4.3.3: reordering only permutes a tile's words (same multiset, same offsets) and
    every group drawn while all banks still hold words has pairwise distinct banks."""
    W, _ = wl.make_inputs(wl.CONFIGS["C1"])
    W = W[:256, :256]
    b0 = oracle_mod.ref_compress(W, policy=0)
    b1 = oracle_mod.ref_compress(W, policy=1, banks=banks, group=group)
    h0, tiles, o0, w0 = _split(b0)
    h1, _, o1, w1 = _split(b1)
    assert h1["policy"] == 1 and np.array_equal(o0, o1) and h0["nnz"] == h1["nnz"]
    conflict_free = 0
    for t in range(tiles):
        a, b = w0[o0[t]:o0[t + 1]], w1[o1[t]:o1[t + 1]]
        assert np.array_equal(np.sort(a), np.sort(b))
        real = b[(b & 0xFFFF) < 128 * 32]
        bank = ((real & 0xFFFF) >> 1) % banks
        remaining = np.bincount(bank, minlength=banks)
        for s in range(0, real.size, group):
            grp = bank[s:s + group]
            live = int((remaining > 0).sum())
            distinct = np.unique(grp).size
            assert distinct == min(live, grp.size) or distinct == grp.size
            if distinct == grp.size:
                conflict_free += 1
            remaining -= np.bincount(grp, minlength=banks)
    assert conflict_free > 0
    assert np.array_equal(oracle_mod.ref_decompress(b1, 256, 256), W)


def test_malformed_blobs_are_rejected(oracle_mod):
    W, _ = wl.make_inputs(wl.CONFIGS["C1"])
    blob = oracle_mod.ref_compress(W[:128, :64])
    bad = blob.copy(); bad[0] ^= 1
    assert oracle_mod.ref_inspect(bad)["rc"] != 0
    bad = blob.copy(); bad[4] = 9
    assert oracle_mod.ref_inspect(bad)["rc"] != 0
    assert oracle_mod.ref_inspect(blob[:-4])["rc"] != 0
    with pytest.raises(ValueError):
        oracle_mod.ref_decompress(blob, 128, 128)
    with pytest.raises(ValueError):
        oracle_mod.ref_compress(np.zeros((100, 64), dtype=np.uint16))
