"""Pins of the oracle's format version 2 (Tiled-CSL in groups of four entries that share one word of locations:
the first in full, the others as 6-bit distances; 3 bytes per nonzero).

What fixes it besides itself: a tile encoded by hand from the format's rules (tests/golden/), a decoder written
here independently of the oracle's, bit-exact round trips on the cases a plausible mistake breaks (a gap of
exactly 63 / 64 / 126 / 127 locations, a first element beyond location 63, the last location of a tile,
empty and full tiles, -0.0 / NaN / Inf / subnormal patterns), and sizes from a closed form computed with numpy
from the sorted locations."""
import json
import os

import numpy as np
import pytest

import fls_workloads as wl

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "tiled_csl_v2_hand_tile.json")


def _locs(W, tile_m, tile_k):
    """Per tile (band-major): sorted locations of the stored elements, with their bit patterns."""
    M, K = W.shape
    out = []
    for i in range(M // tile_m):
        for j in range(K // tile_k):
            t = W[i * tile_m:(i + 1) * tile_m, j * tile_k:(j + 1) * tile_k]
            x, y = np.nonzero(t)
            loc = (y // 8) * (tile_m * 8) + x * 8 + y % 8
            order = np.argsort(loc, kind="stable")
            out.append((loc[order], t[x[order], y[order]]))
    return out


def _independent_decode(blob, M, K):
    """A decoder written from the format's description, sharing nothing with the oracle's."""
    u32 = blob[:32].view(np.uint32)
    u64 = blob[32:64].view(np.uint64)
    assert u32[0] == 0x32534C46 and u32[1] == 2 and u32[4] == 4
    tile_m, tile_k = int(u32[2]), int(u32[3])
    tiles = (M // tile_m) * (K // tile_k)
    n_off = (tiles + 4 + 15) // 16 * 16
    offs = blob[64:64 + 4 * n_off].view(np.uint32)
    words = blob[64 + 4 * n_off:].view(np.uint32)
    assert words.size == int(u64[3])
    W = np.zeros((M, K), dtype=np.uint16)
    for t in range(tiles):
        i, j = divmod(t, K // tile_k)
        g = words[offs[t]:offs[t + 1]].reshape(-1, 3)
        vals = np.stack([g[:, 0] & 0xFFFF, g[:, 0] >> 16, g[:, 1] & 0xFFFF, g[:, 1] >> 16], axis=1).reshape(-1)
        assert not (g[:, 2] >> 30).any()
        # every group by itself: its first location, then three distances added up
        steps = np.stack([g[:, 2] & 0xFFF] + [(g[:, 2] >> s) & 0x3F for s in (12, 18, 24)], axis=1).astype(np.int64)
        loc = np.cumsum(steps, axis=1).reshape(-1)
        assert (np.diff(loc) > 0).all()  # ascending through the tile, group after group
        keep = vals != 0
        loc, vals = loc[keep], vals[keep]
        assert (loc < tile_m * tile_k).all()
        x, y = (loc % (tile_m * 8)) // 8, (loc // (tile_m * 8)) * 8 + loc % 8
        W[i * tile_m + x, j * tile_k + y] = vals.astype(np.uint16)
    return W


def test_hand_encoded_tile(oracle_mod):
    g = json.load(open(GOLDEN))
    W = np.zeros((g["M"], g["K"]), dtype=np.uint16)
    for x, y, bits in g["elements"]:
        W[x, y] = bits
    blob = oracle_mod.ref_compress_v2(W, tile_m=g["tile_m"], tile_k=g["tile_k"])
    assert blob.size == g["bytes_total"]
    assert list(blob[:32].view(np.uint32)) == g["header_u32"]
    assert list(blob[32:64].view(np.uint64)) == g["header_u64"]
    assert list(blob[64:128].view(np.uint32)) == g["offsets"]
    assert list(blob[128:].view(np.uint32)) == g["words"]
    assert np.array_equal(oracle_mod.ref_decompress_v2(blob, g["M"], g["K"]), W)
    assert np.array_equal(_independent_decode(blob, g["M"], g["K"]), W)


def _closed_form_words(W, tile_m, tile_k):
    total, longest = 0, 0
    for loc, _ in _locs(W, tile_m, tile_k):
        gaps = np.diff(np.concatenate([[0], loc]))                     # distance of every stored element from the entry before
        bridges = int(np.where(gaps > 0, (gaps - 1) // 63, 0).sum())   # steps of 63 that fit strictly before it
        words = -(-(loc.size + bridges) // 4) * 3
        total += words
        longest = max(longest, words)
    return total, longest


@pytest.mark.parametrize("beta", [0.0, 0.5, 0.8, 0.9, 0.99, 0.999, 1.0])
def test_round_trip_and_sizes_random(oracle_mod, beta):
    M, K = 384, 160
    W32 = wl.gen_weights_f32(M, K, 11)
    W = np.zeros((M, K), np.uint16) if beta >= 1 else (wl.dense_bits(W32) if beta <= 0 else wl.prune_uniform(W32, beta, 12))
    blob = oracle_mod.ref_compress_v2(W)
    info = oracle_mod.ref_inspect_v2(blob)
    assert info["rc"] == 0 and info["nnz"] == int(np.count_nonzero(W)) and info["bytes_total"] == blob.size
    total, longest = _closed_form_words(W, 128, 32)
    assert info["total_words"] == total and info["max_tile_words"] == longest
    assert np.array_equal(oracle_mod.ref_decompress_v2(blob, M, K), W)
    assert np.array_equal(_independent_decode(blob, M, K), W)
    offs = blob[64:64 + info["bytes_offsets"]].view(np.uint32)
    assert (np.diff(offs.astype(np.int64)) >= 0).all() and (offs % 3 == 0).all() and offs[info["num_tiles"]:].min() == total
    assert blob.size <= oracle_mod.ref_compress_bound_v2(M, K)
    if beta <= 0:
        assert blob.size == oracle_mod.ref_compress_bound_v2(M, K) == 64 + 4 * info["n_off"] + 3 * M * K
    if 0 < beta <= 0.9:  # 3 bytes per nonzero where bridges are rare: the point of the format
        assert 2.99 <= info["bytes_nonzeros"] / info["nnz"] <= 3.1


def test_gap_edges_and_special_values(oracle_mod):
    """One 128 x 32 tile per case: gaps of exactly 63 (no bridge), 64 (one), 126 (one), 127 (two); a first
    element at location 63 / 64 / 4095; the tile's last location; special bit patterns."""
    def at(loc):  # location -> (row, column) of a 128 x 32 tile
        return (loc % 1024) // 8, (loc // 1024) * 8 + loc % 8

    cases = {"gaps": [0, 63, 127, 253, 380, 4095], "late-start-63": [63, 64], "late-start-64": [64],
             "only-last": [4095], "first-and-last": [0, 4095], "dense-run": list(range(1000, 1300))}
    expected_bridges = {"gaps": 0 + 0 + 1 + 1 + 2 + (4095 - 380 - 1) // 63, "late-start-63": 0, "late-start-64": 1,
                        "only-last": (4095 - 1) // 63, "first-and-last": (4095 - 1) // 63, "dense-run": (1000 - 1) // 63}
    special = [0x8000, 0x7C00, 0xFC00, 0x7E00, 0xFFFF, 0x0001, 0x83FF, 0x3C00]
    for name, locs in cases.items():
        W = np.zeros((128, 32), dtype=np.uint16)
        for q, loc in enumerate(locs):
            W[at(loc)] = special[q % len(special)]
        blob = oracle_mod.ref_compress_v2(W)
        info = oracle_mod.ref_inspect_v2(blob)
        entries = len(locs) + expected_bridges[name]
        assert info["total_words"] == -(-entries // 4) * 3, name
        assert np.array_equal(oracle_mod.ref_decompress_v2(blob, 128, 32), W), name
        assert np.array_equal(_independent_decode(blob, 128, 32), W), name


def test_both_format_versions_decode_to_the_same_matrix(oracle_mod):
    W = wl.prune_magnitude(wl.gen_weights_f32(256, 256, 21), 0.8)
    b1, b2 = oracle_mod.ref_compress(W), oracle_mod.ref_compress_v2(W)
    assert np.array_equal(oracle_mod.ref_decompress(b1, 256, 256), oracle_mod.ref_decompress_v2(b2, 256, 256))
    i1, i2 = oracle_mod.ref_inspect(b1), oracle_mod.ref_inspect_v2(b2)
    assert i1["nnz"] == i2["nnz"] and 0.74 < i2["bytes_nonzeros"] / i1["bytes_nonzeros"] < 0.76
    # a version-1 blob is not a version-2 blob and the other way round
    assert oracle_mod.ref_inspect_v2(b1)["rc"] != 0 and oracle_mod.ref_inspect(b2)["rc"] != 0


def test_malformed_blobs_are_rejected(oracle_mod):
    W = wl.prune_uniform(wl.gen_weights_f32(128, 64, 31), 0.8, 32)
    blob = oracle_mod.ref_compress_v2(W)
    bad = blob.copy()
    bad[64 + 4] += 1  # an offset that is not a multiple of 3
    with pytest.raises(ValueError):
        oracle_mod.ref_decompress_v2(bad, 128, 64)
    with pytest.raises(ValueError):
        oracle_mod.ref_decompress_v2(blob[:-12], 128, 64)  # truncated
    with pytest.raises(ValueError):
        oracle_mod.ref_decompress_v2(blob, 256, 64)        # another shape
    info = oracle_mod.ref_inspect_v2(blob)
    w2 = 64 + info["bytes_offsets"] + 8                    # the first group's word of locations
    bad = blob.copy()
    bad[w2:w2 + 4].view(np.uint32)[0] &= ~np.uint32(0x3F << 12)  # a distance of 0: the same location twice
    with pytest.raises(ValueError):
        oracle_mod.ref_decompress_v2(bad, 128, 64)
    bad = blob.copy()
    bad[w2:w2 + 4].view(np.uint32)[0] |= np.uint32(1 << 31)      # a bit that no field owns
    with pytest.raises(ValueError):
        oracle_mod.ref_decompress_v2(bad, 128, 64)
