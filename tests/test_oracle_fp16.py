"""Pins for the oracle's fp16 <-> fp64 conversions (the arithmetic base of every other check)."""
import numpy as np


def test_half_to_double_exhaustive_vs_numpy(oracle_mod):
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    got = oracle_mod.half_to_double(bits)
    ref = bits.view(np.float16).astype(np.float64)
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint64), ref[~nan].view(np.uint64))  # incl. sign of zero


def test_half_to_double_closed_form_points(oracle_mod):
    pts = {0x0000: 0.0, 0x0001: 2.0 ** -24, 0x03FF: 1023 * 2.0 ** -24, 0x0400: 2.0 ** -14, 0x3C00: 1.0,
           0x3C01: 1.0 + 2.0 ** -10, 0x7BFF: 65504.0, 0xC000: -2.0, 0x3555: 0.333251953125}
    bits = np.array(list(pts), dtype=np.uint16)
    assert oracle_mod.half_to_double(bits).tolist() == list(pts.values())
    assert np.isinf(oracle_mod.half_to_double(np.array([0x7C00, 0xFC00], dtype=np.uint16))).all()


def test_double_to_half_roundtrip_is_identity(oracle_mod):
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    d = oracle_mod.half_to_double(bits)
    back = oracle_mod.double_to_half(d)
    nan = np.isnan(d)
    assert np.array_equal(back[~nan], bits[~nan])
    assert ((back[nan] & 0x7C00) == 0x7C00).all() and ((back[nan] & 0x03FF) != 0).all()


def test_double_to_half_rne_vs_numpy(oracle_mod):
    g = np.random.Generator(np.random.Philox(11))
    vals = np.concatenate([
        g.standard_normal(200000) * 3.0,
        g.standard_normal(100000) * 1e-6,          # subnormal range
        g.standard_normal(100000) * 3e4,           # near overflow
        np.array([0.0, -0.0, 65504.0, 65519.999, 65520.0, 65536.0, 1e9, -1e9, 2.0 ** -25, 2.0 ** -25 * 1.0000001,
                  2.0 ** -24 * 1.5, 2.0 ** -24 * 2.5, 2.0 ** -14, 2.0 ** -14 - 2.0 ** -25, np.inf, -np.inf]),
    ])
    got = oracle_mod.double_to_half(vals)
    ref = vals.astype(np.float16).view(np.uint16)
    assert np.array_equal(got, ref)


def test_double_to_half_every_tie_goes_to_even(oracle_mod):
    # midpoints between consecutive finite halves: exactly representable in fp64
    bits = np.arange(0, 0x7BFF, dtype=np.uint32).astype(np.uint16)
    lo = oracle_mod.half_to_double(bits)
    hi = oracle_mod.half_to_double((bits + 1).astype(np.uint16))
    mid = (lo + hi) / 2
    got = oracle_mod.double_to_half(mid)
    expect = np.where(bits % 2 == 0, bits, bits + 1).astype(np.uint16)
    assert np.array_equal(got, expect)
    # a hair off the midpoint goes to the nearer neighbour
    assert np.array_equal(oracle_mod.double_to_half(np.nextafter(mid, np.inf)), (bits + 1).astype(np.uint16))
    assert np.array_equal(oracle_mod.double_to_half(np.nextafter(mid, -np.inf)), bits)
