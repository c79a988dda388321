"""Pins for the oracle's fp16 conversions against numpy's IEEE binary16."""
import numpy as np


def test_half_to_float_all_bit_patterns(oracle_mod):
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    ref = bits.view(np.float16).astype(np.float32)
    got = np.array([oracle_mod.half_to_float(int(b)) for b in bits], dtype=np.float32)
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), ref[~nan].view(np.uint32))


def test_double_to_half_matches_numpy_single_rounding(oracle_mod):
    rng = np.random.default_rng(7)
    xs = np.concatenate([
        rng.standard_normal(20000) * 10.0 ** rng.integers(-9, 5, 20000),
        # exact halves and the ties between neighbouring halves (round-half-to-even cases)
        np.arange(65536, dtype=np.uint32).astype(np.uint16).view(np.float16).astype(np.float64)[::7],
        np.array([65504.0, 65519.999, 65520.0, 70000.0, 2.0 ** -25, 2.0 ** -25 * 1.0000001, 2.0 ** -24 * 1.5,
                  2.0 ** -24 * 2.5, 2.0 ** -14, 2.0 ** -14 - 2.0 ** -26, 0.0, -0.0, 1.0 + 2.0 ** -11,
                  1.0 + 3 * 2.0 ** -11, 2047.5, 2048.5, 2049.0, -2050.0 - 1.0]),
    ])
    xs = xs[np.isfinite(xs)]
    ties = []
    h = np.arange(0x0001, 0x7bff, 13, dtype=np.uint32).astype(np.uint16).view(np.float16).astype(np.float64)
    hn = np.arange(0x0002, 0x7c00, 13, dtype=np.uint32).astype(np.uint16).view(np.float16).astype(np.float64)
    ties = (h + hn) / 2.0          # exactly between two neighbouring halves
    xs = np.concatenate([xs, ties, -ties])
    with np.errstate(over="ignore"):
        ref = xs.astype(np.float16).view(np.uint16)
    got = np.array([oracle_mod.double_to_half_bits(float(x)) for x in xs], dtype=np.uint16)
    assert np.array_equal(got, ref)
