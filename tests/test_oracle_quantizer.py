"""Pins for the oracle's quantizer (Section 3.2, Eq. 2) that do not come from the oracle itself:
hand-worked groups, exact rational arithmetic, the s/2 error bound and structural invariants."""
import os
from fractions import Fraction

import numpy as np
import pytest

GOLD = os.path.join(os.path.dirname(__file__), "golden", "eq2_handworked_groups.txt")


def _golden_rows():
    rows = []
    with open(GOLD) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            bits, vals, s, z, codes = [p.strip() for p in line.split("|")]
            rows.append((int(bits), [float(v) for v in vals.split()], float(s), float(z),
                         [int(c) for c in codes.split()]))
    return rows


@pytest.mark.parametrize("row", _golden_rows())
def test_handworked_groups(oracle_mod, row):
    bits, vals, s, z, codes = row
    x = np.array(vals, dtype=np.float16).astype(np.float32)
    assert np.array_equal(x.astype(np.float64), np.array(vals))      # fixture values are exact halves
    gs, gz, gc = oracle_mod.quantize_group(x, bits)
    assert float(gs) == s and float(gz) == z
    assert gc.tolist() == codes


# ---- exact rational model of the fp32 pipeline, independent of any float hardware ----

def _rne_int(fr: Fraction) -> int:
    fl = fr.numerator // fr.denominator
    rem = fr - fl
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1):
        return fl + 1
    return fl


def _rne_f32(fr: Fraction) -> Fraction:
    """Round a rational to the nearest IEEE binary32 value (ties to even), as a rational."""
    if fr == 0:
        return fr
    sign = -1 if fr < 0 else 1
    a = abs(fr)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1                      # now 2^e <= a < 2^(e+1)
    assert Fraction(2) ** e <= a < Fraction(2) ** (e + 1)
    e = max(e, -126)
    quantum = Fraction(2) ** (e - 23)
    return sign * _rne_int(a / quantum) * quantum


def _model_group(halves, bits):
    xs = [Fraction(float(h)) for h in halves]
    qmax = (1 << bits) - 1
    z = min(xs)
    rng = _rne_f32(max(xs) - z)
    s = _rne_f32(rng / qmax)
    codes = []
    for x in xs:
        if s == 0:
            codes.append(0)
            continue
        t = _rne_f32(_rne_f32(x - z) / s)
        codes.append(min(max(_rne_int(t), 0), qmax))
    return s, z, codes


def _check_against_model(oracle_mod, halves, bits):
    s, z, codes = oracle_mod.quantize_group(halves.astype(np.float32), bits)
    ms, mz, mc = _model_group(halves, bits)
    assert Fraction(float(s)) == ms
    assert Fraction(float(z)) == mz
    assert codes.tolist() == mc


@pytest.mark.parametrize("bits", [2, 4, 8])
def test_exact_rational_model_random_groups(oracle_mod, bits):
    rng = np.random.default_rng(100 + bits)
    for trial in range(60):
        scale = 10.0 ** rng.integers(-4, 3)
        offset = rng.standard_normal() * 20.0 * (trial % 3)
        halves = (rng.standard_normal(32) * scale + offset).astype(np.float16)
        _check_against_model(oracle_mod, halves, bits)


@pytest.mark.parametrize("bits", [2, 4, 8])
def test_exact_rational_model_tie_heavy_grids(oracle_mod, bits):
    """Values on a coarse dyadic grid make exact .5 quotients common: pins the tie rule and the division."""
    rng = np.random.default_rng(200 + bits)
    qmax = (1 << bits) - 1
    n_ties = 0
    for trial in range(60):
        step = 2.0 ** rng.integers(-6, 2)
        lo = float(rng.integers(-2000, 2000)) * step
        ks = rng.integers(0, 2 * qmax + 1, 32)
        ks[0], ks[1] = 0, 2 * qmax            # range = 2*qmax*step, so s = 2*step and odd k are ties
        halves = (lo + ks * step).astype(np.float16)
        if not np.array_equal(halves.astype(np.float64), lo + ks * step):
            continue                           # grid fell off the fp16 lattice; skip
        n_ties += int(np.sum(ks % 2 == 1))
        _check_against_model(oracle_mod, halves, bits)
        s, z, codes = oracle_mod.quantize_group(halves.astype(np.float32), bits)
        assert float(s) == 2 * step
        expect = [(k // 2) + ((k // 2) % 2 if k % 2 else 0) for k in ks]   # k/2 rounded half-to-even
        assert codes.tolist() == expect
    assert n_ties > 100


def test_exact_rational_model_all_fp16_values_in_a_fixed_range(oracle_mod):
    """Every fp16 value inside [z, z + range] for a few fixed (z, range), 31 at a time."""
    allh = np.arange(65536, dtype=np.uint32).astype(np.uint16).view(np.float16)
    allh = allh[np.isfinite(allh)]
    for bits, zv, top in [(2, -1.0, 2.0), (4, 0.0, 1.0), (8, -3.0, 5.0)]:
        inside = allh[(allh >= np.float16(zv)) & (allh <= np.float16(top))]
        inside = inside[:: max(1, inside.size // 2000)]
        for i in range(0, inside.size, 30):
            halves = np.concatenate([[np.float16(zv), np.float16(top)], inside[i:i + 30]]).astype(np.float16)
            _check_against_model(oracle_mod, halves, bits)


# ---- what Eq. 2 guarantees mathematically ----

@pytest.mark.parametrize("bits", [2, 4, 8])
def test_reconstruction_error_at_most_half_a_step(oracle_mod, bits):
    rng = np.random.default_rng(300 + bits)
    qmax = (1 << bits) - 1
    for trial in range(200):
        halves = (rng.standard_normal(32) * (1 + 9 * (trial % 2)) + rng.standard_normal() * 20).astype(np.float16)
        x = halves.astype(np.float64)
        s, z, codes = oracle_mod.quantize_group(halves.astype(np.float32), bits)
        xhat = codes.astype(np.float64) * float(s) + float(z)
        slack = float(s) / 2 * (1 + 2.0 ** -20) + 4 * np.spacing(np.float32(max(np.abs(x).max(), abs(float(z)))))
        assert np.all(np.abs(x - xhat) <= slack)
        assert float(z) == x.min()
        assert codes[np.argmin(x)] == 0
        if s > 0:
            assert codes[np.argmax(x)] == qmax
        assert codes.max() <= qmax
        # scale is the fp32 quotient of the range, within one rounding of the real number
        assert abs(float(s) - (x.max() - x.min()) / qmax) <= 2.0 ** -22 * float(s)


@pytest.mark.parametrize("bits", [2, 4, 8])
def test_constant_group_is_exact(oracle_mod, bits):
    halves = np.full(32, -7.25, dtype=np.float16)
    s, z, codes = oracle_mod.quantize_group(halves.astype(np.float32), bits)
    assert float(s) == 0.0 and float(z) == -7.25 and not codes.any()


@pytest.mark.parametrize("bits", [2, 4, 8])
def test_shift_equivariance_with_representable_shifts(oracle_mod, bits):
    """Adding a constant that keeps every value exactly representable leaves codes and s alone and shifts z."""
    rng = np.random.default_rng(400 + bits)
    for trial in range(50):
        base = (rng.integers(-64, 64, 32) / 8.0)          # multiples of 1/8 in [-8, 8)
        shift = float(rng.integers(-40, 40))              # integer shift: still multiples of 1/8, < 64 in size
        a = base.astype(np.float16)
        b = (base + shift).astype(np.float16)
        assert np.array_equal(b.astype(np.float64), base + shift)
        s1, z1, c1 = oracle_mod.quantize_group(a.astype(np.float32), bits)
        s2, z2, c2 = oracle_mod.quantize_group(b.astype(np.float32), bits)
        assert float(s1) == float(s2) and float(z2) == float(z1) + shift
        assert np.array_equal(c1, c2)


def test_eight_bit_requantization_is_idempotent(oracle_mod):
    """Quantizing X^ of a group whose step is a power of two (so X^ is exact in fp16) returns the same codes."""
    rng = np.random.default_rng(5)
    for trial in range(50):
        codes0 = rng.integers(0, 256, 32)
        codes0[0], codes0[1] = 0, 255
        z0 = float(rng.integers(-100, 100)) / 4.0
        x = (codes0 * 0.25 + z0).astype(np.float16)       # s = 0.25 exactly
        assert np.array_equal(x.astype(np.float64), codes0 * 0.25 + z0)
        s, z, codes = oracle_mod.quantize_group(x.astype(np.float32), 8)
        assert float(s) == 0.25 and float(z) == z0 and np.array_equal(codes, codes0)
        xhat = (codes.astype(np.float64) * float(s) + float(z)).astype(np.float16)
        s2, z2, codes2 = oracle_mod.quantize_group(xhat.astype(np.float32), 8)
        assert float(s2) == 0.25 and np.array_equal(codes2, codes0)


def test_error_shrinks_with_bits_on_gaussian_groups(oracle_mod):
    """i.i.d. N(0,1) groups of 32: mean |x - x^| is about range / (4 (2^B - 1)) with E[range] ~ 4.1."""
    rng = np.random.default_rng(6)
    means = {}
    for bits in (2, 4, 8):
        errs = []
        for trial in range(300):
            halves = rng.standard_normal(32).astype(np.float16)
            s, z, codes = oracle_mod.quantize_group(halves.astype(np.float32), bits)
            errs.append(np.abs(halves.astype(np.float64) - (codes * float(s) + float(z))).mean())
        means[bits] = float(np.mean(errs))
    assert means[8] < means[4] < means[2]
    for bits, expect in ((8, 4.1 / (4 * 255)), (4, 4.1 / (4 * 15)), (2, 4.1 / (4 * 3))):
        assert 0.75 * expect < means[bits] < 1.25 * expect


# ---- narrow-metadata variant: scale rounded once to fp16, zero-point unchanged ----

def _rne_f16(fr: Fraction) -> Fraction:
    """Round a non-negative rational to the nearest IEEE binary16 value (ties to even), as a rational."""
    if fr == 0:
        return fr
    e = fr.numerator.bit_length() - fr.denominator.bit_length()
    if Fraction(2) ** e > fr:
        e -= 1
    e = max(e, -14)                       # subnormals share the quantum 2^-24
    quantum = Fraction(2) ** (e - 10)
    r = _rne_int(fr / quantum) * quantum
    assert r < 65520
    return r


def _model_group_fp16_scale(halves, bits):
    xs = [Fraction(float(h)) for h in halves]
    qmax = (1 << bits) - 1
    z = min(xs)
    s = _rne_f16(_rne_f32(_rne_f32(max(xs) - z) / qmax))
    codes = []
    for x in xs:
        if s == 0:
            codes.append(0)
            continue
        t = _rne_f32(_rne_f32(x - z) / s)
        codes.append(min(max(_rne_int(t), 0), qmax))
    return s, z, codes


@pytest.mark.parametrize("bits", [2, 4, 8])
def test_fp16_scale_variant_matches_rational_model_and_numpy_rounding(oracle_mod, bits):
    rng = np.random.default_rng(700 + bits)
    differs = 0
    for trial in range(80):
        scale = 10.0 ** rng.integers(-4, 3)
        offset = rng.standard_normal() * 20.0 * (trial % 3)
        halves = (rng.standard_normal(32) * scale + offset).astype(np.float16)
        x = halves.astype(np.float32)
        s32, z32, c32 = oracle_mod.quantize_group(x, bits)
        s16, z16, c16 = oracle_mod.quantize_group(x, bits, scale_fp16=True)
        # the stored scale is numpy's fp16 rounding of the fp32 scale; the zero-point is untouched and is an fp16 number
        assert np.float32(np.float32(s32).astype(np.float16)) == s16
        assert z16 == z32 and np.float32(np.float16(z16)) == z16
        ms, mz, mc = _model_group_fp16_scale(halves, bits)
        assert Fraction(float(s16)) == ms and Fraction(float(z16)) == mz and c16.tolist() == mc
        differs += int(not np.array_equal(c16, c32))
        # error bound: half a (rounded) step, plus the clamp's share where the code saturated
        xhat = c16.astype(np.float64) * float(s16) + float(z16)
        qmax = (1 << bits) - 1
        slack = 0.5 * float(s16) * (1 + 2.0 ** -20) + 4 * np.spacing(np.float32(np.abs(x).max()))
        bound = np.where(c16 == qmax, slack + qmax * abs(float(s32) - float(s16)), slack)
        assert np.all(np.abs(xhat - x.astype(np.float64)) <= bound)
    if bits == 8:
        assert differs > 0      # with fine steps the rounded scale really gives a different encoding


def test_fp16_scale_variant_special_cases(oracle_mod):
    # a scale that is an fp16 number: the variant changes nothing
    x = np.array([0.0, 3.0] + [1.5] * 30, dtype=np.float32)
    assert all(np.array_equal(a, b) for a, b in zip(oracle_mod.quantize_group(x, 2), oracle_mod.quantize_group(x, 2, True)))
    # a range so small that the scale rounds to zero in fp16: all codes 0, like a constant group
    tiny = np.array([0.0, 2.0 ** -24] + [0.0] * 30, dtype=np.float32)          # two neighbouring fp16 subnormals
    s, z, c = oracle_mod.quantize_group(tiny, 8, True)
    assert s == 0.0 and z == 0.0 and not c.any()
    s, z, c = oracle_mod.quantize_group(tiny, 8)
    assert s > 0 and c[1] == 255
    # a scale that becomes an fp16 subnormal loses most of its bits: the clamp is what keeps codes in range
    x = np.zeros(32, dtype=np.float32)
    x[1] = 2.0 ** -24 * 700                  # range 700 * 2^-24, s = 2.745 * 2^-24 -> fp16 subnormal 3 * 2^-24
    x[2] = 2.0 ** -24 * 699
    s, z, c = oracle_mod.quantize_group(x, 8, True)
    assert s == np.float32(3 * 2.0 ** -24) and c[1] == 233 and c[2] == 233
    x[1] = 2.0 ** -24 * 300                  # s = 1.18 * 2^-24 -> 1 * 2^-24: quotient 300 > 255 is clamped
    x[2] = 2.0 ** -24 * 100
    s, z, c = oracle_mod.quantize_group(x, 8, True)
    assert s == np.float32(2.0 ** -24) and c[1] == 255 and c[2] == 100


def _bits32(x):
    return int(np.float32(x).view(np.uint32))


@pytest.mark.parametrize("bits", [2, 4, 8])
@pytest.mark.parametrize("scale_fp16", [False, True])
def test_zero_extremes_are_stored_as_plus_zero(oracle_mod, bits, scale_fp16):
    """Eq. 2 takes min(X) and max(X) as numbers; zero has two encodings.  The reading: a zero minimum (and a zero
    maximum) is +0 whichever zeros the group holds and in whichever order, so z and s have one bit pattern each and
    the result cannot depend on the order of the elements.  Expected bits are written out, not computed."""
    pz, nz = np.float32(0.0), np.float32(-0.0)
    assert _bits32(nz) == 0x80000000
    qmax = (1 << bits) - 1
    # minimum zero: both orders of (+0, -0), only -0, only +0; the rest positive (max = qmax -> s = 1 exactly)
    for head in ([pz, nz], [nz, pz], [nz, nz], [pz, pz]):
        x = np.array(head + [np.float32(qmax)] + [np.float32(1.0)] * 29, dtype=np.float32)
        s, z, c = oracle_mod.quantize_group(x, bits, scale_fp16)
        assert _bits32(z) == 0x00000000, head
        assert _bits32(s) == 0x3F800000                       # 1.0
        assert c.tolist() == [0, 0, qmax] + [1] * 29
    # maximum zero: the rest negative (min = -qmax): s = (0 - (-qmax)) / qmax = 1, never -0-tainted
    for head in ([pz, nz], [nz, pz], [nz, nz]):
        x = np.array(head + [np.float32(-qmax)] + [np.float32(-1.0)] * 29, dtype=np.float32)
        s, z, c = oracle_mod.quantize_group(x, bits, scale_fp16)
        assert _bits32(z) == _bits32(np.float32(-qmax)) and _bits32(s) == 0x3F800000
        assert c.tolist() == [qmax, qmax, 0] + [qmax - 1] * 29
    # a group of zeros only: z = +0, s = +0 (not -0, which max - min would give for max = -0, min = +0), codes 0
    for vals in ([nz] * 32, [pz, nz] * 16, [nz, pz] * 16):
        s, z, c = oracle_mod.quantize_group(np.array(vals, dtype=np.float32), bits, scale_fp16)
        assert _bits32(z) == 0 and _bits32(s) == 0 and not c.any()


@pytest.mark.parametrize("key_per_token", [False, True])
def test_zero_extremes_through_the_cache_export(oracle_mod, key_per_token):
    """The same reading through quantize_append and the canonical export, keys and values, both key groupings:
    k_zero / v_zero / k_scale / v_scale bits do not depend on the order in which +0 and -0 appear in a group."""
    rng = np.random.default_rng(5)
    B, H, T, D = 1, 1, 64, 128
    base = np.abs(rng.standard_normal((B, H, T, D))).astype(np.float16) + np.float16(0.5)
    dumps = []
    for first, second in ((0.0, -0.0), (-0.0, 0.0)):
        K, V = base.copy(), base.copy()
        # keys per channel: tokens 3 and 17 of each key group hold the zeros; values (and per-token keys): channels 5, 9 of a group
        K[:, :, 3::32, :] = np.float16(first); K[:, :, 17::32, :] = np.float16(second)
        K[:, :, :, 5::32] = np.float16(first); K[:, :, :, 9::32] = np.float16(second)
        V[:, :, :, 5::32] = np.float16(first); V[:, :, :, 9::32] = np.float16(second)
        o = oracle_mod.OracleCache(1, B, 4, H, D, [4], [2], residual=0, key_per_token=key_per_token)
        o.quantize_append(0, K, V)
        dumps.append(o.export(0))
        o.close()
    a, b = dumps
    for key in ("k_zero", "v_zero", "k_scale", "v_scale", "k_codes", "v_codes"):
        assert np.array_equal(a[key].view(np.uint8), b[key].view(np.uint8)), key
    for key in ("k_zero", "v_zero"):
        assert not a[key].view(np.uint32).any()               # every group's minimum is zero: all-zero bits, never 0x80000000
