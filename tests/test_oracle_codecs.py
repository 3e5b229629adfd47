"""Pins of the oracle's number formats against what the paper and the
mathematics fix (no GPU).  Every check compares the oracle with something that
is not the oracle: Table 1 as printed, exact rational nearest-value search,
numpy's rint / float16 casts, torch's float8_e4m3fn cast."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

import mofq_inputs as mi
from oracle import mofq_oracle as orc

FP4, FP4I, FP8, I4, I8 = orc.FP4_E2M1, orc.FP4_E2M1_IEEE, orc.FP8_E4M3, orc.INT4, orc.INT8


def _read_table1(golden_dir):
    rows = []
    for line in open(os.path.join(golden_dir, "fp4_e2m1_table1.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        code, ieee, ours = line.split()
        rows.append((int(code), ieee, ours))
    assert len(rows) == 16
    return rows


def _same_value(got: float, printed: str) -> bool:
    if printed == "NaN":
        return math.isnan(got)
    if printed == "Inf":
        return math.isinf(got)
    want = float(printed)
    return got == want and math.copysign(1.0, got) == math.copysign(1.0, want)


def test_e2m1_table1_redesigned_row(golden_dir):
    """Table 1, row without NaN/Inf: all sixteen values, including -0 at code 8."""
    for code, _, ours in _read_table1(golden_dir):
        assert _same_value(orc.decode(FP4, code), ours), (code, ours)


def test_e2m1_table1_ieee_row(golden_dir):
    for code, ieee, _ in _read_table1(golden_dir):
        assert _same_value(orc.decode(FP4I, code), ieee), (code, ieee)


def test_e2m1_added_values_are_4_and_6():
    """Section 4.2: the reassigned codes give exactly +-4 and +-6."""
    ours = {orc.decode(FP4, c) for c in range(16)}
    ieee = {orc.decode(FP4I, c) for c in range(16) if math.isfinite(orc.decode(FP4I, c))}
    assert ours - ieee == {4.0, 6.0, -4.0, -6.0}


def test_code_counts():
    """A b-bit format has 2^b codes: every code decodes, INT grids have step 1."""
    for fmt, n in ((I4, 16), (I8, 256)):
        vals = sorted(orc.decode(fmt, c) for c in range(n))
        assert len(set(vals)) == n
        assert all(b - a == 1.0 for a, b in zip(vals, vals[1:]))
    assert sorted(orc.decode(I4, c) for c in range(16))[0] == -8.0
    assert sorted(orc.decode(I8, c) for c in range(256))[-1] == 127.0


def test_e4m3_decode_matches_torch_cast():
    """All 256 E4M3 bit patterns against torch's own float8_e4m3fn decoding."""
    codes = torch.arange(256, dtype=torch.int32).to(torch.uint8)
    ref = codes.view(torch.float8_e4m3fn).to(torch.float32).numpy()
    for c in range(256):
        got = orc.decode(FP8, c)
        if np.isnan(ref[c]):
            assert math.isnan(got) and (c & 0x7F) == 0x7F
        else:
            assert got == float(ref[c]) and math.copysign(1, got) == math.copysign(1, ref[c]), c


def test_e4m3_grid_closed_form():
    mags = [orc.decode(FP8, c) for c in range(127)]
    assert all(b > a for a, b in zip(mags, mags[1:]))       # strictly increasing with code
    assert mags[0] == 0.0 and mags[1] == 2.0 ** -9 and mags[8] == 2.0 ** -6
    assert mags[-1] == 448.0 == orc.qmax(FP8)
    assert orc.qmax(FP4) == 6.0 and orc.qmax(I4) == 7.0 and orc.qmax(I8) == 127.0


def _nearest_even_code(fmt, n_mag, t: Fraction) -> int:
    """Independent nearest-value search in exact rationals."""
    mags = [Fraction(orc.decode(fmt, c)) for c in range(n_mag)]
    a = abs(t)
    best, best_d = None, None
    for c, m in enumerate(mags):
        d = abs(a - m)
        if best is None or d < best_d or (d == best_d and c % 2 == 0):
            best, best_d = c, d
    return best


def _interesting_points(n_mag, fmt):
    mags = [orc.decode(fmt, c) for c in range(n_mag)]
    pts = set(mags)
    for a, b in zip(mags, mags[1:]):
        mid = np.float32((a + b) / 2)
        assert float(mid) == (a + b) / 2
        for v in (mid, np.nextafter(mid, np.float32(np.inf)), np.nextafter(mid, np.float32(-np.inf)),
                  np.nextafter(np.float32(b), np.float32(-np.inf)),
                  np.nextafter(np.float32(b), np.float32(np.inf))):
            pts.add(float(v))
    top = mags[-1]
    pts.update([top * 1.0001, top * 2, top * 1e6, 3.0e38, 1e-45, 1e-30])
    return sorted(pts)


@pytest.mark.parametrize("fmt,n_mag,signbit", [(FP4, 8, 8), (FP8, 127, 0x80), (FP4I, 6, 8)])
def test_fp_encode_nearest_even_exact(fmt, n_mag, signbit):
    """Every grid value, every midpoint and its two fp32 neighbours, binade
    edges, saturation and tiny values, both signs, against exact rationals."""
    for v in _interesting_points(n_mag, fmt):
        for sgn in (1.0, -1.0):
            t = np.float32(sgn * v)
            want = _nearest_even_code(fmt, n_mag, Fraction(float(t)))
            if sgn < 0:
                want |= signbit
            assert orc.encode(fmt, t) == want, (fmt, float(t))


def test_e2m1_midpoints_listed():
    """The seven midpoints of the E2M1 grid resolve to the even code."""
    want = {0.25: 0.0, 0.75: 1.0, 1.25: 1.0, 1.75: 2.0, 2.5: 2.0, 3.5: 4.0, 5.0: 4.0}
    for t, g in want.items():
        assert orc.decode(FP4, orc.encode(FP4, t)) == g
        assert orc.decode(FP4, orc.encode(FP4, -t)) == -g
    assert orc.decode(FP4, orc.encode(FP4, 1e9)) == 6.0
    assert orc.decode(FP4, orc.encode(FP4, -7.0)) == -6.0


def test_negative_zero_code():
    """A negative value that rounds to zero keeps its sign bit (code 8 / 0x80)."""
    assert orc.encode(FP4, -0.1) == 8 and orc.encode(FP4, 0.1) == 0
    assert orc.encode(FP4, -0.0) == 8
    assert orc.encode(FP8, -1e-6) == 0x80 and orc.encode(FP8, 1e-6) == 0
    assert orc.encode(I4, -0.2) == 0 and orc.encode(I8, -0.5) == 0   # two's complement has no -0


def test_roundtrip_all_codes():
    for fmt, n in ((FP4, 16), (I4, 16), (I8, 256)):
        for c in range(n):
            assert orc.encode(fmt, np.float32(orc.decode(fmt, c))) == c
    for c in range(256):
        if (c & 0x7F) != 0x7F:
            assert orc.encode(FP8, np.float32(orc.decode(FP8, c))) == c


def test_e4m3_encode_matches_torch_cast_random():
    """Independent library cast: torch rounds fp32 to float8_e4m3fn to nearest
    even; inside |t| <= 448 it must agree with the oracle bit for bit."""
    rng = np.random.default_rng(0)
    t = np.concatenate([
        rng.standard_normal(200000).astype(np.float32) * 100,
        rng.standard_normal(100000).astype(np.float32) * 0.01,
        (rng.random(100000).astype(np.float32) * 2 - 1) * 448,
        (rng.random(50000).astype(np.float32) * 2 - 1) * 2.0 ** -6,
        np.array(_interesting_points(127, FP8), dtype=np.float32),
        -np.array(_interesting_points(127, FP8), dtype=np.float32),
    ])
    t = t[np.abs(t) <= 448].astype(np.float32)
    ref = torch.from_numpy(t).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = orc.encode_array(FP8, t)
    assert np.array_equal(got, ref)


def test_int_encode_matches_numpy_rint():
    rng = np.random.default_rng(1)
    t = np.concatenate([rng.standard_normal(100000).astype(np.float32) * 5,
                        rng.standard_normal(100000).astype(np.float32) * 100,
                        np.arange(-300, 300, 0.5, dtype=np.float32),
                        np.array([1e30, -1e30, 2.5, 3.5, -2.5, -3.5, 7.5, -8.5], dtype=np.float32)])
    for fmt, lo, hi, mask in ((I4, -8, 7, 0xF), (I8, -128, 127, 0xFF)):
        ref = (np.clip(np.rint(t.astype(np.float64)), lo, hi).astype(np.int64) & mask).astype(np.uint8)
        assert np.array_equal(orc.encode_array(fmt, t), ref)


def test_fp_encode_monotone_and_odd():
    t = np.linspace(-8, 8, 20001).astype(np.float32)
    for fmt in (FP4, FP8):
        v = orc.decode_array(fmt, orc.encode_array(fmt, t))
        assert np.all(np.diff(v) >= 0)
        assert np.array_equal(v, -v[::-1])


def test_round_fp16_matches_numpy():
    rng = np.random.default_rng(2)
    v = np.concatenate([np.exp(rng.uniform(-20, 11, 100000)).astype(np.float32),
                        np.array([0.0, 65504.0, 65519.9, 65520.0, 1e6, 6e-8, 2.98e-8, 2.9802322e-08,
                                  3e-8, 1e-9, 2.0 ** -14, 2.0 ** -24], dtype=np.float32)])
    with np.errstate(over="ignore"):
        ref = v.astype(np.float16).astype(np.float32)
    ref = np.where(np.isinf(ref), np.float32(65504.0), ref)
    got = np.array([orc.round_fp16(x) for x in v], dtype=np.float32)
    assert np.array_equal(got, ref)


def test_scale_formula():
    """s = fl32(fl32(r*a)/qmax); fp16 rounding; degenerate units get scale 1."""
    rng = np.random.default_rng(3)
    for _ in range(2000):
        a = np.float32(abs(rng.standard_normal()) * 0.1 + 1e-6)
        r = np.float32(rng.uniform(0.5, 1.0))
        for fmt in (I4, FP4, I8, FP8):
            ra = np.float32(a * r)                       # one fp32 multiply
            ref = np.float32(ra / np.float32(orc.qmax(fmt)))   # one fp32 divide
            assert orc.scale(a, r, fmt) == float(ref)
            h = float(np.float32(np.float16(ref)))
            assert orc.scale(a, r, fmt, True) == (h if h > 0 else 1.0)
    for fmt in (I4, FP4, I8, FP8):
        assert orc.scale(0.0, 1.0, fmt) == 1.0
        assert orc.scale(1e-44, 1.0, fmt) == 1.0
        assert orc.scale(1e-9, 1.0, fmt, True) == 1.0     # rounds to fp16 zero
        assert orc.scale(1e7, 1.0, I4, True) == 65504.0


# ---- E5M2, the other 8-bit floating-point option of Section 2.2 ---------------------------

FP8B = orc.FP8_E5M2


def test_e5m2_decode_matches_torch_cast():
    """All 256 E5M2 bit patterns against torch's own float8_e5m2 decoding (IEEE layout:
    infinities at 0x7C / 0xFC, NaN above them)."""
    codes = torch.arange(256, dtype=torch.int32).to(torch.uint8)
    ref = codes.view(torch.float8_e5m2).to(torch.float32).numpy()
    for c in range(256):
        got = orc.decode(FP8B, c)
        if np.isnan(ref[c]):
            assert math.isnan(got) and (c & 0x7F) > 0x7C
        else:
            assert got == float(ref[c]) and math.copysign(1, got) == math.copysign(1, ref[c]), c
    assert orc.decode(FP8B, 0x7B) == 57344.0 == orc.qmax(FP8B)
    assert orc.decode(FP8B, 0x01) == 2.0 ** -16 and orc.decode(FP8B, 0x04) == 2.0 ** -14
    assert orc.bits(FP8B) == 8


def test_e5m2_encode_matches_torch_cast_and_saturates():
    """torch rounds fp32 to float8_e5m2 to nearest even; inside the finite range the
    oracle must agree bit for bit; beyond it the oracle saturates at +-57344 (no Inf)."""
    rng = np.random.default_rng(5)
    t = np.concatenate([
        rng.standard_normal(200000).astype(np.float32) * 1000,
        rng.standard_normal(100000).astype(np.float32) * 1e-4,
        (rng.random(100000).astype(np.float32) * 2 - 1) * 57344,
        (rng.random(50000).astype(np.float32) * 2 - 1) * 2.0 ** -14,
        np.array([orc.decode(FP8B, c) for c in range(0x7C)], dtype=np.float32),
        np.array([0.5 * (orc.decode(FP8B, c) + orc.decode(FP8B, c + 1)) for c in range(0x7B)], dtype=np.float32),
    ])
    t = np.concatenate([t, -t])
    # torch rounds values at or above the midpoint between 57344 and 65536 to Inf
    t = t[np.abs(t) < 61440].astype(np.float32)
    ref = torch.from_numpy(t).to(torch.float8_e5m2).view(torch.uint8).numpy()
    assert np.array_equal(orc.encode_array(FP8B, t), ref)
    for big in (61440.0, 65504.0, 1e9, 3.4e38):
        assert orc.encode(FP8B, np.float32(big)) == 0x7B and orc.encode(FP8B, np.float32(-big)) == 0xFB
    for c in range(256):
        if (c & 0x7F) < 0x7C:
            assert orc.encode(FP8B, np.float32(orc.decode(FP8B, c))) == c


def test_e5m2_trades_precision_for_range_against_e4m3():
    """Two mantissa bits instead of three: on Gaussian weights (no range problem) the
    E5M2 tensor error is about 4x the E4M3 one (step twice as coarse)."""
    w = mi.to_f32_numpy(mi.llama_like_weight(32, 1024, seed=21))
    one = np.ones(1, dtype=np.float32)
    r = orc.quantize(w, FP8B, orc.PER_CHANNEL, one).err / orc.quantize(w, FP8, orc.PER_CHANNEL, one).err
    assert 3.0 < r < 5.5

