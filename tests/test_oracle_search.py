"""Pins of the oracle's scale search, error sums and per-layer select (no GPU).

The clip search, group-wise units and fp16 scales are not in the paper; they are
pinned here by exact rational brute force on tiny tensors, closed forms,
invariances and reductions to one another, never by the oracle's own output."""
from fractions import Fraction

import numpy as np
import pytest

import mofq_inputs as mi
from oracle import mofq_oracle as orc

I4, FP4, I8, FP8, FP4I = orc.INT4, orc.FP4_E2M1, orc.INT8, orc.FP8_E4M3, orc.FP4_E2M1_IEEE
PT, PC, PG = orc.PER_TENSOR, orc.PER_CHANNEL, orc.PER_GROUP
QMAX = {I4: 7.0, FP4: 6.0, I8: 127.0, FP8: 448.0}
ONE = np.ones(1, dtype=np.float32)


def _grid(fmt):
    n = 16 if orc.bits(fmt) == 4 else 256
    vals = []
    for c in range(n):
        v = orc.decode(fmt, c)
        if np.isfinite(v):
            vals.append((c, Fraction(v)))
    return vals


def _brute_unit(x32: np.ndarray, fmt: int, clip: np.ndarray, f16: bool):
    """Exact reference for one unit: fp32 scale arithmetic done with numpy
    scalars, grid choice and error in exact rationals."""
    a = np.float32(np.max(np.abs(x32))) if x32.size else np.float32(0)
    grid = _grid(fmt)
    is_int = fmt in (I4, I8)
    sse_k, codes_k, s_k = [], [], []
    for r in clip:
        ra = np.float32(np.float32(r) * a)
        s = np.float32(ra / np.float32(QMAX[fmt]))
        if f16:
            with np.errstate(over="ignore"):
                h = np.float32(np.float16(s))
            s = np.float32(65504.0) if np.isinf(h) else h
        if not s >= np.float32(2.0 ** -126):
            s = np.float32(1.0)
        inv = np.float32(np.float32(1.0) / s)
        sse = Fraction(0)
        codes = []
        for x in x32:
            t = np.float32(x * inv)
            tf = Fraction(float(t))
            if is_int:
                # nearest integer of the range, exact tie -> the even integer
                best = min(((abs(tf - g), int(g) % 2, c, g) for c, g in grid))
                code, gval = best[2], best[3]
            else:
                # nearest non-negative magnitude, exact tie -> the even code; the
                # sign bit of t is carried over (so -tiny gives the "-0" code)
                sign_mask = 8 if orc.bits(fmt) == 4 else 0x80
                mags = [(c, g) for c, g in grid if c < sign_mask]
                best = min(((abs(abs(tf) - g), c % 2, c, g) for c, g in mags))
                neg = bool(np.signbit(t))
                code = best[2] | (sign_mask if neg else 0)
                gval = -best[3] if neg else best[3]
            codes.append(code)
            d = Fraction(float(x)) - gval * Fraction(float(s))
            sse += d * d
        sse_k.append(sse)
        codes_k.append(codes)
        s_k.append(float(s))
    k_star = min(range(len(clip)), key=lambda k: (sse_k[k], k))
    return k_star, s_k[k_star], sse_k, codes_k[k_star]


@pytest.mark.parametrize("fmt", [I4, FP4, I8, FP8])
@pytest.mark.parametrize("f16", [False, True])
def test_search_brute_force_exact(fmt, f16):
    """Tiny tensors, K = 8: winner index, scale, codes and every candidate's
    error against exact rational arithmetic (ties resolve to the first)."""
    rng = np.random.default_rng(10 + fmt)
    clip = mi.clip_ratios(8)
    for trial in range(6):
        w = (rng.standard_normal((4, 16)) * 0.03).astype(np.float32)
        w[rng.integers(4), rng.integers(16)] *= 8
        if trial == 0:
            w[1] = 0.0                                   # a zero unit
        if trial == 1:
            w = w.astype(np.float16).astype(np.float32)
        q = orc.quantize(w, fmt, PC, clip, scale_f16=f16, want_table=True)
        for r in range(4):
            k, s, sse, codes = _brute_unit(w[r], fmt, clip, f16)
            assert q.clip_idx[r] == k
            assert float(q.scale[r]) == s
            assert list(q.codes[r]) == codes
            for kk in range(8):
                ex = float(sse[kk])
                assert abs(q.table[r, kk] - ex) <= 1e-13 * max(ex, 1e-300)
            assert abs(q.unit_err[r] - float(sse[k])) <= 1e-13 * max(float(sse[k]), 1e-300)


def test_zero_unit():
    w = np.zeros((3, 32), dtype=np.float32)
    for fmt in (I4, FP4, I8, FP8):
        q = orc.quantize(w, fmt, PC, mi.clip_ratios(5))
        assert np.all(q.scale == 1.0) and np.all(q.clip_idx == 0) and np.all(q.unit_err == 0.0)
        assert np.all(q.codes == 0)


@pytest.mark.parametrize("fmt", [I4, FP4, I8, FP8])
def test_absmax_scale_closed_form(fmt):
    """Ratio 1: scale = absmax/qmax, the largest element lands on +-qmax and
    nothing is clipped; INT error of every element is at most half a step."""
    rng = np.random.default_rng(20)
    w = (rng.standard_normal((16, 256)) * 0.02).astype(np.float32)
    q = orc.quantize(w, fmt, PC, ONE)
    a = np.max(np.abs(w), axis=1)
    assert np.array_equal(q.scale, (a / np.float32(QMAX[fmt])).astype(np.float32))
    g = orc.decode_array(fmt, q.codes)
    for r in range(16):
        j = int(np.argmax(np.abs(w[r])))
        assert abs(g[r, j]) == QMAX[fmt]
        assert np.max(np.abs(g[r])) == QMAX[fmt]
    if fmt in (I4, I8):
        err = np.abs(w.astype(np.float64) - g * q.scale.astype(np.float64)[:, None])
        assert np.all(err <= 0.5 * q.scale.astype(np.float64)[:, None] * (1 + 1e-6))


@pytest.mark.parametrize("fmt", [I4, FP4, I8, FP8])
@pytest.mark.parametrize("gran,group", [(PC, 0), (PG, 32), (PT, 0)])
def test_on_grid_identity_zero_error(fmt, gran, group):
    """x = g * 2^e built from random codes with one top code per unit: codes
    come back unchanged, scale is exactly 2^e, error is exactly zero."""
    rng = np.random.default_rng(30 + fmt)
    rows, cols = 6, 64
    nbits = orc.bits(fmt)
    allowed = [c for c in range(1 << nbits)
               if np.isfinite(orc.decode(fmt, c)) and abs(orc.decode(fmt, c)) <= QMAX[fmt]
               and not (fmt in (I4, I8) and orc.decode(fmt, c) < -QMAX[fmt])]
    allowed = [c for c in allowed if orc.decode(fmt, c) >= -QMAX[fmt]]
    codes = rng.choice(allowed, size=(rows, cols)).astype(np.uint8)
    top = [c for c in allowed if orc.decode(fmt, c) == QMAX[fmt]][0]
    nu = orc.num_units(rows, cols, gran, group)
    e = rng.integers(-12, 3, size=nu)
    exps = np.zeros((rows, cols))
    if gran == PC:
        codes[:, 3] = top
        exps[:] = e[:, None]
    elif gran == PG:
        codes[:, 5::group] = top
        exps[:] = np.repeat(e.reshape(rows, cols // group), group, axis=1)
    else:
        codes[2, 7] = top
        exps[:] = e[0]
    w = (orc.decode_array(fmt, codes) * 2.0 ** exps).astype(np.float32)
    q = orc.quantize(w, fmt, gran, ONE, group=group)
    assert np.array_equal(q.codes, codes)
    assert np.array_equal(q.scale, (2.0 ** e).astype(np.float32))
    assert np.all(q.unit_err == 0.0) and q.err == 0.0


@pytest.mark.parametrize("fmt", [I4, FP4, I8, FP8])
@pytest.mark.parametrize("p", [-7, 5])
def test_power_of_two_equivariance(fmt, p):
    """W -> 2^p W: same codes and winners, scales times 2^p, errors times 4^p,
    all bit for bit (every fp32 step commutes with a power of two)."""
    w = mi.to_f32_numpy(mi.llama_like_weight(8, 512, seed=5, outlier_frac=5e-3))
    clip = mi.clip_ratios(20)
    # fp16 scales only where none of them is an fp16 subnormal on either side
    # (4-bit formats, scaling up): rounding into subnormals does not commute.
    for gran, group, f16 in ((PC, 0, False), (PG, 128, p > 0 and fmt in (I4, FP4)), (PT, 0, False)):
        a = orc.quantize(w, fmt, gran, clip, group, f16, want_table=True)
        b = orc.quantize((w * np.float32(2.0 ** p)), fmt, gran, clip, group, f16, want_table=True)
        assert np.array_equal(a.codes, b.codes)
        assert np.array_equal(a.clip_idx, b.clip_idx)
        assert np.array_equal(a.scale * np.float32(2.0 ** p), b.scale)
        assert np.array_equal(a.table * 4.0 ** p, b.table)
        assert a.err * 4.0 ** p == b.err


def test_permutation_within_unit():
    rng = np.random.default_rng(40)
    w = mi.to_f32_numpy(mi.llama_like_weight(4, 256, seed=6, outlier_frac=1e-2))
    clip = mi.clip_ratios(16)
    perm = rng.permutation(256)
    for fmt in (I4, FP4):
        a = orc.quantize(w, fmt, PC, clip)
        b = orc.quantize(w[:, perm], fmt, PC, clip)
        assert np.array_equal(a.clip_idx, b.clip_idx) and np.array_equal(a.scale, b.scale)
        assert np.array_equal(a.codes[:, perm], b.codes)
        assert np.allclose(a.unit_err, b.unit_err, rtol=1e-13, atol=0)


def test_group_and_tensor_units_reduce_to_channels():
    """Per-group on [R, C] equals per-channel on [R*C/g, g]; per-tensor equals
    per-channel on the flattened row (pins the unit slicing)."""
    w = mi.to_f32_numpy(mi.llama_like_weight(6, 384, seed=7, outlier_frac=5e-3))
    clip = mi.clip_ratios(12)
    for fmt in (I4, FP4):
        g = orc.quantize(w, fmt, PG, clip, group=128, scale_f16=True)
        c = orc.quantize(w.reshape(-1, 128), fmt, PC, clip, scale_f16=True)
        assert np.array_equal(g.scale, c.scale) and np.array_equal(g.clip_idx, c.clip_idx)
        assert np.array_equal(g.codes.reshape(-1, 128), c.codes)
        assert np.array_equal(g.unit_err, c.unit_err)
        t = orc.quantize(w, fmt, PT, clip)
        f = orc.quantize(w.reshape(1, -1), fmt, PC, clip)
        assert np.array_equal(t.scale, f.scale) and np.array_equal(t.codes.reshape(1, -1), f.codes)
        assert t.err == f.err


def test_partial_unit_range_matches_full():
    w = mi.to_f32_numpy(mi.llama_like_weight(16, 256, seed=8))
    clip = mi.clip_ratios(10)
    full = orc.sweep(w, FP4, PC, clip)
    part = orc.sweep(w, FP4, PC, clip, unit_first=5, unit_count=4)
    assert np.array_equal(full.scale[5:9], part.scale[5:9])
    assert np.array_equal(full.err[5:9], part.err[5:9])
    assert np.all(part.err[:5] == 0) and np.all(part.err[9:] == 0)


def test_clip_search_finds_clipping_with_outliers():
    """A lone huge outlier makes a ratio below 1 strictly better, and the
    winner's error is the minimum of the table (first on ties)."""
    rng = np.random.default_rng(41)
    w = (rng.standard_normal((4, 1024)) * 0.02).astype(np.float32)
    w[:, 17] = 0.5
    s = orc.sweep(w, I4, PC, mi.clip_ratios(100), want_table=True)
    assert np.all(s.clip_idx > 0)
    assert np.array_equal(s.clip_idx, np.argmin(s.table, axis=1))
    assert np.array_equal(s.err, s.table.min(axis=1))


def test_pack4_layout():
    codes = np.arange(16, dtype=np.uint8)
    p = orc.pack4(codes)
    assert list(p) == [(2 * j) | ((2 * j + 1) << 4) for j in range(8)]


# ---- Algorithm 1 ------------------------------------------------------------------

def test_select_rule_strict_less_first_wins():
    assert orc.select([1.0, 1.0]) == 0
    assert orc.select([2.0, 1.0]) == 1
    assert orc.select([1.0, 2.0]) == 0
    assert orc.select([0.0, 0.0, 0.0]) == 0
    assert orc.select([3.0, 2.0, 2.0, 1.0]) == 3
    assert orc.select([float("inf"), float("inf")]) == -1     # nothing beats the initial infinity


def test_select_int_grid_tensor_picks_int():
    rng = np.random.default_rng(50)
    q = rng.integers(-7, 8, size=(8, 64))
    q[:, 0] = 7
    q[:, 1] = 5                                              # 5 is not on the E2M1 grid
    w = (q * 2.0 ** -6).astype(np.float32)
    for cands in ([I4, FP4], [FP4, I4]):
        s = orc.select_layer_w_only(w, cands, PC, ONE)
        assert cands[s.best] == I4 and s.errs[cands.index(I4)] == 0.0 and s.errs[cands.index(FP4)] > 0


def test_select_e2m1_grid_tensor_picks_fp():
    rng = np.random.default_rng(51)
    vals = np.array([0, 0.5, 1, 1.5, 2, 3, 4, 6, -0.5, -1, -1.5, -2, -3, -4, -6])
    w = rng.choice(vals, size=(8, 64))
    w[:, 0] = 6
    w[:, 1] = 1.5
    w = (w * 2.0 ** -5).astype(np.float32)
    s = orc.select_layer_w_only(w, [I4, FP4], PC, ONE)
    assert s.best == 1 and s.errs[1] == 0.0 and s.errs[0] > 0
    assert np.array_equal(orc.decode_array(FP4, s.w.codes) * 2.0 ** -5, w)


def test_select_tie_goes_to_first_candidate():
    """Values in {0, +-a} lie on both grids; with a = 42*2^e both a/7 and a/6
    are exact, so both errors are exactly zero and the first listed candidate
    is kept whichever it is."""
    rng = np.random.default_rng(52)
    a = 42 * 2.0 ** -8
    w = (rng.integers(-1, 2, size=(4, 32)) * a).astype(np.float32)
    w[:, 0] = a
    for cands in ([I4, FP4], [FP4, I4]):
        s = orc.select_layer_w_only(w, cands, PC, ONE)
        assert s.errs == [0.0, 0.0] and s.best == 0 and s.w.fmt == cands[0]


def test_select_returns_requantized_winner_and_energy():
    w = mi.to_f32_numpy(mi.llama_like_weight(32, 256, seed=9))
    clip = mi.clip_ratios(10)
    s = orc.select_layer_w_only(w, [I4, FP4], PC, clip)
    alone = orc.quantize(w, [I4, FP4][s.best], PC, clip)
    assert np.array_equal(s.w.codes, alone.codes) and np.array_equal(s.w.scale, alone.scale)
    assert s.errs[s.best] == min(s.errs)
    assert abs(s.ref_energy - float(np.sum(w.astype(np.float64) ** 2))) < 1e-12 * s.ref_energy


# ---- the paper's qualitative findings, as loose sanity ranges -------------------------

def test_paper_trends_hold_on_synthetic_tensors():
    """Section 3.2 / 4.2 in kind: the redesigned E2M1 has clearly lower error
    than the IEEE-aligned one; at 8 bits INT beats FP on Gaussian weights; on
    activations with outlier channels FP8 beats INT8 by a wide margin."""
    w = mi.to_f32_numpy(mi.llama_like_weight(64, 1024, seed=11))
    e_ours = orc.quantize(w, FP4, PC, ONE).err
    e_ieee = orc.quantize(w, FP4I, PC, ONE).err
    assert 0.3 < e_ours / e_ieee < 0.95
    assert orc.quantize(w, I8, PC, ONE).err < orc.quantize(w, FP8, PC, ONE).err
    x = mi.to_f32_numpy(mi.activations(64, 1024, seed=12))
    assert orc.quantize(x, FP8, PT, ONE).err < 0.2 * orc.quantize(x, I8, PT, ONE).err
