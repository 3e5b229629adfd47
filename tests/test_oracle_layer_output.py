"""Pins of the oracle's layer-output error (A_out = W * A_in with both inputs
quantized, Section 3.2 layer analysis) and of the weight-activation select."""
from fractions import Fraction

import numpy as np
import pytest
import torch

import mofq_inputs as mi
from oracle import mofq_oracle as orc

I8, FP8 = orc.INT8, orc.FP8_E4M3
PT, PC = orc.PER_TENSOR, orc.PER_CHANNEL
ONE = np.ones(1, dtype=np.float32)


def _on_grid(fmt, shape, rng, e):
    """Random tensor of grid values times 2^e that contains the top value, so a
    per-tensor absmax scale is exactly 2^e."""
    top = 127 if fmt == I8 else 448.0
    if fmt == I8:
        g = rng.integers(-127, 128, size=shape).astype(np.float64)
    else:
        codes = rng.integers(0, 127, size=shape)
        g = orc.decode_array(fmt, codes) * rng.choice([-1.0, 1.0], size=shape)
    g.flat[0] = top
    return (g * 2.0 ** e).astype(np.float32)


@pytest.mark.parametrize("fmt", [I8, FP8])
def test_on_grid_inputs_give_zero_output_error(fmt):
    rng = np.random.default_rng(60)
    x = _on_grid(fmt, (12, 40), rng, -3)
    w = _on_grid(fmt, (9, 40), rng, -9)
    s = orc.select_layer_wa(x, w, [fmt])
    assert s.errs == [0.0]
    assert s.x.scale[0] == 2.0 ** -3 and s.w.scale[0] == 2.0 ** -9
    assert s.ref_energy > 0


def test_small_integer_product_is_exact_and_oriented():
    """Small-integer X [tokens, in] and W [out, in]: Y[t,o] = sum_i X[t,i] W[o,i]
    exactly; compared with Python integers (pins the transposition and shapes)."""
    rng = np.random.default_rng(61)
    x = rng.integers(-5, 6, size=(7, 13)).astype(np.float32)
    w = rng.integers(-5, 6, size=(4, 13)).astype(np.float32)
    x[0, 0] = 127                                # INT8 per-tensor scale = 1 exactly
    w[0, 0] = 127
    qx = orc.quantize(x, I8, PT, ONE)
    qw = orc.quantize(w, I8, PT, ONE)
    e, p = orc.layer_output_error(x, w, qx, qw)
    y = [[sum(int(x[t, i]) * int(w[o, i]) for i in range(13)) for o in range(4)] for t in range(7)]
    assert e == 0.0 and p == float(sum(v * v for row in y for v in row))


@pytest.mark.parametrize("fmt", [I8, FP8])
@pytest.mark.parametrize("w_gran", [PT, PC])
def test_layer_output_error_brute_force(fmt, w_gran):
    """Tiny case in exact rationals from the oracle's own codes and scales:
    checks the product, the scale factors and the squared-difference sum."""
    x = mi.to_f32_numpy(mi.activations(5, 24, seed=70, n_outlier=2))
    w = mi.to_f32_numpy(mi.llama_like_weight(6, 24, seed=71, dtype=torch.bfloat16))
    qx = orc.quantize(x, fmt, PT, ONE)
    qw = orc.quantize(w, fmt, w_gran, ONE)
    e, p = orc.layer_output_error(x, w, qx, qw, w_gran)
    F = lambda v: Fraction(float(v))
    ee, pp = Fraction(0), Fraction(0)
    for t in range(5):
        for o in range(6):
            y = sum(F(x[t, i]) * F(w[o, i]) for i in range(24))
            acc = sum(F(orc.decode(fmt, qx.codes[t, i])) * F(orc.decode(fmt, qw.codes[o, i]))
                      for i in range(24))
            sw = qw.scale[0] if w_gran == PT else qw.scale[o]
            d = y - F(qx.scale[0]) * F(sw) * acc
            ee += d * d
            pp += y * y
    assert abs(e - float(ee)) <= 1e-12 * float(ee)
    assert abs(p - float(pp)) <= 1e-12 * float(pp)


def test_wa_select_prefers_fp8_with_outlier_channels_and_int8_without():
    """Section 3.2 in kind: per-tensor INT8 collapses on activations with
    outlier channels, so the layer picks FP8; with tame activations and Gaussian
    weights INT8 wins.  The noise-to-signal ratio orders candidates like the
    error sum."""
    w = mi.to_f32_numpy(mi.llama_like_weight(48, 256, seed=72, dtype=torch.bfloat16))
    x_out = mi.to_f32_numpy(mi.activations(32, 256, seed=73))
    s = orc.select_layer_wa(x_out, w, [I8, FP8])
    assert s.best == 1 and s.errs[1] < 0.75 * s.errs[0]
    x_tame = mi.to_f32_numpy(mi.activations(32, 256, seed=74, n_outlier=0))
    s2 = orc.select_layer_wa(x_tame, w, [I8, FP8])
    assert s2.best == 0
    for sel in (s, s2):
        nsr = [e / sel.ref_energy for e in sel.errs]
        assert int(np.argmin(nsr)) == sel.best and all(e >= 0 for e in sel.errs)


def test_wa_select_shares_one_format_per_layer():
    w = mi.to_f32_numpy(mi.llama_like_weight(16, 64, seed=75, dtype=torch.bfloat16))
    x = mi.to_f32_numpy(mi.activations(8, 64, seed=76))
    s = orc.select_layer_wa(x, w, [I8, FP8])
    assert s.w.fmt == s.x.fmt == [I8, FP8][s.best]
