"""Pins of the oracle's weight-only layer-output error (Section 3.2, layer analysis:
A_out = W * A_in with quantized W and the 16-bit input; Section 4.1 names it as one of
the two metrics that suffice for the weight-only select)."""
from fractions import Fraction

import numpy as np
import pytest

import mofq_inputs as mi
from oracle import mofq_oracle as orc

I4, FP4 = orc.INT4, orc.FP4_E2M1
PT, PC = orc.PER_TENSOR, orc.PER_CHANNEL
ONE = np.ones(1, dtype=np.float32)


def _bf16(a):
    import torch
    return torch.from_numpy(np.asarray(a, dtype=np.float32)).to(torch.bfloat16).to(torch.float32).numpy()


def test_identity_input_reduces_to_the_tensor_error():
    """X = I: the layer output is W^T itself, so the output error is the tensor error of
    the same quantization and the reference energy is sum W^2 (ties this function to the
    tensor-error search, which has its own pins)."""
    rng = np.random.default_rng(70)
    w = _bf16(rng.normal(0, 0.03, size=(24, 32)))
    x = np.eye(32, dtype=np.float32)
    clip = mi.clip_ratios(9)
    for f in (I4, FP4):
        q = orc.quantize(w, f, PC, clip)
        e, p = orc.layer_output_error_w_only(x, w, q, PC)
        assert np.isclose(e, q.err, rtol=1e-13, atol=0.0)
        assert np.isclose(p, float(np.sum(w.astype(np.float64) ** 2)), rtol=1e-13)


def test_on_grid_weights_give_zero_output_error():
    rng = np.random.default_rng(71)
    x = _bf16(rng.normal(0, 1, size=(10, 16)))
    w = (rng.integers(-7, 8, size=(6, 16)) * 2.0 ** -5).astype(np.float32)
    w[:, 0] = 7 * 2.0 ** -5                       # per-channel absmax scale = 2^-5 exactly
    s = orc.select_layer_w_only_output(x, w, [I4], PC)
    assert s.errs == [0.0] and s.best == 0 and s.ref_energy > 0
    g = np.array([0, 0.5, 1, 1.5, 2, 3, 4, 6])
    w2 = (rng.choice(g, size=(6, 16)) * rng.choice([-1.0, 1.0], size=(6, 16)) * 2.0 ** -4).astype(np.float32)
    w2[:, 0] = 6 * 2.0 ** -4
    s2 = orc.select_layer_w_only_output(x, w2, [FP4], PC)
    assert s2.errs == [0.0]


@pytest.mark.parametrize("w_gran", [PT, PC])
def test_brute_force_in_rationals(w_gran):
    """Tiny case in exact rationals from the oracle's own codes and scales: checks the
    orientation of the product, the per-channel scale factor and the squared sum."""
    rng = np.random.default_rng(72)
    x = _bf16(rng.normal(0, 1, size=(3, 8)))
    w = _bf16(rng.normal(0, 0.05, size=(4, 8)))
    for f in (I4, FP4):
        q = orc.quantize(w, f, w_gran, ONE)
        e, p = orc.layer_output_error_w_only(x, w, q, w_gran)
        gw = orc.decode_array(f, q.codes)
        E = Fraction(0)
        P = Fraction(0)
        for t in range(3):
            for o in range(4):
                s = Fraction(float(q.scale[o if w_gran == PC else 0]))
                y = sum(Fraction(float(x[t, i])) * Fraction(float(w[o, i])) for i in range(8))
                yq = s * sum(Fraction(float(x[t, i])) * Fraction(float(gw[o, i])) for i in range(8))
                E += (y - yq) ** 2
                P += y * y
        assert np.isclose(e, float(E), rtol=1e-12) and np.isclose(p, float(P), rtol=1e-12)


def test_select_uses_the_output_error_and_keeps_first_on_ties():
    rng = np.random.default_rng(73)
    x = _bf16(rng.normal(0, 1, size=(16, 64)))
    w = _bf16(rng.normal(0, 0.02, size=(8, 64)))
    s = orc.select_layer_w_only_output(x, w, [I4, FP4], PC, mi.clip_ratios(5))
    assert s.best == int(np.argmin(s.errs)) and len(s.errs) == 2
    assert s.w.fmt == [I4, FP4][s.best]
    # both candidates the same format: equal errors, the first one is kept
    t = orc.select_layer_w_only_output(x, w, [FP4, FP4], PC, mi.clip_ratios(5))
    assert t.errs[0] == t.errs[1] and t.best == 0


def test_output_metric_can_disagree_with_tensor_metric_only_through_the_input():
    """Scaling every input column by the same factor c scales both errors by c^2 and
    leaves the choice unchanged (the metric is homogeneous in X)."""
    rng = np.random.default_rng(74)
    x = _bf16(rng.normal(0, 1, size=(12, 32)))
    w = _bf16(rng.normal(0, 0.02, size=(8, 32)))
    a = orc.select_layer_w_only_output(x, w, [I4, FP4], PC)
    b = orc.select_layer_w_only_output(x * 4.0, w, [I4, FP4], PC)
    assert a.best == b.best
    assert np.allclose(np.array(b.errs), 16.0 * np.array(a.errs), rtol=1e-12)
