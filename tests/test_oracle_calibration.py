"""Pins of the oracle's static calibration of dynamic tensors (Section 3.2, dynamic
tensor analysis: the scale is the largest value over the calibration batches)."""
import numpy as np
import pytest

import mofq_inputs as mi
from oracle import mofq_oracle as orc

I8, FP8 = orc.INT8, orc.FP8_E4M3
ONE = np.ones(1, dtype=np.float32)


def _batches(n, seed):
    return [mi.to_f32_numpy(b) for b in mi.activation_batches(n, 32, 256, seed=seed)]


def test_calibrating_on_the_batch_itself_is_the_per_tensor_quantization():
    (x,) = _batches(1, 1)
    a = orc.calibrate_absmax([x])
    assert a == np.max(np.abs(x))
    for f in (I8, FP8):
        q = orc.quantize_calibrated(x, f, a)
        ref = orc.quantize(x, f, orc.PER_TENSOR, ONE)
        assert np.array_equal(q.codes, ref.codes) and q.scale[0] == ref.scale[0]
        assert np.isclose(q.err, ref.err, rtol=1e-13)


def test_running_maximum_over_batches():
    bs = _batches(5, 2)
    a = orc.calibrate_absmax(bs)
    assert a == max(float(np.max(np.abs(b))) for b in bs)
    assert orc.calibrate_absmax(bs[:2]) <= a
    assert orc.calibrate_absmax([np.zeros((2, 8), np.float32)]) == 0.0


def test_values_beyond_the_calibrated_range_saturate():
    x = np.array([[0.0, 1.0, -1.0, 2.5, -3.0, 100.0, -100.0, 0.26]], dtype=np.float32)
    q = orc.quantize_calibrated(x, I8, np.float32(1.27))          # scale 0.01 exactly? 1.27/127 in fp32
    s = float(q.scale[0])
    g = orc.decode_array(I8, q.codes)[0]
    assert list(g[:3]) == [0.0, round(1.0 / s), -round(1.0 / s)]
    assert g[5] == 127 and g[6] == -128 and g[3] == 127            # beyond the range: clamp
    d = x[0].astype(np.float64) - g * s
    assert np.isclose(q.err, float(np.sum(d * d)), rtol=1e-14)
    qf = orc.quantize_calibrated(x, FP8, np.float32(448.0 * 2.0 ** -8))   # scale 2^-8
    gf = orc.decode_array(FP8, qf.codes)[0]
    assert qf.scale[0] == 2.0 ** -8 and gf[5] == 448.0 and gf[6] == -448.0
    assert gf[1] == 256.0 and gf[3] == 448.0                       # 2.5 / 2^-8 = 640 > 448: saturates


def test_zero_calibration_gives_unit_scale():
    x = np.array([[0.5, -2.0, 0.0, 3.0, 0, 0, 0, 0]], dtype=np.float32)
    q = orc.quantize_calibrated(x, I8, np.float32(0.0))
    assert q.scale[0] == 1.0 and list(orc.decode_array(I8, q.codes)[0][:4]) == [0.0, -2.0, 0.0, 3.0]


def test_oversized_scales_favour_fp8_as_the_paper_reports():
    """With the scale taken from the largest of many batches, most batches are quantized
    with a larger-than-suitable scale; FP8 then has the lower error (Section 3.2)."""
    cal = _batches(16, 3)
    a = orc.calibrate_absmax(cal)
    unseen = _batches(6, 4)
    wins = 0
    for x in unseen:
        s = orc.select_calibrated(x, [I8, FP8], a)
        wins += s.best == 1
        assert s.errs[1] < s.errs[0]
    assert wins == len(unseen)
    # select rule: strict, first wins ties
    t = orc.select_calibrated(unseen[0], [FP8, FP8], a)
    assert t.best == 0 and t.errs[0] == t.errs[1]
