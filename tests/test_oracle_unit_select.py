"""Pins of the oracle's per-unit (channel / group) format select: the finer granularity
the paper leaves as future work (Section 4.1, conclusion item 2)."""
import numpy as np
import pytest

import mofq_inputs as mi
from oracle import mofq_oracle as orc

I4, FP4, I8, FP8 = orc.INT4, orc.FP4_E2M1, orc.INT8, orc.FP8_E4M3
PC, PG = orc.PER_CHANNEL, orc.PER_GROUP


def _w(rows, cols, seed):
    return mi.to_f32_numpy(mi.llama_like_weight(rows, cols, seed=seed))


@pytest.mark.parametrize("gran,group", [(PC, 0), (PG, 64)])
def test_each_unit_takes_its_own_smallest_error(gran, group):
    w = _w(12, 256, 100)
    clip = mi.clip_ratios(5)
    s = orc.select_units(w, [I4, FP4], gran, clip, group)
    qa, qb = s.per_candidate
    for u in range(s.unit_format.size):
        want = 1 if qb.unit_err[u] < qa.unit_err[u] else 0      # strict: a tie keeps the first candidate
        assert s.unit_format[u] == want
        assert s.unit_err[u] == min(qa.unit_err[u], qb.unit_err[u])
        assert s.scale[u] == (qa, qb)[want].scale[u] and s.clip_idx[u] == (qa, qb)[want].clip_idx[u]
    # never worse than the layer-wise choice, and equal to the sum of the per-unit minima
    assert s.err <= min(s.errs) * (1 + 1e-15)
    assert np.isclose(s.err, float(np.sum(np.minimum(qa.unit_err, qb.unit_err))), rtol=1e-14)


def test_codes_come_from_the_chosen_format_unit_by_unit():
    w = _w(6, 256, 101)
    w[0] = (np.random.default_rng(0).integers(-7, 8, 256) * 2.0 ** -6).astype(np.float32)   # on the INT4 grid
    w[0, 0] = 7 * 2.0 ** -6
    s = orc.select_units(w, [FP4, I4], PG, np.ones(1, np.float32), 128)
    qa, qb = s.per_candidate
    for r in range(6):
        for g in range(2):
            u = r * 2 + g
            src = (qa, qb)[s.unit_format[u]]
            assert np.array_equal(s.codes[r, g * 128:(g + 1) * 128], src.codes[r, g * 128:(g + 1) * 128])
    assert s.unit_format[0] == 1 and s.unit_err[0] == 0.0          # the on-grid row goes to INT4, exactly
    # decoding each unit with its own table and scale reproduces the unit errors
    for u in (0, 3, 7):
        r, g = divmod(u, 2)
        f = [FP4, I4][s.unit_format[u]]
        xh = orc.decode_array(f, s.codes[r, g * 128:(g + 1) * 128]) * float(s.scale[u])
        d = w[r, g * 128:(g + 1) * 128].astype(np.float64) - xh
        assert np.isclose(float(np.sum(d * d)), s.unit_err[u], rtol=1e-12, atol=0.0)


def test_same_format_twice_and_ties_keep_the_first():
    w = _w(5, 128, 102)
    s = orc.select_units(w, [FP4, FP4], PC, mi.clip_ratios(3))
    assert not s.unit_format.any()
    z = np.zeros((3, 128), dtype=np.float32)
    t = orc.select_units(z, [I8, FP8], PC, np.ones(1, np.float32))
    assert not t.unit_format.any() and t.err == 0.0


def test_single_dominant_format_reduces_to_the_layer_select():
    """The redesigned FP4 beats the IEEE-aligned one on every channel of a Gaussian
    tensor, so the per-unit select equals the layer select."""
    w = _w(16, 256, 103)
    cands = [orc.FP4_E2M1_IEEE, FP4]
    s = orc.select_units(w, cands, PC, np.ones(1, np.float32))
    layer = orc.select_layer_w_only(w, cands, PC, np.ones(1, np.float32))
    assert s.unit_format.all() and layer.best == 1
    assert np.array_equal(s.codes, layer.w.codes) and s.err == layer.errs[1]
