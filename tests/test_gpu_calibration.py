"""GPU parity of the static calibration path (running absmax over batches, per-tensor
select of unseen batches with the calibrated scale) against the CPU oracle."""
import numpy as np
import pytest
import torch

import mofq_inputs as mi
from oracle import mofq_oracle as orc
from tests.gpu_util import ERR_RTOL, scales_to_f32, unpack_codes

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
I8, FP8, I4, FP4 = orc.INT8, orc.FP8_E4M3, orc.INT4, orc.FP4_E2M1


@pytest.fixture(scope="module")
def mq():
    from paper_2305_12356_amd import binding
    assert torch.cuda.is_available()
    return binding


def _ws(mq, x, n_cand):
    cfg = mq.Cfg(mq.PER_TENSOR, mi.clip_ratios(1))
    return torch.empty(mq.workspace_bytes(x, None, n_cand, mq.ERR_TENSOR, cfg), dtype=torch.uint8, device=DEV)


def calibrate(mq, batches):
    a = torch.zeros(1, dtype=torch.float32, device=DEV)
    ws = _ws(mq, batches[0], 1)
    for b in batches:
        mq.calibrate_absmax(b, a, ws)
    torch.cuda.synchronize()
    return a


def check_batch(mq, x, cands, a_dev):
    print(f"[case] calibrated select X={tuple(x.shape)} dtype={x.dtype} cands={cands}", flush=True)
    cfg = mq.Cfg(mq.PER_TENSOR, mi.clip_ratios(1))
    bits = orc.bits(cands[0])
    out = mq.alloc_qbuffers(x.shape[0], x.shape[1], bits, cfg, DEV)
    res = mq.alloc_result(DEV)
    mq.select_calibrated(x, cands, a_dev, out, res, _ws(mq, x, len(cands)))
    torch.cuda.synchronize()
    r = mq.read_result(res)
    x32 = mi.to_f32_numpy(x)
    ref = orc.select_calibrated(x32, cands, np.float32(a_dev.item()))
    assert np.allclose(list(r.err)[:len(cands)], ref.errs, rtol=ERR_RTOL, atol=1e-300)
    assert r.best == ref.best
    assert np.isclose(r.ref_energy, ref.ref_energy, rtol=1e-12)
    assert np.array_equal(unpack_codes(out.codes, *x.shape, bits), ref.w.codes)
    assert scales_to_f32(out.scales)[0] == ref.w.scale[0]
    return r


def test_running_absmax_and_unseen_batches(mq):
    cal = mi.activation_batches(8, 256, 1024, seed=7, device=DEV)
    a = calibrate(mq, cal)
    assert a.item() == float(orc.calibrate_absmax([mi.to_f32_numpy(b) for b in cal]))
    fp_wins = 0
    for x in mi.activation_batches(4, 256, 1024, seed=8, device=DEV):
        fp_wins += check_batch(mq, x, [I8, FP8], a).best == 1
    assert fp_wins == 4          # oversized scale: FP8 has the lower error (Section 3.2)


def test_saturation_beyond_the_calibrated_range_and_other_formats(mq):
    cal = mi.activation_batches(2, 64, 512, seed=9, device=DEV, spread=0.0)
    a = calibrate(mq, cal)
    big = mi.activation_batches(1, 64, 512, seed=10, device=DEV)[0] * 3.0     # exceeds the calibrated range
    assert big.abs().max().item() > a.item()
    check_batch(mq, big, [I8, FP8], a)
    check_batch(mq, big, [FP8, I8], a)
    check_batch(mq, big.to(torch.float32), [I4, FP4], a)
    check_batch(mq, big.to(torch.float16), [orc.FP8_E5M2], a)


def test_zero_calibration_and_ragged_sizes(mq):
    x = mi.activations(3, 40, seed=11, device=DEV)
    a = torch.zeros(1, dtype=torch.float32, device=DEV)                        # never calibrated: scale 1
    check_batch(mq, x, [I8, FP8], a)
    b = calibrate(mq, [x])
    assert b.item() == x.abs().max().item()
    check_batch(mq, x, [I8, FP8], b)
