"""GPU parity of the per-unit (channel / group) format select against the CPU oracle,
through the C ABI: unit formats, codes, scales, clip indices bit for bit (near-ties under
the rule in gpu_util), error sums to ERR_RTOL."""
import numpy as np
import pytest
import torch

import mofq_inputs as mi
from oracle import mofq_oracle as orc
from tests.gpu_util import ERR_RTOL, TIE_TAU, scales_to_f32, unpack_codes

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
I4, FP4, I8, FP8 = orc.INT4, orc.FP4_E2M1, orc.INT8, orc.FP8_E4M3


@pytest.fixture(scope="module")
def mq():
    from paper_2305_12356_amd import binding
    assert torch.cuda.is_available()
    return binding


def run(mq, w, cands, gran, clip, group=0, f16=False):
    cfg = mq.Cfg(gran, clip, group, f16)
    rows, cols = w.shape
    units = mq.num_units(rows, cols, gran, group)
    out = mq.alloc_qbuffers(rows, cols, orc.bits(cands[0]), cfg, DEV)
    tags = torch.full((units,), 255, dtype=torch.uint8, device=DEV)
    res = mq.alloc_result(DEV)
    mixed = torch.zeros(1, dtype=torch.float64, device=DEV)
    n = mq.select_units_workspace_bytes(w, len(cands), cfg)
    assert n > 0
    ws = torch.empty(n, dtype=torch.uint8, device=DEV)
    mq.select_units(w, cands, cfg, out, tags, res, mixed, ws)
    torch.cuda.synchronize()
    return mq.read_result(res), out, tags.cpu().numpy(), float(mixed.item())


def check(mq, w, cands, gran, clip, group=0, f16=False, label=""):
    print(f"[case] {label} shape={tuple(w.shape)} dtype={w.dtype} gran={gran} group={group} K={len(clip)} cands={cands}", flush=True)
    w32 = mi.to_f32_numpy(w)
    clip = np.asarray(clip, dtype=np.float32)
    ref = orc.select_units(w32, cands, gran, clip, group, f16)
    r, out, tags, mixed = run(mq, w, cands, gran, clip, group, f16)
    rows, cols = w.shape
    codes = unpack_codes(out.codes, rows, cols, orc.bits(cands[0]))
    scale = scales_to_f32(out.scales)
    idx = out.clip_idx.cpu().numpy()
    uerr = out.unit_err.cpu().numpy()
    # layer-wise view
    assert np.allclose(list(r.err)[:len(cands)], ref.errs, rtol=ERR_RTOL, atol=1e-300)
    assert r.best == orc.select(ref.errs)
    assert np.isclose(mixed, ref.err, rtol=ERR_RTOL, atol=1e-300)
    assert mixed <= min(list(r.err)[:len(cands)]) * (1 + 1e-12)
    assert np.allclose(uerr, ref.unit_err, rtol=ERR_RTOL, atol=1e-300)
    # per unit: same format unless the two best errors are a near-tie; then the unit's
    # outputs must be those of the format the library chose
    upr = 1 if gran == orc.PER_CHANNEL else cols // group
    width = cols // upr
    band = 0
    for u in np.nonzero(tags != ref.unit_format)[0]:
        ea = sorted(q.unit_err[u] for q in ref.per_candidate)
        assert ea[1] - ea[0] <= TIE_TAU * max(ea[1], 1e-300), (u, ea)
        band += 1
    for u in range(tags.size):
        q = ref.per_candidate[tags[u]]
        rr, gg = divmod(u, upr)
        sl = slice(gg * width, (gg + 1) * width)
        if q.clip_idx[u] == idx[u]:
            assert scale[u] == q.scale[u]
            assert np.array_equal(codes[rr, sl], q.codes[rr, sl]), u
        else:   # near-tie inside the clip search of that format: covered by the weight-only tests
            assert abs(uerr[u] - q.unit_err[u]) <= TIE_TAU * max(q.unit_err[u], 1e-300)
    return band


@pytest.mark.parametrize("gran,group,f16", [(orc.PER_CHANNEL, 0, False), (orc.PER_GROUP, 128, True), (orc.PER_GROUP, 32, False)])
def test_four_bit_units(mq, gran, group, f16):
    w = mi.llama_like_weight(37, 2048, seed=110, device=DEV, outlier_frac=2e-3)
    check(mq, w, [I4, FP4], gran, mi.clip_ratios(20), group, f16, "units-4bit")
    check(mq, w, [FP4, I4], gran, mi.clip_ratios(1), group, f16, "units-order")


def test_mixed_rows_pick_different_formats(mq):
    """Half of the rows lie on the INT4 grid (INT4 exact), the others are Gaussian with
    outliers (FP4 better): both tags must occur."""
    g = torch.Generator().manual_seed(5)
    w = (torch.randn(16, 1024, generator=g) * 0.02)
    w[::2] = torch.randint(-7, 8, (8, 1024), generator=g).float() * 2.0 ** -6
    w[::2, 0] = 7 * 2.0 ** -6
    w = w.to(torch.float16).to(DEV)
    check(mq, w, [I4, FP4], orc.PER_CHANNEL, mi.clip_ratios(1), label="mixed")
    cfg_tags = run(mq, w, [I4, FP4], orc.PER_CHANNEL, mi.clip_ratios(1))[2]
    assert set(cfg_tags[::2]) == {0} and set(cfg_tags[1::2]) == {1}


def test_eight_bit_and_three_candidates(mq):
    x = mi.activations(64, 1024, seed=111, device=DEV)
    check(mq, x, [I8, FP8], orc.PER_CHANNEL, mi.clip_ratios(1), label="units-8bit")
    w = mi.llama_like_weight(20, 1024, seed=112, dtype=torch.bfloat16, device=DEV)
    check(mq, w, [orc.FP4_E2M1_IEEE, I4, FP4], orc.PER_GROUP, mi.clip_ratios(6), 128, True, "units-3cand")


def test_llama_shaped_tensor(mq):
    w = mi.llama_like_weight(4096, 4096, seed=113, device=DEV)
    w32 = mi.to_f32_numpy(w[:64])
    clip = mi.clip_ratios(100)
    r, out, tags, mixed = run(mq, w, [I4, FP4], orc.PER_CHANNEL, clip)
    ref = orc.select_units(w32, [I4, FP4], orc.PER_CHANNEL, clip)
    assert np.array_equal(tags[:64], ref.unit_format)
    assert np.allclose(out.unit_err[:64].cpu().numpy(), ref.unit_err, rtol=ERR_RTOL)
    assert mixed <= min(r.err[0], r.err[1])


def test_rejects_per_tensor(mq):
    w = mi.llama_like_weight(8, 256, seed=114, device=DEV)
    cfg = mq.Cfg(mq.PER_TENSOR, mi.clip_ratios(1))
    assert mq.select_units_workspace_bytes(w, 2, cfg) == 0
