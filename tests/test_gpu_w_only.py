"""GPU parity of the weight-only path (scale search, select, emit) against the CPU
oracle, through the C ABI.  Codes, scales, clip indices and format choices are
compared bit for bit (near-ties of the clip search under the rule in gpu_util);
error sums to ERR_RTOL."""
import numpy as np
import pytest
import torch

import mofq_inputs as mi
from oracle import mofq_oracle as orc
from tests.gpu_util import ERR_RTOL, compare_quantized, scales_to_f32, unpack_codes

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


@pytest.fixture(scope="module")
def mq():
    from paper_2305_12356_amd import binding
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return binding


def _ws(mq, w, n_cand, cfg):
    n = mq.workspace_bytes(w, None, n_cand, mq.ERR_TENSOR, cfg)
    assert n > 0
    return torch.empty(n, dtype=torch.uint8, device=DEV)


def run_quantize(mq, w, fmt, cfg):
    rows, cols = w.shape
    out = mq.alloc_qbuffers(rows, cols, orc.bits(fmt), cfg, DEV)
    terr = torch.zeros(1, dtype=torch.float64, device=DEV)
    mq.quantize(w, fmt, cfg, out, terr, _ws(mq, w, 1, cfg))
    torch.cuda.synchronize()
    return (unpack_codes(out.codes, rows, cols, orc.bits(fmt)), scales_to_f32(out.scales),
            out.clip_idx.cpu().numpy(), out.unit_err.cpu().numpy(), float(terr.item()))


def run_select(mq, w, cands, cfg):
    rows, cols = w.shape
    out = mq.alloc_qbuffers(rows, cols, orc.bits(cands[0]), cfg, DEV)
    res = mq.alloc_result(DEV)
    mq.select_layer(w, None, cands, mq.ERR_TENSOR, cfg, out, None, res, _ws(mq, w, len(cands), cfg))
    torch.cuda.synchronize()
    r = mq.read_result(res)
    return (r, unpack_codes(out.codes, rows, cols, orc.bits(cands[0])), scales_to_f32(out.scales),
            out.clip_idx.cpu().numpy(), out.unit_err.cpu().numpy())


def check_tensor(mq, w_dev, cands, gran, clip, group=0, f16=False, label=""):
    """Every candidate through mofq_quantize, then mofq_select_layer, against the oracle."""
    print(f"[case] {label} shape={tuple(w_dev.shape)} dtype={w_dev.dtype} gran={gran} group={group} "
          f"K={len(clip)} f16={f16} cands={cands}", flush=True)
    w32 = mi.to_f32_numpy(w_dev)
    cfg = mq.Cfg(gran, clip, group, f16)
    clip = np.asarray(clip, dtype=np.float32)
    refs, band = [], 0
    for f in cands:
        ref = orc.quantize(w32, f, gran, clip, group, f16, want_table=True)
        codes, scale, idx, uerr, terr = run_quantize(mq, w_dev, f, cfg)
        band += compare_quantized(w32, f, gran, group, f16, clip, ref, codes, scale, idx, uerr)
        assert np.isclose(terr, ref.err, rtol=ERR_RTOL, atol=1e-300)
        refs.append(ref)
    r, codes, scale, idx, uerr = run_select(mq, w_dev, cands, cfg)
    errs = [q.err for q in refs]
    best = orc.select(errs)
    assert r.n == len(cands)
    assert np.allclose(list(r.err)[:len(cands)], errs, rtol=ERR_RTOL, atol=1e-300)
    assert r.best == best, (r.best, best, errs)
    energy = float(np.sum(w32.astype(np.float64) ** 2))
    assert np.isclose(r.ref_energy, energy, rtol=1e-12, atol=1e-300)
    band += compare_quantized(w32, cands[best], gran, group, f16, clip, refs[best], codes, scale, idx, uerr)
    return band


def test_config0_fp32_1024_absmax(mq):
    """1024x1024 fp32, seed 0, per-channel absmax scale (one ratio), INT4 vs E2M1."""
    w = mi.config0_weight(0, device=DEV)
    band = check_tensor(mq, w, [orc.INT4, orc.FP4_E2M1], orc.PER_CHANNEL, mi.clip_ratios(1), label="cfg0")
    assert band == 0


@pytest.mark.parametrize("cols", [8, 1000, 2048, 4096, 5000, 11008, 22016, 32768])
def test_per_channel_clip_search_row_lengths(mq, cols):
    """fp16 rows across every register-tiling variant, including ragged tails."""
    rows = 7 if cols > 12000 else 19
    w = mi.llama_like_weight(rows, cols, seed=100 + cols, device=DEV, outlier_frac=2e-3)
    check_tensor(mq, w, [orc.INT4, orc.FP4_E2M1], orc.PER_CHANNEL, mi.clip_ratios(100), label="rows")


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_per_channel_other_dtypes(mq, dtype):
    w = mi.llama_like_weight(13, 4096, seed=7, dtype=dtype, device=DEV)
    check_tensor(mq, w, [orc.INT4, orc.FP4_E2M1], orc.PER_CHANNEL, mi.clip_ratios(33), label="dtype")


def test_repeated_and_dense_clip_ratios(mq):
    """Clip tables whose candidates tie exactly (repeats) or differ by a few ulp: the winner of
    each row has rivals within any rounding margin, so the per-channel search has to settle them
    element by element; rows of several tilings, wide (|x| >= 2) and narrow magnitudes."""
    w = mi.llama_like_weight(11, 4096, seed=21, device=DEV)
    w[3] *= 64.0
    base = mi.clip_ratios(12)
    rep = np.repeat(base, 2)[:20].astype(np.float32)
    check_tensor(mq, w, [orc.INT4, orc.FP4_E2M1], orc.PER_CHANNEL, rep, label="repeats")
    dense = np.array([np.nextafter(np.float32(0.8), np.float32(1.0 if i % 2 else 0.0)) for i in range(4)]
                     + [0.8] * 4 + list(base), dtype=np.float32)
    check_tensor(mq, w, [orc.INT4, orc.FP4_E2M1], orc.PER_CHANNEL, dense, label="dense")
    w2 = mi.llama_like_weight(5, 11008, seed=22, device=DEV)
    check_tensor(mq, w2, [orc.FP4_E2M1, orc.INT4], orc.PER_CHANNEL, rep, label="repeats-11008")


def test_candidate_order_and_single_candidate(mq):
    w = mi.llama_like_weight(9, 1024, seed=8, device=DEV)
    clip = mi.clip_ratios(10)
    check_tensor(mq, w, [orc.FP4_E2M1, orc.INT4], orc.PER_CHANNEL, clip, label="reversed")
    check_tensor(mq, w, [orc.FP4_E2M1], orc.PER_CHANNEL, clip, label="single")
    check_tensor(mq, w, [orc.INT4, orc.INT4, orc.FP4_E2M1], orc.PER_CHANNEL, clip, label="repeat")


@pytest.mark.parametrize("group,cols,rows", [(128, 11008, 5), (128, 4096, 9), (32, 256, 3), (64, 640, 70), (256, 1024, 4)])
def test_group_wise_fp16_scales(mq, group, cols, rows):
    """Groups along the input dimension, fp16 scales, 50 ratios; unit counts that
    do not fill the last workgroup."""
    w = mi.llama_like_weight(rows, cols, seed=200 + cols, device=DEV, outlier_frac=2e-3)
    check_tensor(mq, w, [orc.INT4, orc.FP4_E2M1], orc.PER_GROUP, mi.clip_ratios(50), group, True, label="group")


def test_group_wise_fp32_scales_and_odd_k(mq):
    w = mi.llama_like_weight(6, 1024, seed=9, device=DEV)
    check_tensor(mq, w, [orc.INT4, orc.FP4_E2M1], orc.PER_GROUP, mi.clip_ratios(7), 128, False, label="group-f32")


@pytest.mark.parametrize("n_clip", [1, 2, 33, 64, 128])
def test_group_wise_candidate_counts(mq, n_clip):
    """Candidate counts around the 32-candidate words of the survivor masks, the single
    candidate (no first pass) and the maximum."""
    w = mi.llama_like_weight(7, 2048, seed=300 + n_clip, device=DEV, outlier_frac=2e-3)
    check_tensor(mq, w, [orc.INT4, orc.FP4_E2M1], orc.PER_GROUP, mi.clip_ratios(n_clip), 128, True,
                 label="group-k")


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_group_wise_other_dtypes_and_formats(mq, dtype):
    w = mi.llama_like_weight(5, 1536, seed=41, dtype=dtype, device=DEV)
    check_tensor(mq, w, [orc.INT4, orc.FP4_E2M1], orc.PER_GROUP, mi.clip_ratios(12), 64, False, label="group-dtype")
    check_tensor(mq, w, [orc.INT8, orc.FP8_E4M3], orc.PER_GROUP, mi.clip_ratios(6), 128, True, label="group-8bit")
    check_tensor(mq, w, [orc.FP4_E2M1], orc.PER_GROUP, mi.clip_ratios(9), 128, True, label="group-single")


@pytest.mark.parametrize("cands", [[orc.FP4_E2M1_IEEE], [orc.INT4, orc.FP4_E2M1_IEEE],
                                   [orc.FP4_E2M1_IEEE, orc.FP4_E2M1], [orc.FP8_E5M2],
                                   [orc.INT8, orc.FP8_E5M2], [orc.FP8_E5M2, orc.FP8_E4M3]])
def test_ieee_fp4_and_e5m2_grids(mq, cands):
    """The IEEE-aligned FP4 of Table 1 (saturating at 3) and FP8-E5M2: every granularity,
    alone and against the other formats of their bit-width (such pairs are scored in
    separate launches)."""
    w = mi.llama_like_weight(9, 2048, seed=50, device=DEV, outlier_frac=2e-3)
    check_tensor(mq, w, cands, orc.PER_CHANNEL, mi.clip_ratios(20), label="grids-channel")
    check_tensor(mq, w, cands, orc.PER_CHANNEL, mi.clip_ratios(1), label="grids-absmax")
    check_tensor(mq, w, cands, orc.PER_GROUP, mi.clip_ratios(10), 128, True, label="grids-group")
    wb = mi.llama_like_weight(40, 512, seed=51, dtype=torch.bfloat16, device=DEV)
    check_tensor(mq, wb, cands, orc.PER_TENSOR, mi.clip_ratios(3), label="grids-tensor")
    # values far outside the grid, subnormals of the 8-bit format, signed zeros
    e = torch.zeros(4, 256, dtype=torch.float32)
    e[0] = torch.linspace(-70000, 70000, 256)
    e[1] = torch.linspace(-4, 4, 256) * 2.0 ** -15
    e[2, ::2] = -0.0
    e[2, 1] = 1.0
    e[3] = torch.linspace(-3.6, 3.6, 256)
    check_tensor(mq, e.to(DEV), cands, orc.PER_TENSOR, mi.clip_ratios(1), label="grids-edge")
    check_tensor(mq, e.to(DEV), cands, orc.PER_CHANNEL, mi.clip_ratios(2), label="grids-edge-channel")


@pytest.mark.parametrize("fmt_pair", [(orc.INT8, orc.FP8_E4M3), (orc.INT4, orc.FP4_E2M1)])
def test_per_tensor(mq, fmt_pair):
    x = mi.activations(300, 1024, seed=10, device=DEV)
    check_tensor(mq, x, list(fmt_pair), orc.PER_TENSOR, mi.clip_ratios(1), label="tensor-x")
    w = mi.llama_like_weight(64, 4096, seed=11, dtype=torch.bfloat16, device=DEV)
    check_tensor(mq, w, list(fmt_pair), orc.PER_TENSOR, mi.clip_ratios(4), label="tensor-w")


def test_eight_bit_per_channel(mq):
    w = mi.llama_like_weight(11, 4096, seed=12, dtype=torch.bfloat16, device=DEV)
    check_tensor(mq, w, [orc.INT8, orc.FP8_E4M3], orc.PER_CHANNEL, mi.clip_ratios(5), label="w8")


def test_degenerate_units(mq):
    """Zero rows, a single non-zero, fp16 subnormals, large magnitudes, negative
    zeros, and rows already on a grid (zero error, tie between the formats)."""
    w = torch.zeros(12, 1024, dtype=torch.float16)
    w[1, 5] = 0.37
    w[2] = 6e-8                                  # fp16 subnormal everywhere
    w[3] = torch.randn(1024) * 2000.0            # large values
    w[4] = -0.0
    w[5] = torch.randn(1024) * 1e-6
    a = 42 * 2.0 ** -8
    w[6] = (torch.randint(-1, 2, (1024,)) * a)   # on both grids
    w[6, 0] = a
    w[7] = torch.randint(-7, 8, (1024,)).float() * 2.0 ** -6   # on the INT4 grid
    w[7, 0] = 7 * 2.0 ** -6
    w[8, :] = 65504.0
    w[9] = torch.randn(1024) * 0.02
    w[9, 100] = -3.0
    check_tensor(mq, w.to(DEV), [orc.INT4, orc.FP4_E2M1], orc.PER_CHANNEL, mi.clip_ratios(20), label="degenerate")
    check_tensor(mq, w.to(DEV), [orc.INT4, orc.FP4_E2M1], orc.PER_GROUP, mi.clip_ratios(20), 128, True, label="degenerate-g")
    z = torch.zeros(4, 256, dtype=torch.float32, device=DEV)
    check_tensor(mq, z, [orc.INT8, orc.FP8_E4M3], orc.PER_TENSOR, mi.clip_ratios(1), label="all-zero")


def test_tie_keeps_first_candidate(mq):
    a = 42 * 2.0 ** -8
    g = torch.Generator().manual_seed(3)
    w = (torch.randint(-1, 2, (16, 512), generator=g) * a).to(torch.float16)
    w[:, 0] = a
    for cands in ([orc.INT4, orc.FP4_E2M1], [orc.FP4_E2M1, orc.INT4]):
        r, *_ = run_select(mq, w.to(DEV), cands, mq.Cfg(orc.PER_CHANNEL, mi.clip_ratios(1)))
        assert r.best == 0 and list(r.err)[:2] == [0.0, 0.0]


def test_strided_rows(mq):
    """ld > cols: a column slice of a wider matrix."""
    big = mi.llama_like_weight(10, 4096, seed=13, device=DEV)
    w = big[:, 1024:3072]
    assert w.stride(0) == 4096
    w32 = mi.to_f32_numpy(w)
    cfg = mq.Cfg(orc.PER_CHANNEL, mi.clip_ratios(16))
    ref = orc.quantize(w32, orc.FP4_E2M1, orc.PER_CHANNEL, mi.clip_ratios(16), want_table=True)
    codes, scale, idx, uerr, terr = run_quantize(mq, w, orc.FP4_E2M1, cfg)
    compare_quantized(w32, orc.FP4_E2M1, orc.PER_CHANNEL, 0, False, mi.clip_ratios(16), ref, codes, scale, idx, uerr)


def test_score_matches_quantize_error(mq):
    w = mi.llama_like_weight(33, 4096, seed=14, device=DEV)
    clip = mi.clip_ratios(25)
    cfg = mq.Cfg(orc.PER_CHANNEL, clip)
    w32 = mi.to_f32_numpy(w)
    for f in (orc.INT4, orc.FP4_E2M1):
        err = torch.zeros(1, dtype=torch.float64, device=DEV)
        en = torch.zeros(1, dtype=torch.float64, device=DEV)
        mq.score(w, None, f, mq.ERR_TENSOR, cfg, err, en, _ws(mq, w, 1, cfg))
        torch.cuda.synchronize()
        ref = orc.quantize(w32, f, orc.PER_CHANNEL, clip)
        assert np.isclose(err.item(), ref.err, rtol=ERR_RTOL)
        assert np.isclose(en.item(), float(np.sum(w32.astype(np.float64) ** 2)), rtol=1e-12)


def test_deterministic_across_runs(mq):
    w = mi.llama_like_weight(64, 11008, seed=15, device=DEV)
    cfg = mq.Cfg(orc.PER_CHANNEL, mi.clip_ratios(100))
    a = run_select(mq, w, [orc.INT4, orc.FP4_E2M1], cfg)
    b = run_select(mq, w, [orc.INT4, orc.FP4_E2M1], cfg)
    assert list(a[0].err) == list(b[0].err) and a[0].best == b[0].best
    for x, y in zip(a[1:], b[1:]):
        assert np.array_equal(x, y)


def test_unsupported_and_errors_raise(mq):
    w = mi.llama_like_weight(4, 64, seed=16, device=DEV)
    cfg = mq.Cfg(orc.PER_GROUP, mi.clip_ratios(2), 128)
    out = mq.alloc_qbuffers(4, 64, 4, mq.Cfg(orc.PER_CHANNEL, mi.clip_ratios(2)), DEV)
    ws = torch.empty(1 << 16, dtype=torch.uint8, device=DEV)
    with pytest.raises(mq.MofqError) as e:
        mq.quantize(w, orc.INT4, cfg, out, None, ws)
    assert e.value.status == -2
    cfg = mq.Cfg(orc.PER_CHANNEL, mi.clip_ratios(2))
    with pytest.raises(mq.MofqError) as e:
        mq.quantize(w, orc.INT4, cfg, out, None, ws[:8])
    assert e.value.status == -4
