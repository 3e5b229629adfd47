"""GPU parity of the weight-only select by layer-output error (16-bit input, quantized
weights, matrix cores) against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import mofq_inputs as mi
from oracle import mofq_oracle as orc
from tests.gpu_util import compare_quantized, scales_to_f32, unpack_codes

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
I4, FP4, I8, FP8 = orc.INT4, orc.FP4_E2M1, orc.INT8, orc.FP8_E4M3
# fp32 accumulation inside the matrix cores against fp64 in the oracle: the products are
# exact on both sides, sums of K <= 11008 terms differ by ~sqrt(K)*2^-24 of |Y|, and the
# 4-bit quantization differences are ~1e-1 |Y|, so the error sums agree far inside 1e-5.
E_RTOL = 1e-5


@pytest.fixture(scope="module")
def mq():
    from paper_2305_12356_amd import binding
    assert torch.cuda.is_available()
    return binding


def run_select(mq, x, w, cands, gran, clip, f16=False):
    cfg = mq.Cfg(gran, clip, 0, f16)
    bits = orc.bits(cands[0])
    w_out = mq.alloc_qbuffers(w.shape[0], w.shape[1], bits, cfg, DEV)
    res = mq.alloc_result(DEV)
    n = mq.workspace_bytes(w, x, len(cands), mq.ERR_LAYER_OUTPUT_W_ONLY, cfg)
    assert n > 0
    ws = torch.empty(n, dtype=torch.uint8, device=DEV)
    mq.select_layer(w, x, cands, mq.ERR_LAYER_OUTPUT_W_ONLY, cfg, w_out, None, res, ws)
    torch.cuda.synchronize()
    return mq.read_result(res), w_out


def run_score(mq, x, w, fmt, gran, clip, f16=False):
    cfg = mq.Cfg(gran, clip, 0, f16)
    err = torch.zeros(1, dtype=torch.float64, device=DEV)
    en = torch.zeros(1, dtype=torch.float64, device=DEV)
    ws = torch.empty(mq.workspace_bytes(w, x, 1, mq.ERR_LAYER_OUTPUT_W_ONLY, cfg), dtype=torch.uint8, device=DEV)
    mq.score(w, x, fmt, mq.ERR_LAYER_OUTPUT_W_ONLY, cfg, err, en, ws)
    torch.cuda.synchronize()
    return err.item(), en.item()


def check_layer(mq, x, w, cands, gran, clip, label, f16=False):
    print(f"[case] {label} X={tuple(x.shape)} W={tuple(w.shape)} gran={gran} K={len(clip)} cands={cands}", flush=True)
    x32, w32 = mi.to_f32_numpy(x), mi.to_f32_numpy(w)
    clip = np.asarray(clip, dtype=np.float32)
    ref = orc.select_layer_w_only_output(x32, w32, cands, gran, clip, f16)
    r, w_out = run_select(mq, x, w, cands, gran, clip, f16)
    assert r.n == len(cands)
    assert np.allclose(list(r.err)[:len(cands)], ref.errs, rtol=E_RTOL, atol=1e-300), (list(r.err), ref.errs)
    assert np.isclose(r.ref_energy, ref.ref_energy, rtol=E_RTOL)
    assert r.best == ref.best, (r.best, ref.best, ref.errs)
    # codes, scales and clip indices of the winner: the tensor-error search, bit for bit
    fmt = cands[ref.best]
    q = orc.quantize(w32, fmt, gran, clip, 0, f16, want_table=True)
    compare_quantized(w32, fmt, gran, 0, f16, clip, q, unpack_codes(w_out.codes, *w.shape, orc.bits(fmt)),
                      scales_to_f32(w_out.scales), w_out.clip_idx.cpu().numpy(), w_out.unit_err.cpu().numpy())
    for f in set(cands):
        e, p = run_score(mq, x, w, f, gran, clip, f16)
        assert np.isclose(e, ref.errs[cands.index(f)], rtol=E_RTOL, atol=1e-300)
        assert np.isclose(p, ref.ref_energy, rtol=E_RTOL)
    return r


@pytest.mark.parametrize("gran", [orc.PER_TENSOR, orc.PER_CHANNEL])
def test_four_bit_pair(mq, gran):
    x = mi.activations(300, 1024, seed=80, device=DEV)
    w = mi.llama_like_weight(200, 1024, seed=81, dtype=torch.bfloat16, device=DEV)
    check_layer(mq, x, w, [I4, FP4], gran, mi.clip_ratios(1), "absmax")
    check_layer(mq, x, w, [FP4, I4], gran, mi.clip_ratios(1), "order")


def test_clip_search_and_fp16_scales(mq):
    x = mi.activations(130, 2048, seed=82, device=DEV)
    w = mi.llama_like_weight(260, 2048, seed=83, dtype=torch.bfloat16, device=DEV, outlier_frac=2e-3)
    check_layer(mq, x, w, [I4, FP4], orc.PER_CHANNEL, mi.clip_ratios(20), "clip-20")
    check_layer(mq, x, w, [I4, FP4], orc.PER_CHANNEL, mi.clip_ratios(100), "clip-100-f16", f16=True)


@pytest.mark.parametrize("m,n,k", [(1, 1, 64), (257, 129, 192), (300, 130, 64), (48, 520, 1088)])
def test_ragged_tiles(mq, m, n, k):
    x = mi.activations(m, k, seed=84 + m, device=DEV)
    w = mi.llama_like_weight(n, k, seed=85 + n, dtype=torch.bfloat16, device=DEV)
    check_layer(mq, x, w, [I4, FP4], orc.PER_CHANNEL, mi.clip_ratios(3), "ragged")


@pytest.mark.parametrize("k", [64, 2048, 8192, 11008, 16384, 24576, 32768])
def test_absmax_pair_every_row_length(mq, k):
    """Per-channel absmax scales and a pair of formats: the scoring pass writes both candidates'
    grid values itself; one case per instance of that kernel (row lengths up to the limit)."""
    x = mi.activations(70, k, seed=92 + k, device=DEV)
    w = mi.llama_like_weight(40, k, seed=93 + k, dtype=torch.bfloat16, device=DEV)
    check_layer(mq, x, w, [FP4, I4], orc.PER_CHANNEL, mi.clip_ratios(1), f"absmax-pair-{k}")
    if k in (64, 11008):
        check_layer(mq, x, w, [I8, FP8], orc.PER_CHANNEL, np.array([0.8], dtype=np.float32), f"absmax-pair8-{k}")


def test_single_candidate_and_eight_bit_weights(mq):
    x = mi.activations(128, 512, seed=86, device=DEV)
    w = mi.llama_like_weight(256, 512, seed=87, dtype=torch.bfloat16, device=DEV)
    check_layer(mq, x, w, [FP4], orc.PER_CHANNEL, mi.clip_ratios(4), "single")
    check_layer(mq, x, w, [I8, FP8], orc.PER_CHANNEL, mi.clip_ratios(1), "w8a16")
    check_layer(mq, x, w, [orc.FP4_E2M1_IEEE, FP4], orc.PER_CHANNEL, mi.clip_ratios(1), "ieee-vs-redesigned")
    check_layer(mq, x, w, [orc.FP8_E5M2, FP8], orc.PER_TENSOR, mi.clip_ratios(1), "e5m2-vs-e4m3")


def test_llama_shape_block(mq):
    """One LLaMA-7B attention projection at full size (2048 tokens); the oracle's fp64
    products take a few seconds."""
    x = mi.activations(2048, 4096, seed=88, device=DEV)
    w = mi.llama_like_weight(4096, 4096, seed=89, dtype=torch.bfloat16, device=DEV)
    check_layer(mq, x, w, [I4, FP4], orc.PER_CHANNEL, mi.clip_ratios(1), "7b-q")


def test_rejects_what_it_cannot_do(mq):
    x = mi.activations(64, 256, seed=90, device=DEV)
    w = mi.llama_like_weight(64, 256, seed=91, dtype=torch.bfloat16, device=DEV)
    cfg = mq.Cfg(mq.PER_GROUP, mi.clip_ratios(1), 128, True)
    assert mq.workspace_bytes(w, x, 2, mq.ERR_LAYER_OUTPUT_W_ONLY, cfg) == 0     # group scales vary along K
    cfg = mq.Cfg(mq.PER_CHANNEL, mi.clip_ratios(1))
    out = mq.alloc_qbuffers(64, 256, 4, cfg, DEV)
    res = mq.alloc_result(DEV)
    ws = torch.empty(1 << 22, dtype=torch.uint8, device=DEV)
    with pytest.raises(mq.MofqError):     # fp16 weights: the matrix path takes bf16
        mq.select_layer(w.to(torch.float16), x, [I4, FP4], mq.ERR_LAYER_OUTPUT_W_ONLY, cfg, out, None, res, ws)
    with pytest.raises(mq.MofqError):     # three candidates
        mq.select_layer(w, x, [I4, FP4, I4], mq.ERR_LAYER_OUTPUT_W_ONLY, cfg, out, None, res, ws)
    torch.cuda.synchronize()
