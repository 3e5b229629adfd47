"""GPU parity of the weight-activation path (per-tensor / per-channel 8-bit
quantization of W and X, layer-output error through the matrix cores, select)
against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import mofq_inputs as mi
from oracle import mofq_oracle as orc
from tests.gpu_util import scales_to_f32, unpack_codes

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
I8, FP8 = orc.INT8, orc.FP8_E4M3
# fp32 accumulation inside the matrix cores (the oracle adds in fp64): K <= 11008
# terms, relative error of a sum ~ sqrt(K)*2^-24 of |Y|, and the quantization
# differences are >= 1e-2 |Y|, so error sums agree to ~1e-6; the target is 1e-5.
E_RTOL = 1e-5


@pytest.fixture(scope="module")
def mq():
    from paper_2305_12356_amd import binding
    assert torch.cuda.is_available()
    return binding


def run_wa_select(mq, x, w, cands, w_gran):
    cfg = mq.Cfg(w_gran, mi.clip_ratios(1))
    xcfg = mq.Cfg(mq.PER_TENSOR, mi.clip_ratios(1))
    w_out = mq.alloc_qbuffers(w.shape[0], w.shape[1], 8, cfg, DEV)
    x_out = mq.alloc_qbuffers(x.shape[0], x.shape[1], 8, xcfg, DEV)
    res = mq.alloc_result(DEV)
    n = mq.workspace_bytes(w, x, len(cands), mq.ERR_LAYER_OUTPUT, cfg)
    assert n > 0
    ws = torch.empty(n, dtype=torch.uint8, device=DEV)
    mq.select_layer(w, x, cands, mq.ERR_LAYER_OUTPUT, cfg, w_out, x_out, res, ws)
    torch.cuda.synchronize()
    return mq.read_result(res), w_out, x_out


def run_wa_score(mq, x, w, fmt, w_gran):
    cfg = mq.Cfg(w_gran, mi.clip_ratios(1))
    err = torch.zeros(1, dtype=torch.float64, device=DEV)
    en = torch.zeros(1, dtype=torch.float64, device=DEV)
    ws = torch.empty(mq.workspace_bytes(w, x, 1, mq.ERR_LAYER_OUTPUT, cfg), dtype=torch.uint8, device=DEV)
    mq.score(w, x, fmt, mq.ERR_LAYER_OUTPUT, cfg, err, en, ws)
    torch.cuda.synchronize()
    return err.item(), en.item()


def check_layer(mq, x, w, cands, w_gran, label, want_ref=False):
    print(f"[case] {label} X={tuple(x.shape)} W={tuple(w.shape)} w_gran={w_gran} cands={cands}", flush=True)
    x32, w32 = mi.to_f32_numpy(x), mi.to_f32_numpy(w)
    ref = orc.select_layer_wa(x32, w32, cands, w_gran)
    r, w_out, x_out = run_wa_select(mq, x, w, cands, w_gran)
    assert r.n == len(cands)
    assert np.allclose(list(r.err)[:len(cands)], ref.errs, rtol=E_RTOL, atol=1e-300), (list(r.err), ref.errs)
    assert np.isclose(r.ref_energy, ref.ref_energy, rtol=E_RTOL)
    assert r.best == ref.best
    # codes and scales of the winner, bit for bit
    assert np.array_equal(unpack_codes(w_out.codes, *w.shape, 8), ref.w.codes)
    assert np.array_equal(unpack_codes(x_out.codes, *x.shape, 8), ref.x.codes)
    assert np.array_equal(scales_to_f32(w_out.scales), ref.w.scale)
    assert np.array_equal(scales_to_f32(x_out.scales), ref.x.scale)
    assert np.allclose(w_out.unit_err.cpu().numpy(), ref.w.unit_err, rtol=1e-9, atol=1e-300)
    for f in set(cands):
        e, p = run_wa_score(mq, x, w, f, w_gran)
        assert np.isclose(e, ref.errs[cands.index(f)], rtol=E_RTOL, atol=1e-300)
        assert np.isclose(p, ref.ref_energy, rtol=E_RTOL)
    return (r, ref) if want_ref else r


@pytest.mark.parametrize("w_gran", [orc.PER_TENSOR, orc.PER_CHANNEL])
@pytest.mark.parametrize("M,N,K", [(128, 128, 64), (200, 300, 256), (96, 520, 1024), (257, 129, 11008)])
def test_layer_output_ragged_tiles(mq, w_gran, M, N, K):
    x = mi.activations(M, K, seed=300 + M, device=DEV)
    w = mi.llama_like_weight(N, K, seed=400 + N, dtype=torch.bfloat16, device=DEV)
    check_layer(mq, x, w, [I8, FP8], w_gran, "ragged")


def test_candidate_orders(mq):
    x = mi.activations(130, 512, seed=20, device=DEV)
    w = mi.llama_like_weight(140, 512, seed=21, dtype=torch.bfloat16, device=DEV)
    check_layer(mq, x, w, [FP8, I8], orc.PER_TENSOR, "reversed")
    check_layer(mq, x, w, [FP8], orc.PER_CHANNEL, "single-fp8")
    check_layer(mq, x, w, [I8], orc.PER_TENSOR, "single-int8")


def test_tame_activations_prefer_int8(mq):
    x = mi.activations(256, 1024, seed=22, n_outlier=0, device=DEV)
    w = mi.llama_like_weight(384, 1024, seed=23, dtype=torch.bfloat16, device=DEV)
    r = check_layer(mq, x, w, [I8, FP8], orc.PER_CHANNEL, "tame")
    assert r.best == 0


def test_small_integers_exact(mq):
    """Small-integer operands: every product and sum is exact in every precision, so
    the INT8 error is exactly zero and the energy equals the integer sum."""
    g = torch.Generator().manual_seed(5)
    M, N, K = 150, 170, 192
    x = torch.randint(-5, 6, (M, K), generator=g).float()
    w = torch.randint(-5, 6, (N, K), generator=g).float()
    x[0, 0] = 127.0
    w[0, 0] = 127.0
    r, _, _ = run_wa_select(mq, x.to(torch.bfloat16).to(DEV), w.to(torch.bfloat16).to(DEV), [I8, FP8], orc.PER_TENSOR)
    y = x.double() @ w.double().T
    assert list(r.err)[0] == 0.0 and r.best == 0
    assert r.ref_energy == float((y * y).sum())


@pytest.mark.parametrize("fmt", [I8, FP8])
def test_on_grid_with_per_channel_power_of_two_scales(mq, fmt):
    """W rows on the 8-bit grid with a different power-of-two scale per row, X on the
    grid: the error is exactly zero only if each output column meets its own scale."""
    rng = np.random.default_rng(6)
    M, N, K = 160, 200, 128
    if fmt == I8:
        gx = rng.integers(-127, 128, size=(M, K)).astype(np.float64)
        gw = rng.integers(-127, 128, size=(N, K)).astype(np.float64)
        top = 127.0
    else:
        gx = orc.decode_array(fmt, rng.integers(0, 127, size=(M, K))) * rng.choice([-1.0, 1.0], size=(M, K))
        gw = orc.decode_array(fmt, rng.integers(0, 127, size=(N, K))) * rng.choice([-1.0, 1.0], size=(N, K))
        top = 448.0
    # 8-bit grid values have at most 7 significant bits: exact in bf16
    gx[0, 0] = top
    gw[:, 0] = top
    e = rng.integers(-8, 1, size=N)
    x = torch.from_numpy(gx * 2.0 ** -2).to(torch.bfloat16)
    w = torch.from_numpy(gw * (2.0 ** e)[:, None]).to(torch.bfloat16)
    assert np.array_equal(x.float().numpy(), (gx * 2.0 ** -2).astype(np.float32))
    assert np.array_equal(w.float().numpy(), (gw * (2.0 ** e)[:, None]).astype(np.float32))
    err, en = run_wa_score(mq, x.to(DEV), w.to(DEV), fmt, orc.PER_CHANNEL)
    assert err == 0.0 and en > 0


def run_fp8_unit(mq, x, w, w_gran):
    cfg = mq.Cfg(w_gran, mi.clip_ratios(1))
    w_out = mq.alloc_qbuffers(w.shape[0], w.shape[1], 8, cfg, DEV)
    res = mq.alloc_result(DEV)
    ws = torch.empty(mq.workspace_bytes(w, x, 2, mq.ERR_LAYER_OUTPUT_FP8_UNIT, cfg), dtype=torch.uint8, device=DEV)
    mq.select_layer(w, x, [I8, FP8], mq.ERR_LAYER_OUTPUT_FP8_UNIT, cfg, w_out, None, res, ws)
    torch.cuda.synchronize()
    return mq.read_result(res), w_out


# The fp8 matrix unit aligns the 8 products of each group of 8 consecutive k to the group's
# largest exponent sum and drops what lies more than 13 bits below it (towards zero); group
# sums and the accumulator are then added like fp32 numbers.  With the activation's outlier
# columns inside the fp8 product, the dropped bits moved the FP8 error sum by 1e-6 .. 3e-5 at
# full size and by up to 1e-4 on small layers.  The fused path (INT8 / E4M3 pair, per-tensor
# scales) therefore splits those columns off into one exact K step on the bf16 matrix cores:
# measured deviations are then below 1e-6 on small layers and below 4e-7 at full size, and the
# fp8-unit form of the metric is held to the same 1e-5 as the exact one.
FP8_UNIT_RTOL = E_RTOL


@pytest.mark.parametrize("M,N,K,seed", [(384, 512, 1024, 26), (128, 128, 64, 1), (257, 129, 11008, 2), (96, 520, 1024, 3)])
def test_fp8_unit_metric_small_layers(mq, M, N, K, seed):
    """The E4M3 product on the fp8 matrix cores (outlier columns split off): same INT8 error,
    same codes, same decision; FP8 error within the 1e-5 of the exact form."""
    x = mi.activations(M, K, seed=seed, device=DEV)
    w = mi.llama_like_weight(N, K, seed=seed + 1, dtype=torch.bfloat16, device=DEV)
    ref = orc.select_layer_wa(mi.to_f32_numpy(x), mi.to_f32_numpy(w), [I8, FP8], orc.PER_TENSOR)
    print(f"[case] fp8 unit {M}x{N}x{K}", flush=True)
    r, w_out = run_fp8_unit(mq, x, w, orc.PER_TENSOR)
    dev = r.err[1] / ref.errs[1] - 1
    print(f"fp8-unit deviation of the FP8 error sum: {dev:+.3e}", flush=True)
    assert np.isclose(r.err[0], ref.errs[0], rtol=E_RTOL)
    assert abs(dev) <= FP8_UNIT_RTOL
    assert r.best == ref.best
    assert np.array_equal(unpack_codes(w_out.codes, N, K, 8), ref.w.codes)


@pytest.mark.parametrize("name,o,n", [("q", 4096, 4096), ("gate", 11008, 4096), ("down", 4096, 11008)])
def test_llama_shaped_linear(mq, name, o, n):
    """The three distinct linear shapes of a 7B decoder block at full size (2048 tokens),
    in the launch configuration bench.py times; the oracle's fp64 products take seconds.
    Both forms of the metric: the E4M3 product from grid values on the bf16 matrix cores, and
    the E4M3 codes on the fp8 matrix cores (outlier columns split off), both within the 1e-5
    tolerance of the oracle's error sums."""
    lin = mi.LINEAR_NAMES.index(name)
    x = mi.activations(2048, n, seed=mi.tensor_seed(3, 0, lin, 1), device=DEV)
    w = mi.llama_like_weight(o, n, seed=mi.tensor_seed(3, 0, lin), dtype=torch.bfloat16, device=DEV)
    r, ref = check_layer(mq, x, w, [I8, FP8], orc.PER_TENSOR, "llama-" + name, want_ref=True)
    assert r.best == 1        # FP8 wins with outlier channels (Section 3.2)
    u, w_out = run_fp8_unit(mq, x, w, orc.PER_TENSOR)
    dev = u.err[1] / ref.errs[1] - 1
    print(f"fp8-unit deviation of the FP8 error sum at 2048x{o}x{n}: {dev:+.3e}", flush=True)
    assert np.allclose(list(u.err)[:2], ref.errs, rtol=E_RTOL, atol=1e-300), (list(u.err), ref.errs)
    assert np.isclose(u.ref_energy, ref.ref_energy, rtol=E_RTOL)
    assert u.best == ref.best
    assert np.array_equal(unpack_codes(w_out.codes, o, n, 8), ref.w.codes)
    assert np.array_equal(scales_to_f32(w_out.scales), ref.w.scale)


def test_wa_argument_errors(mq):
    x = mi.activations(64, 128, seed=24, device=DEV)
    w16 = mi.llama_like_weight(64, 128, seed=25, dtype=torch.float16, device=DEV)
    wb = w16.to(torch.bfloat16)
    cfg = mq.Cfg(mq.PER_TENSOR, mi.clip_ratios(1))
    err = torch.zeros(1, dtype=torch.float64, device=DEV)
    ws = torch.empty(1 << 20, dtype=torch.uint8, device=DEV)
    with pytest.raises(mq.MofqError) as e:      # fp16 weights are not accepted for the bf16 reference product
        mq.score(w16, x, I8, mq.ERR_LAYER_OUTPUT, cfg, err, None, ws)
    assert e.value.status == -2
    with pytest.raises(mq.MofqError) as e:      # 4-bit candidates have no matrix-core path
        mq.score(wb, x, orc.INT4, mq.ERR_LAYER_OUTPUT, cfg, err, None, ws)
    assert e.value.status == -2
    with pytest.raises(mq.MofqError) as e:      # inner dimensions differ
        mq.score(wb[:, :64].contiguous(), x, I8, mq.ERR_LAYER_OUTPUT, cfg, err, None, ws)
    assert e.value.status == -1


def test_calls_on_two_caller_streams_equal_serial_calls(mq):
    """The library keeps no state: calls for different linears may run concurrently on two
    streams of the caller (own workspace and outputs per stream) and give, bit for bit, what
    the same calls give one after the other."""
    shapes = [(512, 1024), (300, 1024), (1024, 512), (129, 2048), (512, 1024), (640, 512)]
    xs = {k: mi.activations(384, k, seed=900 + k, device=DEV) for k in {n for _, n in shapes}}
    ws_ = [mi.llama_like_weight(o, n, seed=910 + i, dtype=torch.bfloat16, device=DEV) for i, (o, n) in enumerate(shapes)]
    cands = [I8, FP8]
    cfg = mq.Cfg(orc.PER_TENSOR, mi.clip_ratios(1))
    xcfg = mq.Cfg(mq.PER_TENSOR, mi.clip_ratios(1))
    nbytes = max(mq.workspace_bytes(w, xs[w.shape[1]], 2, mq.ERR_LAYER_OUTPUT, cfg) for w in ws_)

    def run(streams):
        res = mq.alloc_result(DEV, len(shapes))
        wsp = [torch.empty(nbytes, dtype=torch.uint8, device=DEV) for _ in streams]
        w_out = [mq.alloc_qbuffers(o, n, 8, cfg, DEV) for o, n in shapes]
        x_out = [mq.alloc_qbuffers(384, n, 8, xcfg, DEV) for _, n in shapes]
        torch.cuda.synchronize()
        for rep in range(3):                      # several rounds, so that the calls really overlap
            for i, w in enumerate(ws_):
                s = i % len(streams)
                mq.select_layer(w, xs[w.shape[1]], cands, mq.ERR_LAYER_OUTPUT, cfg, w_out[i], x_out[i], res[i],
                                wsp[s], streams[s])
        torch.cuda.synchronize()
        return mq.read_results(res), w_out, x_out

    r1, w1, x1 = run([torch.cuda.current_stream()])
    r2, w2, x2 = run([torch.cuda.Stream(), torch.cuda.Stream()])
    for i in range(len(shapes)):
        assert r1[i].best == r2[i].best and list(r1[i].err) == list(r2[i].err) and r1[i].ref_energy == r2[i].ref_energy
        assert torch.equal(w1[i].codes, w2[i].codes) and torch.equal(w1[i].scales, w2[i].scales)
        assert torch.equal(x1[i].codes, x2[i].codes) and torch.equal(x1[i].scales, x2[i].scales)


@pytest.mark.parametrize("n_outlier,scale", [(0, 1.0), (1, 60.0), (64, 60.0), (100, 60.0), (6, 5.0)])
def test_fp8_unit_column_split_cases(mq, n_outlier, scale):
    """The column split of the fp8-unit product at its edges: no outlier column, one, exactly as
    many as the side step takes (64), more than that (the rest stays in the fp8 product: the
    sum is the same, only less protected), and outliers mild enough to stay in.  Decisions, codes
    and the INT8 error are the oracle's in every case; the E4M3 error within 1e-5 wherever all
    outlier columns fit into the side step."""
    M, N, K = 200, 300, 1024
    x = mi.activations(M, K, seed=500 + n_outlier, device=DEV, n_outlier=n_outlier, outlier_scale=scale)
    w = mi.llama_like_weight(N, K, seed=501 + n_outlier, dtype=torch.bfloat16, device=DEV)
    ref = orc.select_layer_wa(mi.to_f32_numpy(x), mi.to_f32_numpy(w), [I8, FP8], orc.PER_TENSOR)
    r, w_out = run_fp8_unit(mq, x, w, orc.PER_TENSOR)
    dev = r.err[1] / ref.errs[1] - 1
    print(f"[case] column split, {n_outlier} outlier columns x{scale}: deviation {dev:+.3e}", flush=True)
    assert np.isclose(r.err[0], ref.errs[0], rtol=E_RTOL)
    assert np.isclose(r.ref_energy, ref.ref_energy, rtol=E_RTOL)
    assert abs(dev) <= (FP8_UNIT_RTOL if n_outlier <= 64 else 1e-3)
    assert r.best == ref.best
    assert np.array_equal(unpack_codes(w_out.codes, N, K, 8), ref.w.codes)


@pytest.mark.parametrize("K", [12288, 16384, 32768])
def test_fp8_unit_wide_rows(mq, K):
    """Rows beyond what the column pick keeps in LDS (12288 columns), up to the longest row the
    layer-output metric takes: both forms of the metric against the oracle."""
    M, N = 72, 136
    x = mi.activations(M, K, seed=520 + K, device=DEV)
    w = mi.llama_like_weight(N, K, seed=521 + K, dtype=torch.bfloat16, device=DEV)
    check_layer(mq, x, w, [I8, FP8], orc.PER_TENSOR, f"wide-{K}")
    ref = orc.select_layer_wa(mi.to_f32_numpy(x), mi.to_f32_numpy(w), [I8, FP8], orc.PER_TENSOR)
    r, w_out = run_fp8_unit(mq, x, w, orc.PER_TENSOR)
    dev = r.err[1] / ref.errs[1] - 1
    print(f"[case] fp8 unit, {K} columns: deviation {dev:+.3e}", flush=True)
    assert np.isclose(r.err[0], ref.errs[0], rtol=E_RTOL)
    assert abs(dev) <= FP8_UNIT_RTOL + 1e-3 / np.sqrt(M * N)   # 9792 outputs: see test_gpu_random_layers.py
    assert r.best == ref.best
    assert np.array_equal(unpack_codes(w_out.codes, N, K, 8), ref.w.codes)
