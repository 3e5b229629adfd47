"""GPU tests of mofq_select_layers_wa (the weight-activation select of the linear layers of a
model in one call): against the CPU oracle layer by layer, and against mofq_select_layer bit
for bit, with shared activations, with both formats winning, through the C ABI."""
import numpy as np
import pytest
import torch

import mofq_inputs as mi
from oracle import mofq_oracle as orc
from tests.gpu_util import scales_to_f32, unpack_codes

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
I8, FP8 = orc.INT8, orc.FP8_E4M3
E_RTOL = 1e-5      # fp32 accumulation in the matrix cores against fp64 in the oracle (see test_gpu_wa.py)


@pytest.fixture(scope="module")
def mq():
    from paper_2305_12356_amd import binding
    assert torch.cuda.is_available()
    return binding


def block_like(tokens, hidden, ffn, seed, tame=()):
    """The seven linears of a decoder block at reduced size: q, k, v share one activation,
    o has its own, gate and up share one, down has its own.  Layers named in `tame` get an
    activation without outlier channels (INT8 then wins, Section 3.2)."""
    names = ["q", "k", "v", "o", "gate", "up", "down"]
    shapes = {"q": (hidden, hidden), "k": (hidden, hidden), "v": (hidden, hidden), "o": (hidden, hidden),
              "gate": (ffn, hidden), "up": (ffn, hidden), "down": (hidden, ffn)}
    share = {"q": "attn_in", "k": "attn_in", "v": "attn_in", "o": "attn_out", "gate": "mlp_in", "up": "mlp_in",
             "down": "mlp_mid"}
    acts = {}
    ws, xs = [], []
    for i, n in enumerate(names):
        o, k = shapes[n]
        key = share[n]
        if key not in acts:
            acts[key] = mi.activations(tokens, k, seed=seed + 10 * len(acts), device=DEV,
                                       **({"n_outlier": 0} if key in tame else {}))
        ws.append(mi.llama_like_weight(o, k, seed=seed + 100 + i, dtype=torch.bfloat16, device=DEV))
        xs.append(acts[key])
    return names, ws, xs


def blocks_like(n_blocks, tokens, hidden, ffn, seed, tame=()):
    """Several such blocks one after the other (the call works in groups of up to 8 layers, so
    three blocks span three groups whose borders fall inside blocks)."""
    ws, xs = [], []
    for b in range(n_blocks):
        _, w, x = block_like(tokens, hidden, ffn, seed + 1000 * b, tame)
        ws += w
        xs += x
    return ws, xs


def alloc_outs(mq, ws, xs, cfg, with_x=True):
    xcfg = mq.Cfg(mq.PER_TENSOR, mi.clip_ratios(1))
    w_out = [mq.alloc_qbuffers(w.shape[0], w.shape[1], 8, cfg, DEV) for w in ws]
    x_out = [mq.alloc_qbuffers(x.shape[0], x.shape[1], 8, xcfg, DEV) for x in xs] if with_x else None
    return w_out, x_out


def run_batched(mq, ws, xs, cands, metric, cfg, with_x=True, reps=1):
    w_out, x_out = alloc_outs(mq, ws, xs, cfg, with_x)
    batch = mq.WaLayerBatch(ws, xs, w_out, x_out)
    n = batch.workspace_bytes(len(cands), metric, cfg)
    assert n > 0
    wsp = torch.empty(n, dtype=torch.uint8, device=DEV)
    res = mq.alloc_result(DEV, len(ws))
    for _ in range(reps):
        mq.select_layers_wa(batch, cands, metric, cfg, res, wsp)
    torch.cuda.synchronize()
    return mq.read_results(res), w_out, x_out


def run_single(mq, ws, xs, cands, metric, cfg):
    w_out, x_out = alloc_outs(mq, ws, xs, cfg)
    res = mq.alloc_result(DEV, len(ws))
    for i, (w, x) in enumerate(zip(ws, xs)):
        wsp = torch.empty(mq.workspace_bytes(w, x, len(cands), metric, cfg), dtype=torch.uint8, device=DEV)
        mq.select_layer(w, x, cands, metric, cfg, w_out[i], x_out[i], res[i], wsp)
    torch.cuda.synchronize()
    return mq.read_results(res), w_out, x_out


def same_outputs(a, b, with_x=True):
    ra, wa, xa = a
    rb, wb, xb = b
    for i in range(len(ra)):
        assert ra[i].best == rb[i].best and ra[i].n == rb[i].n, i
        assert list(ra[i].err) == list(rb[i].err) and ra[i].ref_energy == rb[i].ref_energy, i
        assert torch.equal(wa[i].codes, wb[i].codes) and torch.equal(wa[i].scales, wb[i].scales), i
        assert torch.equal(wa[i].unit_err, wb[i].unit_err) and torch.equal(wa[i].clip_idx, wb[i].clip_idx), i
        if with_x:
            assert torch.equal(xa[i].codes, xb[i].codes) and torch.equal(xa[i].scales, xb[i].scales), i
            assert torch.equal(xa[i].unit_err, xb[i].unit_err), i


def against_oracle(mq, got, ws, xs, cands, w_gran, exact=True):
    r, w_out, x_out = got
    for i, (w, x) in enumerate(zip(ws, xs)):
        ref = orc.select_layer_wa(mi.to_f32_numpy(x), mi.to_f32_numpy(w), cands, w_gran)
        print(f"[layer {i}] W={tuple(w.shape)} best={r[i].best} oracle={ref.best}", flush=True)
        assert r[i].n == len(cands)
        if exact:
            assert np.allclose(list(r[i].err)[:len(cands)], ref.errs, rtol=E_RTOL, atol=1e-300), (list(r[i].err), ref.errs)
        assert np.isclose(r[i].ref_energy, ref.ref_energy, rtol=E_RTOL)
        assert r[i].best == ref.best
        assert np.array_equal(unpack_codes(w_out[i].codes, *w.shape, 8), ref.w.codes)
        assert np.array_equal(scales_to_f32(w_out[i].scales), ref.w.scale)
        assert np.allclose(w_out[i].unit_err.cpu().numpy(), ref.w.unit_err, rtol=1e-9, atol=1e-300)
        assert int(w_out[i].clip_idx.cpu()[0]) == 0
        if x_out is not None:
            assert np.array_equal(unpack_codes(x_out[i].codes, *x.shape, 8), ref.x.codes)
            assert np.array_equal(scales_to_f32(x_out[i].scales), ref.x.scale)
            assert np.allclose(x_out[i].unit_err.cpu().numpy(), ref.x.unit_err, rtol=1e-9, atol=1e-300)


@pytest.mark.parametrize("cands", [[I8, FP8], [FP8, I8]])
def test_block_against_oracle_both_formats_win(mq, cands):
    """A block whose attention input is tame (INT8 wins on q, k, v: their codes are copied
    over the E4M3 codes the quantize pass left in the output buffer) and whose other
    activations have outlier channels (E4M3 wins: the codes are already in place)."""
    ws, xs = blocks_like(2, 200, 256, 704, seed=7000, tame=("attn_in",))
    cfg = mq.Cfg(orc.PER_TENSOR, mi.clip_ratios(1))
    print(f"[case] two blocks cands={cands}", flush=True)
    got = run_batched(mq, ws, xs, cands, mq.ERR_LAYER_OUTPUT, cfg, reps=2)
    against_oracle(mq, got, ws, xs, cands, orc.PER_TENSOR)
    chosen = [cands[r.best] for r in got[0]]
    print("chosen formats:", chosen, flush=True)
    assert FP8 in chosen


def test_int8_wins_and_its_codes_replace_the_e4m3_codes(mq):
    """Small-integer operands: the INT8 product is exact (error exactly 0), so INT8 is chosen
    in every layer and its codes -- the integers themselves -- must end up in the output
    buffers, which hold the E4M3 codes until the select."""
    g = torch.Generator().manual_seed(11)
    shapes = [(150, 192), (170, 192), (130, 192), (192, 320)] * 3
    tokens = 140
    xs_f, ws_f = {}, []
    for o, k in shapes:
        if k not in xs_f:
            x = torch.randint(-5, 6, (tokens, k), generator=g).float()
            x[0, 0] = 127.0
            xs_f[k] = x
        w = torch.randint(-5, 6, (o, k), generator=g).float()
        w[0, 0] = -127.0
        ws_f.append(w)
    ws = [w.to(torch.bfloat16).to(DEV) for w in ws_f]
    xdev = {k: x.to(torch.bfloat16).to(DEV) for k, x in xs_f.items()}
    xs = [xdev[k] for _, k in shapes]
    cfg = mq.Cfg(orc.PER_TENSOR, mi.clip_ratios(1))
    r, w_out, x_out = run_batched(mq, ws, xs, [FP8, I8], mq.ERR_LAYER_OUTPUT, cfg, reps=2)
    for i, (o, k) in enumerate(shapes):
        y = xs_f[k].double() @ ws_f[i].double().T
        assert r[i].best == 1 and r[i].err[1] == 0.0 and r[i].err[0] > 0.0
        assert r[i].ref_energy == float((y * y).sum())
        assert np.array_equal(unpack_codes(w_out[i].codes, o, k, 8).astype(np.int8), ws_f[i].numpy().astype(np.int8))
        assert np.array_equal(unpack_codes(x_out[i].codes, tokens, k, 8).astype(np.int8), xs_f[k].numpy().astype(np.int8))
        assert float(w_out[i].scales.cpu()[0]) == 1.0 and float(x_out[i].scales.cpu()[0]) == 1.0
        assert float(w_out[i].unit_err.cpu()[0]) == 0.0


@pytest.mark.parametrize("metric_name", ["ERR_LAYER_OUTPUT", "ERR_LAYER_OUTPUT_FP8_UNIT"])
def test_batched_equals_single_calls(mq, metric_name):
    """One call for three blocks gives bit for bit what 21 mofq_select_layer calls give (ragged
    tile edges, a clip ratio below 1 for W; the partial error sums of a tensor do not depend on
    how many tensors share its launch)."""
    metric = getattr(mq, metric_name)
    ws, xs = blocks_like(3, 130, 320, 576, seed=7100, tame=("mlp_in",))
    cfg = mq.Cfg(orc.PER_TENSOR, np.array([0.9], dtype=np.float32))
    print(f"[case] batched == single, {metric_name}", flush=True)
    single = run_single(mq, ws, xs, [I8, FP8], metric, cfg)
    same_outputs(run_batched(mq, ws, xs, [I8, FP8], metric, cfg, reps=2), single)


def test_fp8_unit_block_decisions_and_codes(mq):
    names, ws, xs = block_like(200, 256, 704, seed=7200, tame=("attn_out",))
    cfg = mq.Cfg(orc.PER_TENSOR, mi.clip_ratios(1))
    got = run_batched(mq, ws, xs, [I8, FP8], mq.ERR_LAYER_OUTPUT_FP8_UNIT, cfg)
    # with the activations' outlier columns split off into an exact K step, the E4M3 product on
    # the fp8 matrix cores meets the same tolerance as the exact form
    against_oracle(mq, got, ws, xs, [I8, FP8], orc.PER_TENSOR, exact=True)


def test_without_activation_outputs(mq):
    names, ws, xs = block_like(96, 128, 192, seed=7300)
    cfg = mq.Cfg(orc.PER_TENSOR, mi.clip_ratios(1))
    a = run_batched(mq, ws, xs, [I8, FP8], mq.ERR_LAYER_OUTPUT, cfg, with_x=False)
    b = run_single(mq, ws, xs, [I8, FP8], mq.ERR_LAYER_OUTPUT, cfg)
    same_outputs(a, b, with_x=False)


@pytest.mark.parametrize("cands,w_gran", [([I8, FP8], orc.PER_CHANNEL), ([FP8], orc.PER_TENSOR), ([I8, FP8, I8], orc.PER_TENSOR)])
def test_general_path_inside_the_batched_call(mq, cands, w_gran):
    """Per-channel weight scales and candidate lists other than the format pair go layer by
    layer through the general path: same results as the single calls, and the oracle's."""
    names, ws, xs = block_like(100, 128, 256, seed=7400, tame=("attn_in",))
    cfg = mq.Cfg(w_gran, mi.clip_ratios(1))
    got = run_batched(mq, ws, xs, cands, mq.ERR_LAYER_OUTPUT, cfg)
    same_outputs(got, run_single(mq, ws, xs, cands, mq.ERR_LAYER_OUTPUT, cfg))
    r, w_out, x_out = got
    for i, (w, x) in enumerate(zip(ws, xs)):
        ref = orc.select_layer_wa(mi.to_f32_numpy(x), mi.to_f32_numpy(w), cands, w_gran)
        assert r[i].best == ref.best
        assert np.allclose(list(r[i].err)[:len(cands)], ref.errs, rtol=E_RTOL, atol=1e-300)
        assert np.array_equal(unpack_codes(w_out[i].codes, *w.shape, 8), ref.w.codes)


def test_argument_errors(mq):
    names, ws, xs = block_like(64, 128, 128, seed=7500)
    cfg = mq.Cfg(orc.PER_TENSOR, mi.clip_ratios(1))
    w_out, x_out = alloc_outs(mq, ws, xs, cfg)
    batch = mq.WaLayerBatch(ws, xs, w_out, x_out)
    res = mq.alloc_result(DEV, len(ws))
    need = batch.workspace_bytes(2, mq.ERR_LAYER_OUTPUT, cfg)
    small = torch.empty(need - 256, dtype=torch.uint8, device=DEV)
    with pytest.raises(mq.MofqError) as e:
        mq.select_layers_wa(batch, [I8, FP8], mq.ERR_LAYER_OUTPUT, cfg, res, small)
    assert e.value.status == -4
    big = torch.empty(need, dtype=torch.uint8, device=DEV)
    with pytest.raises(mq.MofqError) as e:      # the tensor-error metric has its own entry point
        mq.select_layers_wa(batch, [I8, FP8], mq.ERR_TENSOR, cfg, res, big)
    assert e.value.status == -1
    with pytest.raises(mq.MofqError) as e:      # 4-bit candidates have no matrix-core path
        mq.select_layers_wa(batch, [orc.INT4, orc.FP4_E2M1], mq.ERR_LAYER_OUTPUT, cfg, res, big)
    assert e.value.status == -2
    x_wrong = mi.activations(64, 256, seed=1, device=DEV)
    bad = mq.WaLayerBatch(ws, xs[:-1] + [x_wrong], w_out, x_out[:-1] + [mq.alloc_qbuffers(64, 256, 8, cfg, DEV)])
    with pytest.raises(mq.MofqError) as e:      # inner dimensions of the last layer differ
        mq.select_layers_wa(bad, [I8, FP8], mq.ERR_LAYER_OUTPUT, cfg, res, big)
    assert e.value.status == -1
    torch.cuda.synchronize()


@pytest.mark.parametrize("seed", range(6))
def test_random_batches_equal_single_calls_and_oracle(mq, seed):
    """Random layer lists (1 to 20 layers, so up to three groups), random shapes, activations
    shared by runs of consecutive layers, some tensors as views with rows further apart than
    their length: the batched call equals the single calls bit for bit, and one layer of each
    list is held to the oracle."""
    rng = np.random.default_rng(8100 + seed)
    n_layers = int(rng.integers(1, 21))
    tokens = int(rng.integers(1, 300))
    ws, xs = [], []
    x = None
    for i in range(n_layers):
        k = 64 * int(rng.integers(1, 12))
        if x is None or x.shape[1] != k or rng.random() < 0.5:
            pad = 64 if rng.random() < 0.3 else 0
            full = mi.activations(tokens, k + pad, seed=int(rng.integers(1 << 30)), device=DEV,
                                  n_outlier=int(rng.integers(0, 7)))
            x = full[:, :k]                      # rows `k + pad` elements apart
        o = int(rng.integers(1, 400))
        pad = 8 * int(rng.integers(0, 3))
        wfull = mi.llama_like_weight(o, k + pad, seed=int(rng.integers(1 << 30)), dtype=torch.bfloat16, device=DEV)
        ws.append(wfull[:, :k])
        xs.append(x)
    cands = [[I8, FP8], [FP8, I8]][int(rng.integers(2))]
    metric = [mq.ERR_LAYER_OUTPUT, mq.ERR_LAYER_OUTPUT_FP8_UNIT][int(rng.integers(2))]
    cfg = mq.Cfg(orc.PER_TENSOR, np.array([float(rng.choice([1.0, 0.75]))], dtype=np.float32))
    print(f"[case] random batch {seed}: {n_layers} layers, {tokens} tokens, cands={cands}, metric={metric}", flush=True)
    got = run_batched(mq, ws, xs, cands, metric, cfg)
    same_outputs(got, run_single(mq, ws, xs, cands, metric, cfg))
    if cfg.c.clip_ratios[0] == 1.0 and metric == mq.ERR_LAYER_OUTPUT:
        i = int(rng.integers(n_layers))
        ref = orc.select_layer_wa(mi.to_f32_numpy(xs[i].contiguous()), mi.to_f32_numpy(ws[i].contiguous()), cands,
                                  orc.PER_TENSOR)
        r, w_out, x_out = got
        assert r[i].best == ref.best
        assert np.allclose(list(r[i].err)[:2], ref.errs, rtol=E_RTOL, atol=1e-300)
        assert np.array_equal(unpack_codes(w_out[i].codes, *ws[i].shape, 8), ref.w.codes)
        assert np.array_equal(unpack_codes(x_out[i].codes, *xs[i].shape, 8), ref.x.codes)


def test_degenerate_layers(mq):
    """Zero activations, zero weights, a one-token one-output layer and on-grid operands, all in
    one call: zero tensors get scale 1 and codes 0 (the degenerate-unit rule), equal errors keep
    the first candidate (Algorithm 1's strict less), and everything equals the oracle."""
    k = 128
    x0 = torch.zeros(40, k, dtype=torch.bfloat16, device=DEV)
    x1 = mi.activations(40, k, seed=8301, device=DEV)
    w0 = torch.zeros(24, k, dtype=torch.bfloat16, device=DEV)
    w1 = mi.llama_like_weight(24, k, seed=8302, dtype=torch.bfloat16, device=DEV)
    xt = mi.activations(1, k, seed=8303, device=DEV)
    wt = mi.llama_like_weight(1, k, seed=8304, dtype=torch.bfloat16, device=DEV)
    g = torch.Generator().manual_seed(3)
    xg = torch.randint(-3, 4, (40, k), generator=g).float()
    wg = torch.randint(-3, 4, (24, k), generator=g).float()
    xg[0, 0] = 127.0
    wg[0, 0] = 127.0
    ws = [w1, w0, w0, wt, wg.to(torch.bfloat16).to(DEV)]
    xs = [x0, x1, x0, xt, xg.to(torch.bfloat16).to(DEV)]
    cfg = mq.Cfg(orc.PER_TENSOR, mi.clip_ratios(1))
    for cands in ([I8, FP8], [FP8, I8]):
        got = run_batched(mq, ws, xs, cands, mq.ERR_LAYER_OUTPUT, cfg)
        r, w_out, x_out = got
        for i in range(len(ws)):
            ref = orc.select_layer_wa(mi.to_f32_numpy(xs[i]), mi.to_f32_numpy(ws[i]), cands, orc.PER_TENSOR)
            print(f"[layer {i}] cands={cands} errs={list(r[i].err)[:2]} oracle={ref.errs} best={r[i].best}/{ref.best}", flush=True)
            assert r[i].best == ref.best
            # A single output is one difference of two nearly equal numbers: the fp32 accumulation
            # of the matrix cores (2^-24 of |Y| per addition) is not averaged out over outputs as it
            # is in a real layer, so the error "sum" of the 1 x 1 layer agrees to 1e-3 only.
            rtol = 1e-3 if xs[i].shape[0] * ws[i].shape[0] == 1 else E_RTOL
            assert np.allclose(list(r[i].err)[:2], ref.errs, rtol=rtol, atol=1e-30)
            assert np.isclose(r[i].ref_energy, ref.ref_energy, rtol=E_RTOL, atol=1e-30)
            assert np.array_equal(unpack_codes(w_out[i].codes, *ws[i].shape, 8), ref.w.codes)
            assert np.array_equal(unpack_codes(x_out[i].codes, *xs[i].shape, 8), ref.x.codes)
            assert np.array_equal(scales_to_f32(w_out[i].scales), ref.w.scale)
            assert np.array_equal(scales_to_f32(x_out[i].scales), ref.x.scale)
        # zero operands: both errors are exactly 0 and the first candidate stays
        for i in (0, 1, 2):
            assert r[i].best == 0 and r[i].err[0] == 0.0 and r[i].err[1] == 0.0 and r[i].ref_energy == 0.0
        assert float(x_out[0].scales.cpu()[0]) == 1.0 and float(w_out[1].scales.cpu()[0]) == 1.0
