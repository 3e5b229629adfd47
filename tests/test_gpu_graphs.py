"""The library's calls only enqueue kernels (and, with a side stream, an event fork / join): they
can be recorded into a HIP graph and replayed.  Every replay must give what the eager call gave,
with eager work and synchronisations of the program between the replays."""
import pytest
import torch

import mofq_inputs as mi
from oracle import mofq_oracle as orc

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
CANDS4 = [orc.INT4, orc.FP4_E2M1]
CANDS8 = [orc.INT8, orc.FP8_E4M3]


@pytest.fixture(scope="module")
def mq():
    from paper_2305_12356_amd import binding
    assert torch.cuda.is_available()
    return binding


def replays_equal_eager(name, run, outs, res, n_replays=3):
    """run(stream) enqueues the call; outs are QBuffers whose codes and scales it writes."""
    print(f"[case] graph capture of {name}", flush=True)
    run(torch.cuda.current_stream())
    torch.cuda.synchronize()
    want_res = res.clone()
    want = [(o.codes.clone(), o.scales.clone()) for o in outs]
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(s):
        with torch.cuda.graph(g, stream=s):
            run(s)
    scratch = torch.empty(1 << 20, dtype=torch.float32, device=DEV)
    for rep in range(n_replays):
        res.zero_()
        for o in outs:
            o.codes.zero_()
            o.scales.zero_()
        scratch.normal_()                 # eager work of the program between the replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(res, want_res), (name, rep)
        for o, (c, sc) in zip(outs, want):
            assert torch.equal(o.codes, c) and torch.equal(o.scales, sc), (name, rep)


def test_weight_only_calls_in_a_graph(mq):
    cfg = mq.Cfg(mq.PER_CHANNEL, mi.clip_ratios(100))
    shapes = [(64, 4096), (48, 4096), (40, 11008), (32, 2048)]
    ws = [mi.llama_like_weight(r, c, seed=8400 + i, device=DEV) for i, (r, c) in enumerate(shapes)]
    out = mq.alloc_qbuffers(*shapes[0], 4, cfg, DEV)
    res = mq.alloc_result(DEV)
    wsp = torch.empty(mq.workspace_bytes(ws[0], None, 2, mq.ERR_TENSOR, cfg), dtype=torch.uint8, device=DEV)
    replays_equal_eager("mofq_select_layer", lambda s: mq.select_layer(ws[0], None, CANDS4, mq.ERR_TENSOR, cfg, out, None, res, wsp, s),
                        [out], res)
    # the workspace-free form (its first, eager call looks the built-in workspace up)
    replays_equal_eager("mofq_select_layer_static", lambda s: mq.select_layer_static(ws[0], CANDS4, cfg, out, res, s), [out], res)
    outs = [mq.alloc_qbuffers(r, c, 4, cfg, DEV) for r, c in shapes]
    batch = mq.LayerBatch(ws, outs)
    res_n = mq.alloc_result(DEV, len(ws))
    ws_n = torch.empty(batch.workspace_bytes(2, cfg), dtype=torch.uint8, device=DEV)
    replays_equal_eager("mofq_select_layers", lambda s: mq.select_layers(batch, CANDS4, cfg, res_n, ws_n, s), outs, res_n)
    side = torch.cuda.Stream()
    replays_equal_eager("mofq_select_layers with a side stream",
                        lambda s: mq.select_layers(batch, CANDS4, cfg, res_n, ws_n, s, side_stream=side), outs, res_n)


@pytest.mark.parametrize("metric_name", ["ERR_LAYER_OUTPUT", "ERR_LAYER_OUTPUT_FP8_UNIT"])
def test_weight_activation_call_in_a_graph(mq, metric_name):
    metric = getattr(mq, metric_name)
    ws = [mi.llama_like_weight(o, 256, seed=8500 + i, dtype=torch.bfloat16, device=DEV) for i, o in enumerate([256, 256, 320, 128])]
    x = mi.activations(200, 256, seed=8510, device=DEV)
    xs = [x, x, x, mi.activations(200, 256, seed=8511, device=DEV)]
    cfg = mq.Cfg(mq.PER_TENSOR, mi.clip_ratios(1))
    w_out = [mq.alloc_qbuffers(w.shape[0], w.shape[1], 8, cfg, DEV) for w in ws]
    x_out = [mq.alloc_qbuffers(a.shape[0], a.shape[1], 8, cfg, DEV) for a in xs]
    batch = mq.WaLayerBatch(ws, xs, w_out, x_out)
    wsp = torch.empty(batch.workspace_bytes(2, metric, cfg), dtype=torch.uint8, device=DEV)
    res = mq.alloc_result(DEV, len(ws))
    replays_equal_eager(f"mofq_select_layers_wa ({metric_name})",
                        lambda s: mq.select_layers_wa(batch, CANDS8, metric, cfg, res, wsp, s), w_out + x_out, res)
