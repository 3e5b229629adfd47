"""The batched weight-only select (mofq_select_layers) must give, tensor by tensor, exactly
what mofq_select_layer gives (which the other tests hold to the oracle), and is also
compared with the oracle directly on a few tensors."""
import numpy as np
import pytest
import torch

import mofq_inputs as mi
from oracle import mofq_oracle as orc
from tests.gpu_util import compare_quantized, scales_to_f32, unpack_codes

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


@pytest.fixture(scope="module")
def mq():
    from paper_2305_12356_amd import binding
    assert torch.cuda.is_available()
    return binding


def _single(mq, w, cands, cfg, bits):
    out = mq.alloc_qbuffers(w.shape[0], w.shape[1], bits, cfg, DEV)
    res = mq.alloc_result(DEV)
    ws = torch.empty(mq.workspace_bytes(w, None, len(cands), mq.ERR_TENSOR, cfg), dtype=torch.uint8, device=DEV)
    mq.select_layer(w, None, cands, mq.ERR_TENSOR, cfg, out, None, res, ws)
    torch.cuda.synchronize()
    return out, mq.read_result(res)


@pytest.mark.parametrize("gran,group,f16,n_clip", [(orc.PER_CHANNEL, 0, False, 100), (orc.PER_CHANNEL, 0, True, 1),
                                                   (orc.PER_GROUP, 128, True, 12), (orc.PER_TENSOR, 0, False, 3)])
@pytest.mark.parametrize("two_streams", [False, True, "same"])
def test_batched_equals_single(mq, gran, group, f16, n_clip, two_streams):
    # more than four batches, mixed shapes; group-wise ones above the per-launch unit limit too;
    # runs of one shape (tensors of one row length in a batch are searched in one launch: 4, 2,
    # and 11 = more than a launch takes), one of
    # them with a member of another dtype and one with a member whose rows are strided
    shapes = [(7, 1024), (64, 4096), (3, 256), (300, 2048), (17, 11008)] * 5 + [(200, 12288), (5, 512), (1, 8 * 40), (130, 1536)]
    shapes += [(64, 4096)] * 4 + [(17, 11008)] * 2 + [(3, 256)] * 11 + [(33, 2048)] * 3 + [(9, 1024)] * 3
    shapes = [(r, c) for r, c in shapes if gran != orc.PER_GROUP or c % group == 0]
    ws_ = [mi.llama_like_weight(r, c, seed=700 + i, device=DEV, outlier_frac=2e-3) for i, (r, c) in enumerate(shapes)]
    mid33 = [i for i, sh in enumerate(shapes) if sh == (33, 2048)][1]
    ws_[mid33] = ws_[mid33].to(torch.bfloat16)
    mid9 = [i for i, sh in enumerate(shapes) if sh == (9, 1024)][1]
    ws_[mid9] = torch.cat([ws_[mid9], ws_[mid9]], dim=1)[:, :1024]      # row stride 2048
    assert ws_[mid9].stride(0) == 2048
    cands = [mq.INT4, mq.FP4_E2M1]
    cfg = mq.Cfg(gran, mi.clip_ratios(n_clip), group, f16)
    outs = [mq.alloc_qbuffers(r, c, 4, cfg, DEV) for r, c in shapes]
    batch = mq.LayerBatch(ws_, outs)
    results = mq.alloc_result(DEV, len(shapes))
    ws = torch.empty(batch.workspace_bytes(2, cfg), dtype=torch.uint8, device=DEV)
    e0 = [torch.cuda.Event(enable_timing=True) for _ in shapes]
    e1 = [torch.cuda.Event(enable_timing=True) for _ in shapes]
    side = {False: None, True: torch.cuda.Stream(), "same": torch.cuda.current_stream()}[two_streams]
    mq.select_layers(batch, cands, cfg, results, ws, None, e0, e1, side_stream=side)
    # the caller's stream alone orders what follows: copies enqueued on it right away must see
    # the finished outputs, whichever stream wrote them
    snap = [(o.codes.clone(), o.scales.clone(), o.clip_idx.clone(), o.unit_err.clone()) for o in outs]
    results_snap = results.clone()
    torch.cuda.synchronize()
    # events bracket each search launch: begin of its first tensor, end of its last
    first = batch.search_groups(cands)
    assert all(f <= i and first[f] == f and i - f < 12 for i, f in enumerate(first))
    assert all(ws_[i].shape[1] == ws_[f].shape[1] and ws_[i].dtype == ws_[f].dtype for i, f in enumerate(first))
    last = {f: i for i, f in enumerate(first)}
    assert all(first.count(f) <= 8 for f in last)
    assert max(first.count(f) for f in last) >= 4
    assert all(e0[f].elapsed_time(e1[l]) >= 0.0 for f, l in last.items())
    res = mq.read_results(results_snap)
    for i, w in enumerate(ws_):
        ref_out, ref_res = _single(mq, w, cands, cfg, 4)
        assert res[i].best == ref_res.best and list(res[i].err) == list(ref_res.err)
        assert res[i].ref_energy == ref_res.ref_energy
        assert torch.equal(snap[i][0], ref_out.codes)
        assert torch.equal(snap[i][1], ref_out.scales)
        assert torch.equal(snap[i][2], ref_out.clip_idx)
        assert torch.equal(snap[i][3], ref_out.unit_err)
    # and against the oracle, directly
    for i in (0, 3, len(shapes) - 1):
        w32 = mi.to_f32_numpy(ws_[i])
        clip = mi.clip_ratios(n_clip)
        ref = orc.select_layer_w_only(w32, cands, gran, clip, group, f16, want_table=True)
        assert res[i].best == ref.best
        compare_quantized(w32, cands[ref.best], gran, group, f16, clip, ref.w,
                          unpack_codes(outs[i].codes, *shapes[i], 4), scales_to_f32(outs[i].scales),
                          outs[i].clip_idx.cpu().numpy(), outs[i].unit_err.cpu().numpy())


def test_batched_rejects_before_enqueueing(mq):
    w = [mi.llama_like_weight(8, 256, seed=1, device=DEV), mi.llama_like_weight(8, 252, seed=2, device=DEV)]
    cfg = mq.Cfg(mq.PER_CHANNEL, mi.clip_ratios(2))
    outs = [mq.alloc_qbuffers(8, 256, 4, cfg, DEV), mq.alloc_qbuffers(8, 256, 4, cfg, DEV)]
    batch = mq.LayerBatch(w, outs)
    assert batch.workspace_bytes(2, cfg) > 0       # sizes alone are fine; the 252 columns are not
    results = mq.alloc_result(DEV, 2)
    ws = torch.empty(1 << 20, dtype=torch.uint8, device=DEV)
    with pytest.raises(mq.MofqError):        # second tensor: 252 columns is not a multiple of 8
        mq.select_layers(batch, [mq.INT4, mq.FP4_E2M1], cfg, results, ws)
    torch.cuda.synchronize()


@pytest.mark.parametrize("cands_name", ["int4,fp4,ieee", "int4,fp4,ieee,int4", "fp4,fp4,int4", "int8,e4m3,e5m2"])
def test_batched_three_and_four_candidates(mq, cands_name):
    """Candidate lists longer than one search launch takes (two formats): every tensor goes
    through launches of at most two formats; results equal the single-tensor call and the
    oracle, tensor by tensor."""
    fmt = {"int4": mq.INT4, "fp4": mq.FP4_E2M1, "ieee": mq.FP4_E2M1_IEEE, "int8": mq.INT8,
           "e4m3": mq.FP8_E4M3, "e5m2": mq.FP8_E5M2}
    cands = [fmt[c] for c in cands_name.split(",")]
    bits = 8 if cands[0] in (mq.INT8, mq.FP8_E4M3, mq.FP8_E5M2) else 4
    shapes = [(40, 4096), (12, 1024), (40, 4096), (9, 11008), (40, 4096)]
    ws_ = [mi.llama_like_weight(r, c, seed=900 + i, device=DEV, outlier_frac=2e-3) for i, (r, c) in enumerate(shapes)]
    clip = mi.clip_ratios(10)
    cfg = mq.Cfg(mq.PER_CHANNEL, clip)
    outs = [mq.alloc_qbuffers(r, c, bits, cfg, DEV) for r, c in shapes]
    batch = mq.LayerBatch(ws_, outs)
    assert batch.search_groups(cands) == list(range(len(shapes)))     # nothing is joined
    results = mq.alloc_result(DEV, len(shapes))
    ws = torch.empty(batch.workspace_bytes(len(cands), cfg), dtype=torch.uint8, device=DEV)
    print(f"[case] select_layers with candidates {cands_name}", flush=True)
    mq.select_layers(batch, cands, cfg, results, ws, side_stream=torch.cuda.Stream())
    torch.cuda.synchronize()
    res = mq.read_results(results)
    for i, w in enumerate(ws_):
        ref_out, ref_res = _single(mq, w, cands, cfg, bits)
        assert res[i].n == len(cands)
        assert res[i].best == ref_res.best and list(res[i].err) == list(ref_res.err)
        assert torch.equal(outs[i].codes, ref_out.codes) and torch.equal(outs[i].scales, ref_out.scales)
        assert torch.equal(outs[i].clip_idx, ref_out.clip_idx) and torch.equal(outs[i].unit_err, ref_out.unit_err)
        w32 = mi.to_f32_numpy(w)
        ref = orc.select_layer_w_only(w32, cands, orc.PER_CHANNEL, clip, want_table=True)
        assert res[i].best == ref.best
        assert np.allclose(list(res[i].err)[:len(cands)], ref.errs, rtol=1e-9)
        compare_quantized(w32, cands[ref.best], orc.PER_CHANNEL, 0, False, clip, ref.w,
                          unpack_codes(outs[i].codes, *shapes[i], bits), scales_to_f32(outs[i].scales),
                          outs[i].clip_idx.cpu().numpy(), outs[i].unit_err.cpu().numpy())
