"""mofq_select_layer_static (the entry point that allocates nothing: its workspace is an
array inside the library's device image) against mofq_select_layer with a caller workspace:
identical outputs, on two calls in a row of which the second has the smaller input, so
that what the first call left in the shared array cannot leak into the second."""
import ctypes as C

import pytest
import torch

import mofq_inputs as mi

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def mq():
    from paper_2305_12356_amd import binding
    assert torch.cuda.is_available()
    return binding


def _reference(mq, w, cands, cfg, bits):
    out = mq.alloc_qbuffers(w.shape[0], w.shape[1], bits, cfg, DEV)
    res = mq.alloc_result(DEV)
    ws = torch.empty(mq.workspace_bytes(w, None, len(cands), mq.ERR_TENSOR, cfg), dtype=torch.uint8, device=DEV)
    mq.select_layer(w, None, cands, mq.ERR_TENSOR, cfg, out, None, res, ws)
    torch.cuda.synchronize()
    return out, mq.read_result(res)


def _static_raw(mq, w, cands, cfg, out, res):
    """Straight through the C ABI."""
    wd = mq.tensor_desc(w)
    cand = (C.c_int32 * len(cands))(*cands)
    oc = out.c()
    return mq._lib.mofq_select_layer_static(C.byref(wd), cand, len(cands), C.byref(cfg.c), C.byref(oc),
                                            C.c_void_p(res.data_ptr()),
                                            C.c_void_p(torch.cuda.current_stream().cuda_stream))


@pytest.mark.parametrize("gran,group,f16,n_clip", [(1, 0, False, 100), (2, 128, True, 12), (0, 0, False, 3)])
def test_static_workspace_equals_caller_workspace(mq, gran, group, f16, n_clip):
    cands = [mq.INT4, mq.FP4_E2M1]
    cfg = mq.Cfg(gran, mi.clip_ratios(n_clip), group, f16)
    # the larger input first, then a smaller one that reuses the front of the same array
    for i, (rows, cols) in enumerate([(300, 4096), (37, 1024)]):
        w = mi.llama_like_weight(rows, cols, seed=4000 + 10 * gran + i, device=DEV, outlier_frac=2e-3)
        out = mq.alloc_qbuffers(rows, cols, 4, cfg, DEV)
        res = mq.alloc_result(DEV)
        print(f"[case] static workspace gran={gran} shape={rows}x{cols} K={n_clip}", flush=True)
        assert _static_raw(mq, w, cands, cfg, out, res) == 0
        torch.cuda.synchronize()
        r = mq.read_result(res)
        ref_out, ref = _reference(mq, w, cands, cfg, 4)
        assert r.best == ref.best and r.n == ref.n
        assert list(r.err) == list(ref.err) and r.ref_energy == ref.ref_energy
        assert torch.equal(out.codes, ref_out.codes) and torch.equal(out.scales, ref_out.scales)
        assert torch.equal(out.clip_idx, ref_out.clip_idx) and torch.equal(out.unit_err, ref_out.unit_err)


def test_static_workspace_rejects_what_does_not_fit(mq):
    # 8 MiB hold about 200 000 per-channel units with two candidates: 262144 rows do not fit
    rows, cols = 262144, 64
    w = torch.zeros(rows, cols, dtype=torch.float16, device=DEV)
    cfg = mq.Cfg(mq.PER_CHANNEL, mi.clip_ratios(1))
    assert mq.workspace_bytes(w, None, 2, mq.ERR_TENSOR, cfg) > mq.STATIC_WORKSPACE_BYTES
    out = mq.alloc_qbuffers(rows, cols, 4, cfg, DEV)
    res = mq.alloc_result(DEV)
    with pytest.raises(mq.MofqError) as e:
        mq.select_layer_static(w, [mq.INT4, mq.FP4_E2M1], cfg, out, res)
    assert e.value.status == -4
    torch.cuda.synchronize()
    # and one candidate of the same tensor fits (the limit is on the bytes needed, not on the shape)
    assert mq.workspace_bytes(w, None, 1, mq.ERR_TENSOR, cfg) <= mq.STATIC_WORKSPACE_BYTES
    mq.select_layer_static(w, [mq.INT4], cfg, out, res)
    torch.cuda.synchronize()
    assert mq.read_result(res).err[0] == 0.0
