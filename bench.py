#!/usr/bin/env python3
"""Benchmark of the MoFQ weight-only hot path on one MI355X.

Workload (`config.workload`): the LLaMA-7B-shaped weight set, fp16, 32 blocks x 7
linears = 224 tensors, 4-bit weight-only, per-channel scales searched over 100
clip ratios in [0.5, 1], INT4 vs FP4-E2M1, per-layer select and emit of the codes.
A step is one pass of the whole path (scale search + select + emit) over all 224
tensors, which are resident in HBM before the timed region starts.

Prints ONE JSON line: the elements x candidates scored per second (and the
full-model select time), the roofline of the dominant kernel measured with HIP
events inside the timed region, and the CPU oracle timed on a bounded sample of
the same workload on the host cores.

`--workload` selects two further workloads of the same path, each with its own
JSON line (same keys; no CPU baseline): `w4_group128` (group-wise scales, 50 clip
ratios) and `w8a8` (weight-activation, layer-output error through the matrix
cores, 2048 tokens).  `k1_hbm` is the memory-bound case: configs[0]'s recipe (fp32,
absmax scale, no clip search) on a 16384 x 16384 tensor (1 GiB).  The default,
`w4_channel`, is the headline workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

N_CLIP = 100
N_CLIP_GROUP = 50
GROUP = 128
TOKENS = 2048
N_FMT = 2
# Published dense matrix-core peaks (TFLOP/s or TOP/s) per operand type.
MFMA_PEAK = {"bf16": 2500.0, "int8": 5000.0, "fp8": 5000.0}
# Algorithmic work of the scale search per element, candidate and format: scale
# (1 multiply), round (1), clamp/saturate (1), residual x - g*s (2), error
# accumulation d*d + acc (2).
FLOPS_PER_ELEM_CAND_FMT = 7
# Vector-ALU peak the exhaustive search is priced against.  Of the 7 flop, 3 are fp32
# (published fp32 vector peak 157.3 TFLOP/s) and 4 are fp64 (published fp64 vector peak
# 78.6 TFLOP/s): 7 / (3/157.3 + 4/78.6) = 100.0 TFLOP/s.
ALU_PEAK_TFLOPS = 7.0 / (3.0 / 157.3 + 4.0 / 78.6)
# HBM bytes per launch of the search kernel from rocprofv3 FETCH_SIZE / WRITE_SIZE runs of this command,
# scaled by what the same counters read for a plain 1 GiB copy (profiles/w_only_7b_k100_hbm_traffic.txt):
# a launch over 46592 rows of 4096 fp16 columns reads 373 230 KiB (1.0013 x its 2 bytes per element) and
# writes 10 192 KiB (224 bytes of per-channel records per row).  Only the 7B per-channel workload has
# been measured.
MEASURED_READ_PER_INPUT_BYTE = 373230.0 / (46592 * 4096 * 2 / 1024)
MEASURED_WRITE_BYTES_PER_ROW = 10192.0 * 1024 / 46592


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=8)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--model", default="7b", choices=["7b", "65b"],
                    help="65b = configs[4]: 560 linears, 129.5 GB of fp16 weights resident in HBM")
    ap.add_argument("--workload", default="w4_channel",
                    choices=["w4_channel", "w4_group128", "w8a8", "w4a16_output", "k1_hbm", "fp4_variants", "w4_units"])
    ap.add_argument("--fp8-unit", action="store_true",
                    help="w8a8: E4M3 code product on the fp8 matrix cores (not within 1e-5 of the exact sum)")
    ap.add_argument("--blocks", type=int, default=0, help="debug: use only the first N blocks")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--single-stream", action="store_true",
                    help="w4_channel: no second stream (kernels run one at a time; for counter runs)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy (reference for rocprofv3 byte counters)")
    return ap.parse_args()


def cpu_baseline(weights, outs, clip, cands):
    """Time the oracle (as it stands) on a bounded sample of the same tensors and
    check the library's results on those rows against it."""
    import numpy as np
    import mofq_inputs as mi
    from oracle import mofq_oracle as orc
    from tests.gpu_util import compare_quantized, scales_to_f32

    # rows of block 0: q (4096 cols), gate (4096 cols), down (11008 cols)
    plan = [(0, 4096), (4, 3072), (6, 2048)]     # about 11 s of oracle time on 16 host threads
    threads = orc.max_threads()
    total_ec, total_t, checked, band = 0, 0.0, 0, 0
    desc = []
    for idx, n_rows in plan:
        w_dev, out, res = weights[idx], outs[idx][0], outs[idx][1]
        n_rows = min(n_rows, w_dev.shape[0])
        cols = w_dev.shape[1]
        w32 = mi.to_f32_numpy(w_dev[:n_rows])
        t0 = time.perf_counter()
        ref = [orc.quantize(w32, f, orc.PER_CHANNEL, clip, want_table=True, threads=threads)
               for f in cands]
        total_t += time.perf_counter() - t0
        total_ec += n_rows * cols * N_CLIP * N_FMT
        desc.append(f"{n_rows}x{cols}")
        best = res.best
        codes = out.codes[: n_rows * cols // 2].cpu().numpy()
        un = np.empty(n_rows * cols, dtype=np.uint8)
        un[0::2] = codes & 0xF
        un[1::2] = codes >> 4
        band += compare_quantized(w32, cands[best], orc.PER_CHANNEL, 0, False, clip, ref[best],
                                  un.reshape(n_rows, cols), scales_to_f32(out.scales[:n_rows]),
                                  out.clip_idx[:n_rows].cpu().numpy(),
                                  out.unit_err[:n_rows].cpu().numpy())
        checked += n_rows
    return {
        "value": total_ec / total_t, "unit": "elem*cand/s", "cores": threads, "kind": "oracle",
        "sample": "first rows of block 0 q/gate/down (" + ", ".join(desc) +
                  "), both formats x 100 clip ratios, full oracle search",
        "seconds": round(total_t, 3),
        "rows_checked_bit_exact": checked, "near_tie_rows": band,
    }


def run_w8a8(args, shapes, dev, w_only=False):
    """configs[3]: per linear, X [2048, in] bf16 with outlier channels, W bf16; per-tensor
    INT8 vs FP8-E4M3 for both; layer-output error through the matrix cores; select + emit.
    With w_only: the weight-only select by layer-output error (X stays bf16; W per-channel
    absmax scales, INT4 vs FP4-E2M1)."""
    import torch

    import mofq_inputs as mi
    from paper_2305_12356_amd import binding as mq

    metric = mq.ERR_LAYER_OUTPUT_FP8_UNIT if args.fp8_unit else mq.ERR_LAYER_OUTPUT
    cands = [mq.INT8, mq.FP8_E4M3]
    cfg = mq.Cfg(mq.PER_TENSOR, mi.clip_ratios(1))
    bits = 8
    if w_only:
        metric, cands, bits = mq.ERR_LAYER_OUTPUT_W_ONLY, [mq.INT4, mq.FP4_E2M1], 4
        cfg = mq.Cfg(mq.PER_CHANNEL, mi.clip_ratios(1))
    xcfg = mq.Cfg(mq.PER_TENSOR, mi.clip_ratios(1))
    xs = {}
    weights, wouts, xouts = [], [], {}
    results = mq.alloc_result(dev, len(shapes))
    ws_bytes = 0
    for b, name, o, n in shapes:
        if n not in xs:
            xs[n] = mi.activations(TOKENS, n, seed=mi.tensor_seed(3, 0, 0, n), device=dev)
            xouts[n] = None if w_only else mq.alloc_qbuffers(TOKENS, n, 8, xcfg, dev)
        w = mi.llama_like_weight(o, n, seed=mi.tensor_seed(1, b, mi.LINEAR_NAMES.index(name)),
                                 dtype=torch.bfloat16, device=dev)
        weights.append(w)
        ws_bytes = max(ws_bytes, mq.workspace_bytes(w, xs[n], len(cands), metric, cfg))
    # one output buffer per distinct weight shape (the codes are not read back here)
    for b, name, o, n in shapes:
        if (o, n) not in xouts:
            xouts[(o, n)] = mq.alloc_qbuffers(o, n, bits, cfg, dev)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream()

    def step(events=None):
        for i, w in enumerate(weights):
            _, _, o, n = shapes[i]
            e0 = e1 = None
            if events is not None:
                e0 = torch.cuda.Event(enable_timing=True)
                e1 = torch.cuda.Event(enable_timing=True)
                events.append((i, e0, e1))
            mq.select_layer(w, xs[n], cands, metric, cfg, xouts[(o, n)], xouts[n], results[i], ws,
                            stream, e0, e1)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    events = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(events)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / args.steps * 1e3

    # the same pass with the linears dealt alternately to two streams of the caller (own
    # workspace and output buffers per stream): the short memory-bound quantize passes of one
    # linear then run beside the matrix-core kernel of another
    two = [torch.cuda.Stream(), torch.cuda.Stream()]
    ws2 = [ws, torch.empty_like(ws)]
    xo2 = [xouts, {k: (None if v is None else mq.alloc_qbuffers(TOKENS if not isinstance(k, tuple) else k[0],
                                                                 k if not isinstance(k, tuple) else k[1],
                                                                 8 if not isinstance(k, tuple) else bits,
                                                                 xcfg if not isinstance(k, tuple) else cfg, dev))
                   for k, v in xouts.items()}]

    def step2():
        for i, w in enumerate(weights):
            _, _, o, n = shapes[i]
            mq.select_layer(w, xs[n], cands, metric, cfg, xo2[i & 1][(o, n)], xo2[i & 1][n], results[i], ws2[i & 1],
                            two[i & 1])

    for st in two:
        st.wait_stream(stream)
    step2()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step2()
    torch.cuda.synchronize()
    ms_two = (time.perf_counter() - t0) / args.steps * 1e3

    # dominant kernel: the fused three-product GEMM; one launch per linear
    mnk = sum(TOKENS * o * n for _, _, o, n in shapes)
    gemm_time = sum(e0.elapsed_time(e1) for _, e0, e1 in events) * 1e-3 / args.steps
    kinds = ["bf16", "bf16", "bf16"] if w_only else ["bf16", "int8", "fp8" if args.fp8_unit else "bf16"]
    flops = 2.0 * mnk * len(kinds)
    ideal = sum(2.0 * mnk / (MFMA_PEAK[k] * 1e12) for k in kinds)
    achieved = flops / gemm_time / 1e12
    peak = flops / ideal / 1e12
    res = mq.read_results(results)
    out = {
        "metric": ("W4A16" if w_only else "W8A8") + " layer-output MoFQ select time over the LLaMA-7B linear shapes",
        "value": ms_per_step / 1e3, "unit": "s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": False,
        "ms_per_step_two_caller_streams": ms_two,
        "scaling": "weak", "vs_baseline": None,
        "dtype": ("bf16 reference product, 4-bit grid values on the bf16 matrix cores, f64 error sums" if w_only else
                  "bf16 reference product, int8 codes, " +
                  ("fp8 codes on the fp8 matrix cores" if args.fp8_unit else "e4m3 grid values on the bf16 matrix cores") +
                  ", f64 error sums"),
        "data": "synthetic",
        "config": {"workload": (f"weight-only select by layer-output error: {len(shapes)} linears of the LLaMA-7B shape, "
                                f"X [{TOKENS} x in] bf16 unquantized, W bf16, per-channel absmax scales, "
                                "INT4 vs FP4-E2M1, per-layer select + emit") if w_only else
                               (f"configs[3]: {len(shapes)} linears of the LLaMA-7B shape, X [{TOKENS} x in] bf16 "
                                "with 6 outlier channels x60, W bf16, per-tensor INT8 vs FP8-E4M3, "
                                "layer-output error, per-layer select + emit"),
                   "fp8_product": "fp8 matrix cores" if args.fp8_unit else "exact (bf16 matrix cores)",
                   "fp_percent": 100.0 * sum(1 for r in res if r.best == 1) / len(res)},
        "roofline": {
            "bound": "mfma", "achieved": achieved, "peak": peak, "unit": "TFLOP/s",
            "frac": achieved / peak, "traffic": None,
            "kernel": "wa_gemm_kernel (reference, INT8-code and E4M3 products of one linear)",
            "note": "three products per launch, " + " + ".join(kinds) + "; peak is the rate at which the "
                    "three would finish if each ran at the published dense peak of its own type "
                    "(bf16 2.5, int8 5.0, fp8 5.0 PFLOP/s)",
            "gemm_ms_per_step": gemm_time * 1e3, "launches": len(events),
            "flops_per_launch_avg": flops / len(shapes),
        },
    }
    print(json.dumps(out))


def run_k1_hbm(args, dev):
    """configs[0]'s recipe at a size that does not fit in the caches: one 16384 x 16384 fp32
    tensor, per-channel absmax scale (one candidate), INT4 vs FP4-E2M1, select + emit."""
    import torch

    import mofq_inputs as mi
    from paper_2305_12356_amd import binding as mq

    n = 16384
    w = mi.config0_weight(seed=0, rows=n, cols=n, device=dev)
    cfg = mq.Cfg(mq.PER_CHANNEL, mi.clip_ratios(1))
    cands = [mq.INT4, mq.FP4_E2M1]
    out = mq.alloc_qbuffers(n, n, 4, cfg, dev)
    res = mq.alloc_result(dev)
    ws = torch.empty(mq.workspace_bytes(w, None, 2, mq.ERR_TENSOR, cfg), dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream()
    for _ in range(args.warmup):
        mq.select_layer(w, None, cands, mq.ERR_TENSOR, cfg, out, None, res, ws, stream)
    torch.cuda.synchronize()
    events = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        events.append((e0, e1))
        mq.select_layer(w, None, cands, mq.ERR_TENSOR, cfg, out, None, res, ws, stream, e0, e1)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / args.steps * 1e3
    sweep_s = sum(e0.elapsed_time(e1) for e0, e1 in events) * 1e-3 / args.steps
    read_bytes = n * n * 4
    achieved = read_bytes / sweep_s / 1e9
    r = mq.read_result(res)
    print(json.dumps({
        "metric": "weight-elems x candidates scored/sec (memory-bound case: one scale candidate)",
        "value": n * n * N_FMT / (elapsed / args.steps), "unit": "elem*cand/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32 decisions, f64 errors", "data": "synthetic",
        "config": {"workload": "configs[0]'s recipe on a 16384 x 16384 fp32 tensor (1 GiB): N(0, 0.02^2), 0.1 % of "
                               "entries x10, per-channel absmax scale, INT4 vs FP4-E2M1, tensor error, select + emit",
                   "best": int(r.best), "err": [float(r.err[0]), float(r.err[1])]},
        "roofline": {
            "bound": "hbm", "achieved": achieved, "peak": 8000.0, "unit": "GB/s", "frac": achieved / 8000.0,
            # FETCH_SIZE / WRITE_SIZE of this kernel, scaled by a plain copy's (profiles/k1_hbm_fp32_16384_kernel_stats.txt)
            "traffic": (1048666 + 3642) * 1024.0,
            "kernel": "sweep_channel_single_kernel<F32, INT4, FP4_E2M1, 512 threads, 4 chunks>",
            "note": "algorithmic bytes = 4 B per element read once by the scoring kernel; the emit pass "
                    "(4 B read + 0.5 B written per element) is in ms_per_step but not in this kernel",
            "avg_launch_ms": sweep_s * 1e3, "launches": len(events),
            "algorithmic_bytes_per_launch": read_bytes,
            "select_emit_GBps": n * n * 4.5 / (elapsed / args.steps - sweep_s) / 1e9,
        },
    }))


def run_fp4_variants(args, shapes, dev):
    """Section 4.2 in kind, on the synthetic 7B-shaped set: tensor error of the redesigned
    FP4 (Table 1, without NaN/Inf) against the IEEE-aligned FP4, per-channel absmax scales,
    and how many layers prefer each FP4 over INT4."""
    import torch

    import mofq_inputs as mi
    from paper_2305_12356_amd import binding as mq

    cfg = mq.Cfg(mq.PER_CHANNEL, mi.clip_ratios(1))
    sets = {"redesigned": [mq.INT4, mq.FP4_E2M1], "ieee": [mq.INT4, mq.FP4_E2M1_IEEE]}
    results = {k: mq.alloc_result(dev, len(shapes)) for k in sets}
    stream = torch.cuda.current_stream()
    ws = out = None
    t0 = time.perf_counter()
    for i, (b, name, o, n) in enumerate(shapes):
        w = mi.llama_like_weight(o, n, seed=mi.tensor_seed(1, b, mi.LINEAR_NAMES.index(name)), device=dev)
        need = mq.workspace_bytes(w, None, 2, mq.ERR_TENSOR, cfg)
        if ws is None or ws.numel() < need:
            ws = torch.empty(need, dtype=torch.uint8, device=dev)
        out = mq.alloc_qbuffers(o, n, 4, cfg, dev)
        for k, cands in sets.items():
            mq.select_layer(w, None, cands, mq.ERR_TENSOR, cfg, out, None, results[k][i], ws, stream)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    res = {k: mq.read_results(v) for k, v in results.items()}
    e_int = sum(r.err[0] for r in res["redesigned"])
    e_new = sum(r.err[1] for r in res["redesigned"])
    e_ieee = sum(r.err[1] for r in res["ieee"])
    per_layer = [r1.err[1] / r2.err[1] for r1, r2 in zip(res["redesigned"], res["ieee"])]
    print(json.dumps({
        "metric": "tensor error of the redesigned FP4 relative to the IEEE-aligned FP4 (synthetic 7B-shaped weights)",
        "value": e_new / e_ieee, "unit": "ratio", "n_gpus": 1, "steps": 1, "warmup": 0,
        "ms_per_step": elapsed * 1e3, "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32 decisions, f64 errors", "data": "synthetic",
        "config": {"workload": f"{len(shapes)} linears of the LLaMA-7B shape, fp16, per-channel absmax scales (one candidate)",
                   "error_reduction_percent": 100.0 * (1.0 - e_new / e_ieee),
                   "per_layer_ratio_min_max": [min(per_layer), max(per_layer)],
                   "int4_error_relative_to_redesigned_fp4": e_int / e_new,
                   "layers_preferring_fp4_over_int4_percent": {
                       k: 100.0 * sum(1 for r in v if r.best == 1) / len(v) for k, v in res.items()}},
    }))


def run_w4_units(args, shapes, dev):
    """Per-unit format select (finer than the layer) on the 7B-shaped set, group 128 with
    fp16 scales and 50 clip ratios: time, and the tensor error of the mixed assignment
    against the layer-wise choice."""
    import torch

    import mofq_inputs as mi
    from paper_2305_12356_amd import binding as mq

    clip = mi.clip_ratios(N_CLIP_GROUP)
    cfg = mq.Cfg(mq.PER_GROUP, clip, GROUP, True)
    cands = [mq.INT4, mq.FP4_E2M1]
    weights, outs, tags = [], [], []
    results = mq.alloc_result(dev, len(shapes))
    mixed = torch.zeros(len(shapes), dtype=torch.float64, device=dev)
    ws_bytes = 0
    for b, name, o, n in shapes:
        w = mi.llama_like_weight(o, n, seed=mi.tensor_seed(1, b, mi.LINEAR_NAMES.index(name)), device=dev)
        weights.append(w)
        outs.append(mq.alloc_qbuffers(o, n, 4, cfg, dev))
        tags.append(torch.empty(o * (n // GROUP), dtype=torch.uint8, device=dev))
        ws_bytes = max(ws_bytes, mq.select_units_workspace_bytes(w, 2, cfg))
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream()

    def step():
        for i, w in enumerate(weights):
            mq.select_units(w, cands, cfg, outs[i], tags[i], results[i], mixed[i:i + 1], ws, stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    res = mq.read_results(results)
    layer = sum(min(r.err[0], r.err[1]) for r in res)
    mix = float(mixed.sum().item())
    fp_units = sum(int(t.sum().item()) for t in tags)
    n_units = sum(t.numel() for t in tags)
    n_elems = sum(o * n for _, _, o, n in shapes)
    print(json.dumps({
        "metric": "weight-elems x candidates scored/sec, per-unit format select (group 128)",
        "value": n_elems * N_CLIP_GROUP * N_FMT / (elapsed / args.steps), "unit": "elem*cand/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": elapsed / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32 decisions, f64 errors", "data": "synthetic",
        "config": {"workload": f"{len(shapes)} linears of the LLaMA-7B shape, fp16, group 128, fp16 scales, 50 clip "
                               "ratios, INT4 vs FP4-E2M1 chosen per group",
                   "mixed_error_relative_to_layer_wise": mix / layer,
                   "fp4_units_percent": 100.0 * fp_units / n_units},
    }))


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no second device); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import mofq_inputs as mi
    from paper_2305_12356_amd import binding as mq

    if not torch.cuda.is_available():
        print("bench.py needs an MI355X (cuda:0)", file=sys.stderr)
        sys.exit(2)
    dev = "cuda:0"
    torch.cuda.set_device(0)

    shapes = mi.model_linear_shapes(args.model)
    if args.blocks:
        shapes = [s for s in shapes if s[0] < args.blocks]
    if args.workload in ("w8a8", "w4a16_output"):
        run_w8a8(args, shapes, dev, w_only=args.workload == "w4a16_output")
        return
    if args.workload == "k1_hbm":
        run_k1_hbm(args, dev)
        return
    if args.workload == "fp4_variants":
        run_fp4_variants(args, shapes, dev)
        return
    if args.workload == "w4_units":
        run_w4_units(args, shapes, dev)
        return
    group = args.workload == "w4_group128"
    n_clip = N_CLIP_GROUP if group else N_CLIP
    clip = mi.clip_ratios(n_clip)
    cands = [mq.INT4, mq.FP4_E2M1]
    cfg = mq.Cfg(mq.PER_GROUP, clip, GROUP, True) if group else mq.Cfg(mq.PER_CHANNEL, clip)

    # ---- resident inputs and caller-owned outputs ---------------------------------
    weights, qouts = [], []
    results = mq.alloc_result(dev, len(shapes))
    ws_bytes = 0
    for i, (b, name, o, n) in enumerate(shapes):
        w = mi.llama_like_weight(o, n, seed=mi.tensor_seed(1, b, mi.LINEAR_NAMES.index(name)), device=dev)
        weights.append(w)
        qouts.append(mq.alloc_qbuffers(o, n, 4, cfg, dev))
        ws_bytes = max(ws_bytes, mq.workspace_bytes(w, None, len(cands), mq.ERR_TENSOR, cfg))
    # one call for the whole model (mofq_select_layers): the per-tensor reduce / select /
    # per-unit outputs of up to 12 tensors share a launch, and so do the searches of those of
    # them that have one row length
    batch = mq.LayerBatch(weights, qouts)
    ws = torch.empty(batch.workspace_bytes(len(cands), cfg), dtype=torch.uint8, device=dev)
    n_elems = sum(o * n for _, _, o, n in shapes)
    stream = torch.cuda.current_stream()
    # default priority: select + code emission beside the next batch's searches
    side = None if args.single_stream else torch.cuda.Stream()

    # the events the library records around each search launch, created (and recorded once,
    # so that they exist) before the timed region
    ev_pool = []
    for _ in range(args.steps):
        e0 = [torch.cuda.Event(enable_timing=True) for _ in weights]
        e1 = [torch.cuda.Event(enable_timing=True) for _ in weights]
        for e in e0 + e1:
            e.record()
        ev_pool.append((e0, e1))

    def step(events=None):
        e0 = e1 = None
        if events is not None:
            e0, e1 = ev_pool.pop()
            events.extend((i, a, b) for i, (a, b) in enumerate(zip(e0, e1)))
        mq.select_layers(batch, cands, cfg, results, ws, stream, e0, e1, side_stream=side)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    events = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(events)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    ms_per_step = elapsed / args.steps * 1e3
    elem_cand = n_elems * n_clip * N_FMT
    value = elem_cand / (elapsed / args.steps)

    # ---- dominant kernel: the scale-search instance for 4096-column rows ------------
    # (q, k, v, o, gate, up: 78 % of all elements; the tensors of a batch with one row length
    # share a launch).  Duration from the HIP events the library recorded around each launch: the
    # begin event of a launch's first tensor, the end event of its last.
    first = batch.search_groups(cands)
    last = {f: i for i, f in enumerate(first)}
    by_cols = {}
    for step_i in range(args.steps):
        ev = events[step_i * len(shapes):(step_i + 1) * len(shapes)]
        for f, l in last.items():
            elems = sum(shapes[i][2] * shapes[i][3] for i in range(f, l + 1) if first[i] == f)
            by_cols.setdefault(shapes[f][3], []).append((elems, ev[f][1].elapsed_time(ev[l][2]) * 1e-3))
    dom_cols = max(by_cols, key=lambda c: sum(e for e, _ in by_cols[c]))
    dom = by_cols[dom_cols]
    dom_flops = sum(e for e, _ in dom) * n_clip * N_FMT * FLOPS_PER_ELEM_CAND_FMT
    dom_time = sum(t for _, t in dom)
    achieved = dom_flops / dom_time / 1e12
    traffic = None
    if not group and args.model == "7b":
        per = [o * n * 2 * MEASURED_READ_PER_INPUT_BYTE + o * MEASURED_WRITE_BYTES_PER_ROW
               for _, _, o, n in shapes if n == dom_cols]
        traffic = sum(per) * args.steps / len(by_cols[dom_cols])   # per launch (a launch covers several tensors)
    search_time = sum(t for v in by_cols.values() for _, t in v) / args.steps
    roofline = {
        "bound": "alu", "achieved": achieved, "peak": ALU_PEAK_TFLOPS, "unit": "TFLOP/s",
        "frac": achieved / ALU_PEAK_TFLOPS, "traffic": traffic,
        "kernel": (f"sweep_group_kernel<F16, INT4, FP4_E2M1, {GROUP}> on {dom_cols}-column rows" if group else
                   f"sweep_sorted_kernel<F16, INT4, FP4_E2M1> instance for {dom_cols}-column rows"),
        "note": ("achieved counts the flop of the exhaustive element x candidate scoring" if group else
                 "achieved counts the flop of the exhaustive element x candidate scoring (the "
                 "algorithmic work); the kernel reaches the same result by sorting each row once and "
                 "locating level boundaries by binary search, so frac can exceed 1"),
        "avg_launch_ms": dom_time / len(dom) * 1e3, "launches": len(dom),
        "algorithmic_bytes_per_launch": sum(e for e, _ in dom) * 2 / len(dom),
        "flops_per_elem_cand_fmt": FLOPS_PER_ELEM_CAND_FMT,
        "hbm_GBps_at_this_rate": sum(e for e, _ in dom) * 2 / dom_time / 1e9,
        "search_ms_per_step": search_time * 1e3,
    }
    if not group and args.model == "7b":
        # what the kernel itself does with the vector ALUs (hardware counters, not measured in this run)
        roofline["kernel_valu_active_frac"] = 0.90
        roofline["kernel_valu_active_frac_source"] = "profiles/w_only_sorted_kernel_counters.txt"

    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)          # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    res = mq.read_results(results)
    fp_pct = 100.0 * sum(1 for r in res if r.best == 1) / len(res)

    out = {
        "metric": f"weight-elems x candidates scored/sec (+ LLaMA-{args.model.upper()} full-model MoFQ select time)",
        "value": value, "unit": "elem*cand/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "select_time_s": ms_per_step / 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32 decisions, f64 errors", "data": "synthetic",
        "config": {"workload": ("configs[2]: LLaMA-7B-shaped fp16 weight set, "
                                f"{len(shapes)} linears, {n_elems} weights, 4-bit W-only group-wise "
                                "(128 along the input dim, fp16 scales), 50 clip ratios in [0.5,1], "
                                "INT4 vs FP4-E2M1, per-layer select + emit") if group else
                               (("configs[4]: LLaMA-65B-shaped" if args.model == "65b" else
                                 "configs[1]: LLaMA-7B-shaped") + " fp16 weight set, "
                                f"{len(shapes)} linears, {n_elems} weights, 4-bit W-only per-channel, "
                                "100 clip ratios in [0.5,1], INT4 vs FP4-E2M1, per-layer select + emit"),
                   "n_clip": n_clip, "formats": ["INT4", "FP4_E2M1"], "fp_percent": fp_pct},
        "roofline": roofline,
    }
    if not args.no_cpu_baseline and not group and args.model == "7b":
        outs = [(qouts[i], res[i]) for i in range(len(shapes))]
        out["cpu_baseline"] = cpu_baseline(weights, outs, clip, cands)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
