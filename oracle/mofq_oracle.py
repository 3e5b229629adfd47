"""Python face of the CPU oracle (TEST INFRASTRUCTURE ONLY).

Loads ``libmofq_oracle.so`` (built from ``mofq_oracle.c`` with gcc) through
ctypes and adds the two pieces that are plain library calls on top of it: the
per-layer select of Algorithm 1 and the layer-output error of Section 3.2
(``A_out = W * A_in``) written as fp64 numpy matrix products.

Nothing here is imported by the product package.  Only tests, the smoke check
and the benchmark's cpu_baseline leg use it.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass
from typing import Optional, Sequence

import numpy as np

INT4, FP4_E2M1, INT8, FP8_E4M3, FP4_E2M1_IEEE, FP8_E5M2 = 0, 1, 2, 3, 4, 5
PER_TENSOR, PER_CHANNEL, PER_GROUP = 0, 1, 2

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mofq_oracle.c")
_LIB = os.path.join(_HERE, "libmofq_oracle.so")

GCC_FLAGS = ["-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
             "-fPIC", "-shared", "-Wall", "-Wextra"]


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (seconds)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.run(["gcc", *GCC_FLAGS, _SRC, "-o", tmp, "-lm"], check=True)
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        f32p, i32p, f64p, u8p = (C.POINTER(C.c_float), C.POINTER(C.c_int32),
                                 C.POINTER(C.c_double), C.POINTER(C.c_uint8))
        L.orc_decode.restype = C.c_double
        L.orc_decode.argtypes = [C.c_int, C.c_int]
        L.orc_encode.restype = C.c_int
        L.orc_encode.argtypes = [C.c_int, C.c_float]
        L.orc_qmax.restype = C.c_double
        L.orc_qmax.argtypes = [C.c_int]
        L.orc_round_fp16.restype = C.c_float
        L.orc_round_fp16.argtypes = [C.c_float]
        L.orc_scale.restype = C.c_float
        L.orc_scale.argtypes = [C.c_float, C.c_float, C.c_int, C.c_int]
        L.orc_num_units.restype = C.c_int64
        L.orc_num_units.argtypes = [C.c_int64, C.c_int64, C.c_int, C.c_int64]
        L.orc_sweep.restype = C.c_int
        L.orc_sweep.argtypes = [f32p, C.c_int64, C.c_int64, C.c_int, C.c_int64, C.c_int, C.c_int,
                                f32p, C.c_int, C.c_int64, C.c_int64, f32p, i32p, f64p, f64p, C.c_int]
        L.orc_emit.restype = C.c_int
        L.orc_emit.argtypes = [f32p, C.c_int64, C.c_int64, C.c_int, C.c_int64, C.c_int, f32p, u8p]
        L.orc_pack4.restype = C.c_int
        L.orc_pack4.argtypes = [u8p, C.c_int64, u8p]
        L.orc_tensor_err.restype = C.c_double
        L.orc_tensor_err.argtypes = [f64p, C.c_int64]
        L.orc_select.restype = C.c_int
        L.orc_select.argtypes = [f64p, C.c_int]
        L.orc_max_threads.restype = C.c_int
        L.orc_init()
        _lib = L
    return _lib


def _p(a: np.ndarray, ct):
    return a.ctypes.data_as(C.POINTER(ct))


def _f32c(w) -> np.ndarray:
    a = np.ascontiguousarray(w, dtype=np.float32)
    if a.ndim != 2:
        raise ValueError("expected a 2-D array")
    return a


# ---- scalars -----------------------------------------------------------------

def decode(fmt: int, code: int) -> float:
    return float(lib().orc_decode(fmt, int(code)))


def encode(fmt: int, t) -> int:
    return int(lib().orc_encode(fmt, C.c_float(float(np.float32(t)))))


def encode_array(fmt: int, t: np.ndarray) -> np.ndarray:
    """Codes of an fp32 array of already scaled values (scale 1 per element)."""
    t = np.ascontiguousarray(t, dtype=np.float32).reshape(1, -1)
    out = np.empty(t.shape, dtype=np.uint8)
    one = np.ones(1, dtype=np.float32)
    rc = lib().orc_emit(_p(t, C.c_float), 1, t.shape[1], PER_TENSOR, 0, fmt,
                        _p(one, C.c_float), _p(out, C.c_uint8))
    assert rc == 0
    return out.reshape(-1)


def decode_array(fmt: int, codes: np.ndarray) -> np.ndarray:
    lut = np.array([decode(fmt, c) for c in range(256 if bits(fmt) == 8 else 16)])
    return lut[np.asarray(codes, dtype=np.int64)]


def bits(fmt: int) -> int:
    return 8 if fmt in (INT8, FP8_E4M3, FP8_E5M2) else 4


def qmax(fmt: int) -> float:
    return float(lib().orc_qmax(fmt))


def round_fp16(v) -> float:
    return float(lib().orc_round_fp16(C.c_float(float(np.float32(v)))))


def scale(absmax, ratio, fmt: int, scale_f16: bool = False) -> float:
    return float(lib().orc_scale(C.c_float(float(np.float32(absmax))),
                                 C.c_float(float(np.float32(ratio))), fmt, int(scale_f16)))


def num_units(rows: int, cols: int, gran: int, group: int = 0) -> int:
    return int(lib().orc_num_units(rows, cols, gran, group))


def max_threads() -> int:
    return int(lib().orc_max_threads())


# ---- sweep / emit ------------------------------------------------------------

@dataclass
class Sweep:
    scale: np.ndarray        # [units] fp32 winner scale
    clip_idx: np.ndarray     # [units] int32 winner candidate
    err: np.ndarray          # [units] fp64 winner error (sum of squares)
    table: Optional[np.ndarray]  # [units, n_clip] fp64 error of every candidate, or None
    units: tuple             # (first, count) range that was computed


def sweep(w, fmt: int, gran: int, clip: Sequence[float], group: int = 0,
          scale_f16: bool = False, unit_first: int = 0, unit_count: Optional[int] = None,
          want_table: bool = False, threads: int = 0) -> Sweep:
    """Scale search of one tensor in one format (results indexed by absolute
    unit; entries outside [unit_first, unit_first+unit_count) are not written)."""
    w = _f32c(w)
    rows, cols = w.shape
    clip = np.ascontiguousarray(clip, dtype=np.float32)
    nu = num_units(rows, cols, gran, group)
    if nu < 0:
        raise ValueError("bad granularity / group")
    if unit_count is None:
        unit_count = nu - unit_first
    sc = np.zeros(nu, dtype=np.float32)
    ci = np.zeros(nu, dtype=np.int32)
    er = np.zeros(nu, dtype=np.float64)
    tb = np.zeros((nu, clip.size), dtype=np.float64) if want_table else None
    rc = lib().orc_sweep(_p(w, C.c_float), rows, cols, gran, group, fmt, int(scale_f16),
                         _p(clip, C.c_float), clip.size, unit_first, unit_count,
                         _p(sc, C.c_float), _p(ci, C.c_int32), _p(er, C.c_double),
                         _p(tb, C.c_double) if want_table else None, threads)
    if rc != 0:
        raise ValueError("orc_sweep rejected its arguments")
    return Sweep(sc, ci, er, tb, (unit_first, unit_count))


def emit(w, fmt: int, gran: int, unit_scale: np.ndarray, group: int = 0) -> np.ndarray:
    """Codes, one byte per element, of w quantized with the given unit scales."""
    w = _f32c(w)
    rows, cols = w.shape
    unit_scale = np.ascontiguousarray(unit_scale, dtype=np.float32)
    assert unit_scale.size == num_units(rows, cols, gran, group)
    out = np.empty((rows, cols), dtype=np.uint8)
    rc = lib().orc_emit(_p(w, C.c_float), rows, cols, gran, group, fmt,
                        _p(unit_scale, C.c_float), _p(out, C.c_uint8))
    if rc != 0:
        raise ValueError("orc_emit rejected its arguments")
    return out


def pack4(codes: np.ndarray) -> np.ndarray:
    c = np.ascontiguousarray(codes, dtype=np.uint8).reshape(-1)
    out = np.empty(c.size // 2, dtype=np.uint8)
    rc = lib().orc_pack4(_p(c, C.c_uint8), c.size, _p(out, C.c_uint8))
    if rc != 0:
        raise ValueError("odd number of 4-bit codes")
    return out


def tensor_err(unit_err: np.ndarray) -> float:
    e = np.ascontiguousarray(unit_err, dtype=np.float64)
    return float(lib().orc_tensor_err(_p(e, C.c_double), e.size))


def select(errs: Sequence[float]) -> int:
    e = np.ascontiguousarray(errs, dtype=np.float64)
    return int(lib().orc_select(_p(e, C.c_double), e.size))


# ---- Algorithm 1, one layer ---------------------------------------------------

@dataclass
class Quantized:
    fmt: int
    codes: np.ndarray        # [rows, cols] uint8, one code per element
    scale: np.ndarray        # [units] fp32
    clip_idx: np.ndarray     # [units] int32
    unit_err: np.ndarray     # [units] fp64
    err: float               # tensor error (sum of squares)
    table: Optional[np.ndarray] = None


def quantize(w, fmt: int, gran: int, clip, group: int = 0, scale_f16: bool = False,
             want_table: bool = False, threads: int = 0) -> Quantized:
    sw = sweep(w, fmt, gran, clip, group, scale_f16, want_table=want_table, threads=threads)
    codes = emit(w, fmt, gran, sw.scale, group)
    return Quantized(fmt, codes, sw.scale, sw.clip_idx, sw.err, tensor_err(sw.err), sw.table)


@dataclass
class Selected:
    best: int                # index into candidates
    errs: list               # error per candidate
    ref_energy: float        # sum of x^2 (tensor metric) or sum of Y^2 (layer-output metric)
    w: Quantized             # weights in the chosen format
    x: Optional[Quantized] = None
    per_candidate: Optional[list] = None


def select_layer_w_only(w, candidates: Sequence[int], gran: int, clip, group: int = 0,
                        scale_f16: bool = False, want_table: bool = False,
                        threads: int = 0) -> Selected:
    """Algorithm 1 for one layer with the tensor-error metric: quantize in each
    candidate format, keep the strictly smaller error, quantize again with it."""
    w = _f32c(w)
    qs = [quantize(w, f, gran, clip, group, scale_f16, want_table, threads) for f in candidates]
    errs = [q.err for q in qs]
    best = select(errs)
    energy = float(np.sum(w.astype(np.float64) ** 2))
    return Selected(best, errs, energy, qs[best], None, qs)


# ---- layer-output error (Section 3.2, layer analysis) -------------------------

def layer_output_error(x, w, qx: Quantized, qw: Quantized, w_gran: int = PER_TENSOR):
    """E = sum (X W^T - Xq Wq^T)^2 and P = sum (X W^T)^2 in fp64.

    Xq Wq^T = sx * sw[o] * (Gx Gw^T) with the grid-value product exact in fp64
    (integers for INT8; multiples of 2^-18 below 2^33 for E4M3)."""
    x64 = np.asarray(x, dtype=np.float64)
    w64 = np.asarray(w, dtype=np.float64)
    y = x64 @ w64.T
    gx = decode_array(qx.fmt, qx.codes)
    gw = decode_array(qw.fmt, qw.codes)
    acc = gx @ gw.T
    sx = np.float64(qx.scale[0])
    if w_gran == PER_TENSOR:
        sw = np.float64(qw.scale[0])
        yq = (sx * sw) * acc
    else:
        yq = (sx * qw.scale.astype(np.float64))[None, :] * acc
    d = y - yq
    return float(np.sum(d * d)), float(np.sum(y * y))


def select_layer_wa(x, w, candidates: Sequence[int], w_gran: int = PER_TENSOR,
                    threads: int = 0) -> Selected:
    """Algorithm 1 for one layer in the weight-activation case with the
    layer-output error: W and X share the candidate format (same data type for
    all tensors of a layer), X per-tensor, W per-tensor or per-channel, no clip
    search (ratio 1)."""
    x = _f32c(x)
    w = _f32c(w)
    one = np.ones(1, dtype=np.float32)
    errs, qxs, qws, energy = [], [], [], 0.0
    for f in candidates:
        qx = quantize(x, f, PER_TENSOR, one, threads=threads)
        qw = quantize(w, f, w_gran, one, threads=threads)
        e, energy = layer_output_error(x, w, qx, qw, w_gran)
        errs.append(e)
        qxs.append(qx)
        qws.append(qw)
    best = select(errs)
    return Selected(best, errs, energy, qws[best], qxs[best], list(zip(qxs, qws)))


def layer_output_error_w_only(x, w, qw: Quantized, w_gran: int = PER_CHANNEL):
    """Weight-only layer-output error (Section 3.2, layer analysis, with the input
    left in 16 bits): E = sum (X W^T - X What^T)^2 and P = sum (X W^T)^2 in fp64, with
    What[o, i] = gw[o, i] * sw[o] (per-channel) or gw[o, i] * sw (per-tensor).

    The quantized product is formed as sw[o] * (X Gw^T): every product of a 16-bit input
    and a 4-bit grid value is exact in fp64 and so is their sum (at most 12 + 15 bits of
    length), so the only roundings are the final scaling and the subtraction."""
    x64 = np.asarray(x, dtype=np.float64)
    w64 = np.asarray(w, dtype=np.float64)
    y = x64 @ w64.T
    gw = decode_array(qw.fmt, qw.codes)
    acc = x64 @ gw.T
    if w_gran == PER_TENSOR:
        yq = np.float64(qw.scale[0]) * acc
    elif w_gran == PER_CHANNEL:
        yq = qw.scale.astype(np.float64)[None, :] * acc
    else:
        raise ValueError("layer-output error needs one scale per output channel or per tensor")
    d = y - yq
    return float(np.sum(d * d)), float(np.sum(y * y))


def select_layer_w_only_output(x, w, candidates: Sequence[int], w_gran: int = PER_CHANNEL,
                               clip=(1.0,), scale_f16: bool = False, threads: int = 0) -> Selected:
    """Algorithm 1 for one layer in the weight-only case with the layer-output error as
    the metric: each candidate format quantizes W (scales searched over `clip` by tensor
    error, as in quantize()), the layer is run on the 16-bit input X with the original
    and with the quantized weights, and the format with the smaller output error wins
    (strict less-than, first candidate on ties)."""
    x = _f32c(x)
    w = _f32c(w)
    clip = np.asarray(clip, dtype=np.float32)
    errs, qws, energy = [], [], 0.0
    for f in candidates:
        qw = quantize(w, f, w_gran, clip, 0, scale_f16, threads=threads)
        e, energy = layer_output_error_w_only(x, w, qw, w_gran)
        errs.append(e)
        qws.append(qw)
    best = select(errs)
    return Selected(best, errs, energy, qws[best], None, [(None, q) for q in qws])


@dataclass
class UnitSelected:
    unit_format: np.ndarray  # [units] index into candidates, per scale unit
    codes: np.ndarray        # [rows, cols] codes, each unit in its own format
    scale: np.ndarray        # [units]
    clip_idx: np.ndarray     # [units]
    unit_err: np.ndarray     # [units] error of the chosen format
    err: float               # sum over units, unit order
    errs: list               # tensor error of each candidate used everywhere (layer-wise view)
    per_candidate: list      # Quantized per candidate


def select_units(w, candidates: Sequence[int], gran: int, clip, group: int = 0,
                 scale_f16: bool = False, threads: int = 0) -> UnitSelected:
    """Format select at the granularity of the scale unit (channel or group) instead of
    the layer -- the extension Section 4.1 leaves open and the conclusion lists as future
    work: every unit takes the candidate with its own smallest error, Algorithm 1's rule
    applied per unit (candidates in list order, strictly smaller wins)."""
    w = _f32c(w)
    if gran == PER_TENSOR:
        raise ValueError("a per-tensor unit is the layer itself")
    qs = [quantize(w, f, gran, clip, group, scale_f16, threads=threads) for f in candidates]
    units = qs[0].unit_err.shape[0]
    pick = np.zeros(units, dtype=np.uint8)
    best = qs[0].unit_err.copy()
    for c in range(1, len(qs)):
        better = qs[c].unit_err < best
        pick[better] = c
        best[better] = qs[c].unit_err[better]
    rows, cols = w.shape
    # unit index of every element
    if gran == PER_CHANNEL:
        unit_of = np.repeat(np.arange(rows)[:, None], cols, axis=1)
    else:
        unit_of = np.arange(rows)[:, None] * (cols // group) + (np.arange(cols) // group)[None, :]
    codes = np.zeros((rows, cols), dtype=np.uint8)
    scale = np.zeros(units, dtype=np.float32)
    idx = np.zeros(units, dtype=np.int32)
    for c, q in enumerate(qs):
        m = pick == c
        scale[m] = q.scale[m]
        idx[m] = q.clip_idx[m]
        em = m[unit_of]
        codes[em] = q.codes[em]
    return UnitSelected(pick, codes, scale, idx, best, tensor_err(best), [q.err for q in qs], qs)


def calibrate_absmax(batches) -> np.float32:
    """Static calibration (Section 3.2, dynamic tensor analysis): the largest magnitude
    over all calibration batches."""
    m = np.float32(0.0)
    for b in batches:
        m = np.maximum(m, np.max(np.abs(_f32c(b))))
    return np.float32(m)


def quantize_calibrated(x, fmt: int, absmax) -> Quantized:
    """Per-tensor quantization of a batch that was not part of the calibration: the scale
    comes from the calibrated magnitude (same scale expression as everywhere, ratio 1);
    values beyond the calibrated range saturate at the format's extreme value."""
    x = _f32c(x)
    s = np.array([scale(np.float32(absmax), 1.0, fmt)], dtype=np.float32)
    codes = emit(x, fmt, PER_TENSOR, s)
    xh = decode_array(fmt, codes) * np.float64(s[0])
    d = x.astype(np.float64) - xh
    e = float(np.sum(d * d))
    return Quantized(fmt, codes, s, np.zeros(1, dtype=np.int32), np.array([e]), e, None)


def select_calibrated(x, candidates: Sequence[int], absmax) -> Selected:
    """Algorithm 1's loop body for one dynamic tensor with calibrated scales."""
    x = _f32c(x)
    qs = [quantize_calibrated(x, f, absmax) for f in candidates]
    errs = [q.err for q in qs]
    best = select(errs)
    return Selected(best, errs, float(np.sum(x.astype(np.float64) ** 2)), qs[best], None, qs)

