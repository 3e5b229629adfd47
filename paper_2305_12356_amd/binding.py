"""ctypes binding of libmofq.so: argument marshalling only.

Every step of the path runs in the library's HIP kernels; PyTorch is used for
device memory and streams.  There is no CPU fallback: if the library is not
built, importing this module raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional, Sequence

import numpy as np
import torch

INT4, FP4_E2M1, INT8, FP8_E4M3, FP4_E2M1_IEEE, FP8_E5M2 = 0, 1, 2, 3, 4, 5
F32, F16, BF16 = 0, 1, 2
PER_TENSOR, PER_CHANNEL, PER_GROUP = 0, 1, 2
ERR_TENSOR, ERR_LAYER_OUTPUT, ERR_LAYER_OUTPUT_FP8_UNIT, ERR_LAYER_OUTPUT_W_ONLY = 0, 1, 2, 3
MAX_CANDIDATES = 4

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmofq.so")


class MofqError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


class TensorDesc(C.Structure):
    _fields_ = [("data", C.c_void_p), ("dtype", C.c_int32), ("rows", C.c_int64),
                ("cols", C.c_int64), ("ld", C.c_int64)]


class ScaleCfg(C.Structure):
    _fields_ = [("gran", C.c_int32), ("group_size", C.c_int32), ("scale_dtype", C.c_int32),
                ("n_clip", C.c_int32), ("clip_ratios", C.POINTER(C.c_float))]


class QOut(C.Structure):
    _fields_ = [("codes", C.c_void_p), ("scales", C.c_void_p), ("clip_idx", C.c_void_p),
                ("unit_err", C.c_void_p)]


class Result(C.Structure):
    _fields_ = [("best", C.c_int32), ("n", C.c_int32), ("err", C.c_double * MAX_CANDIDATES),
                ("ref_energy", C.c_double)]


RESULT_BYTES = C.sizeof(Result)


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2305_12356_amd.build` "
            "(there is no fallback path)")
    L = C.CDLL(LIB_PATH)
    vp = C.c_void_p
    L.mofq_quantize.restype = C.c_int
    L.mofq_quantize.argtypes = [C.POINTER(TensorDesc), C.c_int32, C.POINTER(ScaleCfg),
                                C.POINTER(QOut), vp, vp, C.c_size_t, vp]
    L.mofq_score.restype = C.c_int
    L.mofq_score.argtypes = [C.POINTER(TensorDesc), C.POINTER(TensorDesc), C.c_int32, C.c_int32,
                             C.POINTER(ScaleCfg), vp, vp, vp, C.c_size_t, vp]
    L.mofq_select_layer.restype = C.c_int
    L.mofq_select_layer.argtypes = [C.POINTER(TensorDesc), C.POINTER(TensorDesc),
                                    C.POINTER(C.c_int32), C.c_int32, C.c_int32,
                                    C.POINTER(ScaleCfg), C.POINTER(QOut), C.POINTER(QOut),
                                    vp, vp, C.c_size_t, vp]
    L.mofq_select_layer_static.restype = C.c_int
    L.mofq_select_layer_static.argtypes = [C.POINTER(TensorDesc), C.POINTER(C.c_int32), C.c_int32,
                                           C.POINTER(ScaleCfg), C.POINTER(QOut), vp, vp]
    L.mofq_select_layer_timed.restype = C.c_int
    L.mofq_select_layer_timed.argtypes = L.mofq_select_layer.argtypes + [vp, vp]
    L.mofq_workspace_bytes.restype = C.c_size_t
    L.mofq_workspace_bytes.argtypes = [C.POINTER(TensorDesc), C.POINTER(TensorDesc), C.c_int32,
                                       C.c_int32, C.POINTER(ScaleCfg)]
    L.mofq_select_units.restype = C.c_int
    L.mofq_select_units.argtypes = [C.POINTER(TensorDesc), C.POINTER(C.c_int32), C.c_int32,
                                    C.POINTER(ScaleCfg), C.POINTER(QOut), vp, vp, vp, vp, C.c_size_t, vp]
    L.mofq_select_units_workspace_bytes.restype = C.c_size_t
    L.mofq_select_units_workspace_bytes.argtypes = [C.POINTER(TensorDesc), C.c_int32, C.POINTER(ScaleCfg)]
    L.mofq_select_layers.restype = C.c_int
    L.mofq_select_layers.argtypes = [C.c_int32, C.POINTER(TensorDesc), C.POINTER(C.c_int32), C.c_int32,
                                     C.POINTER(ScaleCfg), C.POINTER(QOut), vp, vp, C.c_size_t, vp, vp]
    L.mofq_select_layers_timed.restype = C.c_int
    L.mofq_select_layers_timed.argtypes = L.mofq_select_layers.argtypes + [C.POINTER(vp), C.POINTER(vp)]
    L.mofq_select_layers_search_groups.restype = C.c_int
    L.mofq_select_layers_search_groups.argtypes = [C.c_int32, C.POINTER(TensorDesc), C.POINTER(C.c_int32),
                                                   C.c_int32, C.POINTER(C.c_int32)]
    L.mofq_select_layers_workspace_bytes.restype = C.c_size_t
    L.mofq_select_layers_workspace_bytes.argtypes = [C.c_int32, C.POINTER(TensorDesc), C.c_int32,
                                                     C.POINTER(ScaleCfg)]
    L.mofq_select_layers_wa.restype = C.c_int
    L.mofq_select_layers_wa.argtypes = [C.c_int32, C.POINTER(TensorDesc), C.POINTER(TensorDesc),
                                        C.POINTER(C.c_int32), C.c_int32, C.c_int32, C.POINTER(ScaleCfg),
                                        C.POINTER(QOut), C.POINTER(QOut), vp, vp, C.c_size_t, vp]
    L.mofq_select_layers_wa_timed.restype = C.c_int
    L.mofq_select_layers_wa_timed.argtypes = L.mofq_select_layers_wa.argtypes + [C.POINTER(vp), C.POINTER(vp)]
    L.mofq_select_layers_wa_workspace_bytes.restype = C.c_size_t
    L.mofq_select_layers_wa_workspace_bytes.argtypes = [C.c_int32, C.POINTER(TensorDesc), C.POINTER(TensorDesc),
                                                        C.c_int32, C.c_int32, C.POINTER(ScaleCfg)]
    L.mofq_calibrate_absmax.restype = C.c_int
    L.mofq_calibrate_absmax.argtypes = [C.POINTER(TensorDesc), vp, vp, C.c_size_t, vp]
    L.mofq_select_calibrated.restype = C.c_int
    L.mofq_select_calibrated.argtypes = [C.POINTER(TensorDesc), C.POINTER(C.c_int32), C.c_int32, vp,
                                         C.POINTER(QOut), vp, vp, C.c_size_t, vp]
    L.mofq_device_ceiling.restype = C.c_int
    L.mofq_device_ceiling.argtypes = [C.c_int32, vp, C.c_size_t, C.c_int32, C.POINTER(C.c_double), vp]
    L.mofq_num_units.restype = C.c_int64
    L.mofq_num_units.argtypes = [C.c_int64, C.c_int64, C.c_int32, C.c_int32]
    L.mofq_status_string.restype = C.c_char_p
    L.mofq_status_string.argtypes = [C.c_int]
    return L


_lib = _load()


def status_string(status: int) -> str:
    return _lib.mofq_status_string(int(status)).decode()


def num_units(rows: int, cols: int, gran: int, group_size: int = 0) -> int:
    return int(_lib.mofq_num_units(rows, cols, gran, group_size))


_DTYPES = {torch.float32: F32, torch.float16: F16, torch.bfloat16: BF16}


def tensor_desc(t: torch.Tensor) -> TensorDesc:
    if t.dim() != 2 or t.stride(1) != 1:
        raise ValueError("expected a 2-D tensor with contiguous rows")
    if t.dtype not in _DTYPES:
        raise ValueError(f"unsupported dtype {t.dtype}")
    if not t.is_cuda:
        raise ValueError("the library works on device memory only")
    return TensorDesc(t.data_ptr(), _DTYPES[t.dtype], t.shape[0], t.shape[1], t.stride(0))


class Cfg:
    """Scale-search configuration; keeps the host clip table alive."""

    def __init__(self, gran: int, clip: Sequence[float], group_size: int = 0,
                 scale_f16: bool = False):
        self._clip = np.ascontiguousarray(clip, dtype=np.float32)
        self.gran, self.group_size, self.scale_f16 = gran, group_size, scale_f16
        self.c = ScaleCfg(gran, group_size, F16 if scale_f16 else F32, self._clip.size,
                          self._clip.ctypes.data_as(C.POINTER(C.c_float)))

    @property
    def n_clip(self) -> int:
        return int(self._clip.size)


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream_handle(stream) -> C.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


@dataclass
class QBuffers:
    """Caller-owned device outputs of one quantized tensor."""
    codes: torch.Tensor                  # uint8: rows*cols/2 (4-bit) or rows*cols (8-bit)
    scales: torch.Tensor                 # [units] float32 or float16
    clip_idx: Optional[torch.Tensor]     # [units] int32
    unit_err: Optional[torch.Tensor]     # [units] float64

    def c(self) -> QOut:
        return QOut(_ptr(self.codes), _ptr(self.scales), _ptr(self.clip_idx), _ptr(self.unit_err))


def alloc_qbuffers(rows: int, cols: int, bits: int, cfg: Cfg, device,
                   with_idx: bool = True, with_err: bool = True) -> QBuffers:
    units = num_units(rows, cols, cfg.gran, cfg.group_size)
    if units <= 0:
        raise ValueError("invalid granularity for this shape")
    n_bytes = rows * cols // 2 if bits == 4 else rows * cols
    return QBuffers(
        torch.empty(n_bytes, dtype=torch.uint8, device=device),
        torch.empty(units, dtype=torch.float16 if cfg.scale_f16 else torch.float32, device=device),
        torch.empty(units, dtype=torch.int32, device=device) if with_idx else None,
        torch.empty(units, dtype=torch.float64, device=device) if with_err else None)


def workspace_bytes(w: torch.Tensor, x: Optional[torch.Tensor], n_candidates: int, metric: int,
                    cfg: Cfg) -> int:
    wd = tensor_desc(w)
    xd = tensor_desc(x) if x is not None else None
    return int(_lib.mofq_workspace_bytes(C.byref(wd), C.byref(xd) if xd else None, n_candidates,
                                         metric, C.byref(cfg.c)))


def quantize(t: torch.Tensor, fmt: int, cfg: Cfg, out: QBuffers,
             tensor_err: Optional[torch.Tensor], ws: torch.Tensor, stream=None) -> None:
    """mofq_quantize: enqueue; results land in `out` / `tensor_err` (device)."""
    td = tensor_desc(t)
    oc = out.c()
    rc = _lib.mofq_quantize(C.byref(td), fmt, C.byref(cfg.c), C.byref(oc), _ptr(tensor_err),
                            _ptr(ws), ws.numel() * ws.element_size(), _stream_handle(stream))
    if rc != 0:
        raise MofqError(rc, "mofq_quantize")


def score(w: torch.Tensor, x: Optional[torch.Tensor], fmt: int, metric: int, cfg: Cfg,
          err: torch.Tensor, ref_energy: Optional[torch.Tensor], ws: torch.Tensor,
          stream=None) -> None:
    """mofq_score: enqueue; `err` / `ref_energy` are device float64 scalars."""
    wd = tensor_desc(w)
    xd = tensor_desc(x) if x is not None else None
    rc = _lib.mofq_score(C.byref(wd), C.byref(xd) if xd else None, fmt, metric, C.byref(cfg.c),
                         _ptr(err), _ptr(ref_energy), _ptr(ws), ws.numel() * ws.element_size(),
                         _stream_handle(stream))
    if rc != 0:
        raise MofqError(rc, "mofq_score")


def _event_handle(ev) -> C.c_void_p:
    """Raw hipEvent_t of a torch.cuda.Event (recorded once so that it exists)."""
    if ev is None:
        return None
    if not ev.cuda_event:
        ev.record()
    return C.c_void_p(ev.cuda_event)


def select_layer(w: torch.Tensor, x: Optional[torch.Tensor], candidates: Sequence[int],
                 metric: int, cfg: Cfg, w_out: QBuffers, x_out: Optional[QBuffers],
                 result: torch.Tensor, ws: torch.Tensor, stream=None,
                 ev_begin=None, ev_end=None) -> None:
    """mofq_select_layer (or, with events, mofq_select_layer_timed): enqueue;
    `result` is a device uint8 tensor of RESULT_BYTES bytes (see read_result).
    `ev_begin`/`ev_end` are torch.cuda.Event(enable_timing=True) recorded by the
    library around the scoring kernels."""
    wd = tensor_desc(w)
    xd = tensor_desc(x) if x is not None else None
    cand = (C.c_int32 * len(candidates))(*candidates)
    woc = w_out.c()
    xoc = x_out.c() if x_out is not None else None
    args = (C.byref(wd), C.byref(xd) if xd else None, cand, len(candidates), metric,
            C.byref(cfg.c), C.byref(woc), C.byref(xoc) if xoc else None, _ptr(result), _ptr(ws),
            ws.numel() * ws.element_size(), _stream_handle(stream))
    if ev_begin is None and ev_end is None:
        rc = _lib.mofq_select_layer(*args)
    else:
        rc = _lib.mofq_select_layer_timed(*args, _event_handle(ev_begin), _event_handle(ev_end))
    if rc != 0:
        raise MofqError(rc, "mofq_select_layer")


STATIC_WORKSPACE_BYTES = 8 << 20


def select_layer_static(w: torch.Tensor, candidates: Sequence[int], cfg: Cfg, w_out: QBuffers,
                        result: torch.Tensor, stream=None) -> None:
    """mofq_select_layer_static: the weight-only, tensor-error select of one layer with the
    library's built-in workspace (no workspace argument, nothing allocated); enqueue."""
    wd = tensor_desc(w)
    cand = (C.c_int32 * len(candidates))(*candidates)
    woc = w_out.c()
    rc = _lib.mofq_select_layer_static(C.byref(wd), cand, len(candidates), C.byref(cfg.c), C.byref(woc),
                                       _ptr(result), _stream_handle(stream))
    if rc != 0:
        raise MofqError(rc, "mofq_select_layer_static")


def select_units_workspace_bytes(w: torch.Tensor, n_candidates: int, cfg: Cfg) -> int:
    wd = tensor_desc(w)
    return int(_lib.mofq_select_units_workspace_bytes(C.byref(wd), n_candidates, C.byref(cfg.c)))


def select_units(w: torch.Tensor, candidates: Sequence[int], cfg: Cfg, w_out: QBuffers,
                 unit_format: torch.Tensor, result: torch.Tensor, mixed_err: torch.Tensor,
                 ws: torch.Tensor, stream=None) -> None:
    """mofq_select_units: per-unit format select (weight-only, tensor error); enqueue.
    `unit_format` is a device uint8 tensor [units], `mixed_err` a device float64 scalar."""
    wd = tensor_desc(w)
    cand = (C.c_int32 * len(candidates))(*candidates)
    woc = w_out.c()
    rc = _lib.mofq_select_units(C.byref(wd), cand, len(candidates), C.byref(cfg.c), C.byref(woc),
                                _ptr(unit_format), _ptr(result), _ptr(mixed_err), _ptr(ws),
                                ws.numel() * ws.element_size(), _stream_handle(stream))
    if rc != 0:
        raise MofqError(rc, "mofq_select_units")


def calibrate_absmax(x: torch.Tensor, absmax: torch.Tensor, ws: torch.Tensor, stream=None) -> None:
    """mofq_calibrate_absmax: absmax (device float32 scalar) = max(absmax, max|x|); enqueue."""
    xd = tensor_desc(x)
    rc = _lib.mofq_calibrate_absmax(C.byref(xd), _ptr(absmax), _ptr(ws), ws.numel() * ws.element_size(),
                                    _stream_handle(stream))
    if rc != 0:
        raise MofqError(rc, "mofq_calibrate_absmax")


def select_calibrated(x: torch.Tensor, candidates: Sequence[int], absmax: torch.Tensor,
                      x_out: Optional[QBuffers], result: torch.Tensor, ws: torch.Tensor,
                      stream=None) -> None:
    """mofq_select_calibrated: per-tensor select with the scale from a calibrated absmax."""
    xd = tensor_desc(x)
    cand = (C.c_int32 * len(candidates))(*candidates)
    xoc = x_out.c() if x_out is not None else None
    rc = _lib.mofq_select_calibrated(C.byref(xd), cand, len(candidates), _ptr(absmax),
                                     C.byref(xoc) if xoc else None, _ptr(result), _ptr(ws),
                                     ws.numel() * ws.element_size(), _stream_handle(stream))
    if rc != 0:
        raise MofqError(rc, "mofq_select_calibrated")


class LayerBatch:
    """Host-side descriptor arrays of a set of weight tensors and their output buffers for
    mofq_select_layers (built once, reused for every call)."""

    def __init__(self, weights: Sequence[torch.Tensor], outs: Sequence[QBuffers]):
        assert len(weights) == len(outs) and len(weights) > 0
        self.n = len(weights)
        self._keep = (list(weights), list(outs))
        self.w = (TensorDesc * self.n)(*[tensor_desc(t) for t in weights])
        self.out = (QOut * self.n)(*[o.c() for o in outs])

    def workspace_bytes(self, n_candidates: int, cfg: Cfg) -> int:
        return int(_lib.mofq_select_layers_workspace_bytes(self.n, self.w, n_candidates, C.byref(cfg.c)))

    def search_groups(self, candidates: Sequence[int]):
        """mofq_select_layers_search_groups: for every tensor, the index of the first tensor of
        the search launch it belongs to."""
        cand = (C.c_int32 * len(candidates))(*candidates)
        first = (C.c_int32 * self.n)()
        rc = _lib.mofq_select_layers_search_groups(self.n, self.w, cand, len(candidates), first)
        if rc != 0:
            raise MofqError(rc, "mofq_select_layers_search_groups")
        return list(first)


def select_layers(batch: LayerBatch, candidates: Sequence[int], cfg: Cfg, results: torch.Tensor,
                  ws: torch.Tensor, stream=None, ev_begin=None, ev_end=None, side_stream=None) -> None:
    """mofq_select_layers (or _timed with lists of torch.cuda.Event): weight-only select of
    every tensor of the batch; `results` is the device array from alloc_result(device, n).
    `side_stream`: a torch.cuda.Stream for the select + emission of each batch (None: all on
    `stream`).  The events bracket search launches, which cover several tensors each:
    ev_begin of a launch's first tensor and ev_end of its last are recorded, the others are
    left alone (LayerBatch.search_groups tells which)."""
    cand = (C.c_int32 * len(candidates))(*candidates)
    side = C.c_void_p(side_stream.cuda_stream) if side_stream is not None else C.c_void_p(0)
    args = (batch.n, batch.w, cand, len(candidates), C.byref(cfg.c), batch.out, _ptr(results), _ptr(ws),
            ws.numel() * ws.element_size(), _stream_handle(stream), side)
    if ev_begin is None:
        rc = _lib.mofq_select_layers(*args)
    else:
        e0 = (C.c_void_p * batch.n)(*[_event_handle(e).value for e in ev_begin])
        e1 = (C.c_void_p * batch.n)(*[_event_handle(e).value for e in ev_end])
        rc = _lib.mofq_select_layers_timed(*args, e0, e1)
    if rc != 0:
        raise MofqError(rc, "mofq_select_layers")


class WaLayerBatch:
    """Host-side descriptor arrays of the linear layers of a model for mofq_select_layers_wa:
    weights, their activations (the same tensor object may be given to consecutive layers) and
    the output buffers (`x_outs` may be None: no activation outputs)."""

    def __init__(self, weights: Sequence[torch.Tensor], acts: Sequence[torch.Tensor],
                 w_outs: Sequence[QBuffers], x_outs: Optional[Sequence[QBuffers]]):
        assert len(weights) == len(acts) == len(w_outs) and len(weights) > 0
        assert x_outs is None or len(x_outs) == len(weights)
        self.n = len(weights)
        self._keep = (list(weights), list(acts), list(w_outs), list(x_outs) if x_outs is not None else None)
        self.w = (TensorDesc * self.n)(*[tensor_desc(t) for t in weights])
        self.x = (TensorDesc * self.n)(*[tensor_desc(t) for t in acts])
        self.w_out = (QOut * self.n)(*[o.c() for o in w_outs])
        self.x_out = (QOut * self.n)(*[o.c() for o in x_outs]) if x_outs is not None else None

    def workspace_bytes(self, n_candidates: int, metric: int, cfg: Cfg) -> int:
        return int(_lib.mofq_select_layers_wa_workspace_bytes(self.n, self.w, self.x, n_candidates, metric,
                                                              C.byref(cfg.c)))


def select_layers_wa(batch: WaLayerBatch, candidates: Sequence[int], metric: int, cfg: Cfg,
                     results: torch.Tensor, ws: torch.Tensor, stream=None, ev_begin=None, ev_end=None) -> None:
    """mofq_select_layers_wa (or _timed with lists of torch.cuda.Event recorded around each
    layer's matrix kernel): the weight-activation select of every layer of the batch; enqueue."""
    cand = (C.c_int32 * len(candidates))(*candidates)
    args = (batch.n, batch.w, batch.x, cand, len(candidates), metric, C.byref(cfg.c), batch.w_out, batch.x_out,
            _ptr(results), _ptr(ws), ws.numel() * ws.element_size(), _stream_handle(stream))
    if ev_begin is None:
        rc = _lib.mofq_select_layers_wa(*args)
    else:
        e0 = (C.c_void_p * batch.n)(*[_event_handle(e).value for e in ev_begin])
        e1 = (C.c_void_p * batch.n)(*[_event_handle(e).value for e in ev_end])
        rc = _lib.mofq_select_layers_wa_timed(*args, e0, e1)
    if rc != 0:
        raise MofqError(rc, "mofq_select_layers_wa")


CEILING_COPY, CEILING_FMA_F32, CEILING_FMA_F64, CEILING_MFMA_BF16, CEILING_MFMA_INT8, CEILING_MFMA_FP8, CEILING_READ = range(7)


def device_ceiling(kind: int, scratch: torch.Tensor, iters: int, stream=None) -> float:
    """mofq_device_ceiling: enqueue one rate-measuring micro-kernel (or `iters` plain copies of
    half of `scratch`); returns the work of the launch (bytes or operations)."""
    work = C.c_double(0.0)
    rc = _lib.mofq_device_ceiling(kind, _ptr(scratch), scratch.numel() * scratch.element_size(), iters,
                                  C.byref(work), _stream_handle(stream))
    if rc != 0:
        raise MofqError(rc, "mofq_device_ceiling")
    return work.value


def alloc_result(device, n: int = 1) -> torch.Tensor:
    return torch.zeros(n, RESULT_BYTES, dtype=torch.uint8, device=device)


def read_result(result: torch.Tensor) -> Result:
    """Copy one mofq_result_t back to the host (synchronises)."""
    raw = result.reshape(-1)[:RESULT_BYTES].cpu().numpy().tobytes()
    return Result.from_buffer_copy(raw)


def read_results(results: torch.Tensor):
    raw = results.cpu().numpy()
    return [Result.from_buffer_copy(raw[i].tobytes()) for i in range(raw.shape[0])]
