"""Helpers of the GPU parity tests: run the library through its C ABI, unpack its
outputs, and compare them with the CPU oracle under the near-tie rule."""
from __future__ import annotations

import numpy as np
import torch

from oracle import mofq_oracle as orc

# Relative width of the near-tie band of the clip search.  Both sides add the unit
# errors in fp64 but in different orders (and the GPU fuses d*d+acc), so sums differ
# by at most about n * 2^-52 ~ 3e-12 for the longest rows; two candidates whose
# oracle errors are closer than this are either-or.
TIE_TAU = 1e-10
# Tolerance on error sums (the target asks for 1e-5; fp64 on both sides gives far better).
ERR_RTOL = 1e-9


def unpack_codes(codes: torch.Tensor, rows: int, cols: int, bits: int) -> np.ndarray:
    raw = codes.cpu().numpy()
    if bits == 8:
        return raw.reshape(rows, cols)
    out = np.empty((rows * cols,), dtype=np.uint8)
    out[0::2] = raw & 0xF
    out[1::2] = raw >> 4
    return out.reshape(rows, cols)


def scales_to_f32(scales: torch.Tensor) -> np.ndarray:
    return scales.cpu().to(torch.float32).numpy()


def unit_absmax(w32: np.ndarray, gran: int, group: int) -> np.ndarray:
    a = np.abs(w32)
    if gran == orc.PER_CHANNEL:
        return a.max(axis=1)
    if gran == orc.PER_GROUP:
        return a.reshape(w32.shape[0], -1, group).max(axis=2).reshape(-1)
    return np.array([a.max()], dtype=np.float32)


def compare_quantized(w32: np.ndarray, fmt: int, gran: int, group: int, scale_f16: bool,
                      clip: np.ndarray, ref: "orc.Quantized", got_codes: np.ndarray,
                      got_scale: np.ndarray, got_idx: np.ndarray, got_err: np.ndarray) -> int:
    """Bit-exact parity of chosen candidates, scales and codes; returns the number
    of units that fell into the near-tie band (different index, oracle errors of the
    two indices within TIE_TAU), for which the scale and codes are checked against
    the oracle's arithmetic at the library's index."""
    assert ref.table is not None
    diff = np.nonzero(got_idx != ref.clip_idx)[0]
    exp_scale = ref.scale.copy()
    if diff.size:
        amax = unit_absmax(w32, gran, group)
        for u in diff:
            kg, ko = int(got_idx[u]), int(ref.clip_idx[u])
            assert 0 <= kg < clip.size, f"unit {u}: clip index {kg} out of range"
            e_g, e_o = ref.table[u, kg], ref.table[u, ko]
            assert e_g <= e_o * (1 + TIE_TAU) + 1e-300, (
                f"unit {u}: library chose candidate {kg} (oracle error {e_g!r}) but {ko} "
                f"({e_o!r}) is smaller beyond the tie band")
            exp_scale[u] = orc.scale(amax[u], clip[kg], fmt, scale_f16)
        exp_codes = orc.emit(w32, fmt, gran, exp_scale, group)
        exp_err = ref.unit_err.copy()
        exp_err[diff] = ref.table[diff, got_idx[diff]]
    else:
        exp_codes, exp_err = ref.codes, ref.unit_err
    assert np.array_equal(got_scale, exp_scale), "scales differ"
    bad = np.nonzero(got_codes != exp_codes)
    assert bad[0].size == 0, f"{bad[0].size} codes differ, first at {bad[0][0], bad[1][0]}"
    assert np.allclose(got_err, exp_err, rtol=ERR_RTOL, atol=1e-300), "unit errors differ"
    return int(diff.size)
