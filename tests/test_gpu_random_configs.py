"""Seeded random sweep of weight-only configurations (shape, dtype, granularity, formats,
clip count, scale type, value distribution) through the same element-by-element parity
check as the hand-picked cases: a guard against shape- or value-dependent paths that the
fixed cases do not reach (kernel variants are chosen by row length, clip count, dtype)."""
import numpy as np
import pytest
import torch

import mofq_inputs as mi
from oracle import mofq_oracle as orc
from tests.test_gpu_w_only import check_tensor, mq  # noqa: F401  (fixture)

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
DTYPES = [torch.float16, torch.bfloat16, torch.float32]
FOUR = [[orc.INT4, orc.FP4_E2M1], [orc.FP4_E2M1, orc.INT4], [orc.INT4], [orc.FP4_E2M1], [orc.FP4_E2M1_IEEE, orc.FP4_E2M1]]
EIGHT = [[orc.INT8, orc.FP8_E4M3], [orc.FP8_E4M3], [orc.FP8_E5M2, orc.INT8]]


def _values(rng, rows, cols, kind, dtype):
    g = torch.Generator().manual_seed(int(rng.integers(1 << 30)))
    if kind == 0:      # the weight recipe
        return mi.llama_like_weight(rows, cols, seed=int(rng.integers(1 << 30)), dtype=dtype, device=DEV)
    if kind == 1:      # heavy duplicates: few distinct values per row (ties in the sort, exact ties in errors)
        v = torch.randint(-5, 6, (rows, cols), generator=g).float() * float(2.0 ** rng.integers(-8, 3))
    elif kind == 2:    # wide dynamic range within a row
        v = torch.randn(rows, cols, generator=g) * torch.exp(torch.randn(rows, cols, generator=g) * 2.0) * 0.01
    elif kind == 3:    # tiny magnitudes (fp16 subnormals) and exact zeros
        v = torch.randn(rows, cols, generator=g) * 3e-7
        v[:, ::3] = 0.0
    else:              # one huge outlier per row
        v = torch.randn(rows, cols, generator=g) * 0.02
        v[torch.arange(rows), torch.randint(0, cols, (rows,), generator=g)] = 30.0
    return v.to(dtype).to(DEV)


@pytest.mark.parametrize("seed", range(150))
def test_random_weight_only_config(mq, seed):  # noqa: F811
    rng = np.random.default_rng(1000 + seed)
    gran = [orc.PER_CHANNEL, orc.PER_CHANNEL, orc.PER_GROUP, orc.PER_TENSOR][rng.integers(4)]
    dtype = DTYPES[rng.integers(3)]
    cands = (FOUR if rng.random() < 0.7 else EIGHT)[0:][rng.integers(3)]
    group = 0
    if gran == orc.PER_GROUP:
        group = int([32, 64, 128, 256][rng.integers(4)])
        cols = group * int(rng.integers(1, 40))
        n_clip = int([1, 3, 17, 50, 64][rng.integers(5)])
    elif gran == orc.PER_TENSOR:
        cols = 8 * int(rng.integers(1, 300))
        n_clip = int([1, 2, 5, 8, 9, 20, 64][rng.integers(7)])
    else:
        cols = 8 * int([rng.integers(1, 64), rng.integers(128, 700), rng.integers(1200, 3100)][rng.integers(3)])
        n_clip = int([1, 2, 7, 8, 31, 100, 128][rng.integers(7)])
    rows = int(rng.integers(1, 24))
    f16 = bool(rng.integers(2)) and gran != orc.PER_TENSOR
    w = _values(rng, rows, cols, int(rng.integers(5)), dtype)
    check_tensor(mq, w, list(cands), gran, mi.clip_ratios(n_clip), group, f16, label=f"random-{seed}")
