"""Seeded random sweep aimed at the two per-channel searches that do not score every (element,
candidate) pair (16-bit rows of 1024 to 24576 columns, 4-bit formats, 8 or more clip ratios):
the histogram kernel (clip ratios whose thresholds span few enough bit patterns: every bf16
case here, fp16 with ratios from about 0.1 up) and the sorting kernel (fp16 with smaller
ratios); every row-length instance of both, ragged row ends, one and two formats, fp16 scales,
clip tables in any order, and value distributions with heavy duplicates, wide dynamic range,
subnormals and outliers, through the same element-by-element parity check against the oracle
as the hand-picked cases."""
import numpy as np
import pytest
import torch

import mofq_inputs as mi
from oracle import mofq_oracle as orc
from tests.test_gpu_random_configs import FOUR, _values
from tests.test_gpu_w_only import check_tensor, mq  # noqa: F401  (fixture)

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("seed", range(60))
def test_random_sorted_search_config(mq, seed):  # noqa: F811
    rng = np.random.default_rng(777000 + seed)
    dtype = [torch.float16, torch.bfloat16][rng.integers(2)]
    cands = FOUR[rng.integers(4)]
    cols = 8 * int([rng.integers(128, 256), rng.integers(256, 512), rng.integers(512, 1024),
                    rng.integers(1024, 1536), rng.integers(1536, 3072)][rng.integers(5)])
    if rng.random() < 0.3:
        cols = int([1024, 2048, 4096, 8192, 12288, 24576, 11008, 22016][rng.integers(8)])
    n_clip = int([8, 9, 31, 50, 64, 65, 100, 128][rng.integers(8)])
    rows = int(rng.integers(1, 9))
    f16 = bool(rng.integers(2))
    w = _values(rng, rows, cols, int(rng.integers(5)), dtype)
    check_tensor(mq, w, list(cands), orc.PER_CHANNEL, mi.clip_ratios(n_clip), 0, f16, label=f"sorted-{seed}")


LOW_RATIOS = [0.3, 0.12, 0.05, 0.02]   # fp16: the first two go to the histogram kernel, the others to the sorting one


@pytest.mark.parametrize("seed", range(48))
def test_random_clip_tables(mq, seed):  # noqa: F811
    """Clip ratios down to 0.02, in descending, ascending or shuffled order, with repeats."""
    rng = np.random.default_rng(778000 + seed)
    dtype = [torch.float16, torch.bfloat16][seed % 2]
    cands = FOUR[rng.integers(4)]
    cols = int([1024, 2048, 4096, 8192, 11008, 12288, 22016, 24576][rng.integers(8)]) if rng.random() < 0.5 \
        else 8 * int(rng.integers(128, 3072))
    n_clip = int([8, 16, 33, 100, 128][rng.integers(5)])
    lo = LOW_RATIOS[(seed // 2) % 4]
    clip = mi.clip_ratios(n_clip, lo=lo, hi=float([1.0, 0.9][rng.integers(2)]))
    order = int(rng.integers(3))
    if order == 1:
        clip = clip[::-1].copy()
    elif order == 2:
        clip = rng.permutation(clip)
        clip[int(rng.integers(n_clip))] = clip[0]   # a repeated ratio: the first of the two wins a tie
    rows = int(rng.integers(1, 7))
    f16 = bool(rng.integers(2))
    w = _values(rng, rows, cols, int(rng.integers(5)), dtype)
    check_tensor(mq, w, list(cands), orc.PER_CHANNEL, np.ascontiguousarray(clip, dtype=np.float32), 0, f16,
                 label=f"clip-{seed}")


def _special_rows(cols, dtype):
    """Rows that stress the counting and the INT4 asymmetry: zeros, one value, the type's extremes,
    negative-only and uniform rows (many elements beyond INT4's -7.5 boundary), a lone element."""
    g = torch.Generator().manual_seed(4242 + cols)
    big = 65504.0 if dtype == torch.float16 else 3.0e38
    tiny = 6.0e-8 if dtype == torch.float16 else 1.0e-38
    rows = []
    rows.append(torch.zeros(cols))                                          # all zero: degenerate scale
    rows.append(torch.full((cols,), -0.0))                                  # negative zeros
    rows.append(torch.full((cols,), 0.37))                                  # one value: one counter holds the row
    rows.append(torch.full((cols,), -0.37))                                 # the same, all on INT4's negative side
    r = torch.zeros(cols); r[cols // 3] = -1.0; rows.append(r)              # a lone negative element
    r = torch.randn(cols, generator=g) * 0.02; r[5] = big; r[6] = -big; rows.append(r)      # the largest finite values
    r = torch.randn(cols, generator=g) * tiny * 4; rows.append(r)           # subnormals only
    rows.append(-torch.rand(cols, generator=g))                             # negative only, uniform: a long INT4 tail
    rows.append(torch.rand(cols, generator=g) * 2 - 1)                      # uniform, both signs
    rows.append(-torch.rand(cols, generator=g) * 0.5 - 0.5)                 # every element beyond half the maximum
    r = torch.randn(cols, generator=g); r[r.abs() < 1.0] = 0.0; rows.append(r)              # mostly zeros
    r = (torch.randint(0, 2, (cols,), generator=g).float() * 2 - 1) * 0.75; rows.append(r)  # two values, +-
    return torch.stack(rows).to(dtype).to("cuda")


@pytest.mark.parametrize("dtype", [torch.float16, torch.bfloat16])
@pytest.mark.parametrize("cols", [1024, 4096, 5120, 11008])
@pytest.mark.parametrize("lo", [0.5, 0.02])
def test_special_rows(mq, dtype, cols, lo):  # noqa: F811
    w = _special_rows(cols, dtype)
    for f16 in (False, True):
        check_tensor(mq, w, [orc.INT4, orc.FP4_E2M1], orc.PER_CHANNEL, mi.clip_ratios(100, lo=lo), 0, f16,
                     label=f"special-{cols}-{lo}-{f16}")
