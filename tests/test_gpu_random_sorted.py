"""Seeded random sweep aimed at the sorted per-channel search (16-bit rows of 1024 to 24576
columns, 4-bit formats, 8 or more clip ratios): every instance of the kernel (row-length
tilings up to 1024 threads), ragged row ends, one and two formats, fp16 scales, and value
distributions with heavy duplicates, wide dynamic range, subnormals and outliers, through
the same element-by-element parity check against the oracle as the hand-picked cases."""
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
