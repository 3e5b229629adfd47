"""Seeded random sweep of layer-output configurations (token count, output and input
width, weight granularity, metric, candidate order) through the same parity checks as the
hand-picked cases: the matrix-core kernel's tile edges, K tails and workgroup regrouping
depend on all three sizes."""
import numpy as np
import pytest
import torch

import mofq_inputs as mi
from oracle import mofq_oracle as orc
from tests import test_gpu_wa as wa
from tests import test_gpu_w_only_output as wo
from tests.test_gpu_wa import mq  # noqa: F401  (fixture)

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


@pytest.mark.parametrize("seed", range(36))
def test_random_layer(mq, seed):  # noqa: F811
    rng = np.random.default_rng(5000 + seed)
    m = int([rng.integers(1, 40), rng.integers(200, 600), rng.integers(700, 1100)][rng.integers(3)])
    n = int([rng.integers(1, 40), rng.integers(100, 400), rng.integers(900, 1500)][rng.integers(3)])
    k = 64 * int(rng.integers(1, 24))
    gran = [orc.PER_TENSOR, orc.PER_CHANNEL][rng.integers(2)]
    x = mi.activations(m, k, seed=int(rng.integers(1 << 30)), device=DEV,
                       n_outlier=int(rng.integers(0, 7)), outlier_scale=float(rng.choice([1.0, 20.0, 60.0])))
    w = mi.llama_like_weight(n, k, seed=int(rng.integers(1 << 30)), dtype=torch.bfloat16, device=DEV)
    if rng.random() < 0.5:
        cands = [[orc.INT8, orc.FP8_E4M3], [orc.FP8_E4M3, orc.INT8], [orc.INT8], [orc.FP8_E4M3]][rng.integers(4)]
        wa.check_layer(mq, x, w, cands, gran, f"random-wa-{seed}")
    else:
        cands = [[orc.INT4, orc.FP4_E2M1], [orc.FP4_E2M1, orc.INT4], [orc.FP4_E2M1], [orc.INT8, orc.FP8_E4M3]][rng.integers(4)]
        clip = mi.clip_ratios(int([1, 1, 5, 30][rng.integers(4)]))
        wo.check_layer(mq, x, w, cands, gran, clip, f"random-wo-{seed}")
