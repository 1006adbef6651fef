"""GPU parity on seeded random jagged batches: random model shape and storage type, 1-5 users with random
prefix / suffix / candidate counts (including empty prefixes, empty suffixes and users without candidates),
a random subset of users uncached, random pool page size.  Every case checks ranking on the cached prefix
and full recompute against the CPU oracle, user by user.  The last eight cases use the second attention form
(softmax over the visible keys)."""
import numpy as np
import pytest

import synth
from test_gpu_parity import run_three_routes

pytestmark = pytest.mark.gpu

SHAPES = [(64, 2, "fp32"), (128, 2, "fp32"), (128, 2, "bf16"), (128, 4, "bf16"), (256, 4, "bf16"), (256, 2, "bf16"),
          (512, 8, "bf16"), (128, 2, "fp16"), (256, 4, "fp16"), (512, 4, "fp16")]


@pytest.mark.parametrize("case", range(24))
def test_random_jagged_batch(case):
    rng = np.random.default_rng(1000 + case)
    d, H, dtype = SHAPES[case % len(SHAPES)]
    n = int(rng.integers(1, 6))
    L = [int(x) for x in rng.choice([0, 1, 31, 64, 65, 127, 200, 333, 512, 700], size=n)]
    S = [int(x) for x in rng.choice([0, 0, 1, 5, 63, 64, 65, 130], size=n)]
    M = [int(x) for x in rng.choice([0, 1, 2, 33, 64, 129, 256, 300], size=n)]
    if sum(M) == 0:
        M[0] = 7
    miss = tuple(int(u) for u in range(n) if rng.random() < 0.3)
    cfg = synth.ModelConfig(int(rng.integers(1, 4)), d, H, dtype, attention="softmax" if case >= 16 else "silu")
    run_three_routes(cfg, 2000 + case, L, S, M, page_tokens=int(rng.choice([64, 128, 256])), miss=miss)
