"""GPU parity on seeded random ragged batches: every row of every sequence against the oracle.
Shapes the other tests do not list one by one: random head groupings and dtypes, short prefill
ranges, short ranges over long contexts, decode rows mixed with prefill (some of them forks of
their neighbour), empty and one-token ranges."""
import numpy as np
import pytest

import mc_inputs as mi
from test_gpu_parity import check_attention, small_workload

pytestmark = pytest.mark.gpu

HEADS = [(8, 8), (8, 2), (16, 2), (32, 8), (4, 2), (16, 16), (64, 8)]


def random_workload(case, rng):
    Hq, Hkv = HEADS[int(rng.integers(0, len(HEADS)))]
    dtype = [mi.F16, mi.BF16][int(rng.integers(0, 2))]
    kind = int(rng.integers(0, 4))
    batch = int(rng.integers(1, 9)) if kind != 2 else int(rng.integers(2, 40))
    lens, begins = [], []
    for _ in range(batch):
        if kind == 0:      # short prefill ranges
            n = int(rng.integers(1, 400))
            b = int(rng.integers(0, n + 1))
        elif kind == 1:    # long contexts, short ranges
            n = int(rng.integers(300, 3000))
            b = n - int(rng.integers(0, 40))
        elif kind == 2:    # decode rows with a few prefill ranges
            n = int(rng.integers(1, 2500))
            b = n - 1 if rng.random() < 0.8 else int(rng.integers(0, n + 1))
        else:
            n = int(rng.integers(1, 1200))
            b = int(rng.integers(0, n + 1))
        lens.append(n)
        begins.append(b)
    if sum(n - b for n, b in zip(lens, begins)) == 0:
        begins[0] = max(0, lens[0] - 1)
    w = small_workload(9000 + case, dtype, Hq, Hkv, lens, begins)
    if kind == 2 and rng.random() < 0.5:       # neighbouring decode rows forked from one another
        for s in range(1, batch):
            both_decode = lens[s] - begins[s] == 1 and lens[s - 1] - begins[s - 1] == 1
            if both_decode and rng.random() < 0.7:
                pages = min(begins[s], begins[s - 1]) // 16
                shared = int(rng.integers(0, pages + 1)) * 16
                if shared:
                    w.share_prefix(s, s - 1, shared)
    return w


@pytest.mark.parametrize("chunk", range(6))
def test_random_batches(chunk):
    rng = np.random.default_rng(4000 + chunk)
    for i in range(10):
        check_attention(random_workload(10 * chunk + i, rng))
