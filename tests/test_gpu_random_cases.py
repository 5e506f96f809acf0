"""Seeded random problems (shapes from 1 coordinate to 400,003, 1 to 255 workers, K from
1 to d, six value distributions incl. heavy ties, mostly zeros, a range down to
denormals, identical rows; fp32 and bf16 gradients) through all three kinds of step,
each compared with the oracle element by element over consecutive steps."""
import sys

import numpy as np
import pytest
import torch

from tests.gpu_util import GpuStepper, assert_matches_oracle
from tests.test_gpu_add_drop import GpuAdStepper

pytestmark = pytest.mark.gpu


def draw_case(rng):
    N = int(rng.choice([1, 2, 3, 5, 8, 16, 31, 64, 255]))
    d = int(rng.choice([1, 7, 63, 1000, 4097, 20011, 65537, 150001, 400003]))
    if N * d > 12_000_000:
        d = max(1, 12_000_000 // N)
    K = [1, max(1, d // 1000), max(1, d // 100), max(1, d // 7), d][int(rng.integers(0, 5))]
    K = min(max(K, 1), d)
    dist = int(rng.integers(0, 6))
    if dist == 0:
        g = rng.standard_normal((N, d))
    elif dist == 1:
        g = rng.standard_t(2, (N, d))
    elif dist == 2:
        g = np.round(rng.standard_normal((N, d)) * 3) / 4                           # heavy ties
    elif dist == 3:
        g = rng.standard_normal((N, d)) * (rng.random((1, d)) < 0.01)               # mostly zeros
    elif dist == 4:
        g = rng.standard_normal((N, d)) * 10.0 ** rng.uniform(-20, 10, (1, d))     # down to denormals
    else:
        g = np.tile(rng.standard_normal((1, d)), (N, 1))                            # identical rows
    g = g.astype(np.float32)
    bf16 = bool(rng.integers(0, 4) == 0)
    if bf16:
        g = torch.from_numpy(g).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    e = (rng.standard_normal((N, d)) * rng.choice([0.0, 0.1])).astype(np.float32)
    return N, d, K, dist, bf16, g, e


@pytest.mark.parametrize("block", range(6))
def test_random_cases(oracle, block):
    for case in range(block * 12, block * 12 + 12):
        rng = np.random.default_rng(7_000_000 + case)
        N, d, K, dist, bf16, g, e = draw_case(rng)
        scheme = int(rng.integers(0, 3))
        what = "case %d: N=%d d=%d K=%d values %d bf16=%s scheme %d" % (case, N, d, K, dist, bf16, scheme)
        print("[case] " + what, flush=True)
        sys.stdout.flush()
        if scheme != 1:
            with GpuStepper(N, d, K, bf16=bf16) as gs:
                gs.set_error(e)
                e_ref = e
                for t in range(2):
                    gs.set_grads(g)
                    if scheme == 0:
                        gs.step()
                        ref = oracle.vote_step(g, e_ref, K, threads=8)
                    else:
                        r = rng.standard_exponential(d).astype(np.float32)
                        if rng.integers(0, 3) == 0:
                            r = np.round(r * 4) / 4                                   # equal times
                        gs.step_rs(r)
                        ref = oracle.rs_vote_step(g, e_ref, K, r, threads=8)
                    assert_matches_oracle(gs.fetch(), ref, what + " step %d" % t)
                    e_ref = ref.err
        else:
            k_ad = int(rng.integers(1, K + 1))
            gs = GpuAdStepper(N, d, K, K, bf16=bf16)
            try:
                vote, msum = np.zeros((N, d), np.uint8), np.zeros(d, np.uint8)
                e_ref = np.zeros((N, d), np.float32)
                for t, ka in enumerate([K, k_ad, k_ad]):
                    ref = oracle.ad_vote_step(g, e_ref, K, ka, vote, msum, threads=8)
                    gs.step(g, ka)
                    gs.compare(ref, what + " step %d" % t)
                    vote, msum, e_ref = ref.vote, ref.msum, ref.err
                    g = np.roll(g, 3, axis=1)
            finally:
                gs.close()
