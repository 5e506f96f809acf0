"""Parity of majority voting with random selection (Algorithm 1, the line with
S_rand-weighted) on the GPU against the oracle's exponential-clock statement, on
the same seeded inputs and the same Exp(1) numbers: every output bit-exact.  One
statistical check ties the GPU's masks to the law itself."""
import sys

import numpy as np
import pytest
import torch

from paper_2011_06495_amd import binding as B
from paper_2011_06495_amd import workloads as W
from tests.gpu_util import GpuStepper, assert_matches_oracle
from tests.rs_law import assert_follows_law, successive_sampling_law

pytestmark = pytest.mark.gpu


def say(msg):
    print("[case] " + msg, flush=True)
    sys.stdout.flush()


SMALL = {
    "C1": W.C1.with_size(150001),
    "C2": W.C2.with_size(300007, N=10),
    "C3": W.C3.with_size(257003, N=16),
    "C4": W.C4.with_size(200003, N=16, lattice_shift=6),
    "C5": W.C5.with_size(180005, N=32),
}


@pytest.mark.parametrize("name", sorted(SMALL))
def test_reduced_workloads_three_steps(oracle, name):
    w = SMALL[name]
    say("random selection, reduced %s N=%d d=%d K=%d" % (name, w.N, w.d, w.K))
    e_ref = W.zero_error(w)
    with GpuStepper(w.N, w.d, w.K, bf16=(w.grad_dtype == "bf16")) as gs:
        gs.set_error(e_ref)
        for t in range(3):
            g = W.gradients(w, t)
            r = W.selection_clocks(w, t)
            gs.set_grads(g)
            gs.step_rs(r)
            got = gs.fetch()
            ref = oracle.rs_vote_step(g, e_ref, w.K, r, threads=8)
            assert_matches_oracle(got, ref, "%s step %d" % (name, t))
            assert np.all(ref.votes[got.mask_idx] >= 1)
            e_ref = ref.err


@pytest.mark.parametrize("d,K,N", [(1, 1, 1), (2, 1, 3), (5, 5, 2), (31, 7, 4), (1024, 1024, 2), (1025, 3, 5),
                                   (16385, 100, 3), (70001, 69999, 2), (50000, 500, 255)])
def test_edge_shapes(oracle, d, K, N):
    say("random selection, edge d=%d K=%d N=%d" % (d, K, N))
    rng = np.random.default_rng(d * 7 + K)
    g = rng.standard_normal((N, d)).astype(np.float32)
    e = (rng.standard_normal((N, d)) * 0.1).astype(np.float32)
    r = rng.standard_exponential(d).astype(np.float32)
    with GpuStepper(N, d, K) as gs:
        gs.set_error(e)
        gs.set_grads(g)
        gs.step_rs(r)
        assert_matches_oracle(gs.fetch(), oracle.rs_vote_step(g, e, K, r), "edge")


@pytest.mark.parametrize("clocks", ["all_equal", "all_zero", "few_levels", "one_bin"])
def test_equal_times_go_to_the_lowest_coordinate(oracle, clocks):
    """Numbers chosen so that many times tie (exactly equal quotients), so that all
    of them share the leading bits of their key, or so that nothing but the
    coordinate decides."""
    N, d, K = 6, 120011, 1500
    rng = np.random.default_rng(11)
    g = rng.standard_normal((N, d)).astype(np.float32)
    e = np.zeros_like(g)
    if clocks == "all_equal":
        r = np.ones(d, np.float32)                                   # time = 1 / votes
    elif clocks == "all_zero":
        r = np.zeros(d, np.float32)                                  # every time is zero
    elif clocks == "few_levels":
        r = rng.integers(1, 4, d).astype(np.float32)                 # 1, 2, 3 over votes 1..6
    else:
        r = (1.0 + rng.random(d) * 2.0 ** -12).astype(np.float32)    # a few thousand distinct values in one bin
    say("random selection, ties: %s" % clocks)
    with GpuStepper(N, d, K) as gs:
        gs.set_error(e)
        gs.set_grads(g)
        gs.step_rs(r)
        assert_matches_oracle(gs.fetch(), oracle.rs_vote_step(g, e, K, r), clocks)


def test_random_selection_with_infinite_magnitudes(oracle):
    """Infinite gradients only change who votes: the clocks are the caller's finite numbers."""
    N, d, K = 4, 50003, 300
    say("random selection, infinities N=%d d=%d K=%d" % (N, d, K))
    rng = np.random.default_rng(32)
    sign = np.where(rng.integers(0, 2, size=d) == 1, np.float32(np.inf), np.float32(-np.inf))
    e = np.zeros((N, d), np.float32)
    with GpuStepper(N, d, K) as gs:
        gs.set_error(e)
        for t in range(2):
            g = rng.standard_normal((N, d)).astype(np.float32)
            if t == 0:
                hot = rng.choice(d, size=80, replace=False)
                g[0, hot] = sign[hot]
                g[3, hot[:30]] = sign[hot[:30]]
            r = rng.exponential(size=d).astype(np.float32)
            gs.set_grads(g)
            gs.step_rs(r)
            got = gs.fetch()
            ref = oracle.rs_vote_step(g, e, K, r)
            assert not np.isnan(ref.err).any() and not np.isnan(ref.agg).any()
            assert_matches_oracle(got, ref, "random selection, infinities, step %d" % t)
            e = ref.err


def test_plain_and_random_steps_share_a_context(oracle):
    """The result of either kind of step does not depend on which kind ran before."""
    w = W.C2.with_size(210007, N=8)
    g0, g1 = W.gradients(w, 0), W.gradients(w, 1)
    r0, r1 = W.selection_clocks(w, 0), W.selection_clocks(w, 1)
    e = W.zero_error(w)
    say("random selection, alternating with plain steps")
    with GpuStepper(w.N, w.d, w.K, want_worker_idx=False, want_votes=False) as gs:
        gs.set_error(e)
        for t, (g, r) in enumerate([(g0, r0), (g1, None), (g0, r1), (g1, None), (g1, r0)]):
            gs.set_grads(g)
            if r is None:
                gs.step()
                ref = oracle.vote_step(g, e, w.K, threads=8)
            else:
                gs.step_rs(r)
                ref = oracle.rs_vote_step(g, e, w.K, r, threads=8)
            assert_matches_oracle(gs.fetch(), ref, "mixed step %d" % t)
            e = ref.err


def test_argument_errors():
    N, d, K = 2, 1000, 10
    with GpuStepper(N, d, K) as gs:
        L = B.load()
        st = L.mv_rs_vote_step(gs.ctx, gs.g.data_ptr(), gs.ld_g, gs.e.data_ptr(), gs.ld_e, 0, 0, 0,
                               gs.mask.data_ptr(), gs.agg.data_ptr(), 0)
        assert st == B.MV_ERR_INVALID_ARG                                  # no random numbers
        r = torch.ones(d + 1, dtype=torch.float32, device=gs.dev)
        st = L.mv_rs_vote_step(gs.ctx, gs.g.data_ptr(), gs.ld_g, gs.e.data_ptr(), gs.ld_e, r.data_ptr() + 2, 0, 0,
                               gs.mask.data_ptr(), gs.agg.data_ptr(), 0)
        assert st == B.MV_ERR_INVALID_ARG                                  # misaligned
        torch.cuda.synchronize()


def test_masks_follow_the_law(oracle):
    """A tiny problem whose votes are known: the frequencies of the masks over many
    independent sets of Exp(1) numbers against the closed-form law."""
    N, d, K = 3, 6, 2
    g = np.array([[9, 8, 0.1, 0.2, 0.3, 0.0],
                  [9, 0.1, 8, 0.2, 0.3, 0.0],
                  [9, 0.1, 0.2, 0.3, 8, 0.0]], np.float32)        # votes 3,1,1,0,1,0
    e = np.zeros_like(g)
    votes = oracle.vote_step(g, e, K).votes
    assert votes.tolist() == [3, 1, 1, 0, 1, 0]
    law = successive_sampling_law(votes.tolist(), K)
    rng = np.random.default_rng(2024)
    trials = 3000
    counts = {}
    say("random selection, %d masks against the law" % trials)
    with GpuStepper(N, d, K, want_worker_idx=False, want_votes=False) as gs:
        gs.set_grads(g)
        for _ in range(trials):
            gs.set_error(e)
            gs.step_rs(rng.standard_exponential(d).astype(np.float32))
            torch.cuda.synchronize()
            m = tuple(gs.mask[:K].cpu().numpy().view(np.uint32).tolist())
            counts[m] = counts.get(m, 0) + 1
    assert_follows_law(counts, trials, law, "GPU masks")
