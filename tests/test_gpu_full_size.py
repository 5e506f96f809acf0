"""Parity at the benchmark's full sizes, in the launch configuration bench.py
times (all outputs requested, error buffer carried on the device from step to
step).  The oracle runs the whole step on the host (row-parallel, same
arithmetic) and every output is compared element by element."""
import sys
import time

import numpy as np
import pytest

from paper_2011_06495_amd import workloads as W
from tests.gpu_util import GpuStepper, assert_matches_oracle

pytestmark = pytest.mark.gpu


def say(msg):
    print("[case] " + msg, flush=True)
    sys.stdout.flush()


def run_full(oracle, w, steps, check_ties=False):
    threads = min(16, oracle.max_threads())
    e_ref = W.zero_error(w)
    paths = []
    with GpuStepper(w.N, w.d, w.K, bf16=(w.grad_dtype == "bf16")) as gs:
        gs.set_error(e_ref)
        for t in range(steps):
            t0 = time.time()
            g = W.gradients(w, t, threads=threads)
            gs.set_grads(g)
            gs.step()
            got = gs.fetch()
            ref = oracle.vote_step(g, e_ref, w.K, threads=threads)
            assert_matches_oracle(got, ref, "%s full size, step %d" % (w.name, t))
            cand, _, path = gs.row_stats()
            paths.append(path)
            if check_ties:
                # the lattice workload must exercise both tie-breaks at full size
                a = (g + e_ref) if g.dtype == np.float32 else None
                keys = np.abs(a).view(np.uint32)
                for n in range(w.N):
                    kmin = keys[n][ref.worker_idx[n]].min()
                    n_tied = int(np.count_nonzero(keys[n] == kmin))
                    n_taken = int(np.count_nonzero(keys[n][ref.worker_idx[n]] == kmin))
                    assert n_tied > n_taken >= 1, "row %d: boundary tie group not split" % n
                vmin = ref.votes[ref.mask_idx].min()
                assert np.count_nonzero(ref.votes == vmin) > np.count_nonzero(ref.votes[ref.mask_idx] == vmin)
            e_ref = ref.err
            say("%s step %d ok (%.1f s), candidates/row %d..%d, slow rows %d" %
                (w.name, t, time.time() - t0, min(cand), max(cand), sum(1 for p in path if p == 1)))
    return paths


@pytest.mark.timeout(900)
def test_c1_full(oracle):
    run_full(oracle, W.C1, 1)


@pytest.mark.timeout(900)
def test_c2_full(oracle):
    run_full(oracle, W.C2, 1)


@pytest.mark.timeout(1200)
def test_c3_full_heavy_tails_many_steps(oracle):
    run_full(oracle, W.C3, 20)


@pytest.mark.timeout(1200)
def test_c4_full_lattice_ties_five_steps(oracle):
    paths = run_full(oracle, W.C4, 5, check_ties=True)
    assert all(p != 1 for step in paths for p in step), "the headline workload must not take the slow path"


@pytest.mark.timeout(1200)
def test_c5_full_bf16(oracle):
    run_full(oracle, W.C5, 10)


# ---- majority voting with add-drop (Algorithm 2) at full size

def run_full_ad(oracle, w, k_ads):
    from tests.test_gpu_add_drop import GpuAdStepper
    threads = min(16, oracle.max_threads())
    gs = GpuAdStepper(w.N, w.d, w.K, max(k_ads), bf16=(w.grad_dtype == "bf16"))
    try:
        vote = np.zeros((w.N, w.d), np.uint8)
        msum = np.zeros(w.d, np.uint8)
        e = W.zero_error(w)
        for t, k_ad in enumerate(k_ads):
            t0 = time.time()
            g = W.gradients(w, t, threads=threads)
            gs.step(g, k_ad)
            ref = oracle.ad_vote_step(g, e, w.K, k_ad, vote, msum, threads=threads)
            gs.compare(ref, "%s add-drop full size, step %d" % (w.name, t))
            vote, msum, e = ref.vote, ref.msum, ref.err
            say("%s add-drop step %d (K_ad=%d) ok (%.1f s), added %s.. dropped %s.." %
                (w.name, t, k_ad, time.time() - t0, [x.size for x in ref.add_idx[:3]],
                 [x.size for x in ref.drop_idx[:3]]))
    finally:
        gs.close()


@pytest.mark.timeout(1200)
def test_add_drop_c4_full(oracle):
    # a full first vote, then the regime phi_ad = phi / 10 (Sec. 4.2)
    k_ad = W.C4.K // 10
    run_full_ad(oracle, W.C4, [W.C4.K, k_ad, k_ad, k_ad])


@pytest.mark.timeout(1200)
def test_add_drop_paper_regime_full(oracle):
    # the paper's setting: ResNet-18 size, N = 10 workers, phi = 1e-2, phi_ad = 1e-3 (Sec. 4.1, 4.2)
    w = W.C2.with_size(W.C2.d, K=111740)
    run_full_ad(oracle, w, [w.K, 11174, 11174])


@pytest.mark.timeout(1200)
def test_add_drop_c5_full_bf16(oracle):
    # the largest workload (102 M coordinates, bf16 gradients): a full first vote, then phi_ad = phi / 10
    run_full_ad(oracle, W.C5, [W.C5.K, W.C5.K // 10])


# ---- majority voting with random selection (Algorithm 1, S_rand-weighted) at full size

def run_full_rs(oracle, w, steps):
    threads = min(16, oracle.max_threads())
    e_ref = W.zero_error(w)
    with GpuStepper(w.N, w.d, w.K, bf16=(w.grad_dtype == "bf16")) as gs:
        gs.set_error(e_ref)
        for t in range(steps):
            t0 = time.time()
            g = W.gradients(w, t, threads=threads)
            r = W.selection_clocks(w, t)
            gs.set_grads(g)
            gs.step_rs(r)
            got = gs.fetch()
            ref = oracle.rs_vote_step(g, e_ref, w.K, r, threads=threads)
            assert_matches_oracle(got, ref, "%s random selection full size, step %d" % (w.name, t))
            # what holds at any size: winners have votes, and more votes win more often
            v = ref.votes
            assert np.all(v[got.mask_idx] >= 1)
            inside = np.zeros(w.d, bool)
            inside[got.mask_idx] = True
            rate = [inside[v == lvl].mean() for lvl in (1, 2, 3) if np.count_nonzero(v == lvl) > 2000]
            assert all(a < b for a, b in zip(rate, rate[1:])), "selection rate does not grow with the votes: %s" % rate
            e_ref = ref.err
            say("%s random selection step %d ok (%.1f s), voted coordinates %d, rate by votes %s" %
                (w.name, t, time.time() - t0, int(np.count_nonzero(v)), ["%.3f" % x for x in rate]))


@pytest.mark.timeout(1200)
def test_random_selection_c4_full(oracle):
    run_full_rs(oracle, W.C4, 3)


@pytest.mark.timeout(1200)
def test_random_selection_c5_full_bf16(oracle):
    run_full_rs(oracle, W.C5, 2)


@pytest.mark.timeout(1200)
def test_random_selection_paper_regime_full(oracle):
    # ResNet-18 size, N = 10 workers, phi = 1e-2 (Sec. 4.1, 4.2)
    w = W.C2.with_size(W.C2.d, K=111740)
    run_full_rs(oracle, w, 2)


@pytest.mark.timeout(1200)
def test_paper_regime_full(oracle):
    # the paper's own setting for plain majority voting: ResNet-18 size, N = 10, phi = 1e-2 (Sec. 4.1, 4.2);
    # about 2K = 223,000 candidates per row: the select spread over many workgroups
    w = W.C2.with_size(W.C2.d, K=111740)
    paths = run_full(oracle, w, 2)
    assert all(p != 1 for step in paths for p in step)


@pytest.mark.timeout(900)
def test_rows_longer_than_2_30_coordinates():
    """Two rows of 2^30 + 4099 coordinates: byte offsets inside a row pass 2^32 and
    coordinates pass 2^30.  A full sort on the host would take minutes, so the check
    is by construction: 64 planted values far above a floor of small noise must be
    each worker's vote, the mask, the aggregate, and the only coordinates the error
    buffers lose.  Row 0's noise is uniform (one histogram bin then holds far more
    coordinates than a candidate list: the exact path from memory), row 1's is
    exponential (the candidate-list route)."""
    d, K, N = (1 << 30) + 4099, 64, 2
    rng = np.random.default_rng(99)
    say("two rows of %d coordinates" % d)
    t0 = time.time()
    fixed = np.array([0, 1, 1023, 1024, (1 << 20) + 1, (1 << 30) - 1, 1 << 30, (1 << 30) + 1, d - 1])
    others = np.setdiff1d(np.unique(rng.integers(0, d, 200)), fixed)[:K - fixed.size]
    planted = np.sort(np.concatenate([fixed, others]))
    assert planted.size == K and np.unique(planted).size == K
    sign = np.where(np.arange(K) % 2 == 0, 1.0, -1.0).astype(np.float32)
    vals = [(2.0 + np.arange(K)).astype(np.float32) * sign, (100.0 - np.arange(K)).astype(np.float32) * sign]
    with GpuStepper(N, d, K) as gs:
        gs.e[:, :d].zero_()
        rows = []
        for n in range(N):
            if n == 0:
                g = rng.random(d, dtype=np.float32)
            else:
                g = rng.standard_exponential(d, dtype=np.float32)
            g *= np.float32(1e-3)                       # exponential: the largest of 2^30 is about 0.021
            g[planted] = vals[n]
            gs.g[n, :d].copy_(torch_from(g))
            g[planted] = 0.0
            rows.append(g)
        gs.step()
        got = gs.fetch()
        cand, _, path = gs.row_stats()
    say("  step done after %.1f s, candidates %s path %s" % (time.time() - t0, cand, path))
    assert path[0] == 1 and path[1] != 1, "row 0 is meant for the exact path, row 1 for its candidate list"
    for n in range(N):
        assert np.array_equal(got.worker_idx[n], planted.astype(np.uint32))
        assert np.array_equal(got.err[n], rows[n])
    assert np.array_equal(got.mask_idx, planted.astype(np.uint32))
    assert np.array_equal(np.flatnonzero(got.votes), planted)
    assert np.all(got.votes[planted] == N)
    assert np.array_equal(got.agg, (vals[0] + vals[1]) * np.float32(0.5))


def torch_from(a):
    import torch
    return torch.from_numpy(a)
