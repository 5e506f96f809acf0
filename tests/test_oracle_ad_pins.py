"""Pins of the add-drop oracle (Algorithm 2): a pure-Python set implementation on
tiny inputs, reduction to Algorithm 1 when K_ad = K from an empty state, and the
invariants the paper states (the PS's cumulative sum equals the sum of the
workers' current votes; at most K_ad additions and removals per worker)."""
import struct

import numpy as np
import pytest


def f32_bits(x):
    return struct.unpack("<I", struct.pack("<f", float(x)))[0] & 0x7FFFFFFF


def brute_ad_step(g, e, K, K_ad, votes, msum):
    """Algorithm 2 with Python sets.  votes: list of sets; msum: list of ints."""
    N, d = g.shape
    a = (g + e).astype(np.float32)
    adds, drops, tops = [], [], []
    for n in range(N):
        key = [f32_bits(x) for x in a[n]]
        top = set(sorted(range(d), key=lambda j: (-key[j], j))[:K])
        A = sorted(top - votes[n], key=lambda j: (-key[j], j))[:K_ad]
        D = sorted(votes[n] - top, key=lambda j: (key[j], j))[:K_ad]
        adds.append(sorted(A))
        drops.append(sorted(D))
        tops.append(sorted(top))
    new_votes = []
    msum = list(msum)
    for n in range(N):
        new_votes.append((votes[n] | set(adds[n])) - set(drops[n]))
        for j in adds[n]:
            msum[j] += 1
        for j in drops[n]:
            msum[j] -= 1
    mask = sorted(sorted(range(d), key=lambda j: (-msum[j], j))[:K])
    return tops, adds, drops, new_votes, msum, mask


@pytest.mark.parametrize("d,K,K_ad,N,levels", [(12, 4, 1, 2, 0), (40, 8, 3, 3, 4), (64, 16, 16, 4, 0), (50, 10, 2, 5, 3)])
def test_ad_bruteforce_multi_step(oracle, d, K, K_ad, N, levels):
    rng = np.random.default_rng(d + K)
    vote = np.zeros((N, d), np.uint8)
    msum = np.zeros(d, np.uint8)
    bv = [set() for _ in range(N)]
    bm = [0] * d
    e = np.zeros((N, d), np.float32)
    for t in range(7):
        g = rng.standard_normal((N, d)).astype(np.float32)
        if levels:
            g = np.round(g * levels) / np.float32(levels)          # heavy ties
        r = oracle.ad_vote_step(g, e, K, K_ad, vote, msum)
        tops, adds, drops, bv, bm, mask = brute_ad_step(g, e, K, K_ad, bv, bm)
        for n in range(N):
            assert r.worker_idx[n].tolist() == tops[n]
            assert r.add_idx[n].tolist() == adds[n], (t, n)
            assert r.drop_idx[n].tolist() == drops[n], (t, n)
            assert set(np.flatnonzero(r.vote[n]).tolist()) == bv[n]
        assert r.msum.tolist() == bm
        assert r.mask_idx.tolist() == mask
        vote, msum, e = r.vote, r.msum, r.err


def test_full_first_vote_is_algorithm_1(oracle):
    """From the empty state, K_ad = K adds every top-K coordinate: the step is the
    plain majority vote."""
    from paper_2011_06495_amd import workloads as W
    w = W.C2.with_size(20000, N=6)
    g, e = W.gradients(w, 0), W.zero_error(w)
    mv = oracle.vote_step(g, e, w.K)
    ad = oracle.ad_vote_step(g, e, w.K, w.K, np.zeros((w.N, w.d), np.uint8), np.zeros(w.d, np.uint8))
    assert np.array_equal(ad.worker_idx, mv.worker_idx)
    assert np.array_equal(ad.msum, mv.votes)
    assert np.array_equal(ad.mask_idx, mv.mask_idx)
    assert np.array_equal(ad.agg.view(np.uint32), mv.agg.view(np.uint32))
    assert np.array_equal(ad.err.view(np.uint32), mv.err.view(np.uint32))
    for n in range(w.N):
        assert np.array_equal(ad.add_idx[n], mv.worker_idx[n]) and ad.drop_idx[n].size == 0
        assert np.array_equal(np.flatnonzero(ad.vote[n]).astype(np.uint32), mv.worker_idx[n])


def test_ad_invariants_over_steps(oracle):
    from paper_2011_06495_amd import workloads as W
    w = W.C2.with_size(30000, N=5, K=300)
    K, K_ad = w.K, 30
    vote = np.zeros((w.N, w.d), np.uint8)
    msum = np.zeros(w.d, np.uint8)
    e = W.zero_error(w)
    sizes = []
    for t in range(14):
        g = W.gradients(w, t)
        r = oracle.ad_vote_step(g, e, K, K_ad, vote, msum, threads=4)
        keys = np.abs(g + e).view(np.uint32)
        for n in range(w.N):
            top = np.zeros(w.d, bool)
            top[r.worker_idx[n]] = True
            prev = vote[n].astype(bool)
            A, D = top & ~prev, prev & ~top
            assert r.add_idx[n].size == min(K_ad, int(A.sum()))
            assert r.drop_idx[n].size == min(K_ad, int(D.sum()))
            assert A[r.add_idx[n]].all() and D[r.drop_idx[n]].all()
            if r.add_idx[n].size:       # the added ones are the largest of A
                rest = A.copy()
                rest[r.add_idx[n]] = False
                if rest.any():
                    assert keys[n][r.add_idx[n]].min() >= keys[n][rest].max()
            if r.drop_idx[n].size:      # the dropped ones are the smallest of D
                rest = D.copy()
                rest[r.drop_idx[n]] = False
                if rest.any():
                    assert keys[n][r.drop_idx[n]].max() <= keys[n][rest].min()
            # |A| - |D| = K - |previous vote|: a vote of K coordinates trades one for one
            assert int(A.sum()) - int(D.sum()) == K - int(prev.sum())
            new = prev.copy()
            new[r.add_idx[n]] = True
            new[r.drop_idx[n]] = False
            assert np.array_equal(new, r.vote[n].astype(bool))
        # Sec. 3: the PS's cumulative sum is the sum of the workers' current votes
        assert np.array_equal(r.msum, r.vote.sum(axis=0).astype(np.uint8))
        sizes.append(r.vote.sum(axis=1))
        assert np.all(sizes[-1] <= K)
        vote, msum, e = r.vote, r.msum, r.err
    sizes = np.array(sizes)
    assert np.all(np.diff(sizes, axis=0) >= 0)            # a vote never shrinks
    assert np.all(sizes[0] == K_ad) and sizes[-1].max() > K_ad


def test_ad_converges_to_plain_vote_on_frozen_input(oracle):
    """With the same compensated vectors every step, the add-drop votes reach the
    plain top-K sets after ceil(K / K_ad) steps and then stop changing."""
    rng = np.random.default_rng(5)
    N, d, K, K_ad = 4, 3000, 60, 7
    g = rng.standard_normal((N, d)).astype(np.float32)
    e = np.zeros_like(g)
    mv = oracle.vote_step(g, e, K)
    vote = np.zeros((N, d), np.uint8)
    msum = np.zeros(d, np.uint8)
    for t in range(10):
        r = oracle.ad_vote_step(g, e, K, K_ad, vote, msum)     # e is not carried: the input is frozen
        vote, msum = r.vote, r.msum
        if t >= 9:
            assert all(x.size == 0 for x in r.add_idx) and all(x.size == 0 for x in r.drop_idx)
    assert np.array_equal(msum, mv.votes)
    assert np.array_equal(r.mask_idx, mv.mask_idx)


def test_ad_argument_and_state_errors(oracle):
    g = np.zeros((2, 10), np.float32)
    z = np.zeros((2, 10), np.uint8)
    with pytest.raises(ValueError):
        oracle.ad_vote_step(g, g, 3, 4, z, np.zeros(10, np.uint8))      # K_ad > K
    with pytest.raises(ValueError):
        oracle.ad_vote_step(g, g, 3, 0, z, np.zeros(10, np.uint8))
    # a vote that the sum does not account for
    g = np.arange(20, dtype=np.float32).reshape(2, 10)
    bad = z.copy()
    bad[:, 0] = 1
    with pytest.raises(ValueError):
        oracle.ad_vote_step(g, np.zeros_like(g), 3, 3, bad, np.zeros(10, np.uint8))
