"""Pins of majority voting with random selection (Algorithm 1, the line with
S_rand-weighted; Sec. 2, paragraph after Algorithm 1; Sec. 4.2).

What the paper fixes is the law: winners are drawn with probabilities proportional
to the votes until K distinct ones are selected.  For small vectors that law has a
closed form (sum over the orders in which a set can be drawn of the product of
w_j / (W - weights drawn before)); both statements of the sampler in the oracle --
the sequential draws and the exponential clocks -- are checked against it, and
against each other on a larger case.  Hand-worked draws, special cases (equal votes,
K = number of voted positions, unvoted positions) and the composition of the whole
step complete the pins."""
import numpy as np
import pytest

from tests.rs_law import assert_follows_law, successive_sampling_law


def test_hand_worked_draws(oracle):
    # votes 2,0,1,3: the six votes lie at positions 0,0,2,3,3,3.  u = 0 -> vote 0 -> position 0;
    # u = 0.4 -> vote 2 -> position 2; u = 0.1 -> vote 0 -> position 0 again (in vain);
    # u = 0.99 -> vote 5 -> position 3.  Three distinct positions after four draws.
    votes = np.array([2, 0, 1, 3], np.uint8)
    mask, used = oracle.rs_mask_draws(votes, 3, np.array([0.0, 0.4, 0.1, 0.99, 0.5]))
    assert mask.tolist() == [0, 2, 3] and used == 4
    mask, used = oracle.rs_mask_draws(votes, 1, np.array([0.34]))        # vote 2 -> position 2
    assert mask.tolist() == [2] and used == 1
    with pytest.raises(ValueError):
        oracle.rs_mask_draws(votes, 3, np.array([0.0, 0.1]))             # numbers run out
    with pytest.raises(ValueError):
        oracle.rs_mask_draws(votes, 4, np.zeros(100))                    # only 3 positions have a vote


def test_hand_worked_clocks(oracle):
    # times: 1.0/2 = 0.5, (no vote), 0.4/1 = 0.4, 1.6/3 = 0.533: the first two to ring are 2 and 0
    votes = np.array([2, 0, 1, 3], np.uint8)
    e = np.array([1.0, 0.0, 0.4, 1.6], np.float32)
    assert oracle.rs_mask_keys(votes, 2, e).tolist() == [0, 2]
    assert oracle.rs_mask_keys(votes, 1, e).tolist() == [2]
    assert oracle.rs_mask_keys(votes, 3, e).tolist() == [0, 2, 3]        # all voted positions; never position 1
    with pytest.raises(ValueError):
        oracle.rs_mask_keys(votes, 4, e)
    # equal times: 2/2 = 1/1 = 3/3 -> lowest positions first
    e = np.array([2.0, 0.0, 1.0, 3.0], np.float32)
    assert oracle.rs_mask_keys(votes, 2, e).tolist() == [0, 2]


@pytest.mark.parametrize("votes,K", [([3, 1, 2, 0, 1], 2), ([1, 1, 1, 1], 2), ([5, 1, 1, 0, 2, 1], 3),
                                     ([7, 1], 1)])
def test_both_samplers_follow_the_successive_sampling_law(oracle, votes, K):
    law = successive_sampling_law(votes, K)
    assert abs(sum(law.values()) - 1.0) < 1e-12
    v = np.array(votes, np.uint8)
    rng = np.random.default_rng(len(votes) * 100 + K)
    trials = 20000
    draws, clocks = {}, {}
    for _ in range(trials):
        m, _used = oracle.rs_mask_draws(v, K, rng.random(400))
        draws[tuple(m.tolist())] = draws.get(tuple(m.tolist()), 0) + 1
        m = oracle.rs_mask_keys(v, K, rng.standard_exponential(len(votes)).astype(np.float32))
        clocks[tuple(m.tolist())] = clocks.get(tuple(m.tolist()), 0) + 1
    assert_follows_law(draws, trials, law, "sequential draws")
    assert_follows_law(clocks, trials, law, "exponential clocks")


def test_first_winner_is_proportional_to_the_votes(oracle):
    # K = 1: P(j) = votes[j] / sum(votes), the sentence of Sec. 2 itself
    v = np.array([4, 0, 1, 2, 8, 1], np.uint8)
    rng = np.random.default_rng(5)
    trials = 40000
    hits = np.zeros((2, v.size))
    for _ in range(trials):
        hits[0, oracle.rs_mask_draws(v, 1, rng.random(1))[0][0]] += 1
        hits[1, oracle.rs_mask_keys(v, 1, rng.standard_exponential(v.size).astype(np.float32))[0]] += 1
    p = v / v.sum()
    sigma = np.sqrt(p * (1 - p) / trials)
    assert np.all(np.abs(hits / trials - p) <= 5 * sigma + 1e-12)
    assert hits[0, 1] == 0 and hits[1, 1] == 0


def test_the_two_samplers_agree_on_a_larger_vector(oracle):
    """Inclusion frequencies per position, d = 60, K = 12, votes 0..8."""
    rng = np.random.default_rng(17)
    v = rng.integers(0, 9, 60).astype(np.uint8)
    v[:5] = 0
    K, trials = 12, 6000
    inc = np.zeros((2, v.size))
    for _ in range(trials):
        inc[0, oracle.rs_mask_draws(v, K, rng.random(4000))[0]] += 1
        inc[1, oracle.rs_mask_keys(v, K, rng.standard_exponential(v.size).astype(np.float32))] += 1
    assert inc[:, v == 0].sum() == 0
    f = inc / trials
    pooled = f.mean(axis=0)
    sigma = np.sqrt(2 * pooled * (1 - pooled) / trials)
    assert np.all(np.abs(f[0] - f[1]) <= 5 * sigma + 1e-9)
    # more votes, more often selected (Sec. 4.2, last sentence on the scheme): compare vote levels
    lo, hi = f[1][(v > 0) & (v <= 2)].mean(), f[1][v >= 7].mean()
    assert hi > 2 * lo


def test_clocks_special_cases(oracle):
    rng = np.random.default_rng(23)
    d, K = 5000, 400
    e = rng.standard_exponential(d).astype(np.float32)
    # equal votes: the K smallest numbers, whatever the common vote count (library sort)
    for level in (1, 3):
        v = np.full(d, level, np.uint8)
        want = np.sort(np.argsort(e, kind="stable")[:K])
        assert np.array_equal(oracle.rs_mask_keys(v, K, e), want.astype(np.uint32))
    # K = number of voted positions: exactly the voted positions
    v = (rng.random(d) < 0.1).astype(np.uint8) * rng.integers(1, 16, d).astype(np.uint8)
    voted = np.flatnonzero(v)
    assert np.array_equal(oracle.rs_mask_keys(v, voted.size, e), voted.astype(np.uint32))
    # a vote count multiplies the rate: doubling rand_exp and the votes together changes nothing
    v2 = (v.astype(np.uint16) * 2).astype(np.uint8)
    assert np.array_equal(oracle.rs_mask_keys(v, 100, e), oracle.rs_mask_keys(v2, 100, e * np.float32(2)))
    # overwhelming majority: a position with 255 votes against ones is nearly always in
    v = np.ones(1000, np.uint8)
    v[123] = 255
    inside = sum(123 in oracle.rs_mask_keys(v, 10, rng.standard_exponential(1000).astype(np.float32))
                 for _ in range(300))
    assert inside >= 250            # law: 1 - prod over ten draws of about (1 - 255/1254) ... = 0.90


def test_whole_step_is_algorithm_1_with_the_random_mask(oracle):
    rng = np.random.default_rng(3)
    N, d, K = 5, 3000, 60
    g = rng.standard_normal((N, d)).astype(np.float32)
    e = (rng.standard_normal((N, d)) * 0.1).astype(np.float32)
    r = rng.standard_exponential(d).astype(np.float32)
    plain = oracle.vote_step(g, e, K)
    rs = oracle.rs_vote_step(g, e, K, r)
    assert np.array_equal(rs.worker_idx, plain.worker_idx) and np.array_equal(rs.votes, plain.votes)
    assert np.array_equal(rs.mask_idx, oracle.rs_mask_keys(plain.votes, K, r))
    assert not np.array_equal(rs.mask_idx, plain.mask_idx)
    assert np.all(plain.votes[rs.mask_idx] >= 1)
    a = g + e
    want = a[:, rs.mask_idx].astype(np.float64).mean(axis=0)
    assert np.allclose(rs.agg, want, rtol=1e-5, atol=1e-6)
    left = a.copy()
    left[:, rs.mask_idx] = 0.0
    assert np.array_equal(rs.err, left)
