"""The law of majority voting with random selection on small vectors, in closed
form (Sec. 2, paragraph after Algorithm 1: winners drawn in proportion to their
votes; Sec. 4.2: until K distinct ones are selected), shared by the oracle's pins
and the GPU's statistical check."""
import itertools

import numpy as np


def successive_sampling_law(w, K):
    """P(selected set) when positions are drawn in proportion to w, repeats discarded."""
    W = float(sum(w))
    law = {}
    voted = [j for j, x in enumerate(w) if x > 0]
    for order in itertools.permutations(voted, K):
        p, rest = 1.0, W
        for j in order:
            p *= w[j] / rest
            rest -= w[j]
        key = tuple(sorted(order))
        law[key] = law.get(key, 0.0) + p
    return law


def assert_follows_law(counts, trials, law, what):
    assert set(counts) <= set(law), "%s selected a set of probability zero" % what
    for key, p in law.items():
        f = counts.get(key, 0) / trials
        sigma = np.sqrt(p * (1 - p) / trials)
        assert abs(f - p) <= 5 * sigma + 1e-9, "%s: set %s frequency %.4f, law %.4f" % (what, key, f, p)
