"""Pins of the typical-acceptance oracle.  The criterion itself comes from the work the paper
cites and is unpinned against the paper; these tests fix the arithmetic against library routines
and closed forms, the limits in which the rule must agree with the (pinned) greedy walk or
accept everything / nothing, and the walk against brute force."""
import itertools

import numpy as np
import pytest
import scipy.special
import scipy.stats

import synth
from oracle import typical as ty
from test_oracle_pins import MICRO, make_model


def random_case(rng, T, V, scale=2.0):
    parent, depth = synth.random_tree(T, 5, int(rng.integers(1 << 30)))
    token = synth.distinct_sibling_tokens(parent, V, int(rng.integers(1 << 30)))
    logits = rng.normal(0, scale, (T, V))
    return token, parent, depth, logits


def test_stats_against_library_routines_and_closed_forms():
    rng = np.random.default_rng(0)
    x = rng.normal(0, 3, (6, 50))
    for temp in (1.0, 0.7, 2.5):
        lse, H = ty.node_stats(x, temp)
        assert np.allclose(lse, scipy.special.logsumexp(x / temp, axis=1), rtol=0, atol=1e-12)
        assert np.allclose(H, scipy.stats.entropy(scipy.special.softmax(x / temp, axis=1), axis=1), atol=1e-12)
    lse, H = ty.node_stats(np.full((1, 32), 4.5))
    assert abs(H[0] - np.log(32)) < 1e-12 and abs(lse[0] - (4.5 + np.log(32))) < 1e-12
    _, H = ty.node_stats(np.array([[0.0, -1e4, -1e4]]))      # one-hot: no entropy, no NaN from 0 log 0
    assert H[0] == 0.0
    _, H = ty.node_stats(np.array([[np.log(3.0), 0.0]]))     # p = (3/4, 1/4)
    assert abs(H[0] - (-(0.75 * np.log(0.75) + 0.25 * np.log(0.25)))) < 1e-12


def test_probability_and_threshold_are_the_stated_expressions():
    rng = np.random.default_rng(1)
    token, parent, depth, logits = random_case(rng, 12, 30)
    r = ty.typical_accept(token, parent, depth, logits, 5, 0.09, 0.3, 0.8)
    p = scipy.special.softmax(logits / 0.8, axis=1)
    H = scipy.stats.entropy(p, axis=1)
    for j in range(1, 12):
        q = parent[j]
        assert abs(r["prob"][j] - p[q, token[j]]) < 1e-12
        assert abs(r["threshold"][j] - min(0.09, 0.3 * np.exp(-H[q]))) < 1e-12
        assert r["edge"][j] == (p[q, token[j]] > min(0.09, 0.3 * np.exp(-H[q])))


def test_cold_limit_is_the_greedy_walk():
    """temperature -> 0 makes p one-hot at the argmax with zero entropy: the threshold is
    min(epsilon, delta) < 1, so a token passes exactly when it is the target's argmax."""
    micro = make_model(MICRO)
    rng = np.random.default_rng(2)
    n_multi = 0
    for _ in range(200):
        T = int(rng.integers(1, 14))
        token, parent, depth, logits = random_case(rng, T, 6)
        amax = logits.argmax(1).astype(np.int32)
        for j in range(1, T):                       # make matches likely
            if rng.random() < 0.6:
                token[j] = amax[parent[j]]
        greedy = micro.accept(token, parent, depth, amax, 9)
        r = ty.typical_accept(token, parent, depth, logits, 9, 0.09, 0.3, 1e-3)
        assert {k: r[k] for k in greedy} == greedy
        n_multi += greedy["n_accepted"] > 1
    assert n_multi > 20


def test_accept_everything_and_nothing():
    rng = np.random.default_rng(3)
    token, parent, depth, logits = random_case(rng, 20, 40)
    r = ty.typical_accept(token, parent, depth, logits, 0, 0.0, 0.0)       # p > 0 always
    deepest = max(range(20), key=lambda j: (depth[j], -j))
    assert r["path"][-1] == deepest and r["n_accepted"] == depth[deepest]
    r = ty.typical_accept(token, parent, depth, logits, 0, 2.0, 1e9)       # threshold >= 1 > p
    assert r["n_accepted"] == 0 and r["path"] == [0] and r["bonus_token"] == int(logits[0].argmax())
    assert r["new_ctx_len"] == 1


def test_walk_by_brute_force_and_monotone_in_epsilon():
    rng = np.random.default_rng(4)
    for _ in range(150):
        T = int(rng.integers(2, 9))
        token, parent, depth, logits = random_case(rng, T, 8, scale=1.0)
        r = ty.typical_accept(token, parent, depth, logits, 3, 0.12, 0.4)
        # brute force: every root-descending chain whose edges all pass; longest, then lowest end index
        children = {i: [j for j in range(T) if parent[j] == i] for i in range(T)}
        chains = [[0]]
        grow = [[0]]
        while grow:
            nxt = []
            for c in grow:
                for j in children[c[-1]]:
                    if r["edge"][j]:
                        nxt.append(c + [j])
            chains += nxt
            grow = nxt
        best = max(chains, key=lambda c: (len(c), -c[-1]))
        assert r["path"] == best and r["tokens"] == [int(token[i]) for i in best]
        assert r["bonus_token"] == int(logits[best[-1]].argmax()) and r["new_ctx_len"] == 3 + len(best)
        stricter = ty.typical_accept(token, parent, depth, logits, 3, 0.5, 0.4)
        assert stricter["n_accepted"] <= r["n_accepted"]
        assert not (stricter["edge"] & ~r["edge"]).any()
