"""Host-side tree construction of one cascaded cycle (Alg. 1, stage 2: ChainTree / BuildTree).

The constructor lives in the product library but runs on the host only, so it is checked
here without a GPU: against the definition (the set of root-to-node token sequences is the
draft prefixes plus, per correction, the prefix before it followed by the correction), and,
through the oracle's accept walk, against the literal walk of Alg. 1."""
import numpy as np
import pytest

import paper_2605_11186_amd as cats
import synth
from test_oracle_pins import MICRO, cascade_commit, make_model


def token_paths(token, parent):
    out = set()
    for i in range(len(parent)):
        seq, a = [], i
        while a > 0:
            seq.append(int(token[a]))
            a = int(parent[a])
        out.add(tuple(seq[::-1]))
    return out


def random_cycle(rng, vocab=5):
    g = int(rng.integers(0, 9))
    d = rng.integers(0, vocab, g).astype(np.int32)
    c = np.full(g, -1, dtype=np.int32)
    for i in range(g):
        r = rng.random()
        if r < 0.4:
            c[i] = (d[i] + 1 + rng.integers(0, vocab - 1)) % vocab     # a real correction
        elif r < 0.6:
            c[i] = d[i]                                               # the verifier agrees: no branch
    return d, c


def test_tree_is_the_draft_chain_plus_one_sibling_leaf_per_correction():
    rng = np.random.default_rng(3)
    for _ in range(400):
        d, c = random_cycle(rng)
        g = len(d)
        token, parent, depth, corr_node = cats.cats_build_tree(11, d, c)
        real = [i for i in range(g) if c[i] >= 0 and c[i] != d[i]]
        assert len(parent) == 1 + g + len(real)
        assert synth.is_valid_tree(parent, depth)
        assert token[0] == 11
        want = {tuple(int(t) for t in d[:k]) for k in range(g + 1)}
        want |= {tuple(int(t) for t in d[:i]) + (int(c[i]),) for i in real}
        assert token_paths(token, parent) == want
        # the chain comes first, the corrections after it in position order
        assert list(parent[: g + 1]) == [-1] + list(range(g))
        assert [int(n) for n in corr_node if n >= 0] == list(range(g + 1, len(parent)))
        for i in range(g):
            if i in real:
                n = corr_node[i]
                assert parent[n] == parent[i + 1] == i and depth[n] == depth[i + 1] and token[n] == c[i]
            else:
                assert corr_node[i] == -1
        # same shape as the generator used by the oracle's own pins
        p2, d2, _, _ = synth.chain_with_corrections(g, real)
        assert np.array_equal(parent, p2) and np.array_equal(depth, d2)


def test_no_corrections_is_the_plain_chain():
    token, parent, depth, corr_node = cats.cats_build_tree(3, [5, 6, 7])
    assert list(token) == [3, 5, 6, 7] and list(parent) == [-1, 0, 1, 2] and list(depth) == [0, 1, 2, 3]
    assert list(corr_node) == [-1, -1, -1]
    token, parent, depth, corr_node = cats.cats_build_tree(3, [])
    assert list(token) == [3] and list(parent) == [-1] and list(depth) == [0]


def test_accept_walk_on_built_trees_is_algorithm_1():
    micro = make_model(MICRO)
    rng = np.random.default_rng(4)
    for _ in range(300):
        d, c = random_cycle(rng, vocab=3)
        if len(d) == 0:
            continue
        token, parent, depth, corr_node = cats.cats_build_tree(9, d, c)
        T = len(parent)
        amax = rng.integers(0, 3, T).astype(np.int32)
        c_hat = {i: int(c[i]) for i in range(len(d)) if corr_node[i] >= 0}

        def argmax_at(prefix):
            node = 0
            for t in prefix:
                node = next(j for j in range(T) if parent[j] == node and token[j] == t)
            return int(amax[node])

        acc = micro.accept(token, parent, depth, amax, 0)
        assert acc["tokens"][1:] + [acc["bonus_token"]] == cascade_commit([int(t) for t in d], c_hat, argmax_at)


def test_error_codes():
    with pytest.raises(cats.CatsError) as e:
        cats.cats_build_tree(0, list(range(cats.CATS_MAX_DEPTH + 1)))
    assert e.value.status == cats.CATS_EINVAL
    with pytest.raises(cats.CatsError) as e:
        cats.cats_build_tree(0, [1, 2, 3], [4, 5, 6], capacity=6)
    assert e.value.status == cats.CATS_ECAPACITY
    with pytest.raises(cats.CatsError) as e:
        cats.cats_build_tree(0, [1, 2, 3], [4, 5])
    assert e.value.status == cats.CATS_EINVAL
    lib = cats.library()
    assert lib.cats_build_tree(0, None, 2, None, 8, None, None, None, None, None) == cats.CATS_EINVAL
    assert lib.cats_verify_nodes(None, None, 0, 0, None, None, None, 0, 0, None, None) == cats.CATS_EINVAL
