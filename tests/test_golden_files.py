"""The stored expectations under tests/golden are self-consistent with the CPU oracle's integer
logic (the floating-point part that produced them takes minutes at 7B size and is re-run only by
tests/golden/make_config2_tree.py)."""
from pathlib import Path

import numpy as np

import synth
from oracle.cats_oracle import Oracle


def test_config2_tree_file_is_consistent():
    text = (Path(__file__).parent / "golden" / "config2_tree_7b.txt").read_text()
    g = {k.strip(): v.split() for k, v in (l.split(":", 1) for l in text.splitlines() if l and not l.startswith("#"))}
    parent, depth, rank = synth.product_tree_pruned()
    tok = np.array(g["tokens"], np.int32)
    amax = np.array(g["argmax"], np.int32)
    assert len(tok) == len(amax) == len(parent) == 63
    assert tok.min() >= 0 and tok.max() < synth.V7B.vocab
    for p in range(63):   # siblings carry distinct ids
        kids = [int(tok[j]) for j in range(63) if parent[j] == p]
        assert len(set(kids)) == len(kids)
    orc = Oracle(synth.TINY, [], None, None)   # only the integer walk is used
    acc = orc.accept(tok, parent, depth, amax, 1024)
    assert acc["n_accepted"] == int(g["n_accepted"][0])
    assert acc["path"] == [int(v) for v in g["path"]]
    assert acc["bonus_token"] == int(g["bonus_token"][0])
    assert acc["new_ctx_len"] == 1024 + acc["n_accepted"] + 1
    assert 3 <= acc["n_accepted"] <= 4          # the workload's "roughly 3-4 accepted tokens"
