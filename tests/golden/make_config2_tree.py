#!/usr/bin/env python3
"""Writes tests/golden/config2_tree_7b.txt: the token ids of the 63-node top-k tree of the
7B-shaped benchmark step, and the accept result the float32 oracle gets for it.

Uses only synth/ (seeded inputs) and oracle/ (CPU reference).  The draft ids imitate a
drafter that is right most of the time: level by level, the children of a node are the
best-ranked tokens of the oracle's own logits at that node after a seeded Gaussian
perturbation (sigma below), so that a few levels are accepted and then the chain breaks.
Needs ~16 GB of RAM and a few minutes of CPU time.
"""
import sys
from pathlib import Path

import numpy as np

ROOT = Path(__file__).resolve().parents[2]
sys.path.insert(0, str(ROOT))
import synth  # noqa: E402
from oracle.cats_oracle import Oracle  # noqa: E402

SEED, S, SIGMA = 11186, 1024, 0.18


def main():
    dims = synth.V7B
    parent, depth, rank = synth.product_tree_pruned()
    T = len(parent)
    layers = [synth.layer_weights(dims, SEED, l) for l in range(dims.n_layers)]
    orc = Oracle(dims, layers, synth.final_weights(dims, SEED), synth.embedding(dims, SEED), precision="f32")
    max_ctx = (S + T + 63) // 64 * 64
    kc, vc = orc.new_cache(max_ctx)
    for l in range(dims.n_layers):
        k, v = synth.random_kv_context(dims, SEED, l, S)
        kc[l, :S] = synth.f32_from_bf16_bits(k)
        vc[l, :S] = synth.f32_from_bf16_bits(v)
    rng = np.random.Generator(np.random.SFC64(np.random.SeedSequence((SEED, 63, 2))))
    tok = np.zeros(T, np.int32)
    tok[0] = int(rng.integers(dims.vocab))
    children = {i: [j for j in range(T) if parent[j] == i] for i in range(T)}
    for level in range(int(depth.max())):
        n = int((depth <= level).sum())          # breadth-first numbering: a prefix of the node list
        x = orc.tree_forward(kc, vc, S, parent[:n], depth[:n], tokens=tok[:n])
        logits = orc.lm_head(x)
        for p in np.flatnonzero(depth == level):
            kids = sorted(children[int(p)], key=lambda j: rank[j])
            if not kids:
                continue
            noisy = logits[p] + SIGMA * rng.standard_normal(dims.vocab).astype(np.float32)
            best = np.argsort(-noisy)[: len(kids)]
            for j, t in zip(kids, best):
                tok[j] = int(t)
        print(f"level {level}: {n} nodes forwarded", flush=True)
    x = orc.tree_forward(kc, vc, S, parent, depth, tokens=tok)
    logits = orc.lm_head(x)
    amax, margin = orc.argmax_margin(logits)
    acc = orc.accept(tok, parent, depth, amax, S)
    on_path_margin = [float(margin[i]) for i in acc["path"]]
    out = ROOT / "tests" / "golden" / "config2_tree_7b.txt"
    with open(out, "w") as f:
        f.write("# Written by tests/golden/make_config2_tree.py (float32 CPU oracle + seeded inputs only).\n")
        f.write(f"# 7B-shaped model, seed {SEED}, KV context {S} (seeded N(0,1) rows), 63-node pruned 4/3/2/2/1/1 tree,\n")
        f.write(f"# children = best-ranked tokens of the oracle's logits + N(0,{SIGMA}^2) noise.\n")
        f.write("tokens: " + " ".join(map(str, tok)) + "\n")
        f.write(f"n_accepted: {acc['n_accepted']}\n")
        f.write("path: " + " ".join(map(str, acc["path"])) + "\n")
        f.write(f"bonus_token: {acc['bonus_token']}\n")
        f.write("min_margin_on_path: %.4f\n" % min(on_path_margin))
        f.write("argmax: " + " ".join(map(str, amax)) + "\n")
        f.write("margin: " + " ".join("%.4f" % m for m in margin) + "\n")
    print(out.read_text()[:600])


if __name__ == "__main__":
    main()
