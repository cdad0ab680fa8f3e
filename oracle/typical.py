"""CPU oracle of the typical-acceptance variant of the tree walk (Alg. 1 with Acc = typical).

TEST INFRASTRUCTURE ONLY: imported by the tests.  The GPU library never imports or calls this.

The paper names the criterion only by citation (Sec. 3.2 and Alg. 1 allow Acc to be greedy or typical, citing
Medusa); it prints neither the inequality nor its constants.  PARITY UNPINNED against this paper:
the inequality below restates the cited work's published rule.  A candidate token x judged by
the target distribution p at its parent node is accepted when

    p(x) > min(epsilon, delta * exp(-H(p))),      p = softmax(logits / temperature),

H the entropy of p.  Everything else follows Alg. 1 as the greedy walk does: a node is accepted
when its parent is and its own token passes; the committed path ends at the deepest accepted
node (lowest index among equals); the bonus token is the target's argmax at that node.
Plain numpy in float64.  What the pins fix is the arithmetic (log-sum-exp, entropy, the limits
in which the rule reduces to greedy acceptance or accepts everything / nothing) and the walk.
"""
from __future__ import annotations

import numpy as np


def node_stats(logits, temperature: float = 1.0):
    """Per row: log-sum-exp and entropy of softmax(logits / temperature)."""
    z = np.asarray(logits, dtype=np.float64) / temperature
    m = z.max(axis=-1, keepdims=True)
    e = np.exp(z - m)
    s = e.sum(axis=-1, keepdims=True)
    lse = (m + np.log(s))[..., 0]
    p = e / s
    with np.errstate(divide="ignore", invalid="ignore"):
        plogp = np.where(p > 0, p * np.log(p), 0.0)
    return lse, -plogp.sum(axis=-1)


def typical_accept(token, parent, depth, logits, ctx_len: int, epsilon: float, delta: float,
                   temperature: float = 1.0):
    """The walk of Alg. 1 with the typical criterion.  Returns the same fields as the greedy
    accept result plus per-node diagnostics (probability of the node's token under its parent,
    threshold at its parent, edge decision)."""
    token, parent, depth = (np.asarray(a) for a in (token, parent, depth))
    T = len(parent)
    lse, H = node_stats(logits, temperature)
    z = np.asarray(logits, dtype=np.float64) / temperature
    prob = np.zeros(T)
    thr = np.zeros(T)
    edge = np.zeros(T, dtype=bool)
    ok = np.zeros(T, dtype=bool)
    ok[0] = True
    for j in range(1, T):
        p = int(parent[j])
        prob[j] = np.exp(z[p, token[j]] - lse[p])
        thr[j] = min(epsilon, delta * np.exp(-H[p]))
        edge[j] = prob[j] > thr[j]
        ok[j] = ok[p] and edge[j]
    best = max((j for j in range(T) if ok[j]), key=lambda j: (depth[j], -j))
    path = []
    a = best
    while a >= 0:
        path.append(int(a))
        a = int(parent[a])
    path = path[::-1]
    amax = np.asarray(logits).argmax(axis=-1)
    return {"n_accepted": len(path) - 1, "path": path, "tokens": [int(token[i]) for i in path],
            "bonus_token": int(amax[best]), "new_ctx_len": int(ctx_len) + len(path),
            "prob": prob, "threshold": thr, "edge": edge}
