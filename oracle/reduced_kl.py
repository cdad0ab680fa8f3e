"""CPU oracle of the Reduced KL Loss (Section 3.3, Eq. 2; Appendix B, steps 1-3).

TEST INFRASTRUCTURE ONLY: imported by the tests and by the benchmark's CPU-baseline
leg of the loss workload.  The GPU library never imports or calls this.

Plain numpy in float64, the three steps of the appendix in their order and
notation.  Inputs are logits; p_target and q_draft are their softmaxes.
Readings (the paper is silent on both): ties in the top-K selection go to the
lower vocabulary index; with no unmasked position the loss is 0.
"""
from __future__ import annotations

import numpy as np


def softmax(x):
    """Row-wise softmax with the usual max subtraction."""
    x = np.asarray(x, dtype=np.float64)
    e = np.exp(x - x.max(axis=-1, keepdims=True))
    return e / e.sum(axis=-1, keepdims=True)


def log_softmax(x):
    x = np.asarray(x, dtype=np.float64)
    m = x.max(axis=-1, keepdims=True)
    return x - m - np.log(np.exp(x - m).sum(axis=-1, keepdims=True))


def top_k_set(p_row, K):
    """Appendix B step 1: the K vocabulary indices of highest target probability, most probable
    first; equal probabilities are ordered by index."""
    order = sorted(range(len(p_row)), key=lambda v: (-p_row[v], v))
    return order[:K]


def renormalise(p_row, support):
    """Appendix B step 2: the target distribution restricted to `support` and rescaled to sum to 1
    (zero elsewhere)."""
    p_tilde = np.zeros_like(p_row)
    p_tilde[support] = p_row[support] / p_row[support].sum()
    return p_tilde


def reduced_kl_loss(target_logits, draft_logits, K, mask=None):
    """Appendix B step 3 (= Eq. 2): mean over the unmasked positions M of
    -sum_{v in T_K(t)} p~_target(v|t) log q_draft(v|t).

    Returns (loss, per_position[P] (0 at masked positions), top_k[P][K] int32 (-1 at masked
    positions), p_tilde[P][V])."""
    a = np.asarray(target_logits, dtype=np.float64)
    z = np.asarray(draft_logits, dtype=np.float64)
    P, V = a.shape
    assert z.shape == (P, V) and 1 <= K <= V
    m = np.ones(P, dtype=bool) if mask is None else np.asarray(mask).astype(bool)
    p = softmax(a)
    log_q = log_softmax(z)
    per_pos = np.zeros(P)
    top = np.full((P, K), -1, dtype=np.int32)
    p_tilde = np.zeros((P, V))
    for t in range(P):
        if not m[t]:
            continue
        support = top_k_set(p[t], K)
        p_tilde[t] = renormalise(p[t], support)
        per_pos[t] = -sum(p_tilde[t, v] * log_q[t, v] for v in support)
        top[t] = support
    n = int(m.sum())
    loss = per_pos.sum() / n if n else 0.0
    return loss, per_pos, top, p_tilde


def reduced_kl_grad(target_logits, draft_logits, K, mask=None):
    """d loss / d draft_logits.  With q = softmax(z): d(-sum_v p~_v log q_v)/dz_u = q_u - p~_u
    (p~ sums to 1), divided by |M|; zero rows at masked positions."""
    z = np.asarray(draft_logits, dtype=np.float64)
    m = np.ones(z.shape[0], dtype=bool) if mask is None else np.asarray(mask).astype(bool)
    _, _, _, p_tilde = reduced_kl_loss(target_logits, draft_logits, K, mask)
    n = int(m.sum())
    g = (softmax(z) - p_tilde) / max(n, 1)
    g[~m] = 0.0
    return g
