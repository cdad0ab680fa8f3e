"""Pins of the Reduced KL Loss oracle (Eq. 2 / Appendix B) against things other than itself:
library cross-entropy routines for the cases it reduces to (K = V is Eq. 1; K = 1 is the
hard-label cross-entropy), closed forms, a brute-force subset search for the selection, an
independent library implementation (torch.topk + autograd) and finite differences for the
gradient."""
import itertools

import numpy as np
import pytest
import torch

from oracle import reduced_kl as rk


def rand_logits(rng, P, V, scale=3.0):
    return rng.normal(0, scale, (P, V))


def test_k_equal_v_is_the_full_vocabulary_loss_eq1():
    rng = np.random.default_rng(0)
    a, z = rand_logits(rng, 7, 50), rand_logits(rng, 7, 50)
    loss, per_pos, _, _ = rk.reduced_kl_loss(a, z, 50)
    # library: cross entropy with probability targets, mean over positions
    ref = torch.nn.functional.cross_entropy(torch.from_numpy(z), torch.softmax(torch.from_numpy(a), -1))
    assert abs(loss - ref.item()) < 1e-12
    # and Eq. 1 written as a double sum
    p, lq = rk.softmax(a), rk.log_softmax(z)
    assert abs(loss - (-(p * lq).sum() / 7)) < 1e-12


def test_k_equal_1_is_hard_label_cross_entropy():
    rng = np.random.default_rng(1)
    a, z = rand_logits(rng, 9, 40), rand_logits(rng, 9, 40)
    loss, _, top, _ = rk.reduced_kl_loss(a, z, 1)
    labels = torch.from_numpy(a).argmax(-1)
    ref = torch.nn.functional.cross_entropy(torch.from_numpy(z), labels)
    assert abs(loss - ref.item()) < 1e-12
    assert np.array_equal(top[:, 0], labels.numpy())


def test_closed_forms():
    rng = np.random.default_rng(2)
    a = rand_logits(rng, 5, 30)
    for K in (1, 3, 10, 30):
        # uniform draft: log q = -log V for every token, and p~ sums to 1
        loss, _, _, p_tilde = rk.reduced_kl_loss(a, np.zeros((5, 30)), K)
        assert abs(loss - np.log(30)) < 1e-12
        assert np.allclose(p_tilde.sum(1), 1) and ((p_tilde > 0).sum(1) == K).all()
    # draft == target, K == V: the entropy of p
    loss, _, _, _ = rk.reduced_kl_loss(a, a, 30)
    p = rk.softmax(a)
    assert abs(loss - (-(p * np.log(p)).sum() / 5)) < 1e-12
    # shifting either logit row by a constant changes nothing
    z = rand_logits(rng, 5, 30)
    l0 = rk.reduced_kl_loss(a, z, 4)[0]
    assert abs(rk.reduced_kl_loss(a + 7.5, z - 3.25, 4)[0] - l0) < 1e-12


def test_loss_minus_entropy_is_a_kl_divergence():
    """L_topK = H(p~) + KL(p~ || q): never below the entropy of p~, and equal to it when the
    draft puts all its mass on the support in the same proportions."""
    rng = np.random.default_rng(3)
    a, z = rand_logits(rng, 6, 25), rand_logits(rng, 6, 25)
    K = 5
    _, per_pos, top, p_tilde = rk.reduced_kl_loss(a, z, K)
    for t in range(6):
        pt = p_tilde[t, top[t]]
        H = -(pt * np.log(pt)).sum()
        assert per_pos[t] >= H - 1e-12
        z_match = np.full(25, -1e9)
        z_match[top[t]] = np.log(pt)
        l_match = rk.reduced_kl_loss(a[t:t + 1], z_match[None], K)[1][0]
        assert abs(l_match - H) < 1e-9


def test_selection_by_brute_force_and_ties_to_lower_index():
    rng = np.random.default_rng(4)
    for trial in range(30):
        V, K = 9, int(rng.integers(1, 9))
        a = rand_logits(rng, 1, V)
        if trial % 3 == 0:       # repeated values: the tie rule matters
            a = np.round(a)
        p = rk.softmax(a)[0]
        top = rk.reduced_kl_loss(a, a, K)[2][0]
        # the top-K set carries the largest total mass of all K-subsets (lowest indices among equals)
        best = max(itertools.combinations(range(V), K), key=lambda s: (round(p[list(s)].sum(), 14), [-i for i in s]))
        assert sorted(top) == list(best)
        # ordered by probability, then index
        assert all((p[top[i]], -top[i]) >= (p[top[i + 1]], -top[i + 1]) for i in range(K - 1))
    a = np.array([[1.0, 5.0, 5.0, 0.0, 5.0, 2.0]])
    assert list(rk.reduced_kl_loss(a, a, 2)[2][0]) == [1, 2]
    assert list(rk.reduced_kl_loss(a, a, 4)[2][0]) == [1, 2, 4, 5]


def test_mask_and_mean_over_unmasked_positions():
    rng = np.random.default_rng(5)
    a, z = rand_logits(rng, 8, 20), rand_logits(rng, 8, 20)
    mask = np.array([1, 0, 1, 1, 0, 0, 1, 1], dtype=np.uint8)
    loss, per_pos, top, _ = rk.reduced_kl_loss(a, z, 3, mask)
    keep = mask.astype(bool)
    loss_kept = rk.reduced_kl_loss(a[keep], z[keep], 3)[0]
    assert abs(loss - loss_kept) < 1e-12
    assert (per_pos[~keep] == 0).all() and (top[~keep] == -1).all()
    # repeating every position leaves the mean unchanged
    assert abs(rk.reduced_kl_loss(np.tile(a, (2, 1)), np.tile(z, (2, 1)), 3, np.tile(mask, 2))[0] - loss) < 1e-12
    assert rk.reduced_kl_loss(a, z, 3, np.zeros(8))[0] == 0.0


def torch_reference(a, z, K, mask):
    """Independent implementation on library routines (topk, softmax, log_softmax)."""
    a, z = torch.from_numpy(a), torch.from_numpy(z).requires_grad_(True)
    vals, idx = torch.topk(torch.softmax(a, -1), K, dim=-1)
    p_tilde = vals / vals.sum(-1, keepdim=True)
    lq = torch.log_softmax(z, -1).gather(-1, idx)
    per_pos = -(p_tilde * lq).sum(-1)
    m = torch.from_numpy(mask.astype(np.float64))
    loss = (per_pos * m).sum() / m.sum()
    loss.backward()
    return loss.item(), z.grad.numpy()


@pytest.mark.parametrize("K", [1, 4, 10, 33])
def test_against_library_topk_and_autograd(K):
    rng = np.random.default_rng(6 + K)
    a, z = rand_logits(rng, 12, 33), rand_logits(rng, 12, 33)
    mask = (rng.random(12) < 0.7).astype(np.uint8)
    mask[0] = 1
    ref_loss, ref_grad = torch_reference(a, z, K, mask)
    assert abs(rk.reduced_kl_loss(a, z, K, mask)[0] - ref_loss) < 1e-12
    assert np.abs(rk.reduced_kl_grad(a, z, K, mask) - ref_grad).max() < 1e-12


def test_gradient_by_finite_differences():
    rng = np.random.default_rng(9)
    a, z = rand_logits(rng, 3, 11), rand_logits(rng, 3, 11)
    mask = np.array([1, 1, 0], dtype=np.uint8)
    g = rk.reduced_kl_grad(a, z, 4, mask)
    h = 1e-6
    for t in range(3):
        for v in range(11):
            zp, zm = z.copy(), z.copy()
            zp[t, v] += h
            zm[t, v] -= h
            fd = (rk.reduced_kl_loss(a, zp, 4, mask)[0] - rk.reduced_kl_loss(a, zm, 4, mask)[0]) / (2 * h)
            assert abs(fd - g[t, v]) < 1e-8
    assert (g[2] == 0).all()
    assert np.abs(g.sum(1)).max() < 1e-12      # both q and p~ sum to 1
