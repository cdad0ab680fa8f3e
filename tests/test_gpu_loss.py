"""GPU parity of the Reduced KL loss kernel (Eq. 2 / Appendix B) against the float64 oracle.

Integer output (the top-K sets, most probable first) is exact: both sides order the same
float32 logits, ties by index.  Floating point: the kernel works in float32; the loss per
position is a log-sum-exp over V terms minus a K-term weighted mean, each accurate to a few
1e-7 relative, so |gpu - ref| <= 2e-5 * max(1, |ref|) per position and for the mean; the
gradient (q - p~)/|M| has entries of magnitude <= 1/|M| and is compared with an absolute bound
of 1e-5/|M|."""
import numpy as np
import pytest
import torch

import paper_2605_11186_amd as cats
import synth
from oracle import reduced_kl as rk

pytestmark = pytest.mark.gpu


def run_gpu(a, z, K, mask=None, want_topk=True, want_grad=True):
    P, V = a.shape
    d_a, d_z = torch.from_numpy(a).cuda(), torch.from_numpy(z).cuda()
    d_m = None if mask is None else torch.from_numpy(mask).cuda()
    loss = torch.full((1,), float("nan"), device="cuda")
    per_pos = torch.full((P,), float("nan"), device="cuda")
    topk = torch.full((P, K), -7, dtype=torch.int32, device="cuda") if want_topk else None
    grad = torch.full((P, V), float("nan"), device="cuda") if want_grad else None
    cats.cats_reduced_kl_loss(d_a, d_z, K, loss, per_pos, mask=d_m, topk_idx_out=topk, grad_out=grad)
    torch.cuda.synchronize()
    return (loss.item(), per_pos.cpu().numpy(), None if topk is None else topk.cpu().numpy(),
            None if grad is None else grad.cpu().numpy())


def check(a, z, K, mask=None):
    loss, per_pos, topk, grad = run_gpu(a, z, K, mask)
    r_loss, r_pos, r_top, _ = rk.reduced_kl_loss(a, z, K, mask)
    assert np.array_equal(topk, r_top)
    assert np.abs(per_pos - r_pos).max() <= 2e-5 * max(1.0, np.abs(r_pos).max())
    assert abs(loss - r_loss) <= 2e-5 * max(1.0, abs(r_loss))
    r_grad = rk.reduced_kl_grad(a, z, K, mask)
    n = a.shape[0] if mask is None else max(int(mask.astype(bool).sum()), 1)
    assert np.isfinite(grad).all()
    assert np.abs(grad - r_grad).max() <= 1e-5 / n
    # the optional outputs do not change the required ones
    loss2, per_pos2, _, _ = run_gpu(a, z, K, mask, want_topk=False, want_grad=False)
    assert loss2 == loss and np.array_equal(per_pos2, per_pos)


@pytest.mark.parametrize("P,V,K", [(5, 1024, 10), (3, 4, 4), (9, 1000, 1), (4, 4100, 64), (33, 32000, 10),
                                   (2, 36864, 7)])
def test_lm_like_rows(P, V, K):
    a = synth.lm_like_logits(1, P, V, tag=0)
    z = synth.lm_like_logits(1, P, V, tag=1)
    check(a, z, K)


@pytest.mark.parametrize("V,K", [(2048, 10), (2048, 64), (512, 3)])
def test_ties_monotone_and_constant_rows(V, K):
    """Rows with many equal values (the selection rule decides), sorted rows (every thread's
    maximum is large), a constant row (every element ties: the slow exact path)."""
    a = synth.special_rows(3, V)
    z = synth.lm_like_logits(3, a.shape[0], V, tag=2)
    check(a, z, K)
    check(a, a.copy(), K)     # draft == target
    check(z, a, K)            # special rows as the draft


def test_masked_positions():
    P, V, K = 40, 2048, 10
    a, z = synth.lm_like_logits(5, P, V, tag=0), synth.lm_like_logits(5, P, V, tag=1)
    mask = synth.position_mask(5, P)
    assert 0 < mask.sum() < P
    check(a, z, K, mask)
    check(a, z, K, np.ones(P, np.uint8))
    one = np.zeros(P, np.uint8)
    one[17] = 1
    check(a, z, K, one)
    loss, per_pos, topk, grad = run_gpu(a, z, K, np.zeros(P, np.uint8))
    assert loss == 0.0 and (per_pos == 0).all() and (topk == -1).all() and (grad == 0).all()


def test_runs_are_bitwise_repeatable():
    a, z = synth.lm_like_logits(6, 16, 32000, tag=0), synth.lm_like_logits(6, 16, 32000, tag=1)
    first = run_gpu(a, z, 10)
    for _ in range(3):
        again = run_gpu(a, z, 10)
        assert again[0] == first[0] and all(np.array_equal(x, y) for x, y in zip(again[1:], first[1:]))


def test_argument_errors():
    a = torch.zeros(4, 1024, device="cuda")
    out, pp = torch.zeros(1, device="cuda"), torch.zeros(4, device="cuda")
    for K in (0, 65, 2000):
        with pytest.raises(cats.CatsError) as e:
            cats.cats_reduced_kl_loss(a, a, K, out, pp)
        assert e.value.status == cats.CATS_EINVAL
    with pytest.raises(cats.CatsError) as e:     # vocab not a multiple of 4
        cats.cats_reduced_kl_loss(a[:, :1022].contiguous(), a[:, :1022].contiguous(), 4, out, pp)
    assert e.value.status == cats.CATS_EINVAL
    with pytest.raises(cats.CatsError) as e:     # misaligned rows
        mis = a.view(-1)[1:1025].view(1, 1024)
        cats.cats_reduced_kl_loss(mis, mis, 4, out, pp)
    assert e.value.status == cats.CATS_EINVAL
    big = torch.zeros(1, cats.CATS_LOSS_MAX_VOCAB + 4, device="cuda")
    with pytest.raises(cats.CatsError) as e:
        cats.cats_reduced_kl_loss(big, big, 4, out, pp[:1])
    assert e.value.status == cats.CATS_ECAPACITY
    with pytest.raises(cats.CatsError) as e:
        cats.cats_reduced_kl_loss(a, a, 4, None, pp)
    assert e.value.status == cats.CATS_EINVAL
