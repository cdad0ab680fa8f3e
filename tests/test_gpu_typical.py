"""GPU parity of the typical-acceptance walk (Alg. 1 with Acc = typical) against its oracle.

Two layers of comparison.  (1) On the GPU's own logits (read back from the same call) the
kernel's float32 statistics must match the float64 oracle: log-sum-exp and entropy to 1e-5
(absolute, values are O(10)), probabilities and thresholds to 1e-4 relative; edge decisions
are compared where |p - thr| > 1e-3 * thr (a float decides an integer: nearer than that, either
answer is right), and given those decisions the accept result must be exact.  (2) Against the
oracle's own forward pass the usual 2e-2 bound holds for logits, and the accept result must
agree whenever every decision of the oracle has a margin of 10 %."""
import numpy as np
import pytest
import torch

import paper_2605_11186_amd as cats
import synth
from gpu_common import REL_TOL, Pair, rel_err
from oracle import typical as ty

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def pair():
    p = Pair(synth.TINY, 909, max_ctx=320, max_tree=128, packed=True)
    yield p
    p.close()


def run(pair, ks, vs, S, tok, parent, depth, eps, delta, temp):
    T, d = len(parent), pair.dims
    logits = torch.empty(T, d.vocab, dtype=torch.float32, device="cuda")
    amax = torch.empty(T, dtype=torch.int32, device="cuda")
    stats = [torch.full((T,), float("nan"), device="cuda") for _ in range(4)]
    host = cats.AcceptResult()
    cats.cats_set_tree(pair.ctx, tok, parent, depth)
    cats.cats_set_acceptance(pair.ctx, 1, eps, delta, temp)
    try:
        cats.cats_verify_tree(pair.ctx, pair.layers_arr, 0, pair.L, pair.d_embed, None, pair.d_final["g_final"],
                              pair.d_final["w_lm"], cats.kv_array(ks, vs), S, pair.res_dev, logits_out=logits,
                              argmax_out=amax, out_host=host)
        cats.cats_typical_stats(pair.ctx, *stats)
        torch.cuda.synchronize()
    finally:
        cats.cats_set_acceptance(pair.ctx, 0)
    return logits.cpu().numpy(), amax.cpu().numpy(), [s.cpu().numpy() for s in stats], host.as_dict()


def pick(r, keys=("n_accepted", "path", "tokens", "bonus_token", "new_ctx_len")):
    return {k: r[k] for k in keys}


@pytest.mark.parametrize("eps,delta,temp", [(0.09, 0.3, 1.0), (0.09, 0.3, 0.7), (0.002, 1.0, 1.0), (0.0005, 0.5, 0.25)])
@pytest.mark.parametrize("T,S", [(33, 70), (100, 5), (1, 0)])
def test_typical_walk_matches_oracle(pair, eps, delta, temp, T, S):
    parent, depth = synth.random_tree(T, 8, T + S)
    tok = synth.distinct_sibling_tokens(parent, pair.dims.vocab, T)
    kc, vc = pair.oracle_cache_random(S + 1, S)
    ks, vs = pair.device_cache_from_oracle(kc, vc, S)
    g_logits, g_amax, (g_lse, g_H, g_prob, g_thr), g_acc = run(pair, ks, vs, S, tok, parent, depth, eps, delta, temp)
    # (1) the kernel's arithmetic on its own logits
    lse, H = ty.node_stats(g_logits, temp)
    assert np.abs(g_lse - lse).max() <= 1e-5 * max(1.0, np.abs(lse).max())
    assert np.abs(g_H - H).max() <= 1e-5 * max(1.0, np.abs(H).max())
    ref = ty.typical_accept(tok, parent, depth, g_logits, S, eps, delta, temp)
    if T > 1:
        assert np.abs(g_prob[1:] - ref["prob"][1:]).max() <= 1e-4 * ref["prob"][1:].max()
        assert np.abs(g_thr[1:] - ref["threshold"][1:]).max() <= 1e-4 * ref["threshold"][1:].max()
    clear = np.abs(ref["prob"] - ref["threshold"]) > 1e-3 * ref["threshold"]
    g_edge = g_prob > g_thr
    assert np.array_equal(g_edge[1:][clear[1:]], ref["edge"][1:][clear[1:]])
    if clear[1:].all():
        assert g_acc == pick(ref)
    assert np.array_equal(g_amax, g_logits.argmax(1))
    # (2) against the oracle's own forward pass
    o_hidden = pair.oracle.tree_forward(kc, vc, S, parent, depth, tokens=tok, layer_end=pair.L)
    o_logits = pair.oracle.lm_head(o_hidden)
    assert rel_err(g_logits, o_logits) <= REL_TOL
    o_ref = ty.typical_accept(tok, parent, depth, o_logits, S, eps, delta, temp)
    wide = np.abs(o_ref["prob"] - o_ref["threshold"])[1:] > 0.1 * o_ref["threshold"][1:]
    o_amax, o_margin = pair.oracle.argmax_margin(o_logits)
    if wide.all() and o_margin[o_ref["path"][-1]] > 1e-2:
        assert g_acc == pick(o_ref)
    # the roll-back followed the typical path
    pair.oracle.compact(kc, vc, S, g_acc["path"])
    for l in range(pair.L):
        gk, gv = pair.device_rows(ks, vs, l, g_acc["new_ctx_len"])
        assert rel_err(gk, kc[l, :g_acc["new_ctx_len"]]) <= REL_TOL
        assert rel_err(gv, vc[l, :g_acc["new_ctx_len"]]) <= REL_TOL


def test_accept_everything_nothing_and_cold_limit(pair):
    S, T = 40, 45
    parent, depth = synth.random_tree(T, 6, 3)
    tok = synth.distinct_sibling_tokens(parent, pair.dims.vocab, 3)
    kc, vc = pair.oracle_cache_random(8, S)
    ks, vs = pair.device_cache_from_oracle(kc, vc, S)
    _, g_amax, _, acc = run(pair, ks, vs, S, tok, parent, depth, 0.0, 0.0, 1.0)
    deepest = max(range(T), key=lambda j: (depth[j], -j))
    assert acc["path"][-1] == deepest and acc["n_accepted"] == depth[deepest]
    ks, vs = pair.device_cache_from_oracle(kc, vc, S)
    _, g_amax, _, acc = run(pair, ks, vs, S, tok, parent, depth, 2.0, 1e9, 1.0)
    assert acc["n_accepted"] == 0 and acc["path"] == [0] and acc["bonus_token"] == int(g_amax[0])
    # temperature -> 0: the greedy walk (drafts that follow the GPU's own argmax are accepted)
    tok2 = tok.copy()
    for j in range(1, T):
        if j % 2:
            tok2[j] = g_amax[parent[j]]
    ks, vs = pair.device_cache_from_oracle(kc, vc, S)
    logits, g_amax2, _, acc = run(pair, ks, vs, S, tok2, parent, depth, 0.09, 0.3, 1e-3)
    greedy = pair.oracle.accept(tok2, parent, depth, g_amax2, S)
    top2 = np.sort(logits, axis=1)[:, -2:]
    if ((top2[:, 1] - top2[:, 0]) > 1e-2).all():
        assert acc == greedy


def test_compact_along_and_argument_rules(pair):
    d = pair.dims
    S, T = 20, 9
    parent, depth = synth.chain_tree(T)
    tok = synth.distinct_sibling_tokens(parent, d.vocab, 1)
    ks = [torch.randn(d.n_heads, pair.max_ctx, d.head_dim, device="cuda").to(torch.bfloat16) for _ in range(pair.L)]
    vs = [torch.randn(d.n_heads, d.head_dim, pair.max_ctx, device="cuda").to(torch.bfloat16) for _ in range(pair.L)]
    k0, v0 = [k.clone() for k in ks], [v.clone() for v in vs]
    cats.cats_set_tree(pair.ctx, tok, parent, depth)
    res = cats.AcceptResult()
    res.n_accepted = 2
    path = [0, 3, 7]
    for i, n in enumerate(path):
        res.path[i] = n
    res_dev = cats.accept_result_tensor()
    res_dev.copy_(torch.frombuffer(bytearray(bytes(res)), dtype=res_dev.dtype)[: res_dev.numel()])
    cats.cats_compact_along(pair.ctx, res_dev, cats.kv_array(ks, vs), 0, pair.L, S)
    torch.cuda.synchronize()
    for l in range(pair.L):
        for k, n in enumerate(path):
            assert torch.equal(ks[l][:, S + k], k0[l][:, S + n]) and torch.equal(vs[l][:, :, S + k], v0[l][:, :, S + n])
        assert torch.equal(ks[l][:, S + 3:], k0[l][:, S + 3:]) and torch.equal(ks[l][:, :S], k0[l][:, :S])
    for bad in ((2, 0.1, 0.1, 1.0), (1, -0.1, 0.3, 1.0), (1, 0.1, 0.3, 0.0)):
        with pytest.raises(cats.CatsError) as e:
            cats.cats_set_acceptance(pair.ctx, *bad)
        assert e.value.status == cats.CATS_EINVAL
    with pytest.raises(cats.CatsError) as e:
        cats.cats_compact_along(pair.ctx, None, cats.kv_array(ks, vs), 0, pair.L, S)
    assert e.value.status == cats.CATS_EINVAL
