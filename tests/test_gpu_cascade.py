"""GPU parity of the cascaded cycle's stage 2 + stage 3 wiring (Alg. 1): the main draft chain
goes through the shallow layers first, the shallow verifier's corrections are re-forwarded
alone through the same layers against the K/V rows the chain left behind
(cats_verify_nodes), and the remaining layers then take the whole tree from hidden states
(cats_verify_tree with hidden_in).  By the definition the oracle implements (every node is
the last position of an ordinary causal pass over its own root path) the staged result must
equal the oracle's one-shot tree pass over all layers."""
import numpy as np
import pytest
import torch

import paper_2605_11186_amd as cats
import synth
from gpu_common import MARGIN, REL_TOL, Pair, rel_err

pytestmark = pytest.mark.gpu


def staged_cycle(pair, ks, vs, S, root, drafts, corrections, l_sv):
    """Returns (token, parent, depth, hidden after l_sv layers, final hidden, logits, argmax,
    accept result) of one cycle run in the three enqueues of Alg. 1."""
    d = pair.dims
    g = len(drafts)
    kv_arr = cats.kv_array(ks, vs)
    token, parent, depth, corr_node = cats.cats_build_tree(root, drafts, corrections)
    T = len(parent)
    # main chain (root + drafts) through layers [0, l_sv): all of its nodes, from the embedding
    chain = cats.cats_build_tree(root, drafts)
    cats.cats_set_tree(pair.ctx, *chain[:3])
    h_sv = torch.full((T, d.hidden), float("nan"), dtype=torch.float32, device="cuda")
    cats.cats_verify_nodes(pair.ctx, pair.layers_arr, 0, l_sv, pair.d_embed, None, kv_arr, S, 0, h_sv[: g + 1])
    # corrections only, same layers, against the chain's K/V rows
    cats.cats_set_tree(pair.ctx, token, parent, depth)
    if T > g + 1:
        cats.cats_verify_nodes(pair.ctx, pair.layers_arr, 0, l_sv, pair.d_embed, None, kv_arr, S, g + 1,
                               h_sv[g + 1:])
    # remaining layers on the whole tree from hidden states; then the shallow layers' caches
    # are compacted along the same path
    hidden = torch.empty(T, d.hidden, dtype=torch.float32, device="cuda")
    logits = torch.empty(T, d.vocab, dtype=torch.float32, device="cuda")
    amax = torch.empty(T, dtype=torch.int32, device="cuda")
    host = cats.AcceptResult()
    cats.cats_verify_tree(pair.ctx, pair.layers_arr, l_sv, pair.L, None, h_sv, pair.d_final["g_final"],
                          pair.d_final["w_lm"], kv_arr, S, pair.res_dev, hidden_out=hidden,
                          logits_out=logits, argmax_out=amax, out_host=host)
    host2 = cats.AcceptResult()
    cats.cats_accept_and_compact(pair.ctx, amax, kv_arr, 0, l_sv, S, pair.res_dev, out_host=host2)
    torch.cuda.synchronize()
    assert host.as_dict() == host2.as_dict()
    return (token, parent, depth, h_sv.cpu().numpy(), hidden.cpu().numpy(), logits.cpu().numpy(),
            amax.cpu().numpy(), host.as_dict())


def check_cycle(pair, kc, vc, S, root, drafts, corrections, l_sv):
    ks, vs = pair.device_cache_from_oracle(kc, vc, S)
    token, parent, depth, g_sv, g_hidden, g_logits, g_amax, g_acc = staged_cycle(
        pair, ks, vs, S, root, drafts, corrections, l_sv)
    kc1, vc1 = kc.copy(), vc.copy()
    o_sv = pair.oracle.tree_forward(kc1, vc1, S, parent, depth, tokens=token, layer_end=l_sv)
    o_hidden = pair.oracle.tree_forward(kc, vc, S, parent, depth, tokens=token, layer_end=pair.L)
    o_logits = pair.oracle.lm_head(o_hidden)
    o_amax, o_margin = pair.oracle.argmax_margin(o_logits)
    e = (rel_err(g_sv, o_sv), rel_err(g_hidden, o_hidden), rel_err(g_logits, o_logits))
    print(f"T={len(parent)} l_sv={l_sv}: shallow hidden {e[0]:.2e} final hidden {e[1]:.2e} logits {e[2]:.2e}")
    assert max(e) <= REL_TOL
    safe = o_margin > MARGIN
    assert np.array_equal(g_amax[safe], o_amax[safe])
    assert g_acc == pair.oracle.accept(token, parent, depth, g_amax, S)
    if safe.all():
        assert g_acc == pair.oracle.accept(token, parent, depth, o_amax, S)
    pair.oracle.compact(kc, vc, S, g_acc["path"])
    new_S = g_acc["new_ctx_len"]
    for l in range(pair.L):
        gk, gv = pair.device_rows(ks, vs, l, new_S)
        assert rel_err(gk, kc[l, :new_S]) <= REL_TOL and rel_err(gv, vc[l, :new_S]) <= REL_TOL
    return g_acc


@pytest.fixture(scope="module")
def tiny4():
    """The tiny shape with four layers, so that both stages span more than one layer."""
    dims = synth.ModelDims(4, 256, 4, 64, 688, 1024)
    p = Pair(dims, 77, max_ctx=320, max_tree=32, packed=True)
    yield p
    p.close()


@pytest.mark.parametrize("l_sv", [1, 2, 3])
@pytest.mark.parametrize("corr_pos", [(), (0,), (1, 3), (0, 1, 2, 3, 4)])
def test_staged_cycle_equals_one_shot_tree_pass(tiny4, l_sv, corr_pos):
    S = 97
    rng = np.random.default_rng(len(corr_pos) * 10 + l_sv)
    kc, vc = tiny4.oracle_cache_random(5, S)
    drafts = rng.integers(0, tiny4.dims.vocab, 5).astype(np.int32)
    corrections = np.full(5, -1, dtype=np.int32)
    for i in corr_pos:
        corrections[i] = (drafts[i] + 1 + rng.integers(0, 50)) % tiny4.dims.vocab
    check_cycle(tiny4, kc, vc, S, 123, drafts, corrections, l_sv)


def test_staged_cycle_accepts_a_correction(tiny4):
    """Drafts follow the oracle's greedy stream except position 2, where the correction does:
    the cycle commits draft 0, draft 1, the correction, and the bonus token after it."""
    p = tiny4
    ctx_tokens = synth.context_tokens(p.dims, 31, 50)
    kc, vc = p.oracle_cache_from_prefill(ctx_tokens[:-1])
    S = 49
    kc2, vc2 = kc.copy(), vc.copy()
    stream = [int(ctx_tokens[-1])]
    for i in range(4):
        x = p.oracle.causal_decode(kc2, vc2, S + i, tokens=[stream[-1]], layer_end=p.L)
        amax, margin = p.oracle.argmax_margin(p.oracle.lm_head(x))
        assert margin[0] > MARGIN, "pick another seed: near-tie in the reference stream"
        stream.append(int(amax[0]))
    V = p.dims.vocab
    drafts = np.array([stream[1], stream[2], (stream[3] + 5) % V, 17, 18], dtype=np.int32)
    corrections = np.array([-1, (stream[2] + 9) % V, stream[3], -1, 19], dtype=np.int32)
    acc = check_cycle(p, kc, vc, S, stream[0], drafts, corrections, 2)
    assert acc["n_accepted"] == 3 and acc["tokens"] == stream[:4] and acc["bonus_token"] == stream[4]
    assert acc["path"] == [0, 1, 2, 7]   # nodes: chain 0..5, corrections 6 (pos 1), 7 (pos 2), 8 (pos 4)


def test_verify_nodes_rejects_bad_ranges(tiny4):
    p = tiny4
    ks, vs = p.device_cache_from_oracle(*p.oracle_cache_random(1, 8), 8)
    kv_arr = cats.kv_array(ks, vs)
    cats.cats_set_tree(p.ctx, *cats.cats_build_tree(1, [2, 3])[:3])
    out = torch.empty(3, p.dims.hidden, dtype=torch.float32, device="cuda")
    for node_begin in (-1, 3, 100):
        with pytest.raises(cats.CatsError) as e:
            cats.cats_verify_nodes(p.ctx, p.layers_arr, 0, 1, p.d_embed, None, kv_arr, 8, node_begin, out)
        assert e.value.status == cats.CATS_EINVAL
    with pytest.raises(cats.CatsError) as e:   # no output buffer
        cats.cats_verify_nodes(p.ctx, p.layers_arr, 0, 1, p.d_embed, None, kv_arr, 8, 0, None)
    assert e.value.status == cats.CATS_EINVAL
    with pytest.raises(cats.CatsError) as e:   # both input sources
        cats.cats_verify_nodes(p.ctx, p.layers_arr, 0, 1, p.d_embed, out, kv_arr, 8, 0, out)
    assert e.value.status == cats.CATS_EINVAL
    with pytest.raises(cats.CatsError) as e:
        cats.cats_verify_nodes(p.ctx, p.layers_arr, 0, 1, p.d_embed, None, kv_arr, 320, 0, out)
    assert e.value.status == cats.CATS_ECAPACITY


# ---------------------------------------------------------------------------------------------
# One whole cascaded cycle (Alg. 1, stages 1-3) with synthetic adapters.
#
# The adapters (Sec. 3.3: normalisation, one attention layer, residual, normalisation, shared LM
# head) are attention-only blocks with their own KV caches.  On the oracle side an adapter is a
# decoder layer whose feed-forward matrices are zero (x += 0), appended to the target's layer
# list, so the oracle needs no code of its own for it; its second normalisation is the final
# gain of the LM-head call.
def zero_ffn_layer(dims, adapter):
    z = lambda r, c: np.zeros((r, c), dtype=np.uint16)
    return {"wq": adapter["wq"], "wk": adapter["wk"], "wv": adapter["wv"], "wo": adapter["wo"],
            "g_attn": adapter["g_attn"], "g_ffn": adapter["g_attn"],
            "w_gate": z(dims.ffn, dims.hidden), "w_up": z(dims.ffn, dims.hidden), "w_down": z(dims.hidden, dims.ffn)}


def test_whole_cycle_with_synthetic_adapters(tiny4):
    import dataclasses
    from oracle.cats_oracle import Oracle
    from gpu_common import to_dev_bf16
    p = tiny4
    d = p.dims
    L, L_DM, L_SV, gamma, S = p.L, 1, 2, 4, 61
    seed = 4321
    ad = [synth.adapter_weights(d, seed, w) for w in (0, 1)]          # draft, shallow verifier
    # ---- oracle: target layers 0..3, then the two adapters as layers 4 and 5
    dims6 = dataclasses.replace(d, n_layers=L + 2)
    layers6 = p.layers + [zero_ffn_layer(d, a) for a in ad]
    orc = [Oracle(dims6, layers6, {"g_final": g, "w_lm": p.final["w_lm"]}, p.embed)
           for g in (ad[0]["g_out"], ad[1]["g_out"], p.final["g_final"])]   # LM head behind each norm
    kc, vc = orc[0].new_cache(p.max_ctx)
    for l in range(L + 2):
        k, v = synth.random_kv_context(d, seed, l, S)
        kc[l, :S], vc[l, :S] = synth.f32_from_bf16_bits(k), synth.f32_from_bf16_bits(v)
    # ---- device: the same caches, adapters as attention-only blocks
    saved_L = p.L
    p.L = L + 2
    ks, vs = p.device_cache_from_oracle(kc, vc, S)
    p.L = saved_L
    d_ad = [cats.pack_layer({k: to_dev_bf16(v) for k, v in a.items() if k != "g_out"}) for a in ad]
    d_gout = [to_dev_bf16(a["g_out"]) for a in ad]
    kv_target = cats.kv_array(ks[:L], vs[:L])
    ad_arr = [cats.layer_array([w]) for w in d_ad]
    ad_kv = [cats.kv_array(ks[L + i:L + i + 1], vs[L + i:L + i + 1]) for i in range(2)]
    H = d.hidden
    root = 77

    def next_token_gpu(hidden_row, g_out):
        amax = torch.empty(hidden_row.shape[0], dtype=torch.int32, device="cuda")
        margin = torch.empty(hidden_row.shape[0], dtype=torch.float32, device="cuda")
        cats.cats_lm_head_argmax(p.ctx, hidden_row, g_out, p.d_final["w_lm"], amax, margin_out=margin)
        torch.cuda.synchronize()
        return amax.cpu().numpy(), margin.cpu().numpy()

    # ---- stage 1: draft loop, one token at a time (chain grows, only the new node is forwarded)
    g_tokens, o_tokens = [root], [root]
    h_dm = torch.zeros(gamma + 1, H, dtype=torch.float32, device="cuda")
    o_hdm = np.zeros((gamma + 1, H))
    kc_o, vc_o = kc.copy(), vc.copy()
    for k in range(gamma + 1):
        chain = cats.cats_build_tree(root, g_tokens[1:])
        cats.cats_set_tree(p.ctx, *chain[:3])
        cats.cats_verify_nodes(p.ctx, p.layers_arr, 0, L_DM, p.d_embed, None, kv_target, S, k, h_dm[k:k + 1])
        o_hdm[k] = orc[0].causal_decode(kc_o, vc_o, S + k, tokens=[o_tokens[-1]], layer_end=L_DM)[0]
        if k == gamma:
            break   # the last draft token only needs its hidden state (it is a node of the tree)
        out = torch.empty(1, H, dtype=torch.float32, device="cuda")
        cats.cats_verify_nodes(p.ctx, ad_arr[0], 0, 1, None, h_dm[k:k + 1], ad_kv[0], S, k, out)
        tok, _ = next_token_gpu(out, d_gout[0])
        o_out = orc[0].causal_decode(kc_o, vc_o, S + k, hidden_in=o_hdm[k:k + 1], layer_begin=L, layer_end=L + 1)
        o_amax, o_margin = orc[0].argmax_margin(orc[0].lm_head(o_out))
        assert o_margin[0] > MARGIN, "pick another seed: near-tie in the draft stream"
        assert rel_err(out.cpu().numpy(), o_out) <= REL_TOL
        g_tokens.append(int(tok[0]))
        o_tokens.append(int(o_amax[0]))
    assert g_tokens == o_tokens
    assert rel_err(h_dm.cpu().numpy(), o_hdm) <= REL_TOL
    drafts = np.array(g_tokens[1:], dtype=np.int32)
    # the same stage in one call, the chain growing on the device (no read-back between tokens):
    # same kernels on the same rows, so tokens and hidden states must be identical
    toks_dev = torch.full((gamma + 1,), -1, dtype=torch.int32, device="cuda")
    h_dev = torch.zeros(gamma + 1, H, dtype=torch.float32, device="cuda")
    cats.cats_draft_chain(p.ctx, p.layers_arr, 0, L_DM, ad_arr[0], d_gout[0], p.d_final["w_lm"], p.d_embed,
                          kv_target, ad_kv[0], S, root, gamma, toks_dev, hidden_out=h_dev)
    torch.cuda.synchronize()
    assert toks_dev.cpu().tolist() == g_tokens
    assert torch.equal(h_dev, h_dm)

    # ---- stage 2: shallow layers on all chain positions in parallel, verifier adapter, corrections
    chain = cats.cats_build_tree(root, drafts)
    cats.cats_set_tree(p.ctx, *chain[:3])
    h_sv = torch.zeros(gamma + 1, H, dtype=torch.float32, device="cuda")
    cats.cats_verify_nodes(p.ctx, p.layers_arr, L_DM, L_SV, None, h_dm, kv_target, S, 0, h_sv)
    o_sv_out = torch.empty(gamma + 1, H, dtype=torch.float32, device="cuda")
    cats.cats_verify_nodes(p.ctx, ad_arr[1], 0, 1, None, h_sv, ad_kv[1], S, 0, o_sv_out)
    c_hat, _ = next_token_gpu(o_sv_out, d_gout[1])
    o_hsv = orc[1].tree_forward(kc_o, vc_o, S, chain[1], chain[2], hidden_in=o_hdm, layer_begin=L_DM, layer_end=L_SV)
    o_svo = orc[1].tree_forward(kc_o, vc_o, S, chain[1], chain[2], hidden_in=o_hsv, layer_begin=L + 1, layer_end=L + 2)
    o_chat, o_cm = orc[1].argmax_margin(orc[1].lm_head(o_svo))
    assert rel_err(h_sv.cpu().numpy(), o_hsv) <= REL_TOL and rel_err(o_sv_out.cpu().numpy(), o_svo) <= REL_TOL
    assert (o_cm[:gamma] > MARGIN).all(), "pick another seed: near-tie in the verifier's tokens"
    assert np.array_equal(c_hat[:gamma], o_chat[:gamma])
    corrections = c_hat[:gamma].astype(np.int32)       # position i judges draft i; equal tokens add no branch
    token, parent, depth, corr_node = cats.cats_build_tree(root, drafts, corrections)
    T = len(parent)
    assert T > gamma + 1, "untrained adapters disagree: there must be correction branches"

    # ---- corrections alone through the draft and shallow layers, then stage 3 on the whole tree
    cats.cats_set_tree(p.ctx, token, parent, depth)
    h_all = torch.zeros(T, H, dtype=torch.float32, device="cuda")
    h_all[: gamma + 1] = h_sv
    cats.cats_verify_nodes(p.ctx, p.layers_arr, 0, L_SV, p.d_embed, None, kv_target, S, gamma + 1, h_all[gamma + 1:])
    hidden = torch.empty(T, H, dtype=torch.float32, device="cuda")
    logits = torch.empty(T, d.vocab, dtype=torch.float32, device="cuda")
    amax = torch.empty(T, dtype=torch.int32, device="cuda")
    host = cats.AcceptResult()
    cats.cats_verify_tree(p.ctx, p.layers_arr, L_SV, L, None, h_all, p.d_final["g_final"], p.d_final["w_lm"],
                          kv_target, S, p.res_dev, hidden_out=hidden, logits_out=logits, argmax_out=amax,
                          out_host=host)
    cats.cats_accept_and_compact(p.ctx, amax, kv_target, 0, L_SV, S, p.res_dev)
    torch.cuda.synchronize()
    g_acc = host.as_dict()
    # oracle: the whole tree through the whole target in one pass (fresh target caches)
    o_hidden = orc[2].tree_forward(kc, vc, S, parent, depth, tokens=token, layer_end=L)
    o_logits = orc[2].lm_head(o_hidden)
    o_amax, o_margin = orc[2].argmax_margin(o_logits)
    assert rel_err(hidden.cpu().numpy(), o_hidden) <= REL_TOL and rel_err(logits.cpu().numpy(), o_logits) <= REL_TOL
    safe = o_margin > MARGIN
    assert np.array_equal(amax.cpu().numpy()[safe], o_amax[safe])
    assert g_acc == orc[2].accept(token, parent, depth, amax.cpu().numpy(), S)
    if safe.all():
        assert g_acc == orc[2].accept(token, parent, depth, o_amax, S)
    orc[2].compact(kc, vc, S, g_acc["path"])
    for l in range(L):
        gk, gv = p.device_rows(ks, vs, l, g_acc["new_ctx_len"])
        assert rel_err(gk, kc[l, :g_acc["new_ctx_len"]]) <= REL_TOL
        assert rel_err(gv, vc[l, :g_acc["new_ctx_len"]]) <= REL_TOL


def test_attention_only_block_argument_rules(tiny4):
    p = tiny4
    ks, vs = p.device_cache_from_oracle(*p.oracle_cache_random(1, 8), 8)
    kv_arr = cats.kv_array(ks, vs)
    cats.cats_set_tree(p.ctx, *cats.cats_build_tree(1, [2, 3])[:3])
    out = torch.empty(3, p.dims.hidden, dtype=torch.float32, device="cuda")
    half = dict(p.d_layers[0])
    half["w_up"] = None                               # some but not all feed-forward arrays
    with pytest.raises(cats.CatsError) as e:
        cats.cats_verify_nodes(p.ctx, cats.layer_array([half]), 0, 1, p.d_embed, None, kv_arr, 8, 0, out)
    assert e.value.status == cats.CATS_EINVAL


def test_draft_chain_argument_rules(tiny4):
    """Host-side validation of cats_draft_chain: nothing is enqueued for a bad call."""
    p = tiny4
    d = p.dims
    from gpu_common import to_dev_bf16
    ad = synth.adapter_weights(d, 7, 0)
    d_ad = cats.pack_layer({k: to_dev_bf16(v) for k, v in ad.items() if k != "g_out"})
    g_out = to_dev_bf16(ad["g_out"])
    ad_arr = cats.layer_array([d_ad])
    ks = [torch.zeros(d.n_heads, p.max_ctx, d.head_dim, dtype=torch.bfloat16, device="cuda") for _ in range(p.L + 1)]
    vs = [torch.zeros(d.n_heads, d.head_dim, p.max_ctx, dtype=torch.bfloat16, device="cuda") for _ in range(p.L + 1)]
    kv, kv_ad = cats.kv_array(ks[:p.L], vs[:p.L]), cats.kv_array(ks[p.L:], vs[p.L:])
    toks = torch.zeros(32, dtype=torch.int32, device="cuda")

    def status(**kw):
        a = dict(layer_begin=0, layer_end=1, adapter=ad_arr, ctx_len=10, root=3, gamma=4)
        a.update(kw)
        try:
            cats.cats_draft_chain(p.ctx, p.layers_arr, a["layer_begin"], a["layer_end"], a["adapter"], g_out,
                                  p.d_final["w_lm"], p.d_embed, kv, kv_ad, a["ctx_len"], a["root"], a["gamma"], toks)
        except cats.CatsError as e:
            return e.status
        return cats.CATS_OK

    assert status(gamma=0) == cats.CATS_EINVAL
    assert status(gamma=cats.CATS_MAX_DEPTH + 1) == cats.CATS_EINVAL
    assert status(root=d.vocab) == cats.CATS_EINVAL
    assert status(layer_end=0) == cats.CATS_EINVAL                      # empty layer range
    assert status(adapter=p.layers_arr) == cats.CATS_EINVAL             # a full layer is not an adapter block
    assert status(ctx_len=p.max_ctx - 3) == cats.CATS_ECAPACITY
    assert status() == cats.CATS_OK
    torch.cuda.synchronize()


@pytest.mark.parametrize("packed", [False, True])
def test_greedy_token_inside_the_single_row_lm_head(packed):
    """A single-row LM head call that asks for the token alone takes it inside the product (every
    workgroup holds complete sums for whole tiles; the last one to arrive picks the best).  It must
    name the token that the separate argmax kernel names on the logits of the same call, on a
    vocabulary with a ragged last tile and more tiles than workgroups, and the lowest index among
    equal logits (two identical weight rows)."""
    dims = synth.ModelDims(1, 256, 4, 64, 688, 128 * 300 + 11)
    seed = 991
    final = synth.final_weights(dims, seed)
    w = final["w_lm"].copy()
    rng = np.random.default_rng(seed)
    desc = cats.ModelDesc(dims.n_layers, dims.hidden, dims.n_heads, dims.head_dim, dims.ffn, dims.vocab, 64, 4,
                          dims.rms_eps, dims.rope_base, int(packed))
    ctx = cats.cats_create(desc)
    try:
        g = to_dev_bf16_local(final["g_final"])
        for case in range(6):
            hidden = torch.from_numpy(synth.random_hidden(dims, seed + case, 1).astype(np.float32)).cuda()
            wc = w.copy()
            if case >= 3:   # the winning row once more at a higher and at a lower index
                ref = synth.f32_from_bf16_bits(wc).astype(np.float64) @ (
                    hidden.cpu().numpy()[0].astype(np.float64) * synth.f32_from_bf16_bits(final["g_final"]))
                best = int(ref.argmax())
                others = [i for i in rng.integers(0, dims.vocab, 8) if i != best]
                wc[others[0]] = wc[best]
                wc[others[1]] = wc[best]
            w_dev = to_dev_bf16_local(wc)
            if packed:
                w_dev = cats.cats_pack_matrix(w_dev)
            tok_alone = torch.full((1,), -1, dtype=torch.int32, device="cuda")
            tok_full = torch.full((1,), -1, dtype=torch.int32, device="cuda")
            logits = torch.empty(1, dims.vocab, dtype=torch.float32, device="cuda")
            cats.cats_lm_head_argmax(ctx, hidden, g, w_dev, tok_alone)
            cats.cats_lm_head_argmax(ctx, hidden, g, w_dev, tok_full, logits_out=logits)
            torch.cuda.synchronize()
            lg = logits.cpu().numpy()[0]
            assert int(tok_full[0]) == int(np.flatnonzero(lg == lg.max())[0])
            assert int(tok_alone[0]) == int(tok_full[0]), (case, int(tok_alone[0]), int(tok_full[0]))
            if case >= 3:
                assert int(tok_alone[0]) == min(best, others[0], others[1])
    finally:
        torch.cuda.synchronize()
        cats.cats_destroy(ctx)


def to_dev_bf16_local(bits):
    from gpu_common import to_dev_bf16
    return to_dev_bf16(bits)
