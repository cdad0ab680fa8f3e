"""Pins of the CPU oracle against things other than itself.

Each test names what it fixes: a closed form, a library routine, a textbook
formulation written independently in numpy, brute force on tiny inputs, or a
property the paper states (greedy speculative decoding is lossless: the
Introduction's claim that the output distribution is unchanged; the tree mask
of Fig. 4; Algorithm 1's walk).  None of them needs a GPU.
"""
import itertools
from pathlib import Path

import numpy as np
import pytest
from scipy.special import softmax

import synth
from oracle.cats_oracle import Oracle

MICRO = synth.ModelDims(n_layers=2, hidden=64, n_heads=4, head_dim=16, ffn=96, vocab=61)
SEED = 1234


def make_model(dims, seed=SEED, precision="f64"):
    layers = [synth.layer_weights(dims, seed, l) for l in range(dims.n_layers)]
    return Oracle(dims, layers, synth.final_weights(dims, seed), synth.embedding(dims, seed),
                  precision=precision)


@pytest.fixture(scope="module")
def micro():
    return make_model(MICRO)


def widen(bits):
    return synth.f32_from_bf16_bits(bits).astype(np.float64)


# --------------------------------------------------------------------------
# An independent textbook transformer: whole-sequence matmuls, a lower-
# triangular mask and library softmax; rotary embedding in the "rotate-half"
# formulation.  Written without looking at how the oracle loops.
# --------------------------------------------------------------------------
def textbook_forward(dims, layers, final, embed, tokens):
    H, nh, d = dims.hidden, dims.n_heads, dims.head_dim
    n = len(tokens)
    x = widen(embed)[tokens]
    pos = np.arange(n)[:, None]
    inv = dims.rope_base ** (-np.arange(0, d, 2) / d)
    ang = np.concatenate([pos * inv, pos * inv], axis=1)  # [n][d]
    cos, sin = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]

    def norm(v, g):
        return v / np.sqrt((v * v).mean(-1, keepdims=True) + dims.rms_eps) * widen(g)

    def rot(v):  # [n][nh][d]
        half = np.concatenate([-v[..., d // 2:], v[..., : d // 2]], axis=-1)
        return v * cos + half * sin

    ks, vs = [], []
    for w in layers:
        xn = norm(x, w["g_attn"])
        q = rot((xn @ widen(w["wq"]).T).reshape(n, nh, d))
        k = rot((xn @ widen(w["wk"]).T).reshape(n, nh, d))
        v = (xn @ widen(w["wv"]).T).reshape(n, nh, d)
        ks.append(k.reshape(n, H))
        vs.append(v.reshape(n, H))
        s = np.einsum("ihd,jhd->hij", q, k) / np.sqrt(d)
        s = np.where(np.tril(np.ones((n, n), bool))[None], s, -np.inf)
        p = softmax(s, axis=-1)
        o = np.einsum("hij,jhd->ihd", p, v).reshape(n, H)
        x = x + o @ widen(w["wo"]).T
        xn = norm(x, w["g_ffn"])
        g = xn @ widen(w["w_gate"]).T
        u = xn @ widen(w["w_up"]).T
        x = x + (g / (1 + np.exp(-g)) * u) @ widen(w["w_down"]).T
    logits = norm(x, final["g_final"]) @ widen(final["w_lm"]).T
    return x, logits, ks, vs


# ------------------------------ single operations ---------------------------
def test_bf16_roundtrip_and_rounding():
    # exactly representable values survive; ties go to even
    x = np.array([1.0, -2.5, 0.02, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8], np.float32)
    b = synth.bf16_bits_from_f32(x)
    y = synth.f32_from_bf16_bits(b)
    assert y[0] == 1.0 and y[1] == -2.5
    assert y[3] == 1.0            # halfway between 1 and 1+2^-7: even mantissa wins
    assert y[4] == 1.0 + 2 ** -6  # halfway between 1+2^-7 and 1+2^-6
    assert abs(y[2] - 0.02) <= 0.02 * 2 ** -8


def test_rmsnorm_closed_form(micro):
    H = MICRO.hidden
    g = synth.bf16_bits_from_f32(np.full(H, 1.5, np.float32))
    out = micro.rmsnorm(np.full(H, 3.0), g)
    assert np.allclose(out, 1.5 * 3.0 / np.sqrt(9.0 + MICRO.rms_eps), rtol=1e-12)
    # scale invariance up to eps: doubling x leaves the output (almost) unchanged
    x = np.random.default_rng(0).normal(size=H)
    a, b = micro.rmsnorm(x, g), micro.rmsnorm(2 * x, g)
    assert np.allclose(a, b, rtol=1e-5)
    assert np.allclose(np.sqrt((a * a).mean()), 1.5, rtol=1e-5)


def test_linear_is_matmul_with_transposed_weight(micro):
    rng = np.random.default_rng(1)
    W = synth.normal_bf16((7, 0, 1), (37, 53), 0.02)
    X = rng.normal(size=(5, 53))
    Y = micro.linear(X, W)
    assert Y.shape == (5, 37)
    assert np.allclose(Y, X @ widen(W).T, rtol=1e-12, atol=1e-14)
    # a transposed operand would not even agree in shape semantics: check one entry by hand
    assert np.isclose(Y[2, 3], sum(X[2, k] * widen(W)[3, k] for k in range(53)))


def test_rope_identity_norm_and_relative_position(micro):
    rng = np.random.default_rng(2)
    H, nh, d = MICRO.hidden, MICRO.n_heads, MICRO.head_dim
    q, k = rng.normal(size=H), rng.normal(size=H)
    assert np.array_equal(micro.rope(q, 0), q)                      # position 0: identity
    assert np.allclose(np.linalg.norm(micro.rope(q, 77)), np.linalg.norm(q))
    # per-head dot products depend only on the position difference
    def dots(pq, pk):
        a, b = micro.rope(q, pq).reshape(nh, d), micro.rope(k, pk).reshape(nh, d)
        return (a * b).sum(-1)
    assert np.allclose(dots(9, 4), dots(105, 100), rtol=1e-9, atol=1e-12)
    assert not np.allclose(dots(9, 4), dots(9, 5), rtol=1e-3)
    # closed form for one pair: dims (j, j + d/2) rotate by pos * base^(-2j/d)
    j, pos = 3, 11
    ang = pos * MICRO.rope_base ** (-2 * j / d)
    r = micro.rope(q, pos)
    assert np.isclose(r[j], q[j] * np.cos(ang) - q[j + d // 2] * np.sin(ang))
    assert np.isclose(r[j + d // 2], q[j] * np.sin(ang) + q[j + d // 2] * np.cos(ang))


def test_attend_against_library_softmax(micro):
    rng = np.random.default_rng(3)
    H, nh, d = MICRO.hidden, MICRO.n_heads, MICRO.head_dim
    Kc, Vc, q = rng.normal(size=(9, H)), rng.normal(size=(9, H)), rng.normal(size=H)
    rows = [0, 2, 3, 7]
    out = micro.attend(q, Kc, Vc, rows).reshape(nh, d)
    for h in range(nh):
        sl = slice(h * d, (h + 1) * d)
        p = softmax(Kc[rows][:, sl] @ q[sl] / np.sqrt(d))
        assert np.allclose(out[h], p @ Vc[rows][:, sl], rtol=1e-12)
    # a single visible row returns that row's value exactly
    one = micro.attend(q, Kc, Vc, [5])
    assert np.allclose(one, Vc[5], rtol=1e-15)


# ------------------------------ whole passes ---------------------------------
def test_causal_decode_equals_textbook_transformer(micro):
    tokens = synth.context_tokens(MICRO, 5, 11)
    x_ref, logits_ref, ks, vs = textbook_forward(MICRO, micro.layers, micro.final, micro.embed, tokens)
    kc, vc = micro.new_cache(16)
    x = micro.causal_decode(kc, vc, 0, tokens=tokens)
    assert np.allclose(x, x_ref, rtol=1e-9, atol=1e-12)
    assert np.allclose(micro.lm_head(x), logits_ref, rtol=1e-9, atol=1e-12)
    for l in range(MICRO.n_layers):
        assert np.allclose(kc[l, :11], ks[l], rtol=1e-9, atol=1e-12)
        assert np.allclose(vc[l, :11], vs[l], rtol=1e-9, atol=1e-12)


def prefill(model, tokens, max_ctx):
    kc, vc = model.new_cache(max_ctx)
    if len(tokens):
        model.causal_decode(kc, vc, 0, tokens=tokens)
    return kc, vc


def path_of(parent, i):
    p = []
    while i >= 0:
        p.append(i)
        i = int(parent[i])
    return p[::-1]


def check_nodes_equal_own_paths(model, ctx_tokens, parent, depth, tok, tol=1e-9):
    """Every node's output must equal ordinary decoding of context + its root-to-node path."""
    S = len(ctx_tokens)
    kc, vc = prefill(model, ctx_tokens, S + len(parent) + 1)
    x = model.tree_forward(kc, vc, S, parent, depth, tokens=tok)
    for i in range(len(parent)):
        p = path_of(parent, i)
        kc2, vc2 = prefill(model, ctx_tokens, S + len(p) + 1)
        xi = model.causal_decode(kc2, vc2, S, tokens=tok[p])
        assert np.allclose(x[i], xi[-1], rtol=tol, atol=1e-12), (parent, i)
        # the node's cached key/value rows are those of the path's last position
        for l in range(model.dims.n_layers):
            assert np.allclose(kc[l, S + i], kc2[l, S + len(p) - 1], rtol=tol, atol=1e-12)
            assert np.allclose(vc[l, S + i], vc2[l, S + len(p) - 1], rtol=tol, atol=1e-12)


def test_chain_tree_equals_causal_decoding(micro):
    ctx = synth.context_tokens(MICRO, 6, 7)
    parent, depth = synth.chain_tree(6)
    tok = synth.distinct_sibling_tokens(parent, MICRO.vocab, 1)
    kc, vc = prefill(micro, ctx, 20)
    x = micro.tree_forward(kc, vc, 7, parent, depth, tokens=tok)
    kc2, vc2 = prefill(micro, ctx, 20)
    x2 = micro.causal_decode(kc2, vc2, 7, tokens=tok)
    assert np.allclose(x, x2, rtol=1e-10, atol=1e-13)
    assert np.allclose(kc[:, :13], kc2[:, :13], rtol=1e-10, atol=1e-13)
    assert np.allclose(vc[:, :13], vc2[:, :13], rtol=1e-10, atol=1e-13)
    # and both equal the textbook transformer over context + chain
    x_ref, _, _, _ = textbook_forward(MICRO, micro.layers, micro.final, micro.embed,
                                      np.concatenate([ctx, tok]))
    assert np.allclose(x, x_ref[7:], rtol=1e-9, atol=1e-12)


def test_every_node_equals_its_own_path_all_small_trees(micro):
    ctx = synth.context_tokens(MICRO, 8, 3)
    n_trees = 0
    for T in range(1, 7):
        for parent, depth in synth.all_parent_arrays(T):
            tok = synth.distinct_sibling_tokens(parent, MICRO.vocab, 100 + n_trees)
            check_nodes_equal_own_paths(micro, ctx, parent, depth, tok)
            n_trees += 1
    assert n_trees == 1 + 1 + 2 + 6 + 24 + 120


def test_every_node_equals_its_own_path_binary_tree_and_empty_context(micro):
    parent, depth = synth.complete_binary_tree(3)
    tok = synth.distinct_sibling_tokens(parent, MICRO.vocab, 3)
    check_nodes_equal_own_paths(micro, synth.context_tokens(MICRO, 9, 5), parent, depth, tok)
    check_nodes_equal_own_paths(micro, np.zeros(0, np.int32), parent, depth, tok)


def test_root_only_tree_is_one_vanilla_decode_step(micro):
    ctx = synth.context_tokens(MICRO, 10, 6)
    parent, depth = synth.chain_tree(1)
    tok = np.array([17], np.int32)
    kc, vc = prefill(micro, ctx, 10)
    _, logits, amax, _, acc = micro.verify_step(kc, vc, 6, tok, parent, depth)
    _, logits_ref, _, _ = textbook_forward(MICRO, micro.layers, micro.final, micro.embed,
                                           np.concatenate([ctx, tok]))
    assert np.allclose(logits[0], logits_ref[-1], rtol=1e-9, atol=1e-12)
    assert acc == {"n_accepted": 0, "path": [0], "tokens": [17],
                   "bonus_token": int(np.argmax(logits_ref[-1])), "new_ctx_len": 7}


def test_relabelling_invariance(micro):
    ctx = synth.context_tokens(MICRO, 11, 4)
    parent, depth = synth.random_tree(12, 5, 7)
    tok = synth.distinct_sibling_tokens(parent, MICRO.vocab, 5)
    kc, vc = prefill(micro, ctx, 20)
    x = micro.tree_forward(kc, vc, 4, parent, depth, tokens=tok)
    p2, d2, old_of_new = synth.relabel_topological(parent, 3)
    assert not np.array_equal(old_of_new, np.arange(12))
    kc2, vc2 = prefill(micro, ctx, 20)
    x2 = micro.tree_forward(kc2, vc2, 4, p2, d2, tokens=tok[old_of_new])
    assert np.allclose(x2, x[old_of_new], rtol=1e-11, atol=1e-14)


def test_sibling_subtrees_do_not_influence_a_node(micro):
    ctx = synth.context_tokens(MICRO, 12, 4)
    # 0-1-2 chain plus a side subtree 3,4 under the root
    parent = np.array([-1, 0, 1, 0, 3], np.int32)
    depth = np.array([0, 1, 2, 1, 2], np.int32)
    tok = np.array([5, 6, 7, 8, 9], np.int32)
    kc, vc = prefill(micro, ctx, 12)
    x = micro.tree_forward(kc, vc, 4, parent, depth, tokens=tok)
    kc2, vc2 = prefill(micro, ctx, 12)
    x2 = micro.tree_forward(kc2, vc2, 4, parent[:3], depth[:3], tokens=tok[:3])
    assert np.array_equal(x[:3], x2)   # bit-identical: same operations on the same numbers


# ------------------------------ accept walk ---------------------------------
def brute_force_accept(token, parent, depth, amax):
    """Enumerate every root-descending chain, keep the valid ones, take the longest
    (lowest end node on ties)."""
    T = len(parent)
    best = [0]
    for i in range(T):
        p = path_of(parent, i)
        if all(token[p[k]] == amax[p[k - 1]] for k in range(1, len(p))):
            if len(p) > len(best):
                best = p
    return best, int(amax[best[-1]])


def test_accept_brute_force_small_trees(micro):
    rng = np.random.default_rng(5)
    n = 0
    for T in range(1, 8):
        for parent, depth in itertools.islice(synth.all_parent_arrays(T), 0, None, max(1, T - 3)):
            for _ in range(3):
                token = rng.integers(0, 3, T).astype(np.int32)   # tiny vocabulary: many matches,
                amax = rng.integers(0, 3, T).astype(np.int32)    # duplicate sibling tokens included
                acc = micro.accept(token, parent, depth, amax, 10)
                path, bonus = brute_force_accept(token, parent, depth, amax)
                assert acc["path"] == path and acc["bonus_token"] == bonus
                assert acc["n_accepted"] == len(path) - 1
                assert acc["tokens"] == [int(token[p]) for p in path]
                assert acc["new_ctx_len"] == 10 + len(path)
                n += 1
    assert n > 500


def cascade_commit(d, c_hat, argmax_at):
    """What one cascaded cycle commits (Algorithm 1, walk + bonus token) for a chain of drafts
    d[0..g-1] with shallow-verifier corrections c_hat (dict position -> token), stated as a
    property instead of a walk.  argmax_at(prefix) is the target's greedy token after
    root + prefix.  Let m be the length of the longest draft prefix in which every draft equals
    the target's greedy token after the drafts before it.  The committed tokens are that prefix,
    then the correction at position m if there is one and it equals the target's greedy token
    after the prefix (readings: the correction is judged by the distribution that judged the
    draft it replaces; nothing follows an accepted correction, it is a leaf), then the target's
    own greedy token after all of these (the bonus token)."""
    g = len(d)
    agrees = [d[j] == argmax_at(tuple(d[:j])) for j in range(g)]
    m = agrees.index(False) if False in agrees else g
    y = list(d[:m])
    if m < g and c_hat.get(m) == argmax_at(tuple(y)):
        y.append(c_hat[m])
    return y + [argmax_at(tuple(y))]


def test_general_walk_commits_what_algorithm1_commits_on_chain_plus_corrections(micro):
    rng = np.random.default_rng(6)
    for trial in range(300):
        g = int(rng.integers(1, 7))
        corr_pos = [i for i in range(g) if rng.random() < 0.5]
        parent, depth, main, corr = synth.chain_with_corrections(g, corr_pos)
        T = len(parent)
        token = np.zeros(T, np.int32)
        token[0] = 9
        d = rng.integers(0, 3, g)
        c_hat = {i: int((d[i] + 1 + rng.integers(0, 2)) % 3) for i in corr_pos}  # differs from d[i]
        for i in range(g):
            token[main[i]] = d[i]
        for i, node in corr.items():
            token[node] = c_hat[i]
        amax = rng.integers(0, 3, T).astype(np.int32)

        def argmax_at(prefix):
            node = 0
            for t in prefix:  # descend to the child that carries token t
                node = next(j for j in range(T) if parent[j] == node and token[j] == t)
            return int(amax[node])

        acc = micro.accept(token, parent, depth, amax, 0)
        assert acc["tokens"][1:] + [acc["bonus_token"]] == cascade_commit(list(d), c_hat, argmax_at)


def test_duplicate_siblings_pick_lowest_index(micro):
    parent = np.array([-1, 0, 0], np.int32)
    depth = np.array([0, 1, 1], np.int32)
    acc = micro.accept(np.array([1, 4, 4]), parent, depth, np.array([4, 7, 8]), 0)
    assert acc["path"] == [0, 1] and acc["bonus_token"] == 7


def test_argmax_ties_and_margin(micro):
    logits = np.array([[0.5, 2.0, 2.0, -1.0], [3.0, 1.0, 2.5, 0.0]])
    amax, margin = micro.argmax_margin(logits)
    assert list(amax) == [1, 0]
    assert np.allclose(margin, [0.0, 0.5])


# ------------------------------ compaction ---------------------------------
def test_compaction_moves_rows_in_place_with_overlap(micro):
    kc, vc = micro.new_cache(12)
    kc[:] = np.arange(kc.size).reshape(kc.shape)
    vc[:] = -np.arange(vc.size).reshape(vc.shape)
    k0, v0 = kc.copy(), vc.copy()
    path = [0, 1, 3, 4]    # row 3 is both a destination (of node 4) and a source
    micro.compact(kc, vc, 5, path)
    for k, p in enumerate(path):
        assert np.array_equal(kc[:, 5 + k], k0[:, 5 + p])
        assert np.array_equal(vc[:, 5 + k], v0[:, 5 + p])
    assert np.array_equal(kc[:, :5], k0[:, :5])


# ------------------------------ losslessness ---------------------------------
def greedy_stream(model, ctx_tokens, n_new):
    """Plain greedy autoregressive decoding with the textbook transformer."""
    seq = list(ctx_tokens)
    for _ in range(n_new):
        _, logits, _, _ = textbook_forward(model.dims, model.layers, model.final, model.embed,
                                           np.array(seq))
        seq.append(int(np.argmax(logits[-1])))
    return seq[len(ctx_tokens):]


def test_speculative_greedy_stream_is_lossless(micro):
    """Many verify-accept-compact cycles on trees that mix right and wrong drafts commit
    exactly the plain greedy stream, and the compacted cache equals an ordinary one."""
    rng = np.random.default_rng(8)
    ctx = synth.context_tokens(MICRO, 13, 5)
    truth = greedy_stream(micro, ctx, 40)
    max_ctx = 80
    kc, vc = prefill(micro, ctx[:-1], max_ctx)   # the last context token is the first root
    S = len(ctx) - 1
    committed = []          # tokens after ctx
    root_tok = int(ctx[-1])
    accepted_hist = []
    while len(committed) < 30:
        parent, depth = synth.random_tree(int(rng.integers(1, 14)), 5, int(rng.integers(1 << 30)))
        T = len(parent)
        tok = np.zeros(T, np.int32)
        tok[0] = root_tok
        taken = {}
        for i in range(1, T):
            # the true continuation along this node's path, used with probability 0.7
            true_next = truth[len(committed) + depth[i] - 1]
            sib = taken.setdefault(int(parent[i]), set())
            t = true_next if (rng.random() < 0.7 and true_next not in sib) else int(rng.integers(MICRO.vocab))
            while t in sib:
                t = int(rng.integers(MICRO.vocab))
            sib.add(t)
            tok[i] = t
        _, _, _, _, acc = micro.verify_step(kc, vc, S, tok, parent, depth)
        committed += acc["tokens"][1:] + [acc["bonus_token"]]
        accepted_hist.append(acc["n_accepted"])
        S = acc["new_ctx_len"]
        root_tok = acc["bonus_token"]
    assert committed == truth[: len(committed)]
    assert max(accepted_hist) >= 2 and min(accepted_hist) == 0   # both outcomes were exercised
    # the cache now equals that of ordinary decoding over everything whose K/V is committed
    full = np.concatenate([ctx, np.array(committed[:-1], np.int32)])
    assert len(full) == S
    _, _, ks, vs = textbook_forward(MICRO, micro.layers, micro.final, micro.embed, full)
    for l in range(MICRO.n_layers):
        assert np.allclose(kc[l, :S], ks[l], rtol=1e-8, atol=1e-11)
        assert np.allclose(vc[l, :S], vs[l], rtol=1e-8, atol=1e-11)


# ------------------------------ precision / bytes ---------------------------
def test_f32_build_agrees_with_f64_build():
    m64, m32 = make_model(synth.TINY), make_model(synth.TINY, precision="f32")
    ctx = synth.context_tokens(synth.TINY, 14, 16)
    parent, depth = synth.complete_binary_tree(3)
    tok = synth.distinct_sibling_tokens(parent, synth.TINY.vocab, 2)
    outs = []
    for m in (m64, m32):
        kc, vc = prefill(m, ctx, 40)
        outs.append(m.verify_step(kc, vc, 16, tok, parent, depth))
    assert np.allclose(outs[0][1], outs[1][1], rtol=0, atol=2e-5 * np.abs(outs[0][1]).max())
    assert outs[0][4] == outs[1][4]


def test_weight_bytes_per_token_matches_table4_baseline():
    """Table 4 lists 12.95 GB streamed per token for the non-speculative 32-layer 7B
    baseline; the per-layer element count used for the roofline reproduces it at 2 bytes."""
    golden = (Path(__file__).parent / "golden" / "table4_baseline_bpt.txt").read_text()
    gb = float([l for l in golden.splitlines() if not l.startswith("#")][0])
    total = synth.V7B.n_layers * synth.V7B.layer_weight_elems() * 2
    assert total == 12_952_535_040
    assert round(total / 1e9, 2) == gb


def test_generators_are_deterministic_and_shaped():
    a = synth.layer_weights(synth.TINY, 3, 1)
    b = synth.layer_weights(synth.TINY, 3, 1)
    c = synth.layer_weights(synth.TINY, 3, 0)
    assert all(np.array_equal(a[k], b[k]) for k in a)
    assert not np.array_equal(a["wq"], c["wq"])
    w = synth.f32_from_bf16_bits(a["w_gate"])
    assert w.shape == (688, 256) and abs(w.std() - 0.02) < 1e-3 and abs(w.mean()) < 1e-3
    g = synth.f32_from_bf16_bits(a["g_attn"])
    assert abs(g.mean() - 1.0) < 0.01
    parent, depth, rank = synth.product_tree_pruned()
    assert len(parent) == 63 and synth.is_valid_tree(parent, depth) and depth.max() == 6
    assert [int((depth == k).sum()) for k in range(7)] == [1, 4, 7, 10, 14, 14, 13]
    p, d = synth.random_tree(128, 8, 1)
    assert synth.is_valid_tree(p, d) and d.max() <= 8
