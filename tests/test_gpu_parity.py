"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle
on the same seeded inputs.  Floating point: max |gpu - ref| / max |ref| <= 2e-2
per tensor.  Integer results (accepted length, path, token ids, bonus token,
compacted rows) are exact; greedy decisions are compared where the oracle's
top-2 logit gap exceeds 1e-2."""
import numpy as np
import pytest
import torch

import paper_2605_11186_amd as cats
import synth
from gpu_common import MARGIN, REL_TOL, Pair, bf16_to_f32_np, rel_err, to_dev_bf16

pytestmark = pytest.mark.gpu

SEED = 2024


@pytest.fixture(scope="module", params=[False, True], ids=["rowmajor", "packed"])
def tiny(request):
    """The tiny model with row-major weights and with weights re-tiled by cats_pack_matrix."""
    p = Pair(synth.TINY, SEED, max_ctx=320, max_tree=128, packed=request.param)
    yield p
    p.close()


def trees_for_tests():
    yield "binary15", *synth.complete_binary_tree(3)
    yield "root", *synth.chain_tree(1)
    yield "chain9", *synth.chain_tree(9)
    p, d, _ = synth.product_tree_pruned()
    yield "topk63", p, d
    yield "rand33", *synth.random_tree(33, 8, 5)
    yield "rand100", *synth.random_tree(100, 8, 6)
    yield "rand128", *synth.random_tree(128, 16, 7)


TREES = list(trees_for_tests())


def run_gpu_step(pair, ks, vs, S, tok, parent, depth, want_logits=True):
    T = len(parent)
    d = pair.dims
    kv_arr = cats.kv_array(ks, vs)
    hidden = torch.empty(T, d.hidden, dtype=torch.float32, device="cuda")
    logits = torch.empty(T, d.vocab, dtype=torch.float32, device="cuda") if want_logits else None
    amax = torch.empty(T, dtype=torch.int32, device="cuda")
    margin = torch.empty(T, dtype=torch.float32, device="cuda")
    host = cats.AcceptResult()
    cats.cats_set_tree(pair.ctx, tok, parent, depth)
    cats.cats_verify_tree(pair.ctx, pair.layers_arr, 0, pair.L, pair.d_embed, None,
                          pair.d_final["g_final"], pair.d_final["w_lm"], kv_arr, S, pair.res_dev,
                          hidden_out=hidden, logits_out=logits, argmax_out=amax, margin_out=margin,
                          out_host=host)
    torch.cuda.synchronize()
    return (hidden.cpu().numpy(), None if logits is None else logits.cpu().numpy(),
            amax.cpu().numpy(), margin.cpu().numpy(), host.as_dict())


def check_step(pair, kc, vc, ks, vs, S, tok, parent, depth):
    """Whole verify step on both sides; returns the oracle's accept result."""
    T = len(parent)
    g_hidden, g_logits, g_amax, g_margin, g_acc = run_gpu_step(pair, ks, vs, S, tok, parent, depth)
    # oracle: tree pass first, KV comparison before compaction changes the rows
    o_hidden = pair.oracle.tree_forward(kc, vc, S, parent, depth, tokens=tok, layer_end=pair.L)
    o_logits = pair.oracle.lm_head(o_hidden)
    o_amax, o_margin = pair.oracle.argmax_margin(o_logits)
    assert rel_err(g_hidden, o_hidden) <= REL_TOL
    assert rel_err(g_logits, o_logits) <= REL_TOL
    safe = o_margin > MARGIN
    assert np.array_equal(g_amax[safe], o_amax[safe])
    # margin reported by the GPU is consistent with its own logits
    top2 = np.sort(g_logits, axis=1)[:, -2:]
    assert np.allclose(g_margin, top2[:, 1] - top2[:, 0], atol=1e-6)
    assert np.array_equal(g_amax, g_logits.argmax(1))
    # accept walk: exact given the same per-node argmax ...
    o_acc_same = pair.oracle.accept(tok, parent, depth, g_amax, S)
    assert g_acc == o_acc_same
    # ... and equal to the oracle's own outcome when no decision on the way was a near-tie
    o_acc = pair.oracle.accept(tok, parent, depth, o_amax, S)
    if safe.all():
        assert g_acc == o_acc
    # compaction: bit-exact row moves on the GPU, compared with its own pre-compaction rows
    # through the oracle's compaction applied to the oracle cache
    pair.oracle.compact(kc, vc, S, g_acc["path"])
    new_S = g_acc["new_ctx_len"]
    for l in range(pair.L):
        gk, gv = pair.device_rows(ks, vs, l, new_S)
        assert rel_err(gk, kc[l, :new_S]) <= REL_TOL
        assert rel_err(gv, vc[l, :new_S]) <= REL_TOL
    return g_acc, o_acc, safe.all()


@pytest.mark.parametrize("name,parent,depth", TREES, ids=[t[0] for t in TREES])
def test_verify_tree_tiny_prefilled_context(tiny, name, parent, depth):
    """Config 1: tiny model, 128 prefilled context tokens, several tree shapes."""
    ctx_tokens = synth.context_tokens(synth.TINY, SEED, 128)
    kc, vc = tiny.oracle_cache_from_prefill(ctx_tokens)
    ks, vs = tiny.device_cache_from_oracle(kc, vc, 128)
    tok = synth.distinct_sibling_tokens(parent, synth.TINY.vocab, SEED)
    check_step(tiny, kc, vc, ks, vs, 128, tok, parent, depth)


# Hidden 384 = 3 and FFN 1104 = 8.6 chunks of 128 k-values: an odd chunk count (the second k group
# of the last 256-wide item has nothing to multiply), a ragged last chunk, and a vocabulary that
# ends inside a tile.
ODD = synth.ModelDims(2, 384, 6, 64, 1104, 1000)


@pytest.fixture(scope="module", params=[False, True], ids=["rowmajor", "packed"])
def odd(request):
    p = Pair(ODD, SEED + 5, max_ctx=192, max_tree=128, packed=request.param)
    yield p
    p.close()


@pytest.mark.parametrize("T", [9, 31, 40, 70, 96, 97, 100, 128])
def test_odd_chunk_counts_every_accumulator_depth(odd, T):
    """One to three accumulator blocks per wave (and the two-k-group variant up to 32 rows), and
    beyond 96 rows the paired workgroups (two blocks each; the second of a pair has 33 rows at
    T = 97), on shapes whose k range does not divide into whole items."""
    S = 37
    parent, depth = synth.random_tree(T, 8, T)
    tok = synth.distinct_sibling_tokens(parent, ODD.vocab, T)
    kc, vc = odd.oracle_cache_random(SEED + T, S)
    ks, vs = odd.device_cache_from_oracle(kc, vc, S)
    check_step(odd, kc, vc, ks, vs, S, tok, parent, depth)


@pytest.mark.parametrize("S", [0, 37, 191])
def test_single_row_on_ragged_shapes(odd, S):
    """A one-node tree (plain decoding of one token) runs on the single-row product, which builds
    its own input columns from the partial sums of the product before it: hidden 384 and FFN 1104
    end inside a 256-wide item, the vocabulary inside a tile; both weight layouts."""
    parent, depth = synth.chain_tree(1)
    tok = np.array([S % ODD.vocab], dtype=np.int32)
    kc, vc = odd.oracle_cache_random(SEED + 100 + S, S)
    ks, vs = odd.device_cache_from_oracle(kc, vc, S)
    check_step(odd, kc, vc, ks, vs, S, tok, parent, depth)


@pytest.mark.parametrize("head_dim,S", [(64, 4200), (128, 4200), (64, 9100), (128, 9100)])
def test_single_row_behind_a_long_context(head_dim, S):
    """One token behind a context of more than 32 x 128 keys: the single-query attention then takes
    its key chunks in several passes (4200: two, the second ragged; 9100: three), for both head sizes."""
    dims = synth.ModelDims(1, 256, 256 // head_dim, head_dim, 688, 1000)
    p = Pair(dims, SEED + 7, max_ctx=9216, max_tree=8, packed=True)
    try:
        parent, depth = synth.chain_tree(1)
        kc, vc = p.oracle_cache_random(SEED + S, S)
        ks, vs = p.device_cache_from_oracle(kc, vc, S)
        check_step(p, kc, vc, ks, vs, S, np.array([7], dtype=np.int32), parent, depth)
    finally:
        p.close()


@pytest.mark.parametrize("S", [0, 1, 31, 32, 33, 100, 191])
def test_verify_tree_ragged_context_lengths(tiny, S):
    parent, depth = synth.random_tree(45, 6, S + 1)
    tok = synth.distinct_sibling_tokens(parent, synth.TINY.vocab, S)
    kc, vc = tiny.oracle_cache_random(SEED + S, S)
    ks, vs = tiny.device_cache_from_oracle(kc, vc, S)
    check_step(tiny, kc, vc, ks, vs, S, tok, parent, depth)


@pytest.mark.parametrize("S", [31, 63, 95])
def test_largest_tree_behind_a_context_that_ends_a_key_block(tiny, S):
    """128 nodes whose first row is the last key of a 32-key block: the tree spans five key blocks
    and the low-part window beside the cache is used up to its last row."""
    parent, depth = synth.random_tree(128, 16, S)
    tok = synth.distinct_sibling_tokens(parent, synth.TINY.vocab, S)
    kc, vc = tiny.oracle_cache_random(SEED + S, S)
    ks, vs = tiny.device_cache_from_oracle(kc, vc, S)
    check_step(tiny, kc, vc, ks, vs, S, tok, parent, depth)


def test_accepting_drafts_are_accepted(tiny):
    """A tree whose main chain follows the oracle's greedy continuation is accepted to the end,
    and wrong siblings are not."""
    ctx_tokens = synth.context_tokens(synth.TINY, SEED + 1, 40)
    kc, vc = tiny.oracle_cache_from_prefill(ctx_tokens[:-1])
    S = 39
    # greedy continuation from the oracle (plain decoding)
    kc2, vc2 = kc.copy(), vc.copy()
    stream = [int(ctx_tokens[-1])]
    for i in range(5):
        x = tiny.oracle.causal_decode(kc2, vc2, S + i, tokens=[stream[-1]])
        amax, margin = tiny.oracle.argmax_margin(tiny.oracle.lm_head(x))
        assert margin[0] > MARGIN, "pick another seed: near-tie in the reference stream"
        stream.append(int(amax[0]))
    parent, depth, main, corr = synth.chain_with_corrections(4, [1, 3])
    tok = np.zeros(len(parent), np.int32)
    tok[0] = stream[0]
    for i in range(4):
        tok[main[i]] = stream[i + 1]
    for i, node in corr.items():
        tok[node] = (stream[i + 1] + 1) % synth.TINY.vocab
    ks, vs = tiny.device_cache_from_oracle(kc, vc, S)
    g_acc, o_acc, _ = check_step(tiny, kc, vc, ks, vs, S, tok, parent, depth)
    assert g_acc["n_accepted"] == 4 and g_acc["tokens"] == stream[:5]
    assert g_acc["bonus_token"] == stream[5] and g_acc["path"] == [0, 1, 2, 3, 4]
    # now break the chain at position 2 and let the correction carry the right token
    tok2 = tok.copy()
    tok2[main[1]] = (stream[2] + 7) % synth.TINY.vocab
    tok2[corr[1]] = stream[2]
    kc, vc = tiny.oracle_cache_from_prefill(ctx_tokens[:-1])
    ks, vs = tiny.device_cache_from_oracle(kc, vc, S)
    g_acc, _, _ = check_step(tiny, kc, vc, ks, vs, S, tok2, parent, depth)
    assert g_acc["path"] == [0, 1, corr[1]] and g_acc["bonus_token"] == stream[3]


def test_single_layer_call_matches_oracle(tiny):
    """cats_verify_layer on given hidden states (the stage-3 entry: hidden states, not tokens)."""
    S, T = 77, 37
    parent, depth = synth.random_tree(T, 7, 3)
    tok = synth.distinct_sibling_tokens(parent, synth.TINY.vocab, 3)
    x0 = synth.random_hidden(synth.TINY, 9, T)
    kc, vc = tiny.oracle_cache_random(5, S)
    ks, vs = tiny.device_cache_from_oracle(kc, vc, S)
    cats.cats_set_tree(tiny.ctx, tok, parent, depth)
    hidden = torch.from_numpy(x0).cuda()
    for l in range(tiny.L):
        w = cats.layer_weights_struct(tiny.d_layers[l])
        kv = cats.KVLayer(ks[l].data_ptr(), vs[l].data_ptr())
        cats.cats_verify_layer(tiny.ctx, w, hidden, kv, S)
        torch.cuda.synchronize()
        ref = tiny.oracle.tree_forward(kc, vc, S, parent, depth, hidden_in=x0 if l == 0 else ref,
                                       layer_begin=l, layer_end=l + 1)
        assert rel_err(hidden.cpu().numpy(), ref) <= REL_TOL
        gk, gv = tiny.device_rows(ks, vs, l, S + T)
        assert rel_err(gk, kc[l, :S + T]) <= REL_TOL and rel_err(gv, vc[l, :S + T]) <= REL_TOL


@pytest.mark.parametrize("S,T", [(0, 1), (5, 3), (128, 15), (190, 128), (95, 64)])
def test_tree_attention_alone(tiny, S, T):
    d = synth.TINY
    parent, depth = synth.random_tree(T, 8, S + T)
    tok = synth.distinct_sibling_tokens(parent, d.vocab, 1)
    rng = np.random.default_rng(S * 1000 + T)
    q = synth.f32_from_bf16_bits(synth.bf16_bits_from_f32(rng.normal(size=(T, d.hidden)).astype(np.float32)))
    kc, vc = tiny.oracle_cache_random(31, S + T)      # all S+T rows given, tree rows included
    ks, vs = tiny.device_cache_from_oracle(kc, vc, S + T)
    cats.cats_set_tree(tiny.ctx, tok, parent, depth)
    out = torch.empty(T, d.hidden, dtype=torch.bfloat16, device="cuda")
    kv = cats.KVLayer(ks[0].data_ptr(), vs[0].data_ptr())
    cats.cats_tree_attention(tiny.ctx, torch.from_numpy(q).cuda().to(torch.bfloat16), kv, S, out)
    torch.cuda.synchronize()
    ref = np.zeros((T, d.hidden))
    for i in range(T):
        rows = list(range(S))
        chain = []
        a = i
        while a >= 0:
            chain.append(S + a)
            a = int(parent[a])
        ref[i] = tiny.oracle.attend(q[i], kc[0], vc[0], rows + chain[::-1])
    assert rel_err(bf16_to_f32_np(out), ref) <= REL_TOL


def test_accept_and_compact_alone_is_bit_exact(tiny):
    """Integer path: random per-node argmax arrays, every result field and every moved row exact."""
    d = synth.TINY
    rng = np.random.default_rng(17)
    S = 50
    for trial in range(12):
        T = int(rng.integers(1, 129))
        parent, depth = synth.random_tree(T, 16 if trial % 2 else 4, trial)
        tok = rng.integers(0, 3, T).astype(np.int32)        # many matches, duplicate siblings
        amax = rng.integers(0, 3, T).astype(np.int32)
        ks = [torch.randn(d.n_heads, tiny.max_ctx, d.head_dim, device="cuda").to(torch.bfloat16) for _ in range(tiny.L)]
        vs = [torch.randn(d.n_heads, d.head_dim, tiny.max_ctx, device="cuda").to(torch.bfloat16) for _ in range(tiny.L)]
        k0 = [k.clone() for k in ks]
        v0 = [v.clone() for v in vs]
        cats.cats_set_tree(tiny.ctx, tok, parent, depth)
        host = cats.AcceptResult()
        cats.cats_accept_and_compact(tiny.ctx, torch.from_numpy(amax).cuda(), cats.kv_array(ks, vs), 0,
                                     tiny.L, S, tiny.res_dev, out_host=host)
        ref = tiny.oracle.accept(tok, parent, depth, amax, S)
        assert host.as_dict() == ref
        assert cats.accept_result_from_tensor(tiny.res_dev) == ref
        assert list(host.path[ref["n_accepted"] + 1:]) == [-1] * (cats.CATS_MAX_DEPTH - ref["n_accepted"])
        for l in range(tiny.L):
            for k, p in enumerate(ref["path"]):
                assert torch.equal(ks[l][:, S + k], k0[l][:, S + p])
                assert torch.equal(vs[l][:, :, S + k], v0[l][:, :, S + p])
            assert torch.equal(ks[l][:, :S], k0[l][:, :S]) and torch.equal(vs[l][:, :, :S], v0[l][:, :, :S])
            n = len(ref["path"])
            assert torch.equal(ks[l][:, S + n:], k0[l][:, S + n:])   # nothing else was touched


def test_chain_tree_is_chunked_prefill_and_multi_step_stream_is_lossless(tiny):
    """Prefill the context on the GPU with chain trees (no compaction needed: a chain is fully
    its own path), then run verify-accept-compact cycles; the committed stream must equal the
    oracle's plain greedy stream wherever its decisions are not near-ties."""
    d = synth.TINY
    ctx_tokens = synth.context_tokens(d, SEED + 2, 48)   # seed chosen for a long tie-free reference stream
    # reference: plain greedy decoding by the oracle
    kc, vc = tiny.oracle_cache_from_prefill(ctx_tokens[:-1])
    S0 = 47
    truth, margins = [], []
    last = int(ctx_tokens[-1])
    for i in range(40):
        x = tiny.oracle.causal_decode(kc, vc, S0 + i, tokens=[last])
        amax, margin = tiny.oracle.argmax_margin(tiny.oracle.lm_head(x))
        last = int(amax[0])
        truth.append(last)
        margins.append(float(margin[0]))
    # GPU: prefill 47 tokens as two chain chunks through verify_tree with layer results kept
    ks = [torch.full((d.n_heads, tiny.max_ctx, d.head_dim), float("nan"), device="cuda").to(torch.bfloat16) for _ in range(tiny.L)]
    vs = [torch.full((d.n_heads, d.head_dim, tiny.max_ctx), float("nan"), device="cuda").to(torch.bfloat16) for _ in range(tiny.L)]
    kv_arr = cats.kv_array(ks, vs)
    S = 0
    for chunk in (ctx_tokens[:30], ctx_tokens[30:47]):
        # chains deeper than CATS_MAX_DEPTH are fed in pieces of 16
        for lo in range(0, len(chunk), 16):
            piece = chunk[lo:lo + 16]
            p, dp = synth.chain_tree(len(piece))
            cats.cats_set_tree(tiny.ctx, piece, p, dp)
            # layers only, no roll-back: keep every row
            cats.cats_verify_tree(tiny.ctx, tiny.layers_arr, 0, tiny.L, tiny.d_embed, None,
                                  tiny.d_final["g_final"], tiny.d_final["w_lm"], kv_arr, S, tiny.res_dev)
            torch.cuda.synchronize()
            # the roll-back of a chain whose drafts are not the greedy ones keeps only a prefix, but the
            # rows themselves were all written in place (row S+i for chain node i), so they are all valid
            S += len(piece)
    kc_ref, vc_ref = tiny.oracle_cache_from_prefill(ctx_tokens[:-1])
    for l in range(tiny.L):
        gk, gv = tiny.device_rows(ks, vs, l, S0)
        assert rel_err(gk, kc_ref[l, :S0]) <= REL_TOL and rel_err(gv, vc_ref[l, :S0]) <= REL_TOL
    # verify cycles with drafts that are right with probability 0.7
    rng = np.random.default_rng(3)
    committed = []
    root_tok = int(ctx_tokens[-1])
    S = S0
    while len(committed) < 24:
        parent, depth = synth.random_tree(int(rng.integers(1, 20)), 5, int(rng.integers(1 << 30)))
        T = len(parent)
        tok = np.zeros(T, np.int32)
        tok[0] = root_tok
        taken = {}
        for i in range(1, T):
            true_next = truth[len(committed) + depth[i] - 1]
            sib = taken.setdefault(int(parent[i]), set())
            t = true_next if (rng.random() < 0.7 and true_next not in sib) else int(rng.integers(d.vocab))
            while t in sib:
                t = int(rng.integers(d.vocab))
            sib.add(t)
            tok[i] = t
        host = cats.AcceptResult()
        cats.cats_set_tree(tiny.ctx, tok, parent, depth)
        cats.cats_verify_tree(tiny.ctx, tiny.layers_arr, 0, tiny.L, tiny.d_embed, None,
                              tiny.d_final["g_final"], tiny.d_final["w_lm"], kv_arr, S, tiny.res_dev,
                              out_host=host)
        acc = host.as_dict()
        committed += acc["tokens"][1:] + [acc["bonus_token"]]
        S = acc["new_ctx_len"]
        root_tok = acc["bonus_token"]
    # the streams must agree up to the reference's first near-tie (none within the first 24 here)
    first_tie = next((i for i, m in enumerate(margins) if m <= MARGIN), len(margins))
    assert first_tie >= 24, "reference stream has an early near-tie: pick another seed"
    n = min(len(committed), first_tie)
    assert committed[:n] == truth[:n]
    # compacted cache == plain causal cache over context + committed tokens (bonus excluded)
    full = np.concatenate([ctx_tokens, np.array(committed[:-1], np.int32)])
    kc_ref, vc_ref = tiny.oracle_cache_from_prefill(full)
    assert len(full) == S
    for l in range(tiny.L):
        gk, gv = tiny.device_rows(ks, vs, l, S)
        assert rel_err(gk, kc_ref[l, :S]) <= REL_TOL and rel_err(gv, vc_ref[l, :S]) <= REL_TOL


def test_error_codes_from_host_validation(tiny):
    d = synth.TINY
    ok = (np.array([1, 2], np.int32), np.array([-1, 0], np.int32), np.array([0, 1], np.int32))
    bad = [
        (np.array([1, 2]), np.array([0, 0]), np.array([0, 1])),           # parent[0] != -1
        (np.array([1, 2]), np.array([-1, 1]), np.array([0, 1])),          # parent not earlier
        (np.array([1, 2]), np.array([-1, 0]), np.array([0, 2])),          # depth mismatch
        (np.array([1, d.vocab]), np.array([-1, 0]), np.array([0, 1])),    # token out of range
        (np.array([1, -1]), np.array([-1, 0]), np.array([0, 1])),
    ]
    for tok, par, dep in bad:
        with pytest.raises(cats.CatsError) as e:
            cats.cats_set_tree(tiny.ctx, tok, par, dep)
        assert e.value.status == cats.CATS_EINVAL
    p, dp = synth.chain_tree(18)                                           # deeper than CATS_MAX_DEPTH
    with pytest.raises(cats.CatsError):
        cats.cats_set_tree(tiny.ctx, np.zeros(18, np.int32), p, dp)
    cats.cats_set_tree(tiny.ctx, *ok)
    ks = [torch.zeros(d.n_heads, tiny.max_ctx, d.head_dim, device="cuda", dtype=torch.bfloat16) for _ in range(tiny.L)]
    vs = [torch.zeros(d.n_heads, d.head_dim, tiny.max_ctx, device="cuda", dtype=torch.bfloat16) for _ in range(tiny.L)]
    with pytest.raises(cats.CatsError) as e:
        cats.cats_verify_tree(tiny.ctx, tiny.layers_arr, 0, tiny.L, tiny.d_embed, None,
                              tiny.d_final["g_final"], tiny.d_final["w_lm"], cats.kv_array(ks, vs),
                              tiny.max_ctx - 1, tiny.res_dev)
    assert e.value.status == cats.CATS_ECAPACITY
    with pytest.raises(cats.CatsError) as e:   # both / neither input source
        cats.cats_verify_tree(tiny.ctx, tiny.layers_arr, 0, tiny.L, None, None,
                              tiny.d_final["g_final"], tiny.d_final["w_lm"], cats.kv_array(ks, vs), 0,
                              tiny.res_dev)
    assert e.value.status == cats.CATS_EINVAL
    desc = cats.ModelDesc(2, 256, 4, 64, 688, 1024, 320, 128, 1e-6, 10000.0, 0)
    fresh = cats.cats_create(desc)
    with pytest.raises(cats.CatsError) as e:   # no tree yet
        cats.cats_tree_attention(fresh, ks[0], cats.KVLayer(ks[0].data_ptr(), vs[0].data_ptr()), 0, ks[0])
    assert e.value.status == cats.CATS_ESTATE
    cats.cats_destroy(fresh)
    with pytest.raises(cats.CatsError):
        cats.cats_create(cats.ModelDesc(2, 250, 4, 64, 688, 1024, 320, 128, 1e-6, 10000.0, 0))
    with pytest.raises(cats.CatsError):   # layout flag must be 0 or 1
        cats.cats_create(cats.ModelDesc(2, 256, 4, 64, 688, 1024, 320, 128, 1e-6, 10000.0, 7))


def test_streamed_weights_give_the_same_step(tiny):
    """Offload regime: layer weights in pinned host memory, copied through two staging buffers
    while the previous layer computes.  Same kernels on the same values: results are identical
    to the resident call, bit for bit."""
    d = synth.TINY
    parent, depth = synth.random_tree(40, 6, 11)
    tok = synth.distinct_sibling_tokens(parent, d.vocab, 11)
    T, S = len(parent), 96
    kc, vc = tiny.oracle_cache_random(77, S)
    outs = []
    desc = cats.ModelDesc(d.n_layers, d.hidden, d.n_heads, d.head_dim, d.ffn, d.vocab, tiny.max_ctx, 128,
                          d.rms_eps, d.rope_base, int(tiny.packed))
    nbytes = cats.cats_layer_weight_bytes(desc)
    if not tiny.packed:
        assert nbytes == d.layer_weight_elems() * 2
    # the host copies hold exactly what the device layers hold (packed or not)
    host_layers = [{k: v.cpu().view(torch.int16).pin_memory() for k, v in w.items()} for w in tiny.d_layers]
    assert nbytes == sum(v.numel() * 2 for v in host_layers[0].values())
    staging = [torch.empty(nbytes, dtype=torch.uint8, device="cuda") for _ in range(2)]
    for streamed in (False, True, True):
        ks, vs = tiny.device_cache_from_oracle(kc, vc, S)
        hidden = torch.empty(T, d.hidden, dtype=torch.float32, device="cuda")
        logits = torch.empty(T, d.vocab, dtype=torch.float32, device="cuda")
        host = cats.AcceptResult()
        cats.cats_set_tree(tiny.ctx, tok, parent, depth)
        common = dict(hidden_out=hidden, logits_out=logits, out_host=host)
        if streamed:
            cats.cats_verify_tree_streamed(tiny.ctx, cats.layer_array(host_layers), 0, tiny.L, staging,
                                           tiny.d_embed, None, tiny.d_final["g_final"], tiny.d_final["w_lm"],
                                           cats.kv_array(ks, vs), S, tiny.res_dev, **common)
        else:
            cats.cats_verify_tree(tiny.ctx, tiny.layers_arr, 0, tiny.L, tiny.d_embed, None,
                                  tiny.d_final["g_final"], tiny.d_final["w_lm"], cats.kv_array(ks, vs), S,
                                  tiny.res_dev, **common)
        torch.cuda.synchronize()
        outs.append((hidden.cpu(), logits.cpu(), host.as_dict(), [k.cpu() for k in ks]))
    for o in outs[1:]:
        assert torch.equal(o[0], outs[0][0]) and torch.equal(o[1], outs[0][1]) and o[2] == outs[0][2]
        new_S = o[2]["new_ctx_len"]
        assert all(torch.equal(a[:, :new_S], b[:, :new_S]) for a, b in zip(o[3], outs[0][3]))
    # and against the oracle
    o_hidden = tiny.oracle.tree_forward(kc, vc, S, parent, depth, tokens=tok, layer_end=tiny.L)
    assert rel_err(outs[1][0].numpy(), o_hidden) <= REL_TOL


def test_pack_matrix_layout_is_the_documented_one():
    """cats_pack_matrix against the layout spelled out in the header, computed in numpy."""
    rng = np.random.default_rng(5)
    for rows, cols in [(32, 128), (70, 272), (688, 256), (256, 688)]:
        bits = rng.integers(0, 1 << 16, size=(rows, cols), dtype=np.uint16)
        packed = cats.cats_pack_matrix(to_dev_bf16(bits)).view(torch.int16).cpu().numpy().view(np.uint16)
        C = -(-cols // 128)
        rb_n = -(-rows // 32)
        assert packed.size * 2 == cats.cats_packed_matrix_bytes(rows, cols) == rb_n * C * 8 * 1024
        padded = np.zeros((rb_n * 32, C * 128), np.uint16)
        padded[:rows, :cols] = bits
        ref = np.empty((rb_n, C, 8, 64, 8), np.uint16)
        for l in range(64):
            for j in range(8):
                k0 = 16 * j + 8 * (l // 32)
                ref[:, :, j, l, :] = padded.reshape(rb_n, 32, C, 128)[:, l % 32, :, k0:k0 + 8]
        assert np.array_equal(packed, ref.reshape(-1))
