"""A whole verification call enqueues kernels only (no allocation, no memset, no host
synchronisation), so it can be recorded into a HIP graph.  The graph is replayed several times
with eager work and synchronisations of the program's own in between, and every replay must
reproduce the eager call's outputs bit for bit."""
import numpy as np
import pytest
import torch

import paper_2605_11186_amd as cats
import synth
from gpu_common import Pair

pytestmark = pytest.mark.gpu

SEED = 77


def outputs(pair, T):
    d = pair.dims
    return dict(hidden=torch.zeros(T, d.hidden, dtype=torch.float32, device="cuda"),
                logits=torch.zeros(T, d.vocab, dtype=torch.float32, device="cuda"),
                amax=torch.zeros(T, dtype=torch.int32, device="cuda"),
                res=cats.accept_result_tensor())


def enqueue(pair, kv_arr, S, out, stream):
    cats.cats_verify_tree(pair.ctx, pair.layers_arr, 0, pair.L, pair.d_embed, None,
                          pair.d_final["g_final"], pair.d_final["w_lm"], kv_arr, S, out["res"],
                          hidden_out=out["hidden"], logits_out=out["logits"], argmax_out=out["amax"],
                          stream=stream)


def snapshot(out):
    return (out["hidden"].cpu().numpy().copy(), out["logits"].cpu().numpy().copy(),
            out["amax"].cpu().numpy().copy(), cats.accept_result_from_tensor(out["res"]))


@pytest.mark.parametrize("packed", [False, True], ids=["rowmajor", "packed"])
def test_verify_call_replays_from_a_graph(packed):
    pair = Pair(synth.TINY, SEED, max_ctx=320, max_tree=64, packed=packed)
    try:
        S = 100
        parent, depth = synth.random_tree(45, 6, 3)
        T = len(parent)
        tok = synth.distinct_sibling_tokens(parent, synth.TINY.vocab, SEED)
        kc, vc = pair.oracle_cache_random(SEED, S)
        ks, vs = pair.device_cache_from_oracle(kc, vc, S)
        kv_arr = cats.kv_array(ks, vs)
        cats.cats_set_tree(pair.ctx, tok, parent, depth)
        torch.cuda.synchronize()   # the tree upload ran on the default stream
        stream = torch.cuda.Stream()
        eager, other, replayed = outputs(pair, T), outputs(pair, T), outputs(pair, T)
        with torch.cuda.stream(stream):
            enqueue(pair, kv_arr, S, eager, stream)
            torch.cuda.synchronize()
            want = snapshot(eager)
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=stream):
                enqueue(pair, kv_arr, S, replayed, stream)
            torch.cuda.synchronize()
            for _ in range(4):
                for t in (replayed["hidden"], replayed["logits"], replayed["amax"], replayed["res"]):
                    t.zero_()
                enqueue(pair, kv_arr, S, other, stream)     # eager work between the replays
                torch.cuda.synchronize()
                graph.replay()
                torch.cuda.synchronize()
                got = snapshot(replayed)
                assert np.array_equal(got[0], want[0])
                assert np.array_equal(got[1], want[1])
                assert np.array_equal(got[2], want[2])
                assert got[3] == want[3]
                assert snapshot(other)[3] == want[3]
    finally:
        pair.close()


def test_draft_chain_replays_from_a_graph():
    """The stage-1 draft loop (single-row kernels: products that build their own input, the
    one-launch attention, the LM head that names the token itself through an arrival counter)
    enqueues kernels and one device-to-device copy only; replays must give the eager call's
    tokens and hidden states bit for bit, with eager calls in between."""
    from gpu_common import to_dev_bf16
    pair = Pair(synth.TINY, SEED + 1, max_ctx=320, max_tree=16, packed=True)
    try:
        d = pair.dims
        S, gamma, root = 70, 5, 123
        ad = synth.adapter_weights(d, SEED + 2, 0)
        d_ad = cats.pack_layer({k: to_dev_bf16(v) for k, v in ad.items() if k != "g_out"})
        g_out = to_dev_bf16(ad["g_out"])
        ad_arr = cats.layer_array([d_ad])
        kc, vc = pair.oracle_cache_random(SEED, S)
        ks, vs = pair.device_cache_from_oracle(kc, vc, S)
        kv_arr = cats.kv_array(ks, vs)
        ka, va = pair.device_cache_from_oracle(kc, vc, S)   # a second set: its first layer is the adapter block's cache
        kv_ad = cats.kv_array(ka[:1], va[:1])

        def enqueue_chain(tokens, hidden, stream):
            cats.cats_draft_chain(pair.ctx, pair.layers_arr, 0, pair.L, ad_arr, g_out, pair.d_final["w_lm"],
                                  pair.d_embed, kv_arr, kv_ad, S, root, gamma, tokens, hidden_out=hidden,
                                  stream=stream)

        def fresh():
            return (torch.full((gamma + 1,), -1, dtype=torch.int32, device="cuda"),
                    torch.zeros(gamma + 1, d.hidden, dtype=torch.float32, device="cuda"))

        stream = torch.cuda.Stream()
        (t_eager, h_eager), (t_other, h_other), (t_rep, h_rep) = fresh(), fresh(), fresh()
        with torch.cuda.stream(stream):
            enqueue_chain(t_eager, h_eager, stream)
            torch.cuda.synchronize()
            want_t, want_h = t_eager.cpu().numpy().copy(), h_eager.cpu().numpy().copy()
            assert want_t[0] == root and (want_t[1:] >= 0).all()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=stream):
                enqueue_chain(t_rep, h_rep, stream)
            torch.cuda.synchronize()
            for _ in range(4):
                t_rep.fill_(-1)
                h_rep.zero_()
                enqueue_chain(t_other, h_other, stream)     # eager work between the replays
                torch.cuda.synchronize()
                graph.replay()
                torch.cuda.synchronize()
                assert np.array_equal(t_rep.cpu().numpy(), want_t)
                assert np.array_equal(h_rep.cpu().numpy(), want_h)
                assert np.array_equal(t_other.cpu().numpy(), want_t)
    finally:
        pair.close()
