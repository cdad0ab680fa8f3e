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
