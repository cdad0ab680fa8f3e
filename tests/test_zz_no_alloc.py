"""The entry point that allocates nothing (cats_tree_attention_noalloc) against the existing
cats_tree_attention: same inputs, outputs must be identical bit for bit (same kernels; only the
scratch differs: a fixed array in the library instead of the context's allocation).  Two calls in a
row, the second with a smaller input, so that whatever the first call left in the shared scratch
must not leak into the second."""
import ctypes
import gc

import numpy as np
import pytest
import torch

import paper_2605_11186_amd as cats
import synth

pytestmark = pytest.mark.gpu


def _case(dims, ctx, max_ctx, S, T, seed):
    parent, depth = synth.random_tree(T, 8, seed)
    tok = synth.distinct_sibling_tokens(parent, dims.vocab, seed)
    g = torch.Generator(device="cuda").manual_seed(seed)
    q = torch.randn(T, dims.hidden, device="cuda", generator=g).to(torch.bfloat16)
    k = torch.randn(dims.n_heads, max_ctx, dims.head_dim, device="cuda", generator=g).to(torch.bfloat16)
    v = torch.randn(dims.n_heads, dims.head_dim, max_ctx, device="cuda", generator=g).to(torch.bfloat16)
    k[:, S + T:] = float("nan")        # rows past the tree must stay invisible
    v[:, :, S + T:] = float("nan")
    kv = cats.KVLayer(k.data_ptr(), v.data_ptr())
    ref = torch.empty(T, dims.hidden, dtype=torch.bfloat16, device="cuda")
    cats.cats_set_tree(ctx, tok, parent, depth)
    cats.cats_tree_attention(ctx, q, kv, S, ref)
    out = torch.full((T, dims.hidden), float("nan"), dtype=torch.bfloat16, device="cuda")
    gc.collect()   # tensors of earlier tests that are still waiting for the collector must not be freed in between
    before = torch.cuda.memory_allocated()
    cats.cats_tree_attention_noalloc(q, kv, parent, dims.n_heads, dims.head_dim, max_ctx, S, out)
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    assert torch.isfinite(ref.float()).all()
    assert torch.equal(out.view(torch.int16), ref.view(torch.int16)), (S, T)


@pytest.mark.parametrize("dims_name,max_ctx,first,second", [
    ("TINY", 320, (200, 100), (37, 9)),
    ("V7B", 1152, (1024, 63), (300, 17)),
])
def test_noalloc_attention_equals_context_attention_twice(dims_name, max_ctx, first, second):
    dims = getattr(synth, dims_name)
    desc = cats.ModelDesc(dims.n_layers, dims.hidden, dims.n_heads, dims.head_dim, dims.ffn, dims.vocab,
                          max_ctx, 128, dims.rms_eps, dims.rope_base, 0)
    ctx = cats.cats_create(desc)
    try:
        _case(dims, ctx, max_ctx, first[0], first[1], 5)
        _case(dims, ctx, max_ctx, second[0], second[1], 6)     # smaller input, same shared scratch
    finally:
        torch.cuda.synchronize()
        cats.cats_destroy(ctx)


def test_noalloc_rejects_what_does_not_fit():
    q = torch.zeros(4, 8192, dtype=torch.bfloat16, device="cuda")
    k = torch.zeros(1, device="cuda")
    kv = cats.KVLayer(k.data_ptr(), k.data_ptr())
    lib = cats.library()
    par = np.array([-1, 0, 1, 2], dtype=np.int32)
    call = lambda n, nh, d, mc, S, p=par: lib.cats_tree_attention_noalloc(
        q.data_ptr(), ctypes.byref(kv), p.ctypes.data, n, nh, d, mc, S, q.data_ptr(), None)
    assert call(4, 32, 128, 1024, 1022) == cats.CATS_ECAPACITY          # ctx_len + n_nodes > max_ctx
    assert call(129, 32, 128, 4096, 0) == cats.CATS_ECAPACITY           # more nodes than CATS_MAX_TREE
    assert call(4, 512, 128, 1024, 0) == cats.CATS_ECAPACITY            # partial results exceed the fixed scratch
    assert call(4, 32, 96, 1024, 0) == cats.CATS_EINVAL                 # head_dim
    bad = np.array([-1, 0, 3, 1], dtype=np.int32)
    assert call(4, 32, 128, 1024, 0, bad) == cats.CATS_EINVAL           # parent after child
    assert "no-allocation" in cats.cats_strerror(cats.CATS_ECAPACITY)
