"""Seeded model-shaped arrays: weights, embeddings, contexts, KV contents.

All floating-point arrays are produced directly as bf16 bit patterns
(numpy uint16).  A value is drawn by picking one of 65536 equiprobable
quantiles of the requested normal distribution with a 16-bit uniform integer
from a counter-seeded SFC64 stream, so generation is a table lookup and is
reproducible block by block whatever the number of worker threads.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass
from functools import lru_cache

import numpy as np
from scipy.special import ndtri


@dataclass(frozen=True)
class ModelDims:
    n_layers: int
    hidden: int
    n_heads: int
    head_dim: int
    ffn: int
    vocab: int
    rms_eps: float = 1e-6
    rope_base: float = 10000.0

    def layer_weight_elems(self) -> int:
        """Matrix + gain elements of one decoder layer."""
        h, f = self.hidden, self.ffn
        return 4 * h * h + 3 * h * f + 2 * h


# Shapes named by the benchmark configurations (LLaMA-family layer shapes).
TINY = ModelDims(2, 256, 4, 64, 688, 1024)
V7B = ModelDims(32, 4096, 32, 128, 11008, 32000)
V13B = ModelDims(40, 5120, 40, 128, 13824, 32000)

# Stable small integers that name each array in the seed key.
MATRIX_IDS = {"wq": 1, "wk": 2, "wv": 3, "wo": 4, "w_gate": 5, "w_up": 6,
              "w_down": 7, "g_attn": 8, "g_ffn": 9, "g_final": 10,
              "w_lm": 11, "embed": 12, "kv_k": 13, "kv_v": 14,
              "ctx_tokens": 15, "hidden": 16, "tree": 17, "tree_tokens": 18}

_BLOCK = 1 << 24  # values per independently seeded block


def bf16_bits_from_f32(x: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 (round-to-nearest-even), return the 16 bits."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def f32_from_bf16_bits(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns to float32 exactly."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32)
            << np.uint32(16)).view(np.float32)


@lru_cache(maxsize=16)
def _quantile_table(mean: float, std: float) -> np.ndarray:
    q = ndtri((np.arange(65536, dtype=np.float64) + 0.5) / 65536.0)
    return bf16_bits_from_f32((mean + std * q).astype(np.float32))


def _n_threads() -> int:
    env = os.environ.get("OMP_NUM_THREADS")
    n = int(env) if env and env.isdigit() else (os.cpu_count() or 1)
    return max(1, min(n, 16))


def normal_bf16(key, shape, std: float, mean: float = 0.0) -> np.ndarray:
    """bf16 bits of i.i.d. N(mean, std^2) samples, fully determined by `key`.

    `key` is a tuple of non-negative ints (seed, layer, array id, ...).
    """
    shape = tuple(int(s) for s in np.atleast_1d(shape))
    n = int(np.prod(shape))
    table = _quantile_table(float(mean), float(std))
    out = np.empty(n, dtype=np.uint16)
    key = tuple(int(k) for k in key)

    def fill(blk: int) -> None:
        lo = blk * _BLOCK
        hi = min(n, lo + _BLOCK)
        bg = np.random.SFC64(np.random.SeedSequence(key + (blk,)))
        raw = bg.random_raw((hi - lo + 3) // 4).view(np.uint16)[: hi - lo]
        np.take(table, raw, out=out[lo:hi])

    n_blocks = (n + _BLOCK - 1) // _BLOCK
    if n_blocks <= 1:
        for b in range(n_blocks):
            fill(b)
    else:
        with ThreadPoolExecutor(_n_threads()) as ex:
            list(ex.map(fill, range(n_blocks)))
    return out.reshape(shape)


def layer_weights(dims: ModelDims, seed: int, layer: int) -> dict:
    """One decoder layer: matrices N(0, 0.02) as [out][in]; gains 1 + N(0, 0.02)."""
    h, f = dims.hidden, dims.ffn
    assert dims.n_heads * dims.head_dim == h
    shapes = {"wq": (h, h), "wk": (h, h), "wv": (h, h), "wo": (h, h),
              "w_gate": (f, h), "w_up": (f, h), "w_down": (h, f)}
    w = {name: normal_bf16((seed, layer, MATRIX_IDS[name]), shp, 0.02)
         for name, shp in shapes.items()}
    for name in ("g_attn", "g_ffn"):
        w[name] = normal_bf16((seed, layer, MATRIX_IDS[name]), (h,), 0.02, 1.0)
    return w


def adapter_weights(dims: ModelDims, seed: int, which: int) -> dict:
    """An attention-only adapter block (draft adapter which=0, shallow-verifier adapter which=1):
    the four attention matrices, the gain of the normalisation in front of the attention
    (g_attn) and the gain of the normalisation in front of the shared LM head (g_out).  Drawn
    like a decoder layer's, under layer ids no model reaches."""
    h = dims.hidden
    layer = 100000 + which
    w = {name: normal_bf16((seed, layer, MATRIX_IDS[name]), (h, h), 0.02) for name in ("wq", "wk", "wv", "wo")}
    w["g_attn"] = normal_bf16((seed, layer, MATRIX_IDS["g_attn"]), (h,), 0.02, 1.0)
    w["g_out"] = normal_bf16((seed, layer, MATRIX_IDS["g_final"]), (h,), 0.02, 1.0)
    return w


def final_weights(dims: ModelDims, seed: int) -> dict:
    """Final norm gain and the (untied) LM head [vocab][hidden]."""
    return {
        "g_final": normal_bf16((seed, 0, MATRIX_IDS["g_final"]), (dims.hidden,), 0.02, 1.0),
        "w_lm": normal_bf16((seed, 0, MATRIX_IDS["w_lm"]), (dims.vocab, dims.hidden), 0.02),
    }


def embedding(dims: ModelDims, seed: int) -> np.ndarray:
    """Token embedding table [vocab][hidden], N(0, 0.02)."""
    return normal_bf16((seed, 0, MATRIX_IDS["embed"]), (dims.vocab, dims.hidden), 0.02)


def random_kv_context(dims: ModelDims, seed: int, layer: int, ctx_len: int):
    """Synthetic committed KV rows of one layer: K and V, each [ctx_len][hidden]
    (head h occupies columns h*head_dim..), N(0, 1) as bf16 bits.  Stands in for
    a prefilled context when only the verify step itself is under test."""
    k = normal_bf16((seed, layer, MATRIX_IDS["kv_k"]), (ctx_len, dims.hidden), 1.0)
    v = normal_bf16((seed, layer, MATRIX_IDS["kv_v"]), (ctx_len, dims.hidden), 1.0)
    return k, v


def context_tokens(dims: ModelDims, seed: int, n: int) -> np.ndarray:
    """n context token ids, uniform in [0, vocab)."""
    rng = np.random.Generator(np.random.SFC64(
        np.random.SeedSequence((seed, 0, MATRIX_IDS["ctx_tokens"]))))
    return rng.integers(0, dims.vocab, size=n, dtype=np.int32)


def random_hidden(dims: ModelDims, seed: int, n: int, std: float = 1.0) -> np.ndarray:
    """n hidden-state rows [n][hidden] as float32 (exactly bf16-representable)."""
    bits = normal_bf16((seed, 0, MATRIX_IDS["hidden"]), (n, dims.hidden), std)
    return f32_from_bf16_bits(bits)
