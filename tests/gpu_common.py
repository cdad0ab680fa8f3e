"""Shared set-up for the GPU parity tests: the same seeded inputs are handed to
the CPU oracle (numpy) and to the HIP library (torch device tensors)."""
from __future__ import annotations

import numpy as np
import torch

import paper_2605_11186_amd as cats
import synth
from oracle.cats_oracle import Oracle

REL_TOL = 2e-2      # max |gpu - ref| / max |ref| per tensor (bf16 activations, fp32 accumulate)
MARGIN = 1e-2       # integer decisions are compared where the oracle's top-2 gap exceeds this


def rel_err(gpu, ref) -> float:
    ref = np.asarray(ref, dtype=np.float64)
    gpu = np.asarray(gpu, dtype=np.float64)
    assert gpu.shape == ref.shape, (gpu.shape, ref.shape)
    assert np.isfinite(gpu).all()
    return float(np.abs(gpu - ref).max() / max(np.abs(ref).max(), 1e-30))


def rel_err_elementwise(gpu, ref, floor: float = 1e-3) -> dict:
    """Element-wise relative error |gpu - ref| / |ref| over the entries with
    |ref| > floor * max |ref| (smaller entries have no meaningful relative error in bf16
    arithmetic): its maximum, 99.9th percentile and median.  Reported beside rel_err, which is the
    figure the 2e-2 tolerance applies to; not asserted."""
    ref = np.asarray(ref, dtype=np.float64).ravel()
    gpu = np.asarray(gpu, dtype=np.float64).ravel()
    keep = np.abs(ref) > floor * np.abs(ref).max()
    e = np.abs(gpu[keep] - ref[keep]) / np.abs(ref[keep])
    if e.size == 0:
        return {"max": 0.0, "p999": 0.0, "median": 0.0, "entries": 0}
    return {"max": float(e.max()), "p999": float(np.quantile(e, 0.999)), "median": float(np.median(e)),
            "entries": int(e.size)}


def fmt_elementwise(d: dict) -> str:
    return f"max {d['max']:.2e} / p99.9 {d['p999']:.2e} / median {d['median']:.2e} over {d['entries']} entries"


def to_dev_bf16(bits: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


def bf16_to_f32_np(t: torch.Tensor) -> np.ndarray:
    return t.float().cpu().numpy()


class Pair:
    """One model on both sides."""

    def __init__(self, dims, seed, max_ctx, max_tree, precision="f64", n_layers=None, packed=False):
        self.dims = dims
        self.max_ctx = max_ctx
        L = dims.n_layers if n_layers is None else n_layers
        self.L = L
        self.layers = [synth.layer_weights(dims, seed, l) for l in range(L)]
        self.final = synth.final_weights(dims, seed)
        self.embed = synth.embedding(dims, seed)
        self.oracle = Oracle(dims, self.layers + [None] * (dims.n_layers - L), self.final, self.embed,
                             precision=precision)
        self.packed = packed
        self.d_layers = []
        for w in self.layers:   # packed layout: re-tile on the device, drop the row-major copy
            dw = {k: to_dev_bf16(v) for k, v in w.items()}
            self.d_layers.append(cats.pack_layer(dw) if packed else dw)
        self.d_final = {k: to_dev_bf16(v) for k, v in self.final.items()}
        if packed:
            self.d_final["w_lm"] = cats.cats_pack_matrix(self.d_final["w_lm"])
        self.d_embed = to_dev_bf16(self.embed)
        self.layers_arr = cats.layer_array(self.d_layers)
        desc = cats.ModelDesc(dims.n_layers, dims.hidden, dims.n_heads, dims.head_dim, dims.ffn,
                              dims.vocab, max_ctx, max_tree, dims.rms_eps, dims.rope_base, int(packed))
        self.ctx = cats.cats_create(desc)
        self.res_dev = cats.accept_result_tensor()

    def close(self):
        if self.ctx is not None:
            torch.cuda.synchronize()
            cats.cats_destroy(self.ctx)
            self.ctx = None

    # caches -----------------------------------------------------------------
    def oracle_cache_from_prefill(self, ctx_tokens):
        kc, vc = self.oracle.new_cache(self.max_ctx)
        if len(ctx_tokens):
            self.oracle.causal_decode(kc, vc, 0, tokens=ctx_tokens, layer_end=self.L)
        return kc, vc

    def oracle_cache_random(self, seed, ctx_len):
        kc, vc = self.oracle.new_cache(self.max_ctx)
        for l in range(self.L):
            k, v = synth.random_kv_context(self.dims, seed, l, ctx_len)
            kc[l, :ctx_len] = synth.f32_from_bf16_bits(k)
            vc[l, :ctx_len] = synth.f32_from_bf16_bits(v)
        return kc, vc

    def device_cache_from_oracle(self, kc, vc, rows):
        """Device caches holding the first `rows` oracle rows (rounded to bf16); the rest is
        filled with NaN so that any read of a row that must stay invisible shows up."""
        ks, vs = [], []
        for l in range(self.L):
            kr = torch.from_numpy(kc[l, :rows].astype(np.float32)).cuda().to(torch.bfloat16)
            vr = torch.from_numpy(vc[l, :rows].astype(np.float32)).cuda().to(torch.bfloat16)
            k, v = cats.kv_from_rows(kr, vr, self.dims.n_heads, self.dims.head_dim, self.max_ctx)
            k[:, rows:] = float("nan")
            v[:, :, rows:] = float("nan")
            ks.append(k)
            vs.append(v)
        return ks, vs

    def device_rows(self, ks, vs, l, rows):
        kr, vr = cats.kv_to_rows(ks[l], vs[l], rows)
        return bf16_to_f32_np(kr), bf16_to_f32_np(vr)
