#!/usr/bin/env python3
"""Benchmark of the draft-tree verification step on one MI355X.

A "step" is one pass of the whole hot path: tree ingest, embedding rows, every
decoder layer (weights streamed once for all T tree nodes, tree-masked
attention), final norm + LM head + per-node argmax, greedy acceptance and KV
roll-back.  Inputs are seeded and synthetic and already resident in HBM when the
timed region starts.

Prints ONE JSON line: verify steps/s, the HBM roofline of the dominant
(weight-streaming GEMM) kernel measured with HIP events, and the CPU oracle
timed on this machine's host cores on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from pathlib import Path

ROOT = Path(__file__).resolve().parent
sys.path.insert(0, str(ROOT))

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E peak

WORKLOADS = {
    # BASELINE configs[1]: Vicuna-7B-shaped single verify step
    "7b_t63_s1024": dict(model="V7B", ctx=1024, tree="topk63", label="Vicuna-7B-shaped (32L, H4096, F11008, V32000) verify step, 63-node top-k tree (4/3/2/2/1/1 pruned), KV context 1024"),
    "7b_t64_s1024": dict(model="V7B", ctx=1024, tree="rand64", label="7B-shape, 64-node random tree (depth<=8), KV context 1024"),
    "13b_t64_s2048": dict(model="V13B", ctx=2048, tree="rand64d7", label="13B-shape (40L, H5120, F13824), 64-node tree (depth 7), KV context 2048"),
    # BASELINE configs[4]: offload regime, weights streamed from pinned host memory
    "7b_offload_t128_s1024": dict(model="V7B", ctx=1024, tree="rand128", offload=True, label="7B-shape, layer weights in pinned host memory streamed through two HBM staging buffers, 128-node random tree, KV context 1024"),
    # BASELINE configs[3]: 100 consecutive verify-accept-compact iterations
    "13b_t64_s2048_x100": dict(model="V13B", ctx=2048, tree="rand64d7", iterate=100, label="13B-shape (40L, H5120, F13824), 100 verify-accept-compact iterations, 64-node trees (depth 7), KV context from 2048"),
    # BASELINE configs[2]: tree-size and context sweep on the 7B shape
    "7b_sweep": dict(model="V7B", ctx=4096, tree="rand128", sweep=True, label="7B-shape sweep: tree sizes 16/32/64/128 (random parents, depth<=8) x KV context 512/2048/4096"),
    # the cascaded cycle's own tree shape (Alg. 1): a draft chain of 5 plus correction leaves, shallow layers
    # first (chain, then corrections alone), the remaining layers on the whole tree from hidden states
    "7b_cascade_g5": dict(model="V7B", ctx=1024, tree="cascade", cascade=dict(gamma=5, l_sv=8, corr=(1, 3)),
                          label="7B-shape cascaded cycle: draft chain of 5 + 2 correction leaves (8 nodes); layers 0..7 on the chain, then on the corrections alone, layers 8..31 + LM head on the tree; KV context 1024"),
    # stage 1 of the cascaded cycle: token-at-a-time drafting through the first layers and an attention-only
    # adapter with the shared LM head (T = 1: the matrix-vector corner of the weight-streaming product)
    "7b_draft_loop_g5": dict(model="V7B", ctx=1024, tree="cascade", draft=dict(gamma=5, l_dm=2),
                             label="7B-shape draft loop: 5 tokens one at a time through layers 0..1, an attention-only adapter and the shared LM head; KV context 1024"),
    # adapter-training side kernel (Eq. 2): not a verify step, its own metric and roofline
    "reduced_kl_p4096_v32000_k10": dict(model="V7B", ctx=0, tree="binary15", loss=dict(P=4096, V=32000, K=10),
                                        label="Reduced KL loss + gradient, 4096 positions x vocab 32000, top-10, LM-like seeded logits"),
    "tiny": dict(model="TINY", ctx=128, tree="binary15", label="tiny oracle-check model, 15-node binary tree, KV context 128"),
}


def make_tree(kind, synth):
    if kind == "topk63":
        p, d, _ = synth.product_tree_pruned()
        return p, d
    if kind == "binary15":
        return synth.complete_binary_tree(3)
    if kind == "rand64":
        return synth.random_tree(64, 8, 1)
    if kind == "rand64d7":
        return synth.random_tree(64, 7, 1)
    if kind.startswith("rand"):
        return synth.random_tree(int(kind[4:]), 8, 1)
    raise ValueError(kind)


def algorithmic_bytes(dims, T, S, n_layers):
    """Bytes the method must move per step: every weight once (2 B each), K and V of
    context + tree once per layer.  Small activations are ignored (< 1 %)."""
    w_layers = n_layers * dims.layer_weight_elems() * 2
    w_lm = dims.vocab * dims.hidden * 2
    kv = n_layers * 2 * (S + T) * dims.hidden * 2
    return w_layers + w_lm, kv


def run_iterations(args, wl, dims, cats, synth, torch, np, ctx, layers_arr, kv_arr, d_embed, d_final, res_dev,
                   stream, S0, n_iter, seed):
    """Consecutive verify-accept-compact iterations on a seeded token stream: a reference greedy
    stream is first produced by the same library with root-only trees (plain decoding); every
    iteration then verifies a fresh tree whose first child at each level carries the true next
    token with probability 0.8, and the committed stream must reproduce the reference."""
    L = dims.n_layers
    rng = np.random.default_rng(seed)
    host = cats.AcceptResult()
    one = (np.array([-1], np.int32), np.array([0], np.int32))

    def verify(tok, parent, depth, S):
        cats.cats_set_tree(ctx, tok, parent, depth, stream)
        cats.cats_verify_tree(ctx, layers_arr, 0, L, d_embed, None, d_final["g_final"], d_final["w_lm"],
                              kv_arr, S, res_dev, out_host=host, stream=stream)
        return host.as_dict()

    n_ref = n_iter * 8 + 16
    ref, tok, S = [], int(rng.integers(dims.vocab)), S0
    first = tok
    t0 = time.perf_counter()
    for _ in range(n_ref):
        r = verify(np.array([tok], np.int32), one[0], one[1], S)
        tok = r["bonus_token"]
        ref.append(tok)
        S += 1
    t_ref = time.perf_counter() - t0
    # the K/V rows written above stay valid for the speculative run: it starts from S0 again
    committed, S, root = [], S0, first
    accepted = []
    t0 = time.perf_counter()
    for it in range(n_iter):
        parent, depth = synth.random_tree(64, 7, seed + it)
        T = len(parent)
        tok_arr = np.zeros(T, np.int32)
        tok_arr[0] = root
        first_child = {}
        for i in range(1, T):
            p = int(parent[i])
            want = ref[len(committed) + depth[i] - 1]
            sib = first_child.setdefault(p, set())
            t = want if (not sib and rng.random() < 0.8) else int(rng.integers(dims.vocab))
            while t in sib:
                t = int(rng.integers(dims.vocab))
            sib.add(t)
            tok_arr[i] = t
        r = verify(tok_arr, parent, depth, S)
        committed += r["tokens"][1:] + [r["bonus_token"]]
        accepted.append(r["n_accepted"])
        S, root = r["new_ctx_len"], r["bonus_token"]
    elapsed = time.perf_counter() - t0
    n = len(committed)
    mismatch = next((i for i in range(n) if committed[i] != ref[i]), None)
    return {"metric": "tree-verify steps/sec", "value": round(n_iter / elapsed, 3), "unit": "steps/s",
            "n_gpus": 1, "steps": n_iter, "warmup": 0, "ms_per_step": round(elapsed / n_iter * 1e3, 4),
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
            "data": "synthetic",
            "config": {"workload": wl["label"], "key": args.workload, "tree_nodes": 64, "ctx_len": S0,
                       "layers": L, "seed": seed},
            "iterations": {"mean_accepted": round(float(np.mean(accepted)), 3),
                           "tokens_committed": n, "tokens_per_s": round(n / elapsed, 1),
                           "plain_decode_tokens_per_s": round(n_ref / t_ref, 1),
                           "first_mismatch_vs_plain_greedy": mismatch,
                           "note": "each step ends with a host read-back of the accept result"}}


def bench_loss(args, wl, cats, synth, torch, np):
    """Reduced KL loss (forward + gradient) over P positions: one launch of the per-position kernel
    plus the mean; timed with HIP events on the launch stream."""
    P, V, K = (wl["loss"][k] for k in ("P", "V", "K"))
    rows = 256   # distinct seeded rows, tiled to P positions (generation time, not a property of the kernel)
    a = torch.from_numpy(synth.lm_like_logits(args.seed, rows, V, tag=0)).cuda().repeat(P // rows, 1).contiguous()
    z = torch.from_numpy(synth.lm_like_logits(args.seed, rows, V, tag=1)).cuda().repeat(P // rows, 1).contiguous()
    loss = torch.zeros(1, device="cuda")
    per_pos = torch.zeros(P, device="cuda")
    topk = torch.zeros(P, K, dtype=torch.int32, device="cuda")
    grad = torch.empty(P, V, device="cuda")
    stream = torch.cuda.current_stream()

    def step():
        cats.cats_reduced_kl_loss(a, z, K, loss, per_pos, topk_idx_out=topk, grad_out=grad, stream=stream)

    for _ in range(args.warmup):
        step()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ev[0].record(stream)
    for _ in range(args.steps):
        step()
    ev[1].record(stream)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t1) / args.steps * 1e3
    ms_ev = ev[0].elapsed_time(ev[1]) / args.steps
    alg = 3 * P * V * 4   # both logit rows read once, the gradient row written once
    out = {"metric": "reduced-KL loss positions/sec", "value": round(P / (ms * 1e-3), 1), "unit": "positions/s",
           "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 4),
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
           "config": {"workload": wl["label"], "key": args.workload, "positions": P, "vocab": V, "top_k": K,
                      "seed": args.seed, "loss": round(loss.item(), 6)},
           "roofline": {"bound": "hbm", "kernel": "cats_reduced_kl_positions", "achieved": round(alg / (ms_ev * 1e-3) / 1e9, 1),
                        "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(alg / (ms_ev * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                        "traffic": None, "bytes_per_launch": alg, "avg_launch_us": round(ms_ev * 1e3, 2),
                        "note": "events bracket the position kernel and the one-workgroup mean kernel together"}}
    if not args.no_cpu_baseline:
        from oracle import reduced_kl as rk
        n = 32
        a_h, z_h = a[:n].cpu().numpy(), z[:n].cpu().numpy()
        t1 = time.perf_counter()
        rk.reduced_kl_grad(a_h, z_h, K)
        dt = time.perf_counter() - t1
        out["cpu_baseline"] = {"value": round(n / dt, 2), "unit": "positions/s", "cores": 1, "kind": "oracle",
                               "sample": f"float64 numpy oracle (loss + gradient) on the first {n} positions ({dt:.2f} s)"}
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="7b_t63_s1024", choices=sorted(WORKLOADS))
    ap.add_argument("--tree-nodes", type=int, default=0, help="override: random tree with this many nodes")
    ap.add_argument("--ctx", type=int, default=0, help="override the KV context length")
    ap.add_argument("--seed", type=int, default=11186)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-layers", type=int, default=8)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one 1 GiB device-to-device copy (a known-size kernel that scales "
                         "the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
                 "run it with --gpus 1")

    import numpy as np
    import torch
    import paper_2605_11186_amd as cats
    import synth

    wl = dict(WORKLOADS[args.workload])
    if wl.get("loss"):
        return bench_loss(args, wl, cats, synth, torch, np)
    dims = getattr(synth, wl["model"])
    S = args.ctx or wl["ctx"]
    cascade = wl.get("cascade")
    draft = wl.get("draft")
    if draft:
        casc_tok, parent, depth, _ = cats.cats_build_tree(1, list(range(2, 2 + draft["gamma"])))
    elif cascade:
        rng = np.random.default_rng(args.seed)
        drafts = rng.integers(0, dims.vocab, cascade["gamma"]).astype(np.int32)
        corrections = np.full(cascade["gamma"], -1, dtype=np.int32)
        for i in cascade["corr"]:
            corrections[i] = (drafts[i] + 1 + rng.integers(0, dims.vocab - 1)) % dims.vocab
        root = int(rng.integers(0, dims.vocab))
        casc_tok, parent, depth, _ = cats.cats_build_tree(root, drafts, corrections)
        casc_chain = cats.cats_build_tree(root, drafts)[:3]
    elif args.tree_nodes:
        parent, depth = synth.random_tree(args.tree_nodes, 8, 1)
        wl["label"] += f" [override: {args.tree_nodes}-node random tree]"
    else:
        parent, depth = make_tree(wl["tree"], synth)
    if args.ctx:
        wl["label"] += f" [override: KV context {S}]"
    T = len(parent)
    L = dims.n_layers
    seed = args.seed
    iterate = wl.get("iterate", 0)
    offload = wl.get("offload", False)
    max_ctx = (S + T + (iterate * 9 if iterate else 0) + 63) // 64 * 64
    tok = casc_tok if (cascade or draft) else synth.distinct_sibling_tokens(parent, dims.vocab, seed)
    golden = None
    gfile = ROOT / "tests" / "golden" / "config2_tree_7b.txt"
    if args.workload == "7b_t63_s1024" and seed == 11186 and not args.tree_nodes and not args.ctx and gfile.exists():
        # draft ids chosen by the CPU oracle from perturbed true logits, and the accept result it expects
        golden = {k.strip(): v.split() for k, v in
                  (l.split(":", 1) for l in gfile.read_text().splitlines() if l and not l.startswith("#"))}
        tok = np.array(golden["tokens"], dtype=np.int32)

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    to_dev = lambda bits: torch.from_numpy(bits.view(np.int16)).to(dev).view(torch.bfloat16)

    t0 = time.time()
    host_layers = []   # kept only for the CPU-baseline sample
    d_layers = []
    n_keep = 0 if args.no_cpu_baseline else min(args.cpu_sample_layers, L)
    pinned_layers = []  # offload regime: the weights stay in pinned host memory
    n_model_layers = draft["l_dm"] if draft else L
    for l in range(n_model_layers):
        w = synth.layer_weights(dims, seed, l)
        dw = cats.pack_layer({k: to_dev(v) for k, v in w.items()})   # one-time re-tiling, row-major copy dropped
        if offload:
            pinned_layers.append({k: v.view(torch.int16).cpu().pin_memory() for k, v in dw.items()})
        else:
            d_layers.append(dw)
        if l < n_keep:
            host_layers.append(w)
    final = synth.final_weights(dims, seed)
    embed = synth.embedding(dims, seed)
    d_final = {k: to_dev(v) for k, v in final.items()}
    d_final["w_lm"] = cats.cats_pack_matrix(d_final["w_lm"])
    d_embed = to_dev(embed)
    ks, vs, host_kv = [], [], []
    for l in range(n_model_layers + (1 if draft else 0)):   # the draft adapter has a cache of its own
        k_rows, v_rows = synth.random_kv_context(dims, seed, l, S)
        k, v = cats.kv_from_rows(to_dev(k_rows), to_dev(v_rows), dims.n_heads, dims.head_dim, max_ctx)
        ks.append(k)
        vs.append(v)
        if l < n_keep:
            host_kv.append((k_rows, v_rows))
    gen_s = time.time() - t0

    desc = cats.ModelDesc(L, dims.hidden, dims.n_heads, dims.head_dim, dims.ffn, dims.vocab, max_ctx,
                          max(T, 1), dims.rms_eps, dims.rope_base, 1)
    ctx = cats.cats_create(desc)
    layers_arr = cats.layer_array(pinned_layers if offload else d_layers)
    kv_arr = cats.kv_array(ks, vs)
    if offload:
        layer_bytes = cats.cats_layer_weight_bytes(desc)
        staging = [torch.empty(layer_bytes, dtype=torch.uint8, device=dev) for _ in range(2)]
    res_dev = cats.accept_result_tensor(dev)
    stream = torch.cuda.current_stream()

    def step():
        cats.cats_set_tree(ctx, tok, parent, depth, stream)
        if offload:
            cats.cats_verify_tree_streamed(ctx, layers_arr, 0, L, staging, d_embed, None, d_final["g_final"],
                                           d_final["w_lm"], kv_arr, S, res_dev, stream=stream)
        else:
            cats.cats_verify_tree(ctx, layers_arr, 0, L, d_embed, None, d_final["g_final"], d_final["w_lm"],
                                  kv_arr, S, res_dev, stream=stream)

    if wl.get("sweep"):
        points = []
        for Ts in (16, 32, 64, 128):
            p_s, d_s = synth.random_tree(Ts, 8, 1)
            tok_s = synth.distinct_sibling_tokens(p_s, dims.vocab, seed)
            for Ss in (512, 2048, 4096):
                def step_s():
                    cats.cats_set_tree(ctx, tok_s, p_s, d_s, stream)
                    cats.cats_verify_tree(ctx, layers_arr, 0, L, d_embed, None, d_final["g_final"],
                                          d_final["w_lm"], kv_arr, Ss, res_dev, stream=stream)
                for _ in range(args.warmup):
                    step_s()
                torch.cuda.synchronize()
                t1 = time.perf_counter()
                for _ in range(args.steps):
                    step_s()
                torch.cuda.synchronize()
                ms = (time.perf_counter() - t1) / args.steps * 1e3
                cats.cats_profile_gemm(ctx, True)
                g_ms, g_n = 0.0, 0
                for _ in range(max(1, args.steps // 5)):
                    step_s()
                    a_ms, a_n = cats.cats_profile_gemm_read(ctx)
                    g_ms += a_ms
                    g_n += a_n
                cats.cats_profile_gemm(ctx, False)
                wb, kvb = algorithmic_bytes(dims, Ts, Ss, L)
                gemm_tbs = wb * (g_n / 129) / (g_ms * 1e-3) / 1e12
                # bf16 MFMA work of the GEMMs: 2 flop per weight per node, twice for the hi+lo activation parts
                mfma_util = (2 * 2 * Ts * (wb / 2) * (g_n / 129)) / (g_ms * 1e-3) / 2.5e15
                points.append({"T": Ts, "S": Ss, "ms_per_step": round(ms, 3), "steps_per_s": round(1e3 / ms, 1),
                               "step_gbs": round((wb + kvb) / (ms * 1e-3) / 1e9, 1),
                               "gemm_weight_tbs": round(gemm_tbs, 3), "gemm_frac_of_hbm_peak": round(gemm_tbs / 8, 4),
                               "gemm_mfma_frac_of_bf16_peak": round(mfma_util, 4)})
        cats.cats_destroy(ctx)
        best = max(points, key=lambda q: q["steps_per_s"])
        print(json.dumps({"metric": "tree-verify steps/sec", "value": best["steps_per_s"], "unit": "steps/s",
                          "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
                          "ms_per_step": best["ms_per_step"], "higher_is_better": True, "scaling": "weak",
                          "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
                          "config": {"workload": wl["label"], "key": args.workload, "layers": L, "seed": seed,
                                     "value_is": "fastest point of the sweep"},
                          "sweep": points}))
        return

    if draft:
        g, l_dm = draft["gamma"], draft["l_dm"]
        ad = synth.adapter_weights(dims, seed, 0)
        d_ad = cats.pack_layer({k: to_dev(v) for k, v in ad.items() if k != "g_out"})
        g_out = to_dev(ad["g_out"])
        ad_arr = cats.layer_array([d_ad])
        kv_model = cats.kv_array(ks[:l_dm], vs[:l_dm])
        kv_ad = cats.kv_array(ks[l_dm:], vs[l_dm:])

        toks_dev = torch.empty(g + 1, dtype=torch.int32, device=dev)
        toks_host = torch.empty(g + 1, dtype=torch.int32).pin_memory()

        def draft_cycle():
            # the chain grows on the device: the argmax of step k is the embedding row of step k + 1;
            # one read-back per gamma tokens
            cats.cats_draft_chain(ctx, layers_arr, 0, l_dm, ad_arr, g_out, d_final["w_lm"], d_embed, kv_model,
                                  kv_ad, S, 1, g, toks_dev, stream=stream)
            toks_host.copy_(toks_dev, non_blocking=True)
            torch.cuda.synchronize()
            return toks_host.tolist()

        for _ in range(args.warmup):
            draft_cycle()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(args.steps):
            toks = draft_cycle()
        torch.cuda.synchronize()
        ms_cycle = (time.perf_counter() - t1) / args.steps * 1e3
        w_tok = (l_dm * dims.layer_weight_elems() + 4 * dims.hidden * dims.hidden + dims.vocab * dims.hidden) * 2
        cats.cats_destroy(ctx)
        print(json.dumps({"metric": "draft tokens/sec", "value": round(g / (ms_cycle * 1e-3), 1), "unit": "tokens/s",
                          "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
                          "ms_per_step": round(ms_cycle, 4), "higher_is_better": True, "scaling": "weak",
                          "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
                          "config": {"workload": wl["label"], "key": args.workload, "gamma": g, "l_dm": l_dm,
                                     "ctx_len": S, "seed": seed, "drafted": toks[1:]},
                          "draft": {"us_per_token": round(ms_cycle * 1e3 / g, 1), "weight_bytes_per_token": w_tok,
                                    "weight_gbs": round(w_tok * g / (ms_cycle * 1e-3) / 1e9, 1),
                                    "note": "cats_draft_chain: tokens stay on the device, one host read-back per gamma tokens"}}))
        return

    if cascade:
        g, l_sv = cascade["gamma"], cascade["l_sv"]
        h_sv = torch.empty(T, dims.hidden, dtype=torch.float32, device=dev)
        amax = torch.empty(T, dtype=torch.int32, device=dev)

        def cycle():
            cats.cats_set_tree(ctx, *casc_chain, stream)
            cats.cats_verify_nodes(ctx, layers_arr, 0, l_sv, d_embed, None, kv_arr, S, 0, h_sv[: g + 1], stream)
            cats.cats_set_tree(ctx, tok, parent, depth, stream)
            cats.cats_verify_nodes(ctx, layers_arr, 0, l_sv, d_embed, None, kv_arr, S, g + 1, h_sv[g + 1:], stream)
            cats.cats_verify_tree(ctx, layers_arr, l_sv, L, None, h_sv, d_final["g_final"], d_final["w_lm"],
                                  kv_arr, S, res_dev, argmax_out=amax, stream=stream)
            cats.cats_accept_and_compact(ctx, amax, kv_arr, 0, l_sv, S, res_dev, stream=stream)

        def timed(fn):
            for _ in range(args.warmup):
                fn()
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            for _ in range(args.steps):
                fn()
            torch.cuda.synchronize()
            return (time.perf_counter() - t1) / args.steps * 1e3

        ms_cycle = timed(cycle)
        acc_staged = cats.accept_result_from_tensor(res_dev)
        ms_one_shot = timed(step)
        acc_one = cats.accept_result_from_tensor(res_dev)
        w_layer = dims.layer_weight_elems() * 2
        w_bytes = (L + l_sv) * w_layer + dims.vocab * dims.hidden * 2   # shallow layers are streamed twice
        cats.cats_destroy(ctx)
        print(json.dumps({"metric": "tree-verify steps/sec", "value": round(1e3 / ms_cycle, 3), "unit": "steps/s",
                          "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
                          "ms_per_step": round(ms_cycle, 4), "higher_is_better": True, "scaling": "weak",
                          "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
                          "config": {"workload": wl["label"], "key": args.workload, "tree_nodes": T, "ctx_len": S,
                                     "layers": L, "l_sv": l_sv, "seed": seed},
                          "cascade": {"weight_bytes_streamed": w_bytes,
                                      "weight_gbs": round(w_bytes / (ms_cycle * 1e-3) / 1e9, 1),
                                      "one_shot_same_tree_ms": round(ms_one_shot, 4),
                                      "staged_equals_one_shot_accept": acc_staged == acc_one}}))
        return

    if iterate:
        out = run_iterations(args, wl, dims, cats, synth, torch, np, ctx, layers_arr, kv_arr, d_embed, d_final,
                             res_dev, stream, S, iterate, seed)
        cats.cats_destroy(ctx)
        print(json.dumps(out))
        return

    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    # K timed steps between two synchronisations; an event on the launch stream after every step
    # gives the per-step durations, whose median is the reported step time (the wall-clock mean
    # over the same region is kept beside it)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    marks[0].record(stream)
    for i in range(args.steps):
        step()
        marks[i + 1].record(stream)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start
    per_step = np.array([marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps)])
    ms_wall_mean = elapsed / args.steps * 1e3
    ms_per_step = float(np.median(per_step))
    accepted = cats.accept_result_from_tensor(res_dev)

    # Same K steps again with HIP events around every GEMM launch (on the launch stream): the
    # dominant kernel's average duration.  Kept out of the region above so that the event
    # records do not inflate `value`.
    cats.cats_profile_gemm(ctx, True)
    gemm_ms, gemm_launches = 0.0, 0
    for _ in range(args.steps):
        step()
        ms, n = cats.cats_profile_gemm_read(ctx)
        gemm_ms += ms
        gemm_launches += n
    cats.cats_profile_gemm(ctx, False)
    torch.cuda.synchronize()

    w_bytes, kv_bytes = algorithmic_bytes(dims, T, S, L)
    gemm_bytes_per_launch = w_bytes * args.steps / gemm_launches
    gemm_avg_s = gemm_ms * 1e-3 / gemm_launches
    gemm_gbs = gemm_bytes_per_launch / gemm_avg_s / 1e9
    step_gbs = (w_bytes + kv_bytes) / (ms_per_step * 1e-3) / 1e9

    # HBM traffic (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by a copy of known size) is not
    # measured in this run: it is read from the committed summary of this same workload
    traffic, step_traffic = None, None
    prof = ROOT / "profiles" / f"verify_step_{args.workload}.pmc.txt"
    if prof.exists() and not args.tree_nodes and not args.ctx:
        for line in prof.read_text().splitlines():
            if line.startswith("gemm_traffic_bytes_per_launch:"):
                traffic = int(line.split(":")[1])
            if line.startswith("step_traffic_bytes:"):
                step_traffic = int(line.split(":")[1])

    out = {
        "metric": "tree-verify steps/sec",
        "value": round(1e3 / ms_per_step, 3),
        "unit": "steps/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": wl["label"], "key": args.workload, "tree_nodes": T, "ctx_len": S,
                   "layers": L, "seed": seed, "accepted_per_step": accepted["n_accepted"],
                   "accept_matches_cpu_oracle": None if golden is None else bool(
                       accepted["n_accepted"] == int(golden["n_accepted"][0])
                       and accepted["path"] == [int(v) for v in golden["path"]]
                       and accepted["bonus_token"] == int(golden["bonus_token"][0]))},
        "timing": {"value_is": "1 / median of the per-step times (events on the launch stream between steps)",
                   "median_ms": round(ms_per_step, 4), "wall_mean_ms": round(ms_wall_mean, 4),
                   "min_ms": round(float(per_step.min()), 4), "max_ms": round(float(per_step.max()), 4)},
        "step_hbm": {"algorithmic_bytes": w_bytes + kv_bytes, "weight_bytes": w_bytes, "kv_bytes": kv_bytes,
                     "achieved_gbs": round(step_gbs, 1), "frac_of_peak": round(step_gbs / HBM_PEAK_GBS, 4),
                     "traffic": step_traffic,
                     "traffic_over_algorithmic": None if step_traffic is None else round(step_traffic / (w_bytes + kv_bytes), 3),
                     "traffic_source": None if step_traffic is None else f"profiles/{prof.name} (committed rocprofv3 --pmc summary, all kernels of one step)"},
        "roofline": {"bound": "hbm", "kernel": cats.cats_gemm_kernel_name(),
                     "achieved": round(gemm_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(gemm_gbs / HBM_PEAK_GBS, 4), "traffic": traffic,
                     "traffic_source": None if traffic is None else f"profiles/{prof.name} (committed rocprofv3 --pmc summary)",
                     "launches_per_step": gemm_launches // args.steps,
                     "avg_launch_us": round(gemm_avg_s * 1e6, 2),
                     "bytes_per_launch": int(gemm_bytes_per_launch)},
        "input_generation_s": round(gen_s, 1),
    }

    if offload:
        # copy alone (same pinned tensors, same staging buffers) and compute alone (two layers kept
        # resident, scaled) bound the overlap: hidden = how much of the shorter leg disappears
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for w in pinned_layers:
            off = 0
            buf = staging[0]
            for k in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down", "g_attn", "g_ffn"):
                n = w[k].numel() * 2
                buf[off:off + n].view(torch.int16).copy_(w[k].reshape(-1), non_blocking=True)
                off += n
        torch.cuda.synchronize()
        t_copy = time.perf_counter() - t1
        t_step = ms_per_step * 1e-3
        out["offload"] = {"link_gbs": round(w_bytes / t_step / 1e9, 2),
                          "copy_only_s": round(t_copy, 4), "step_s": round(t_step, 4),
                          "copy_link_gbs": round((w_bytes - dims.vocab * dims.hidden * 2) / t_copy / 1e9, 2),
                          "gemm_compute_s_per_step": round(gemm_ms * 1e-3 / args.steps, 5),
                          "exposed_beyond_copy_s": round(max(0.0, t_step - t_copy), 5)}
        out["roofline"]["note"] = "offload regime: the step is bound by the host link, not by HBM"
    if not args.no_cpu_baseline:
        from oracle.cats_oracle import Oracle
        orc = Oracle(dims, host_layers + [None] * (L - n_keep), final, embed, precision="f32")
        kc, vc = orc.new_cache(max_ctx)
        for l in range(n_keep):
            kc[l, :S] = synth.f32_from_bf16_bits(host_kv[l][0])
            vc[l, :S] = synth.f32_from_bf16_bits(host_kv[l][1])
        # the sampled layers and the LM head are run again and again until about ten seconds of
        # CPU work have been spent (at most 12 passes); the median pass is reported
        passes, spent = [], 0.0
        while len(passes) < 12 and (spent < 10.0 or len(passes) < 3):
            t1 = time.perf_counter()
            x = orc.tree_forward(kc, vc, S, parent, depth, tokens=tok, layer_end=n_keep)
            t_layers = time.perf_counter() - t1
            t1 = time.perf_counter()
            orc.lm_head(x)
            t_lm = time.perf_counter() - t1
            passes.append((t_layers, t_lm))
            spent += t_layers + t_lm
        t_layers = float(np.median([p[0] for p in passes]))
        t_lm = float(np.median([p[1] for p in passes]))
        est = t_layers * L / n_keep + t_lm
        out["cpu_baseline"] = {
            "value": round(1.0 / est, 5), "unit": "steps/s", "cores": orc.num_threads(), "kind": "oracle",
            "sample": f"float32 oracle, same tree and context: layers 0..{n_keep - 1} of {L} "
                      f"({t_layers:.2f} s, scaled by {L}/{n_keep}) plus the full LM head ({t_lm:.2f} s); "
                      f"median of {len(passes)} passes, {spent:.1f} s of CPU work in all",
            "est_s_per_step": round(est, 2)}

    cats.cats_destroy(ctx)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
