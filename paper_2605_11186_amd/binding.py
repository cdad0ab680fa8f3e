"""ctypes binding of libcats.so: the same entry points as include/cats.h.

Argument marshalling only.  Tensors are torch CUDA (ROCm) tensors used as device
memory; bf16 data travels as torch.bfloat16 (or int16/uint16 bit patterns).
Every function raises CatsError on a non-zero status.
"""
from __future__ import annotations

import ctypes as C
from pathlib import Path

import numpy as np

__all__ = ["CATS_MAX_TREE", "CATS_MAX_DEPTH", "CatsError", "ModelDesc", "LayerWeights", "KVLayer",
           "AcceptResult", "library", "library_path", "exported_symbols", "cats_create",
           "cats_destroy", "cats_set_tree", "cats_verify_layer", "cats_tree_attention", "cats_tree_attention_noalloc",
           "CATS_NOALLOC_SCRATCH_BYTES",
           "cats_accept_and_compact", "cats_verify_tree", "cats_verify_nodes", "cats_build_tree", "cats_draft_chain", "cats_reduced_kl_loss", "cats_set_acceptance",
           "cats_typical_stats", "cats_compact_along", "CATS_LOSS_MAX_K", "CATS_LOSS_MAX_VOCAB",
           "cats_lm_head_argmax",
           "cats_gemm_kernel_name", "cats_strerror", "cats_profile_gemm", "cats_profile_gemm_read",
           "cats_verify_tree_streamed", "cats_layer_weight_bytes", "cats_packed_matrix_bytes",
           "cats_pack_matrix", "pack_layer", "MATRIX_FIELDS", "layer_weights_struct", "kv_array",
           "layer_array", "kv_from_rows", "kv_to_rows", "accept_result_tensor",
           "accept_result_from_tensor", "CATS_OK", "CATS_EINVAL", "CATS_ECAPACITY", "CATS_ESTATE",
           "CATS_EHIP"]

CATS_MAX_TREE = 128
CATS_MAX_DEPTH = 16
CATS_LOSS_MAX_K = 64
CATS_LOSS_MAX_VOCAB = 36864
CATS_NOALLOC_SCRATCH_BYTES = 8 << 20
CATS_OK, CATS_EINVAL, CATS_ECAPACITY, CATS_ESTATE, CATS_EHIP = 0, -1, -2, -3, -4

_LIB_PATH = Path(__file__).resolve().parent / "libcats.so"
_lib = None


class CatsError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"cats status {status}: {text}")
        self.status = status


class ModelDesc(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("hidden", C.c_int32), ("n_heads", C.c_int32),
                ("head_dim", C.c_int32), ("ffn", C.c_int32), ("vocab", C.c_int32),
                ("max_ctx", C.c_int32), ("max_tree", C.c_int32),
                ("rms_eps", C.c_float), ("rope_base", C.c_float), ("packed_weights", C.c_int32)]


class LayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in
                ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down", "g_attn", "g_ffn")]


class KVLayer(C.Structure):
    _fields_ = [("k", C.c_void_p), ("v", C.c_void_p)]


class Tree(C.Structure):
    _fields_ = [("token", C.c_void_p), ("parent", C.c_void_p), ("depth", C.c_void_p),
                ("n", C.c_int32)]


class AcceptResult(C.Structure):
    _fields_ = [("n_accepted", C.c_int32), ("path", C.c_int32 * (CATS_MAX_DEPTH + 1)),
                ("tokens", C.c_int32 * (CATS_MAX_DEPTH + 1)), ("bonus_token", C.c_int32),
                ("new_ctx_len", C.c_int32)]

    def as_dict(self):
        n = self.n_accepted
        return {"n_accepted": n, "path": list(self.path[: n + 1]),
                "tokens": list(self.tokens[: n + 1]), "bonus_token": self.bonus_token,
                "new_ctx_len": self.new_ctx_len}


_SIGNATURES = {
    "cats_create": [C.c_void_p, C.c_void_p],
    "cats_destroy": [C.c_void_p],
    "cats_set_tree": [C.c_void_p, C.c_void_p, C.c_void_p],
    "cats_verify_layer": [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p],
    "cats_tree_attention": [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p],
    "cats_accept_and_compact": [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32,
                                C.c_void_p, C.c_void_p, C.c_void_p],
    "cats_verify_tree": [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                         C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p,
                         C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p],
    "cats_verify_tree_streamed": [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                  C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
                                  C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                  C.c_void_p, C.c_void_p],
    "cats_verify_nodes": [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                          C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p],
    "cats_build_tree": [C.c_int32, C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p,
                        C.c_void_p, C.c_void_p, C.c_void_p],
    "cats_reduced_kl_loss": [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32,
                             C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p],
    "cats_set_acceptance": [C.c_void_p, C.c_int32, C.c_float, C.c_float, C.c_float],
    "cats_typical_stats": [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p],
    "cats_compact_along": [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p],
    "cats_pack_matrix": [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p],
    "cats_profile_gemm": [C.c_void_p, C.c_int],
    "cats_profile_gemm_read": [C.c_void_p, C.c_void_p, C.c_void_p],
    "cats_lm_head_argmax": [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                            C.c_void_p, C.c_void_p, C.c_void_p],
    "cats_draft_chain": [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                         C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
                         C.c_void_p, C.c_void_p],
    "cats_tree_attention_noalloc": [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32,
                                    C.c_int32, C.c_int32, C.c_void_p, C.c_void_p],
}


def library_path() -> Path:
    return _LIB_PATH


def exported_symbols():
    """Names every build must export (those declared in include/cats.h)."""
    return sorted(list(_SIGNATURES) + ["cats_gemm_kernel_name", "cats_strerror",
                                       "cats_layer_weight_bytes", "cats_packed_matrix_bytes"])


def library():
    """Load libcats.so once.  There is no fallback: a missing library is an error."""
    global _lib
    if _lib is None:
        if not _LIB_PATH.exists():
            raise FileNotFoundError(
                f"{_LIB_PATH} is missing: build it with `python -m paper_2605_11186_amd.build` "
                "(there is no CPU fallback)")
        lib = C.CDLL(str(_LIB_PATH))
        for name, args in _SIGNATURES.items():
            fn = getattr(lib, name)
            fn.argtypes = args
            fn.restype = C.c_int
        lib.cats_strerror.argtypes = [C.c_int]
        lib.cats_strerror.restype = C.c_char_p
        lib.cats_packed_matrix_bytes.argtypes = [C.c_int32, C.c_int32]
        lib.cats_packed_matrix_bytes.restype = C.c_size_t
        lib.cats_layer_weight_bytes.argtypes = [C.c_void_p]
        lib.cats_layer_weight_bytes.restype = C.c_size_t
        lib.cats_gemm_kernel_name.argtypes = []
        lib.cats_gemm_kernel_name.restype = C.c_char_p
        _lib = lib
    return _lib


def _check(status: int):
    if status != 0:
        raise CatsError(status, library().cats_strerror(status).decode())


def _dp(t):
    """Device (or host) pointer of a tensor / ctypes object / None."""
    if t is None:
        return None
    if hasattr(t, "data_ptr"):
        return C.c_void_p(t.data_ptr())
    if isinstance(t, np.ndarray):
        return t.ctypes.data_as(C.c_void_p)
    if isinstance(t, int):
        return C.c_void_p(t)
    return C.cast(C.byref(t), C.c_void_p)


def _stream(stream):
    if stream is None:
        return None
    if hasattr(stream, "cuda_stream"):
        return C.c_void_p(stream.cuda_stream)
    return C.c_void_p(int(stream))


# ---------------------------------------------------------------- entry points
def cats_strerror(status: int) -> str:
    return library().cats_strerror(status).decode()


def cats_gemm_kernel_name() -> str:
    return library().cats_gemm_kernel_name().decode()


def cats_create(desc: ModelDesc):
    handle = C.c_void_p()
    _check(library().cats_create(C.byref(desc), C.byref(handle)))
    return handle


def cats_destroy(ctx):
    _check(library().cats_destroy(ctx))


def cats_set_tree(ctx, token, parent, depth, stream=None):
    token = np.ascontiguousarray(token, dtype=np.int32)
    parent = np.ascontiguousarray(parent, dtype=np.int32)
    depth = np.ascontiguousarray(depth, dtype=np.int32)
    if not (len(token) == len(parent) == len(depth)):
        raise CatsError(CATS_EINVAL, "token/parent/depth lengths differ")
    tree = Tree(token.ctypes.data, parent.ctypes.data, depth.ctypes.data, len(parent))
    _check(library().cats_set_tree(ctx, C.byref(tree), _stream(stream)))


def cats_verify_layer(ctx, weights: LayerWeights, hidden, kv: KVLayer, ctx_len: int, stream=None):
    _check(library().cats_verify_layer(ctx, C.byref(weights), _dp(hidden), C.byref(kv),
                                       int(ctx_len), _stream(stream)))


def cats_tree_attention(ctx, q, kv: KVLayer, ctx_len: int, out, stream=None):
    _check(library().cats_tree_attention(ctx, _dp(q), C.byref(kv), int(ctx_len), _dp(out),
                                         _stream(stream)))


def cats_tree_attention_noalloc(q, kv: KVLayer, parent, n_heads: int, head_dim: int, max_ctx: int,
                                ctx_len: int, out, stream=None):
    """cats_tree_attention without a context: nothing is allocated (fixed scratch in the library)."""
    parent = np.ascontiguousarray(parent, dtype=np.int32)
    _check(library().cats_tree_attention_noalloc(_dp(q), C.byref(kv), parent.ctypes.data, len(parent),
                                                 int(n_heads), int(head_dim), int(max_ctx), int(ctx_len),
                                                 _dp(out), _stream(stream)))


def cats_accept_and_compact(ctx, node_argmax, kv_arr, layer_begin: int, layer_end: int,
                            ctx_len: int, out_dev, out_host: AcceptResult | None = None,
                            stream=None):
    _check(library().cats_accept_and_compact(
        ctx, _dp(node_argmax), kv_arr, int(layer_begin), int(layer_end), int(ctx_len),
        _dp(out_dev), None if out_host is None else C.byref(out_host), _stream(stream)))


def cats_verify_tree(ctx, layers_arr, layer_begin: int, layer_end: int, embed, hidden_in, g_final,
                     w_lm, kv_arr, ctx_len: int, out_dev, hidden_out=None, logits_out=None,
                     argmax_out=None, margin_out=None, out_host: AcceptResult | None = None,
                     stream=None):
    _check(library().cats_verify_tree(
        ctx, layers_arr, int(layer_begin), int(layer_end), _dp(embed), _dp(hidden_in), _dp(g_final),
        _dp(w_lm), kv_arr, int(ctx_len), _dp(hidden_out), _dp(logits_out), _dp(argmax_out),
        _dp(margin_out), _dp(out_dev), None if out_host is None else C.byref(out_host),
        _stream(stream)))


def cats_verify_nodes(ctx, layers_arr, layer_begin: int, layer_end: int, embed, hidden_in, kv_arr,
                      ctx_len: int, node_begin: int, hidden_out, stream=None):
    _check(library().cats_verify_nodes(
        ctx, layers_arr, int(layer_begin), int(layer_end), _dp(embed), _dp(hidden_in), kv_arr,
        int(ctx_len), int(node_begin), _dp(hidden_out), _stream(stream)))


def cats_draft_chain(ctx, layers_arr, layer_begin: int, layer_end: int, adapter_arr, g_adapter_out, w_lm,
                     embed, kv_arr, kv_adapter_arr, ctx_len: int, root_token: int, gamma: int, tokens_out,
                     hidden_out=None, stream=None):
    """Stage-1 draft loop on the device; adapter_arr / kv_adapter_arr are one-element arrays."""
    _check(library().cats_draft_chain(
        ctx, layers_arr, int(layer_begin), int(layer_end), adapter_arr, _dp(g_adapter_out), _dp(w_lm),
        _dp(embed), kv_arr, kv_adapter_arr, int(ctx_len), int(root_token), int(gamma), _dp(tokens_out),
        _dp(hidden_out), _stream(stream)))


def cats_build_tree(root_token: int, main_tokens, corrections=None, capacity: int = CATS_MAX_TREE):
    """Host-side tree of one cascaded cycle: (token, parent, depth, corr_node) numpy int32 arrays."""
    main = np.ascontiguousarray(main_tokens, dtype=np.int32)
    gamma = len(main)
    corr = None if corrections is None else np.ascontiguousarray(corrections, dtype=np.int32)
    if corr is not None and len(corr) != gamma:
        raise CatsError(CATS_EINVAL, "corrections must have one entry per draft position")
    cap = max(int(capacity), 1)
    token, parent, depth = (np.zeros(cap, dtype=np.int32) for _ in range(3))
    corr_node = np.full(max(gamma, 1), -1, dtype=np.int32)
    n = C.c_int32(0)
    _check(library().cats_build_tree(
        int(root_token), main.ctypes.data if gamma else None, gamma,
        None if corr is None else corr.ctypes.data, int(capacity), token.ctypes.data, parent.ctypes.data,
        depth.ctypes.data, C.byref(n), corr_node.ctypes.data))
    return token[: n.value].copy(), parent[: n.value].copy(), depth[: n.value].copy(), corr_node[:gamma].copy()


def cats_set_acceptance(ctx, mode: int, epsilon: float = 0.09, delta: float = 0.3, temperature: float = 1.0):
    _check(library().cats_set_acceptance(ctx, int(mode), float(epsilon), float(delta), float(temperature)))


def cats_typical_stats(ctx, lse_out=None, entropy_out=None, prob_out=None, threshold_out=None, stream=None):
    _check(library().cats_typical_stats(ctx, _dp(lse_out), _dp(entropy_out), _dp(prob_out),
                                        _dp(threshold_out), _stream(stream)))


def cats_compact_along(ctx, result_dev, kv_arr, layer_begin: int, layer_end: int, ctx_len: int, stream=None):
    _check(library().cats_compact_along(ctx, _dp(result_dev), kv_arr, int(layer_begin), int(layer_end),
                                        int(ctx_len), _stream(stream)))


def cats_reduced_kl_loss(target_logits, draft_logits, top_k: int, loss_out, per_pos_out, mask=None,
                         topk_idx_out=None, grad_out=None, stream=None):
    """Shapes are taken from target_logits [n_pos][vocab]; every tensor lives on the device."""
    n_pos, vocab = target_logits.shape
    for t in (target_logits, draft_logits, grad_out):
        if t is not None and (tuple(t.shape) != (n_pos, vocab) or not t.is_contiguous()):
            raise CatsError(CATS_EINVAL, "logit / gradient tensors must be contiguous [n_pos][vocab]")
    _check(library().cats_reduced_kl_loss(
        _dp(target_logits), _dp(draft_logits), _dp(mask), int(n_pos), int(vocab), int(top_k), _dp(loss_out),
        _dp(per_pos_out), _dp(topk_idx_out), _dp(grad_out), _stream(stream)))


def cats_packed_matrix_bytes(rows: int, cols: int) -> int:
    return int(library().cats_packed_matrix_bytes(int(rows), int(cols)))


def cats_pack_matrix(src, stream=None):
    """Packed copy of a row-major bf16 [rows][cols] device tensor (new device tensor, bf16)."""
    import torch
    rows, cols = src.shape
    dst = torch.empty(cats_packed_matrix_bytes(rows, cols) // 2, dtype=torch.bfloat16, device=src.device)
    _check(library().cats_pack_matrix(_dp(src), _dp(dst), int(rows), int(cols), _stream(stream)))
    return dst


MATRIX_FIELDS = ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down")


def pack_layer(tensors: dict) -> dict:
    """A layer dict with its seven matrices packed (gains unchanged)."""
    return {k: (cats_pack_matrix(v) if k in MATRIX_FIELDS else v) for k, v in tensors.items()}


def cats_layer_weight_bytes(desc: ModelDesc) -> int:
    return int(library().cats_layer_weight_bytes(C.byref(desc)))


def cats_verify_tree_streamed(ctx, host_layers_arr, layer_begin: int, layer_end: int, staging, embed,
                              hidden_in, g_final, w_lm, kv_arr, ctx_len: int, out_dev, hidden_out=None,
                              logits_out=None, argmax_out=None, margin_out=None,
                              out_host: AcceptResult | None = None, stream=None):
    """`host_layers_arr`: LayerWeights array whose pointers are pinned host addresses;
    `staging`: two device tensors of cats_layer_weight_bytes() bytes each."""
    stg = (C.c_void_p * 2)(staging[0].data_ptr(), staging[1].data_ptr())
    _check(library().cats_verify_tree_streamed(
        ctx, host_layers_arr, int(layer_begin), int(layer_end), stg, _dp(embed), _dp(hidden_in),
        _dp(g_final), _dp(w_lm), kv_arr, int(ctx_len), _dp(hidden_out), _dp(logits_out),
        _dp(argmax_out), _dp(margin_out), _dp(out_dev),
        None if out_host is None else C.byref(out_host), _stream(stream)))


def cats_lm_head_argmax(ctx, hidden, g_final, w_lm, argmax_out, logits_out=None, margin_out=None,
                        stream=None):
    """Rows are taken from hidden's shape [n_rows][hidden]."""
    _check(library().cats_lm_head_argmax(ctx, _dp(hidden), int(hidden.shape[0]), _dp(g_final), _dp(w_lm),
                                         _dp(logits_out), _dp(argmax_out), _dp(margin_out), _stream(stream)))


def cats_profile_gemm(ctx, enable: bool):
    _check(library().cats_profile_gemm(ctx, int(bool(enable))))


def cats_profile_gemm_read(ctx):
    """(summed GEMM kernel milliseconds, launches) since the last read."""
    ms, n = C.c_float(), C.c_int32()
    _check(library().cats_profile_gemm_read(ctx, C.byref(ms), C.byref(n)))
    return float(ms.value), int(n.value)


# ---------------------------------------------------------------- marshalling helpers
def layer_weights_struct(tensors: dict) -> LayerWeights:
    """Struct of device pointers from a dict name -> bf16 tensor (kept alive by the caller)."""
    return LayerWeights(**{n: (tensors[n].data_ptr() if tensors.get(n) is not None else None)
                           for n, _ in LayerWeights._fields_})


def layer_array(layer_dicts):
    """LayerWeights array from dicts name -> tensor; names that are missing or None stay NULL
    (an attention-only block has no w_gate / w_up / w_down / g_ffn)."""
    arr = (LayerWeights * len(layer_dicts))()
    for i, t in enumerate(layer_dicts):
        for n, _ in LayerWeights._fields_:
            if t.get(n) is not None:
                setattr(arr[i], n, t[n].data_ptr())
    return arr


def kv_array(k_tensors, v_tensors):
    arr = (KVLayer * len(k_tensors))()
    for i, (k, v) in enumerate(zip(k_tensors, v_tensors)):
        arr[i].k = k.data_ptr()
        arr[i].v = v.data_ptr()
    return arr


def accept_result_tensor(device="cuda"):
    """Device storage for one cats_accept_result (int32 words)."""
    import torch
    return torch.zeros(C.sizeof(AcceptResult) // 4, dtype=torch.int32, device=device)


def accept_result_from_tensor(t) -> dict:
    words = t.cpu().numpy().astype(np.int32)
    res = AcceptResult.from_buffer_copy(words.tobytes())
    return res.as_dict()


def kv_from_rows(k_rows, v_rows, n_heads: int, head_dim: int, max_ctx: int):
    """Lay out row-major caches ([rows][hidden] bf16 tensors on the device) in the
    library's format: keys [heads][max_ctx][dim], values transposed [heads][dim][max_ctx]."""
    import torch
    rows = k_rows.shape[0]
    k = torch.zeros(n_heads, max_ctx, head_dim, dtype=torch.bfloat16, device=k_rows.device)
    v = torch.zeros(n_heads, head_dim, max_ctx, dtype=torch.bfloat16, device=k_rows.device)
    if rows:
        k[:, :rows] = k_rows.view(rows, n_heads, head_dim).permute(1, 0, 2)
        v[:, :, :rows] = v_rows.view(rows, n_heads, head_dim).permute(1, 2, 0)
    return k, v


def kv_to_rows(k, v, rows: int):
    """Inverse of kv_from_rows for the first `rows` rows: two [rows][hidden] tensors."""
    n_heads, _, head_dim = k.shape
    k_rows = k[:, :rows].permute(1, 0, 2).reshape(rows, n_heads * head_dim)
    v_rows = v[:, :, :rows].permute(2, 0, 1).reshape(rows, n_heads * head_dim)
    return k_rows, v_rows
