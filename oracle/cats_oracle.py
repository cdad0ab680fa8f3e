"""ctypes front end of the CPU oracle (cats_oracle.cpp).

TEST INFRASTRUCTURE ONLY: imported by the tests, by the smoke check and by the
benchmark's CPU-baseline leg.  The GPU library never imports or calls this.

Two builds of the same source exist: `f32` (plain float, the one that is timed
as the CPU baseline) and `f64` (double, the reference for parity checks).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "cats_oracle.cpp"
_LIBS = {"f32": _HERE / "libcats_oracle_f32.so", "f64": _HERE / "libcats_oracle_f64.so"}
MAX_PATH = 32


def build(force: bool = True) -> None:
    """Compile both precisions with the host compiler."""
    for prec, out in _LIBS.items():
        if not force and out.exists() and out.stat().st_mtime >= _SRC.stat().st_mtime:
            continue
        cmd = ["g++", "-O3", "-march=x86-64-v3", "-fopenmp", "-fPIC", "-shared", "-std=c++17",
               "-Wall", "-Wextra"]
        if prec == "f64":
            cmd.append("-DCATS_ORACLE_F64")
        cmd += [str(_SRC), "-o", str(out)]
        subprocess.run(cmd, check=True)


class Dims(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("hidden", C.c_int32), ("n_heads", C.c_int32),
                ("head_dim", C.c_int32), ("ffn", C.c_int32), ("vocab", C.c_int32),
                ("rms_eps", C.c_float), ("rope_base", C.c_float)]


class Layer(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in
                ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down", "g_attn", "g_ffn")]


class Accept(C.Structure):
    _fields_ = [("n_accepted", C.c_int32), ("path", C.c_int32 * MAX_PATH),
                ("tokens", C.c_int32 * MAX_PATH), ("bonus_token", C.c_int32),
                ("new_ctx_len", C.c_int32)]


def _ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a


class Oracle:
    """One precision of the oracle bound to one model (dims + bf16-bit weights).

    `layers` is a list of dicts as made by synth.layer_weights; `final` holds
    g_final / w_lm; `embed` is the embedding table (all uint16 bf16 bits).
    """

    def __init__(self, dims, layers, final=None, embed=None, precision: str = "f64"):
        lib_path = _LIBS[precision]
        if not lib_path.exists():
            build(force=False)
        self.lib = C.CDLL(str(lib_path))
        self.real = np.float64 if precision == "f64" else np.float32
        assert self.lib.oracle_real_bytes() == np.dtype(self.real).itemsize
        self.dims = dims
        self.cdims = Dims(dims.n_layers, dims.hidden, dims.n_heads, dims.head_dim, dims.ffn,
                          dims.vocab, dims.rms_eps, dims.rope_base)
        self._keep = [layers, final, embed]
        self.layers = layers
        self.final = final
        self.embed = embed
        arr = (Layer * max(1, len(layers)))()
        for i, w in enumerate(layers):
            if w is None:
                continue
            for name, _ in Layer._fields_:
                a = w[name]
                assert a.dtype == np.uint16 and a.flags.c_contiguous
                setattr(arr[i], name, a.ctypes.data)
        self.clayers = arr

    # -- caches ------------------------------------------------------------
    def new_cache(self, max_ctx: int):
        shape = (self.dims.n_layers, max_ctx, self.dims.hidden)
        return np.zeros(shape, self.real), np.zeros(shape, self.real)

    def num_threads(self) -> int:
        return int(self.lib.oracle_num_threads())

    # -- single ops --------------------------------------------------------
    def rmsnorm(self, x, g_bits):
        x = np.ascontiguousarray(x, self.real)
        out = np.empty_like(x)
        self.lib.oracle_rmsnorm(_ptr(x), _ptr(g_bits), C.c_int(x.shape[-1]),
                                C.c_float(self.dims.rms_eps), _ptr(out))
        return out

    def linear(self, X, W_bits):
        X = np.ascontiguousarray(X, self.real)
        T, K = X.shape
        N = W_bits.shape[0]
        assert W_bits.shape == (N, K) and W_bits.dtype == np.uint16
        Y = np.empty((T, N), self.real)
        self.lib.oracle_linear(_ptr(X), _ptr(W_bits), T, K, N, _ptr(Y))
        return Y

    def rope(self, v, pos: int):
        v = np.array(v, dtype=self.real, order="C", copy=True)
        self.lib.oracle_rope(_ptr(v), self.dims.n_heads, self.dims.head_dim, int(pos),
                             C.c_float(self.dims.rope_base))
        return v

    def attend(self, q, Kc, Vc, rows):
        q = np.ascontiguousarray(q, self.real)
        Kc = np.ascontiguousarray(Kc, self.real)
        Vc = np.ascontiguousarray(Vc, self.real)
        rows = _i32(rows)
        out = np.empty_like(q)
        self.lib.oracle_attend(_ptr(q), _ptr(Kc), _ptr(Vc), _ptr(rows), len(rows),
                               self.dims.n_heads, self.dims.head_dim, _ptr(out))
        return out

    # -- whole passes --------------------------------------------------------
    def causal_decode(self, kc, vc, ctx_len, tokens=None, hidden_in=None,
                      layer_begin=0, layer_end=None):
        """Token-at-a-time decoding.  Returns hidden_out [n][hidden]."""
        layer_end = self.dims.n_layers if layer_end is None else layer_end
        if tokens is not None:
            tokens = _i32(tokens)
            n = len(tokens)
            embed = self.embed
            assert embed is not None
        else:
            hidden_in = np.ascontiguousarray(hidden_in, self.real)
            n = hidden_in.shape[0]
            embed = None
        out = np.empty((n, self.dims.hidden), self.real)
        rc = self.lib.oracle_causal_decode(
            C.byref(self.cdims), self.clayers, layer_begin, layer_end, _ptr(embed),
            _ptr(hidden_in), _ptr(tokens), n, _ptr(kc), _ptr(vc), kc.shape[1], int(ctx_len),
            _ptr(out))
        if rc != 0:
            raise ValueError("context capacity exceeded")
        return out

    def tree_forward(self, kc, vc, ctx_len, parent, depth, tokens=None, hidden_in=None,
                     layer_begin=0, layer_end=None):
        """Batched pass of all tree nodes under the tree mask.  Returns x [T][hidden]."""
        layer_end = self.dims.n_layers if layer_end is None else layer_end
        parent, depth = _i32(parent), _i32(depth)
        T = len(parent)
        if tokens is not None:
            tokens = _i32(tokens)
            embed = self.embed
            assert embed is not None
            x = np.empty((T, self.dims.hidden), self.real)
        else:
            embed = None
            x = np.array(hidden_in, dtype=self.real, order="C", copy=True)
            assert x.shape == (T, self.dims.hidden)
        rc = self.lib.oracle_tree_forward(
            C.byref(self.cdims), self.clayers, layer_begin, layer_end, _ptr(embed), _ptr(tokens),
            _ptr(parent), _ptr(depth), T, _ptr(kc), _ptr(vc), kc.shape[1], int(ctx_len), _ptr(x))
        if rc != 0:
            raise ValueError("context capacity exceeded")
        return x

    def lm_head(self, x):
        x = np.ascontiguousarray(x, self.real)
        T = x.shape[0]
        logits = np.empty((T, self.dims.vocab), self.real)
        self.lib.oracle_lm_head(C.byref(self.cdims), _ptr(self.final["g_final"]),
                                _ptr(self.final["w_lm"]), _ptr(x), T, _ptr(logits))
        return logits

    def argmax_margin(self, logits):
        logits = np.ascontiguousarray(logits, self.real)
        T, V = logits.shape
        amax = np.empty(T, np.int32)
        margin = np.empty(T, self.real)
        self.lib.oracle_argmax_margin(_ptr(logits), T, V, _ptr(amax), _ptr(margin))
        return amax, margin

    def accept(self, token, parent, depth, amax, ctx_len):
        token, parent, depth, amax = _i32(token), _i32(parent), _i32(depth), _i32(amax)
        res = Accept()
        rc = self.lib.oracle_accept(_ptr(token), _ptr(parent), _ptr(depth), _ptr(amax),
                                    len(parent), int(ctx_len), C.byref(res))
        if rc != 0:
            raise ValueError("accepted path too deep")
        n = res.n_accepted
        return {"n_accepted": n, "path": list(res.path[: n + 1]),
                "tokens": list(res.tokens[: n + 1]), "bonus_token": res.bonus_token,
                "new_ctx_len": res.new_ctx_len}

    def compact(self, kc, vc, ctx_len, path):
        path = _i32(path)
        self.lib.oracle_compact(_ptr(kc), _ptr(vc), kc.shape[0], kc.shape[1], kc.shape[2],
                                int(ctx_len), _ptr(path), len(path))

    def verify_step(self, kc, vc, ctx_len, tokens, parent, depth):
        """One whole verify step: tree pass, LM head, argmax, accept, compaction.
        Returns (hidden, logits, amax, margin, accept dict)."""
        x = self.tree_forward(kc, vc, ctx_len, parent, depth, tokens=tokens)
        logits = self.lm_head(x)
        amax, margin = self.argmax_margin(logits)
        acc = self.accept(tokens, parent, depth, amax, ctx_len)
        self.compact(kc, vc, ctx_len, acc["path"])
        return x, logits, amax, margin, acc


if __name__ == "__main__":
    build()
    print("built", ", ".join(str(p) for p in _LIBS.values()))
