"""ctypes wrapper around the CPU oracle (oracle/orc.c).  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this module.
It imports nothing from the GPU package.  Weights are numpy arrays: float32 values or
uint16 bf16 bit patterns; they are borrowed, so the wrapper keeps references alive.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List

import numpy as np

from . import build as _build

_LIB = None


class OrcShape(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "hidden", "n_heads", "n_kv_heads", "head_dim", "ffn", "vocab")] + [
        ("rope_base", C.c_float), ("rms_eps", C.c_float), ("rope_style", C.c_int32), ("weight_dtype", C.c_int32),
        ("max_batch", C.c_int32), ("max_seq", C.c_int32)]


class OrcWeights(C.Structure):
    _fields_ = [("tok_emb", C.c_void_p)] + [(n, C.POINTER(C.c_void_p)) for n in (
        "attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down")] + [
        ("final_norm", C.c_void_p), ("lm_head", C.c_void_p)]


_LAYER_NAMES = ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down")


def lib():
    global _LIB
    if _LIB is None:
        path = _build.LIB
        if not os.path.exists(path) or os.path.getmtime(path) < os.path.getmtime(_build.SRC):
            _build.build()
        L = C.CDLL(path)
        dp, ip, vp = C.POINTER(C.c_double), C.POINTER(C.c_int32), C.c_void_p
        L.orc_linear.argtypes = [vp, C.c_int, C.c_int, C.c_int, dp, C.c_int, dp]
        L.orc_linear.restype = None
        L.orc_rmsnorm.argtypes = [dp, vp, C.c_int, C.c_int, C.c_double, dp]
        L.orc_rmsnorm.restype = None
        L.orc_rope.argtypes = [dp, C.c_int, C.c_int, C.c_double, C.c_int]
        L.orc_rope.restype = None
        L.orc_attend.argtypes = [dp, dp, dp, C.c_int, C.c_int, C.c_size_t, dp]
        L.orc_attend.restype = None
        L.orc_silu.argtypes = [C.c_double]
        L.orc_silu.restype = C.c_double
        L.orc_argmax.argtypes = [dp, C.c_int]
        L.orc_argmax.restype = C.c_int32
        L.orc_sample.argtypes = [dp, C.c_int, C.c_double, C.c_double]
        L.orc_sample.restype = C.c_int32
        L.orc_token_logprob.argtypes = [dp, C.c_int, C.c_int]
        L.orc_token_logprob.restype = C.c_double
        L.orc_param_count.argtypes = [C.POINTER(OrcShape)]
        L.orc_param_count.restype = C.c_int64
        L.orc_kv_bytes_per_token.argtypes = [C.POINTER(OrcShape), C.c_int]
        L.orc_kv_bytes_per_token.restype = C.c_int64
        L.orc_create.argtypes = [C.POINTER(OrcShape), C.POINTER(OrcWeights), C.POINTER(vp)]
        L.orc_create.restype = C.c_int
        L.orc_destroy.argtypes = [vp]
        L.orc_destroy.restype = None
        L.orc_reset.argtypes = [vp]
        L.orc_reset.restype = C.c_int
        L.orc_forward_all.argtypes = [vp, ip, C.c_int, C.c_int, dp]
        L.orc_forward_all.restype = C.c_int
        L.orc_prefill.argtypes = [vp, ip, C.c_int, C.c_int, dp, ip]
        L.orc_prefill.restype = C.c_int
        L.orc_decode_step.argtypes = [vp, ip, dp, ip]
        L.orc_decode_step.restype = C.c_int
        L.orc_extend.argtypes = [vp, ip, C.c_int, dp]
        L.orc_extend.restype = C.c_int
        L.orc_num_threads.argtypes = []
        L.orc_num_threads.restype = C.c_int
        _LIB = L
    return _LIB


def _dp(a: np.ndarray):
    assert a.dtype == np.float64 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(C.POINTER(C.c_double))


def _ip(a: np.ndarray):
    assert a.dtype == np.int32 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(C.POINTER(C.c_int32))


def _wdtype(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return 0
    if a.dtype == np.uint16:
        return 1
    raise TypeError("oracle weights must be float32 values or uint16 bf16 bit patterns")


def make_shape(shape, weight_dtype: int, max_batch: int, max_seq: int) -> OrcShape:
    """shape: any object with the ModelShape field names."""
    return OrcShape(shape.n_layers, shape.hidden, shape.n_heads, shape.n_kv_heads, shape.head_dim, shape.ffn,
                    shape.vocab, shape.rope_base, shape.rms_eps, shape.rope_style, weight_dtype, max_batch, max_seq)


# ---------------------------------------------------------------- sub-functions (for pins and kernel unit tests)

def linear(W: np.ndarray, X: np.ndarray) -> np.ndarray:
    W = np.ascontiguousarray(W)
    X = np.ascontiguousarray(X, dtype=np.float64)
    N, K = W.shape
    M = X.shape[0]
    assert X.shape[1] == K
    Y = np.empty((M, N), dtype=np.float64)
    lib().orc_linear(W.ctypes.data_as(C.c_void_p), _wdtype(W), N, K, _dp(X), M, _dp(Y))
    return Y


def rmsnorm(x: np.ndarray, g: np.ndarray, eps: float) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float64)
    g = np.ascontiguousarray(g)
    y = np.empty_like(x)
    rows = x.reshape(-1, x.shape[-1])
    out = y.reshape(-1, x.shape[-1])
    for i in range(rows.shape[0]):
        lib().orc_rmsnorm(_dp(rows[i]), g.ctypes.data_as(C.c_void_p), _wdtype(g), rows.shape[1], float(eps), _dp(out[i]))
    return y


def rope(v: np.ndarray, pos: int, base: float, style: int) -> np.ndarray:
    out = np.array(v, dtype=np.float64, order="C", copy=True)
    rows = out.reshape(-1, out.shape[-1])
    for i in range(rows.shape[0]):
        lib().orc_rope(_dp(rows[i]), rows.shape[1], int(pos), float(base), int(style))
    return out


def attend(q: np.ndarray, K: np.ndarray, V: np.ndarray) -> np.ndarray:
    """q [hd], K and V [n_ctx, hd] -> o [hd]"""
    q = np.ascontiguousarray(q, dtype=np.float64)
    K = np.ascontiguousarray(K, dtype=np.float64)
    V = np.ascontiguousarray(V, dtype=np.float64)
    o = np.empty_like(q)
    lib().orc_attend(_dp(q), _dp(K), _dp(V), K.shape[0], K.shape[1], K.shape[1], _dp(o))
    return o


def silu(z: float) -> float:
    return lib().orc_silu(float(z))


def argmax(x: np.ndarray) -> int:
    x = np.ascontiguousarray(x, dtype=np.float64)
    return int(lib().orc_argmax(_dp(x), x.shape[0]))


def sample(x: np.ndarray, temperature: float, u: float) -> int:
    x = np.ascontiguousarray(x, dtype=np.float64)
    return int(lib().orc_sample(_dp(x), x.shape[0], float(temperature), float(u)))


def token_logprob(x: np.ndarray, target: int) -> float:
    x = np.ascontiguousarray(x, dtype=np.float64)
    return float(lib().orc_token_logprob(_dp(x), x.shape[0], int(target)))


def sequence_logprobs(logits: np.ndarray, tokens: np.ndarray) -> np.ndarray:
    """logits [B, T, V] of every position, tokens [B, T] -> [B, T-1]: log-probability that position i assigns to the
    token that follows it (Section 2.1: what the inference call over prompt + response returns per token)."""
    B, T, _ = logits.shape
    out = np.empty((B, T - 1), dtype=np.float64)
    for b in range(B):
        for i in range(T - 1):
            out[b, i] = token_logprob(logits[b, i], int(tokens[b, i + 1]))
    return out


def param_count(shape) -> int:
    s = make_shape(shape, 1, 1, 1)
    return int(lib().orc_param_count(C.byref(s)))


def kv_bytes_per_token(shape, elem_bytes: int = 2) -> int:
    s = make_shape(shape, 1, 1, 1)
    return int(lib().orc_kv_bytes_per_token(C.byref(s), elem_bytes))


def num_threads() -> int:
    return int(lib().orc_num_threads())


# ---------------------------------------------------------------- model

class OracleError(RuntimeError):
    def __init__(self, code: int, where: str):
        super().__init__(f"oracle {where} failed with code {code}")
        self.code = code


class OracleModel:
    """weights: {"tok_emb": ndarray, "final_norm": ndarray, "lm_head": ndarray, <layer tensor>: [ndarray]*L}"""

    def __init__(self, shape, weights: Dict[str, object], max_batch: int, max_seq: int):
        self.shape = shape
        wd = _wdtype(np.asarray(weights["tok_emb"]))
        self._keep: List[np.ndarray] = []

        def hold(a) -> int:
            a = np.ascontiguousarray(a)
            if _wdtype(a) != wd:
                raise TypeError("all oracle weights must share one dtype")
            self._keep.append(a)
            return a.ctypes.data

        w = OrcWeights()
        w.tok_emb = hold(weights["tok_emb"])
        w.final_norm = hold(weights["final_norm"])
        w.lm_head = hold(weights["lm_head"])
        self._arrays = []
        L = shape.n_layers
        for name in _LAYER_NAMES:
            arr = (C.c_void_p * max(L, 1))()
            lst = weights.get(name, [])
            if len(lst) != L:
                raise ValueError(f"{name}: expected {L} tensors, got {len(lst)}")
            for l in range(L):
                arr[l] = hold(lst[l])
            self._arrays.append(arr)
            setattr(w, name, C.cast(arr, C.POINTER(C.c_void_p)))
        self._w = w
        self._s = make_shape(shape, wd, max_batch, max_seq)
        h = C.c_void_p()
        rc = lib().orc_create(C.byref(self._s), C.byref(w), C.byref(h))
        if rc != 0:
            raise OracleError(rc, "orc_create")
        self._h = h

    def close(self):
        if getattr(self, "_h", None):
            lib().orc_destroy(self._h)
            self._h = None

    __del__ = close

    def reset(self):
        lib().orc_reset(self._h)

    def forward_all(self, tokens: np.ndarray) -> np.ndarray:
        tokens = np.ascontiguousarray(tokens, dtype=np.int32)
        B, T = tokens.shape
        out = np.empty((B, T, self.shape.vocab), dtype=np.float64)
        rc = lib().orc_forward_all(self._h, _ip(tokens), B, T, _dp(out))
        if rc != 0:
            raise OracleError(rc, "orc_forward_all")
        return out

    def prefill(self, tokens: np.ndarray):
        tokens = np.ascontiguousarray(tokens, dtype=np.int32)
        B, T = tokens.shape
        logits = np.empty((B, self.shape.vocab), dtype=np.float64)
        nxt = np.empty((B,), dtype=np.int32)
        rc = lib().orc_prefill(self._h, _ip(tokens), B, T, _dp(logits), _ip(nxt))
        if rc != 0:
            raise OracleError(rc, "orc_prefill")
        self._B = B
        return logits, nxt

    def extend(self, tokens: np.ndarray, want_logits: bool = True):
        """tokens [B, T]: T further tokens per sequence against the cache; returns the logits [B, V] of the last one (or None)."""
        tokens = np.ascontiguousarray(tokens, dtype=np.int32)
        B, T = tokens.shape
        logits = np.empty((B, self.shape.vocab), dtype=np.float64) if want_logits else None
        rc = lib().orc_extend(self._h, _ip(tokens), T, _dp(logits) if want_logits else None)
        if rc != 0:
            raise OracleError(rc, "orc_extend")
        return logits

    def decode_step(self, tokens: np.ndarray):
        tokens = np.ascontiguousarray(tokens, dtype=np.int32)
        B = tokens.shape[0]
        logits = np.empty((B, self.shape.vocab), dtype=np.float64)
        nxt = np.empty((B,), dtype=np.int32)
        rc = lib().orc_decode_step(self._h, _ip(tokens), _dp(logits), _ip(nxt))
        if rc != 0:
            raise OracleError(rc, "orc_decode_step")
        return logits, nxt


def weights_to_numpy(weights: Dict[str, object], as_bf16_bits: bool = True) -> Dict[str, object]:
    """Converts a dict of torch tensors (workload.make_weights) into the numpy form the oracle borrows.

    bf16 tensors become uint16 bit patterns (as_bf16_bits) or float32 values; float32 tensors stay float32.
    """
    import torch

    def conv(t):
        t = t.detach().cpu().contiguous()
        if t.dtype == torch.bfloat16:
            if as_bf16_bits:
                return t.view(torch.int16).numpy().view(np.uint16)
            return t.to(torch.float32).numpy()
        if t.dtype == torch.float32:
            return t.numpy()
        raise TypeError(t.dtype)

    out: Dict[str, object] = {}
    for k, v in weights.items():
        out[k] = [conv(t) for t in v] if isinstance(v, (list, tuple)) else conv(v)
    return out
