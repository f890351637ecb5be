"""CPU oracle (test infrastructure, never imported by the product).

``oracle.c`` holds the fp64 forward pass and the per-position greedy decode /
confidence; ``slowfast.py`` holds the SlowFast selection rule, stage controller
and decode loop.  This module compiles the C file with gcc and exposes it
through ctypes on numpy arrays.  Nothing here imports or shares code with the
HIP library.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")


def build(force: bool = False) -> str:
    """Compile oracle.c with the host compiler (plain -O2, OpenMP over rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-o", _LIB, _SRC, "-lm"]
        )
    return _LIB


class _Config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("n_layers", "d_model", "n_heads", "head_dim", "d_ffn", "vocab", "mask_id")] + \
               [("rms_eps", C.c_double), ("rope_theta", C.c_double)]


class _Weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("lm_head", C.c_void_p), ("final_norm", C.c_void_p),
                ("attn_norm", C.POINTER(C.c_void_p)), ("wqkv", C.POINTER(C.c_void_p)),
                ("wo", C.POINTER(C.c_void_p)), ("ffn_norm", C.POINTER(C.c_void_p)),
                ("w_gate_up", C.POINTER(C.c_void_p)), ("w_down", C.POINTER(C.c_void_p))]


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_bf16_to_f64.restype = C.c_double
        _lib.orc_bf16_to_f64.argtypes = [C.c_uint16]
        _lib.orc_f64_to_bf16.restype = C.c_uint16
        _lib.orc_f64_to_bf16.argtypes = [C.c_double]
        _lib.orc_softmax_row.restype = C.c_int32
        _lib.orc_forward.restype = C.c_int
    return _lib


def _p(a):
    return a.ctypes.data_as(C.c_void_p)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _u16(a):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16, "bf16 data is passed as its uint16 bit pattern"
    return a


def threads() -> int:
    """Number of OpenMP threads the C part will use."""
    return int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))


# ---- bf16 ------------------------------------------------------------------

def bf16_to_f64(bits):
    bits = _u16(bits)
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def round_to_bf16(x):
    x = _f64(x)
    out = np.empty(x.shape, dtype=np.uint16)
    lib().orc_round_to_bf16(_p(x), C.c_int64(x.size), _p(out))
    return out


# ---- operators ---------------------------------------------------------------

def rmsnorm(x, g_bits, eps):
    x = _f64(x); g_bits = _u16(g_bits)
    rows, d = x.shape
    out = np.empty_like(x)
    lib().orc_rmsnorm(_p(x), _p(g_bits), C.c_int64(rows), C.c_int(d), C.c_double(eps), _p(out))
    return out


def linear(x, w_bits):
    x = _f64(x); w_bits = _u16(w_bits)
    rows, K = x.shape
    N, K2 = w_bits.shape
    assert K == K2
    y = np.empty((rows, N), dtype=np.float64)
    lib().orc_linear(_p(x), _p(w_bits), C.c_int64(rows), C.c_int(K), C.c_int(N), _p(y))
    return y


def rope(x, pos, theta):
    """x: [rows, n_heads, dh]; returns the rotated copy."""
    x = _f64(x).copy()
    rows, H, dh = x.shape
    pos = np.ascontiguousarray(pos, dtype=np.int32)
    assert pos.shape == (rows,)
    lib().orc_rope(_p(x), _p(pos), C.c_int64(rows), C.c_int(H), C.c_int(dh), C.c_double(theta))
    return x


def attention(q, k, v):
    """q, k, v: [L, n_heads, dh] of one sequence."""
    q = _f64(q); k = _f64(k); v = _f64(v)
    L, H, dh = q.shape
    out = np.empty_like(q)
    lib().orc_attention(_p(q), _p(k), _p(v), C.c_int(L), C.c_int(H), C.c_int(dh), _p(out))
    return out


def swiglu(gate, up):
    gate = _f64(gate); up = _f64(up)
    out = np.empty_like(gate)
    lib().orc_swiglu(_p(gate), _p(up), C.c_int64(gate.size), _p(out))
    return out


def _pack(cfg: dict, weights: dict):
    c = _Config(*[int(cfg[k]) for k in
                  ("n_layers", "d_model", "n_heads", "head_dim", "d_ffn", "vocab", "mask_id")],
                float(cfg["rms_eps"]), float(cfg["rope_theta"]))
    nl = c.n_layers
    keep = []

    def arr(name):
        lst = [_u16(a) for a in weights[name]]
        assert len(lst) == nl
        keep.append(lst)
        return (C.c_void_p * max(nl, 1))(*[a.ctypes.data for a in lst])

    single = {k: _u16(weights[k]) for k in ("embed", "lm_head", "final_norm")}
    arrays = {k: arr(k) for k in ("attn_norm", "wqkv", "wo", "ffn_norm", "w_gate_up", "w_down")}
    w = _Weights(single["embed"].ctypes.data, single["lm_head"].ctypes.data,
                 single["final_norm"].ctypes.data,
                 *[C.cast(arrays[k], C.POINTER(C.c_void_p)) for k in
                   ("attn_norm", "wqkv", "wo", "ffn_norm", "w_gate_up", "w_down")])
    return c, w, (keep, single, arrays)


class KVCache:
    """Per-layer keys (after RoPE) and values of every position, float64: the
    features kept by out-of-span caching."""

    def __init__(self, cfg: dict, B: int, L: int):
        self.k = np.zeros((int(cfg["n_layers"]), B * L, int(cfg["d_model"])), dtype=np.float64)
        self.v = np.zeros_like(self.k)


def forward_cached(cfg: dict, weights: dict, tokens, cache: KVCache, rows, skip=None):
    """Forward that recomputes the positions with skip == 0 (all of them when
    skip is None), lets them attend to the cached keys/values of the skipped
    ones, refreshes the cache rows of the recomputed ones, and returns the
    logits [len(rows), V] of the listed rows (indices into B*L, none skipped)."""
    c, w, keep = _pack(cfg, weights)
    tokens = np.ascontiguousarray(tokens, dtype=np.int32)
    B, L = tokens.shape
    assert cache.k.shape == (c.n_layers, B * L, c.d_model) and cache.k.flags.c_contiguous
    rows = np.ascontiguousarray(rows, dtype=np.int32)
    if skip is not None:
        skip = np.ascontiguousarray(skip, dtype=np.uint8).reshape(-1)
        assert skip.shape[0] == B * L
    logits = np.empty((rows.shape[0], c.vocab), dtype=np.float64)
    rc = lib().orc_forward_cached(C.byref(c), C.byref(w), _p(tokens), C.c_int(B), C.c_int(L),
                                  _p(skip) if skip is not None else None, _p(cache.k), _p(cache.v),
                                  _p(rows), C.c_int(rows.shape[0]), _p(logits))
    if rc != 0:
        raise ValueError(f"orc_forward_cached failed with {rc}")
    return logits


def forward(cfg: dict, weights: dict, tokens, rows=None):
    """cfg: dict with the orc_config fields; weights: dict of uint16 arrays
    (per-layer entries are lists).  tokens [B, L] -> logits float64 [B*L, V],
    or [len(rows), V] when `rows` (indices into B*L) is given."""
    c = _Config(*[int(cfg[k]) for k in
                  ("n_layers", "d_model", "n_heads", "head_dim", "d_ffn", "vocab", "mask_id")],
                float(cfg["rms_eps"]), float(cfg["rope_theta"]))
    nl = c.n_layers
    keep = []

    def arr(name):
        lst = [_u16(a) for a in weights[name]]
        assert len(lst) == nl
        keep.append(lst)
        return (C.c_void_p * max(nl, 1))(*[a.ctypes.data for a in lst])

    single = {k: _u16(weights[k]) for k in ("embed", "lm_head", "final_norm")}
    assert single["embed"].shape == (c.vocab, c.d_model)
    assert single["lm_head"].shape == (c.vocab, c.d_model)
    arrays = {k: arr(k) for k in ("attn_norm", "wqkv", "wo", "ffn_norm", "w_gate_up", "w_down")}
    w = _Weights(single["embed"].ctypes.data, single["lm_head"].ctypes.data,
                 single["final_norm"].ctypes.data,
                 *[C.cast(arrays[k], C.POINTER(C.c_void_p)) for k in
                   ("attn_norm", "wqkv", "wo", "ffn_norm", "w_gate_up", "w_down")])
    tokens = np.ascontiguousarray(tokens, dtype=np.int32)
    B, L = tokens.shape
    if rows is not None:
        rows = np.ascontiguousarray(rows, dtype=np.int32)
    n_out = B * L if rows is None else rows.shape[0]
    logits = np.empty((n_out, c.vocab), dtype=np.float64)
    rc = lib().orc_forward(C.byref(c), C.byref(w), _p(tokens), C.c_int(B), C.c_int(L),
                           _p(rows) if rows is not None else None, C.c_int(0 if rows is None else rows.shape[0]),
                           _p(logits))
    if rc != 0:
        raise ValueError(f"orc_forward failed with {rc}")
    return logits


# ---- greedy decode + confidence ---------------------------------------------

def softmax_row(logits_bits, mask_id):
    """Returns (argmax id, confidence, probabilities[V]) of one bf16 row."""
    logits_bits = _u16(logits_bits)
    V = logits_bits.shape[0]
    prob = np.empty(V, dtype=np.float64)
    conf = C.c_double()
    arg = lib().orc_softmax_row(_p(logits_bits), C.c_int(V), C.c_int(mask_id), _p(prob), C.byref(conf))
    return int(arg), conf.value, prob


def row_phase(logits_bits, mask_id, active=None):
    """logits_bits [rows, V] uint16 -> (pred int32 [rows], conf float32 [rows])."""
    logits_bits = _u16(logits_bits)
    rows, V = logits_bits.shape
    pred = np.empty(rows, dtype=np.int32)
    conf = np.empty(rows, dtype=np.float32)
    act = None if active is None else np.ascontiguousarray(active, dtype=np.uint8)
    lib().orc_row_phase(_p(logits_bits), C.c_int64(rows), C.c_int(V), C.c_int(mask_id),
                        _p(act) if act is not None else None, _p(pred), _p(conf))
    return pred, conf
