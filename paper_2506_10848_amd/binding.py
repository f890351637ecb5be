"""Thin ctypes binding of libdllm.so (same names as the C ABI in include/dllm.h).

Argument marshalling only: torch tensors supply device memory and the current
HIP stream; every step of the path runs in the library's kernels.  There is no
fallback: if the shared library is missing, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdllm.so")

OK, EINVAL, ENOMEM, EHIP, ECAPACITY, ESTATE = 0, -1, -2, -3, -4, -5
STAGE_SLOW, STAGE_FAST, STAGE_IDLE = 0, 1, 2
CACHE_OFF, CACHE_REFRESH, CACHE_REUSE = 0, 1, 2
MAX_BATCH = 64


class DllmError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"dllm error {code}: {msg}")
        self.code = code


class Config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_heads", "head_dim", "d_ffn", "vocab", "mask_id")] \
        + [("rms_eps", C.c_float), ("rope_theta", C.c_float), ("max_batch", C.c_int32), ("max_seq", C.c_int32)]


class Weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("lm_head", C.c_void_p), ("final_norm", C.c_void_p)] + \
               [(n, C.POINTER(C.c_void_p)) for n in ("attn_norm", "wqkv", "wo", "ffn_norm", "w_gate_up", "w_down")]


class StageParams(C.Structure):
    _fields_ = [("stage", C.c_int32), ("s_cycle", C.c_int32), ("e_cycle", C.c_int32), ("top_k", C.c_int32),
                ("tau_min_conf", C.c_float), ("tau_high_conf", C.c_float), ("conv_mode", C.c_int32),
                ("gen_start", C.c_int32), ("gen_end", C.c_int32)]


class CommitListC(C.Structure):
    _fields_ = [("capacity", C.c_int32), ("n_commit", C.c_void_p), ("pos", C.c_void_p), ("tok", C.c_void_p),
                ("conf", C.c_void_p), ("e_cand", C.c_void_p), ("first_masked", C.c_void_p),
                ("n_masked_after", C.c_void_p)]


class DecodeParams(C.Structure):
    _fields_ = [("max_steps", C.c_int32), ("k_max", C.c_int32), ("w_hist", C.c_int32), ("k_slow", C.c_int32),
                ("k_fast", C.c_int32), ("conv_mode", C.c_int32), ("sigma2_stable", C.c_float),
                ("tau_min_conf", C.c_float), ("tau_high_conf", C.c_float), ("out_of_span_cache", C.c_int32),
                ("prompt_cache_interval", C.c_int32), ("response_cache_interval", C.c_int32)]


class StepStat(C.Structure):
    _fields_ = [("n_slow", C.c_int32), ("n_fast", C.c_int32), ("n_idle", C.c_int32), ("n_commit", C.c_int32),
                ("ms", C.c_float)]


EXPORTS = ["dllm_create", "dllm_destroy", "dllm_last_error", "dllm_step", "dllm_step_cached", "dllm_decode", "dllm_decode_low_confidence", "dllm_set_fused_selector", "dllm_sync_status", "dllm_debug_reload_env", "dllm_debug_gemm_plan", "dllm_debug_mfma_rate", "dllm_debug_logits",
           "dllm_debug_rows", "dllm_profile_begin", "dllm_profile_end", "dllm_forward", "dllm_select", "dllm_op_linear", "dllm_op_linear_swiglu", "dllm_op_pack_panels", "dllm_op_linear_panels",
           "dllm_op_add_rmsnorm", "dllm_op_rope", "dllm_op_linear_qkv_rope", "dllm_op_linear_qkv_rope_static", "dllm_op_attention"]

_lib = None


def lib() -> C.CDLL:
    """Loads libdllm.so; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2506_10848_amd.build` "
                "(there is no fallback path)")
        _lib = C.CDLL(LIB_PATH)
        _lib.dllm_last_error.restype = C.c_char_p
        _lib.dllm_last_error.argtypes = [C.c_void_p]
        _lib.dllm_destroy.restype = None
        _lib.dllm_destroy.argtypes = [C.c_void_p]
        _lib.dllm_debug_reload_env.restype = None
        _lib.dllm_debug_reload_env.argtypes = []
    return _lib


def debug_mfma_rate(operands, sink, workgroups: int, iters: int) -> float:
    """dllm_debug_mfma_rate on the current stream; returns the flop count of the launch (the caller times it)."""
    _dev(operands, torch.bfloat16, "operands"); _dev(sink, torch.float32, "sink")
    assert operands.numel() % 8 == 0 and sink.numel() >= workgroups * 256
    _check(lib().dllm_debug_mfma_rate(_stream(), _ptr(operands), operands.numel() // 8, _ptr(sink), workgroups, iters))
    return workgroups * 4.0 * iters * 8 * 32768


def gemm_plan(epilogue: int, M: int, N: int, K: int, split_limit: int = 8) -> dict:
    """dllm_debug_gemm_plan as a dict (tile, stage depth, stages, wave grid, splits, kernel kind)."""
    out = (C.c_int32 * 8)()
    _check(lib().dllm_debug_gemm_plan(epilogue, M, N, K, split_limit, out))
    keys = ("bm", "bn", "bk", "stages", "waves_m", "waves_n", "splits", "async_copy")
    return dict(zip(keys, list(out)))


def reload_env() -> None:
    """dllm_debug_reload_env: the library re-reads its DLLM_* environment switches (tests only)."""
    lib().dllm_debug_reload_env()


def _check(rc: int, handle=None):
    if rc != OK:
        raise DllmError(rc, lib().dllm_last_error(handle).decode())


def _stream() -> C.c_void_p:
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t: Optional[torch.Tensor]) -> C.c_void_p:
    return C.c_void_p(0 if t is None else t.data_ptr())


def _dev(t: torch.Tensor, dtype, name: str) -> torch.Tensor:
    if not (t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise TypeError(f"{name}: expected a contiguous {dtype} device tensor")
    return t


def stage_params(stage, s_cycle, e_cycle, top_k, tau_min_conf, tau_high_conf, conv_mode, gen_start, gen_end):
    return StageParams(stage, s_cycle, e_cycle, top_k, tau_min_conf, tau_high_conf, conv_mode, gen_start, gen_end)


class CommitList:
    """Device buffers for the result of a step (dllm_commit_list)."""

    def __init__(self, batch: int, capacity: int, device="cuda"):
        self.batch, self.capacity = batch, capacity
        i32 = dict(dtype=torch.int32, device=device)
        self.n_commit = torch.zeros(batch, **i32)
        self.pos = torch.full((batch, max(capacity, 1)), -1, **i32)
        self.tok = torch.full((batch, max(capacity, 1)), -1, **i32)
        self.conf = torch.zeros((batch, max(capacity, 1)), dtype=torch.float32, device=device)
        self.e_cand = torch.zeros(batch, **i32)
        self.first_masked = torch.zeros(batch, **i32)
        self.n_masked_after = torch.zeros(batch, **i32)

    def c_struct(self) -> CommitListC:
        return CommitListC(self.capacity, *[t.data_ptr() for t in (
            self.n_commit, self.pos, self.tok, self.conf, self.e_cand, self.first_masked, self.n_masked_after)])

    def to_host(self):
        """[(positions, tokens, confidences, e_cand, first_masked, n_masked_after)] per sequence."""
        n = self.n_commit.cpu().tolist()
        pos, tok, conf = self.pos.cpu(), self.tok.cpu(), self.conf.cpu()
        e, f, m = self.e_cand.cpu().tolist(), self.first_masked.cpu().tolist(), self.n_masked_after.cpu().tolist()
        return [(pos[b, :n[b]].tolist(), tok[b, :n[b]].tolist(), conf[b, :n[b]].numpy().copy(), e[b], f[b], m[b])
                for b in range(self.batch)]


def _sp_array(sps: Sequence[StageParams]):
    return (StageParams * len(sps))(*sps)


class Model:
    """Owns a dllm_handle.  `weights` is a dict of bf16 device tensors laid out
    as include/dllm.h documents (per-layer entries are lists); they are kept
    alive here because the library reads them in place."""

    def __init__(self, cfg: dict, weights: dict, max_batch: int, max_seq: int):
        self._h = C.c_void_p()
        self.cfg = dict(cfg)
        self.weights = weights
        nl = cfg["n_layers"]
        c = Config(cfg["n_layers"], cfg["d_model"], cfg["n_heads"], cfg["head_dim"], cfg["d_ffn"], cfg["vocab"],
                   cfg["mask_id"], cfg["rms_eps"], cfg["rope_theta"], max_batch, max_seq)
        for k in ("embed", "lm_head", "final_norm"):
            _dev(weights[k], torch.bfloat16, k)
        arrays = {}
        for k in ("attn_norm", "wqkv", "wo", "ffn_norm", "w_gate_up", "w_down"):
            assert len(weights[k]) == nl
            arrays[k] = (C.c_void_p * max(nl, 1))(*[_dev(t, torch.bfloat16, k).data_ptr() for t in weights[k]])
        w = Weights(weights["embed"].data_ptr(), weights["lm_head"].data_ptr(), weights["final_norm"].data_ptr(),
                    *[C.cast(arrays[k], C.POINTER(C.c_void_p)) for k in
                      ("attn_norm", "wqkv", "wo", "ffn_norm", "w_gate_up", "w_down")])
        _check(lib().dllm_create(C.byref(c), C.byref(w), _stream(), C.byref(self._h)))

    def close(self):
        if self._h:
            lib().dllm_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def forward(self, tokens: torch.Tensor) -> torch.Tensor:
        """dllm_forward + dllm_debug_logits: bf16 logits [B*L, V] (a view of the workspace)."""
        _dev(tokens, torch.int32, "tokens")
        B, L = tokens.shape
        _check(lib().dllm_forward(self._h, B, L, _ptr(tokens)), self._h)
        return self.debug_logits(B * L)

    def debug_logits(self, rows: int) -> torch.Tensor:
        p = C.c_void_p()
        _check(lib().dllm_debug_logits(self._h, C.byref(p)), self._h)
        return _view(p.value, (rows, self.cfg["vocab"]), torch.bfloat16)

    def debug_rows(self, rows: int):
        p, q = C.c_void_p(), C.c_void_p()
        _check(lib().dllm_debug_rows(self._h, C.byref(p), C.byref(q)), self._h)
        return _view(p.value, (rows,), torch.int32), _view(q.value, (rows,), torch.float32)

    def profile_begin(self, max_launches: int) -> None:
        _check(lib().dllm_profile_begin(self._h, max_launches), self._h)

    def profile_end(self):
        """(summed ms, launches) of the bracketed gate/up GEMM launches."""
        ms, n = C.c_float(0), C.c_int32(0)
        _check(lib().dllm_profile_end(self._h, C.byref(ms), C.byref(n)), self._h)
        return ms.value, n.value

    def step(self, tokens, mask, prev_pred, sps: Sequence[StageParams], out: CommitList) -> None:
        _dev(tokens, torch.int32, "tokens"); _dev(mask, torch.uint8, "mask"); _dev(prev_pred, torch.int32, "prev_pred")
        B, L = tokens.shape
        assert len(sps) == B and mask.shape == (B, L) and prev_pred.shape == (B, L)
        cl = out.c_struct()
        _check(lib().dllm_step(self._h, B, L, _ptr(tokens), _ptr(mask), _ptr(prev_pred), _sp_array(sps),
                               C.byref(cl)), self._h)

    def sync_status(self) -> None:
        """dllm_sync_status: waits for the stream; raises if a step read a token id outside [0, vocab)."""
        _check(lib().dllm_sync_status(self._h), self._h)

    def set_fused_selector(self, enable: bool) -> None:
        """dllm_set_fused_selector: greedy decode inside the vocabulary projection (default) or from bf16 logits."""
        _check(lib().dllm_set_fused_selector(self._h, int(bool(enable))), self._h)

    def step_cached(self, tokens, mask, prev_pred, sps, cache_mode, skip, out: "CommitList") -> None:
        """dllm_step_cached: cache_mode is a sequence of B ints, skip a host uint8 array [B, L] or None."""
        _dev(tokens, torch.int32, "tokens"); _dev(mask, torch.uint8, "mask"); _dev(prev_pred, torch.int32, "prev_pred")
        B, L = tokens.shape
        cl = out.c_struct()
        modes = (C.c_int32 * B)(*[int(m) for m in cache_mode])
        sk = None
        if skip is not None:
            import numpy as np
            sk = np.ascontiguousarray(skip, dtype=np.uint8)
            assert sk.shape == (B, L)
        _check(lib().dllm_step_cached(self._h, B, L, _ptr(tokens), _ptr(mask), _ptr(prev_pred), _sp_array(sps), modes,
                                      C.c_void_p(sk.ctypes.data) if sk is not None else None, C.byref(cl)), self._h)

    def decode(self, tokens, mask, gen_start: int, params: DecodeParams, stats_capacity: int = 0):
        _dev(tokens, torch.int32, "tokens"); _dev(mask, torch.uint8, "mask")
        B, L = tokens.shape
        steps = C.c_int32(0)
        stats = (StepStat * max(stats_capacity, 1))()
        _check(lib().dllm_decode(self._h, B, L, gen_start, _ptr(tokens), _ptr(mask), C.byref(params),
                                 C.byref(steps), stats if stats_capacity else None, stats_capacity), self._h)
        n = min(steps.value, stats_capacity)
        return steps.value, [(s.n_slow, s.n_fast, s.n_idle, s.n_commit, s.ms) for s in stats[:n]]


    def decode_low_confidence(self, tokens, mask, gen_start: int, n_steps: int, block_len: int = 0,
                              stats_capacity: int = 0):
        _dev(tokens, torch.int32, "tokens"); _dev(mask, torch.uint8, "mask")
        B, L = tokens.shape
        steps = C.c_int32(0)
        stats = (StepStat * max(stats_capacity, 1))()
        _check(lib().dllm_decode_low_confidence(self._h, B, L, gen_start, _ptr(tokens), _ptr(mask), n_steps, block_len,
                                                C.byref(steps), stats if stats_capacity else None, stats_capacity),
               self._h)
        n = min(steps.value, stats_capacity)
        return steps.value, [(s.n_slow, s.n_fast, s.n_idle, s.n_commit, s.ms) for s in stats[:n]]


def _view(ptr: int, shape, dtype) -> torch.Tensor:
    """A torch view of library-owned device memory (no copy, no ownership)."""
    n = 1
    for s in shape:
        n *= s
    itemsize = torch.empty((), dtype=dtype).element_size()

    class _Holder:
        pass

    holder = _Holder()
    holder.__cuda_array_interface__ = {
        "shape": (n * itemsize,), "typestr": "|u1", "data": (ptr, False), "version": 2}
    return torch.as_tensor(holder, device="cuda").view(dtype).view(*shape)


def select(logits, tokens, mask, prev_pred, sps: Sequence[StageParams], mask_id: int, pred, conf,
           out: CommitList) -> None:
    """dllm_select: the selector alone on caller-provided bf16 logits [B, L, V]."""
    _dev(logits, torch.bfloat16, "logits"); _dev(tokens, torch.int32, "tokens"); _dev(mask, torch.uint8, "mask")
    _dev(prev_pred, torch.int32, "prev_pred"); _dev(pred, torch.int32, "pred"); _dev(conf, torch.float32, "conf")
    B, L, V = logits.shape
    assert len(sps) == B
    cl = out.c_struct()
    _check(lib().dllm_select(_stream(), _ptr(logits), B, L, V, mask_id, _ptr(tokens), _ptr(mask), _ptr(prev_pred),
                             _sp_array(sps), _ptr(pred), _ptr(conf), C.byref(cl)))


def op_linear(A, W):
    _dev(A, torch.bfloat16, "A"); _dev(W, torch.bfloat16, "W")
    M, K = A.shape
    N = W.shape[0]
    Cc = torch.empty((M, N), dtype=torch.bfloat16, device=A.device)
    _check(lib().dllm_op_linear(_stream(), _ptr(A), _ptr(W), _ptr(Cc), M, N, K))
    return Cc


def op_linear_swiglu(A, W):
    _dev(A, torch.bfloat16, "A"); _dev(W, torch.bfloat16, "W")
    M, K = A.shape
    f = W.shape[0] // 2
    out = torch.empty((M, f), dtype=torch.bfloat16, device=A.device)
    _check(lib().dllm_op_linear_swiglu(_stream(), _ptr(A), _ptr(W), _ptr(out), M, f, K))
    return out


def op_add_rmsnorm(x, partials, gain, eps: float):
    """x fp32 [M, d] is updated in place; returns h bf16 [M, d]."""
    _dev(x, torch.float32, "x"); _dev(gain, torch.bfloat16, "gain")
    M, d = x.shape
    n = 0 if partials is None else partials.shape[0]
    if partials is not None:
        _dev(partials, torch.float32, "partials")
    h = torch.empty((M, d), dtype=torch.bfloat16, device=x.device)
    _check(lib().dllm_op_add_rmsnorm(_stream(), _ptr(x), _ptr(partials), n, _ptr(gain), _ptr(h), M, d,
                                     C.c_float(eps)))
    return h


def op_linear_qkv_rope(A, W, B: int, L: int, H: int, dh: int, theta: float):
    _dev(A, torch.bfloat16, "A"); _dev(W, torch.bfloat16, "W")
    qkv = torch.empty((B * L, 3 * H * dh), dtype=torch.bfloat16, device=A.device)
    table = torch.empty((L, dh // 2, 2), dtype=torch.float32, device=A.device)
    _check(lib().dllm_op_linear_qkv_rope(_stream(), _ptr(A), _ptr(W), _ptr(qkv), _ptr(table), B, L, H, dh,
                                         C.c_float(theta)))
    return qkv


def op_pack_panels(src):
    """dllm_op_pack_panels: bf16 [rows, K] -> panel-major bf16 [K // 32, rows, 32]."""
    _dev(src, torch.bfloat16, "src")
    rows, K = src.shape
    dst = torch.empty((K // 32, rows, 32), dtype=torch.bfloat16, device=src.device)
    _check(lib().dllm_op_pack_panels(_stream(), _ptr(src), _ptr(dst), C.c_int64(rows), K))
    return dst


def op_linear_panels(A, W, M: int, N: int, K: int, swiglu: bool, a_panel_rows: int, w_panels: bool, c_panel_rows: int):
    """dllm_op_linear_panels; A / W are device tensors in whichever layout the flags say.  Returns C as
    [M, N] (or [M, N/2]; panel-major output: [N/2 // 32, c_panel_rows, 32])."""
    n_out = N // 2 if swiglu else N
    shape = (n_out // 32, c_panel_rows, 32) if c_panel_rows else (M, n_out)
    out = torch.zeros(shape, dtype=torch.bfloat16, device=A.device)
    _check(lib().dllm_op_linear_panels(_stream(), _ptr(A), _ptr(W), _ptr(out), M, N, K, int(swiglu), a_panel_rows,
                                       int(w_panels), c_panel_rows))
    return out


def op_linear_qkv_rope_static(A, W, qkv, B: int, L: int, H: int, dh: int, theta: float):
    """dllm_op_linear_qkv_rope_static: writes into the caller's qkv [B*L, 3*H*dh]; nothing is allocated."""
    _dev(A, torch.bfloat16, "A"); _dev(W, torch.bfloat16, "W"); _dev(qkv, torch.bfloat16, "qkv")
    assert qkv.shape == (B * L, 3 * H * dh)
    _check(lib().dllm_op_linear_qkv_rope_static(_stream(), _ptr(A), _ptr(W), _ptr(qkv), B, L, H, dh, C.c_float(theta)))
    return qkv


def op_rope(qkv, B: int, L: int, H: int, dh: int, theta: float):
    _dev(qkv, torch.bfloat16, "qkv")
    _check(lib().dllm_op_rope(_stream(), _ptr(qkv), B, L, H, dh, C.c_float(theta)))
    return qkv


def op_attention(qkv, B: int, L: int, H: int, dh: int):
    _dev(qkv, torch.bfloat16, "qkv")
    out = torch.empty((B * L, H * dh), dtype=torch.bfloat16, device=qkv.device)
    _check(lib().dllm_op_attention(_stream(), _ptr(qkv), _ptr(out), B, L, H, dh))
    return out
