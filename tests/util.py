"""Helpers shared by the tests: tensor <-> bf16 bit-pattern conversions and the
comparison rules used for parity."""
import numpy as np
import torch


def bits(t: torch.Tensor) -> np.ndarray:
    """bf16 tensor (any device) -> uint16 numpy array of its bit patterns."""
    assert t.dtype == torch.bfloat16
    return t.detach().cpu().contiguous().view(torch.uint16).numpy()


def weights_bits(w: dict) -> dict:
    return {k: ([bits(a) for a in v] if isinstance(v, list) else bits(v)) for k, v in w.items()}


def from_bits(a: np.ndarray, device="cpu") -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).view(torch.bfloat16).to(device)


class OraclePredictor:
    """The mask predictor + row phase of the oracle as the callable the oracle's
    decode loops want; `.cached` is the variant used with out-of-span caching.
    Keeps the last call's logits (float64, NaN where not computed) for the tests."""

    def __init__(self, mc: dict, wbits: dict, B: int, L: int):
        import oracle
        self.o, self.mc, self.wb, self.B, self.L = oracle, mc, wbits, B, L
        self.cache = oracle.KVCache(mc, B, L)
        self.last = {}
        self.recomputed = []          # rows recomputed by every call

    def _finish(self, logits_rows, rows, active):
        B, L, V = self.B, self.L, self.mc["vocab"]
        full = np.full((B * L, V), np.nan)
        full[rows] = logits_rows
        lb = self.o.round_to_bf16(np.nan_to_num(full))
        pred, conf = self.o.row_phase(lb, self.mc["mask_id"], active.reshape(-1))
        self.last = dict(logits=full, pred=pred.reshape(B, L), conf=conf.reshape(B, L))
        return self.last["pred"], self.last["conf"]

    def __call__(self, tokens, active):
        rows = np.arange(self.B * self.L)
        self.recomputed.append(self.B * self.L)
        return self._finish(self.o.forward(self.mc, self.wb, tokens), rows, active)

    def cached(self, tokens, active, skip):
        rows = np.flatnonzero(skip.reshape(-1) == 0)
        self.recomputed.append(len(rows))
        return self._finish(self.o.forward_cached(self.mc, self.wb, tokens, self.cache, rows, skip), rows, active)
