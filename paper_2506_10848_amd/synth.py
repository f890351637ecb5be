"""Seeded synthetic inputs: model shapes, random-init weights, prompts, masks
and planted-peak logits.

This module holds no arithmetic of the method.  It only draws numbers, so that
the CPU oracle and the HIP library can be handed identical bytes.  Tensors are
drawn with a torch generator on the requested device; a tensor drawn on the GPU
is copied to the host when the oracle needs the same values.

The workloads stand in for the benchmark prompts of the paper's experiments
(generation length 256 with 256 steps; 8-shot prompts with length 1024), which
are not available here: only their shapes are kept.
"""
from __future__ import annotations

import zlib
from typing import Dict, Optional

import torch

# name -> model shape and workload.  "tiny", "medium", "llada8b" and
# "llada8b_long" are full-step workloads; "selector" is logits-only.
CONFIGS: Dict[str, dict] = {
    "tiny": dict(n_layers=2, d_model=256, n_heads=4, head_dim=64, d_ffn=688, vocab=2048,
                 mask_id=2047, rms_eps=1e-5, rope_theta=10000.0, batch=1, prompt=32, gen=64, seed=1001),
    "medium": dict(n_layers=8, d_model=1024, n_heads=16, head_dim=64, d_ffn=2816, vocab=32000,
                   mask_id=31999, rms_eps=1e-5, rope_theta=10000.0, batch=4, prompt=128, gen=256, seed=1002),
    "llada8b": dict(n_layers=32, d_model=4096, n_heads=32, head_dim=128, d_ffn=12288, vocab=126464,
                    mask_id=126336, rms_eps=1e-5, rope_theta=500000.0, batch=1, prompt=256, gen=256,
                    seed=1003),
    "llada8b_long": dict(n_layers=32, d_model=4096, n_heads=32, head_dim=128, d_ffn=12288, vocab=126464,
                         mask_id=126336, rms_eps=1e-5, rope_theta=500000.0, batch=8, prompt=512, gen=1024,
                         seed=1005),
    "selector": dict(vocab=126464, mask_id=126336, batch=16, seq=2048, peak_lo=2.0, peak_hi=8.0,
                     mask_frac=0.5, agree_frac=0.7, seed=1004),
    "selector_peaked": dict(vocab=126464, mask_id=126336, batch=16, seq=2048, peak_lo=8.0, peak_hi=18.0,
                            mask_frac=0.5, agree_frac=0.7, seed=1014),
}

MODEL_KEYS = ("n_layers", "d_model", "n_heads", "head_dim", "d_ffn", "vocab", "mask_id", "rms_eps", "rope_theta")


def model_config(cfg: dict) -> dict:
    return {k: cfg[k] for k in MODEL_KEYS}


def _gen(seed: int, name: str, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed((seed * 1_000_003 + zlib.crc32(name.encode())) & 0x7FFF_FFFF_FFFF)
    return g


def normal_bf16(shape, std: float, seed: int, name: str, device="cpu") -> torch.Tensor:
    """i.i.d. N(0, std^2) rounded to bf16; each named tensor has its own stream."""
    g = _gen(seed, name, device)
    rows = shape[0]
    out = torch.empty(shape, dtype=torch.bfloat16, device=device)
    # draw in row chunks so that the fp32 temporary stays small
    per_row = 1
    for s in shape[1:]:
        per_row *= s
    chunk = max(1, (64 << 20) // max(per_row, 1))
    for r0 in range(0, rows, chunk):
        r1 = min(rows, r0 + chunk)
        t = torch.randn((r1 - r0,) + tuple(shape[1:]), generator=g, device=device, dtype=torch.float32)
        out[r0:r1] = (t * std).to(torch.bfloat16)
    return out


def make_weights(cfg: dict, device="cpu", std: float = 0.02, gain: float = 1.0) -> dict:
    """Random-init weights: every matrix N(0, std^2) in bf16, norm gains = gain.

    Layouts: a linear map is W[N, K] (y = x W^T); wqkv rows are [q | k | v],
    each head-major; w_gate_up rows are [gate | up]."""
    d, f, V, nl, seed = cfg["d_model"], cfg["d_ffn"], cfg["vocab"], cfg["n_layers"], cfg["seed"]
    ones = lambda: torch.full((d,), gain, dtype=torch.bfloat16, device=device)
    w = dict(embed=normal_bf16((V, d), std, seed, "embed", device),
             lm_head=normal_bf16((V, d), std, seed, "lm_head", device),
             final_norm=ones(), attn_norm=[], wqkv=[], wo=[], ffn_norm=[], w_gate_up=[], w_down=[])
    for l in range(nl):
        w["attn_norm"].append(ones())
        w["wqkv"].append(normal_bf16((3 * d, d), std, seed, f"wqkv{l}", device))
        w["wo"].append(normal_bf16((d, d), std, seed, f"wo{l}", device))
        w["ffn_norm"].append(ones())
        w["w_gate_up"].append(normal_bf16((2 * f, d), std, seed, f"w_gate_up{l}", device))
        w["w_down"].append(normal_bf16((d, f), std, seed, f"w_down{l}", device))
    return w


def make_state(cfg: dict, device="cpu", batch: Optional[int] = None):
    """Prompt ids uniform over the non-mask ids followed by `gen` [MASK]
    positions.  Returns tokens int32 [B, L], mask uint8 [B, L], prev_pred int32 [B, L] (= -1)."""
    B = batch or cfg["batch"]
    P, G, V, mid = cfg["prompt"], cfg["gen"], cfg["vocab"], cfg["mask_id"]
    g = _gen(cfg["seed"], "prompt", "cpu")
    ids = torch.randint(0, V - 1, (B, P), generator=g, dtype=torch.int64)
    ids = ids + (ids >= mid).to(torch.int64)          # skip the mask id
    tokens = torch.full((B, P + G), mid, dtype=torch.int32)
    tokens[:, :P] = ids.to(torch.int32)
    mask = torch.zeros((B, P + G), dtype=torch.uint8)
    mask[:, P:] = 1
    prev = torch.full((B, P + G), -1, dtype=torch.int32)
    return tokens.to(device), mask.to(device), prev.to(device)


def make_selector_inputs(cfg: dict, device="cpu", batch: Optional[int] = None, seq: Optional[int] = None,
                         vocab: Optional[int] = None):
    """Planted-peak logits for the selector workload.

    logits[b, i, :] ~ N(0, 1) with +U(peak_lo, peak_hi) added at one seeded id
    per position, rounded to bf16; mask ~ Bernoulli(mask_frac); planted[b, i] is
    the peak's id and agree[b, i] ~ Bernoulli(agree_frac) says whether the
    previous step's prediction should be made to agree with the current arg max
    (the caller fills prev_pred from whichever arg max it computes).
    Returns logits bf16 [B, L, V], mask uint8 [B, L], planted int32 [B, L],
    agree bool [B, L], other int32 [B, L] (a seeded different id)."""
    B = batch or cfg["batch"]
    L = seq or cfg["seq"]
    V = vocab or cfg["vocab"]
    mid = min(cfg["mask_id"], V - 1)
    seed = cfg["seed"]
    g = _gen(seed, "logits", device)
    logits = torch.empty((B, L, V), dtype=torch.bfloat16, device=device)
    gc = _gen(seed, "planted", "cpu")
    planted = torch.randint(0, V - 1, (B, L), generator=gc, dtype=torch.int64)
    planted = planted + (planted >= mid).to(torch.int64)
    peak = torch.rand((B, L), generator=gc) * (cfg["peak_hi"] - cfg["peak_lo"]) + cfg["peak_lo"]
    mask = (torch.rand((B, L), generator=gc) < cfg["mask_frac"]).to(torch.uint8)
    agree = torch.rand((B, L), generator=gc) < cfg["agree_frac"]
    other = torch.randint(0, V - 1, (B, L), generator=gc, dtype=torch.int64)
    other = other + (other >= mid).to(torch.int64)
    rows_per = max(1, (256 << 20) // (V * 4))
    for b in range(B):
        for r0 in range(0, L, rows_per):
            r1 = min(L, r0 + rows_per)
            t = torch.randn((r1 - r0, V), generator=g, device=device, dtype=torch.float32)
            idx = planted[b, r0:r1].to(device)
            t[torch.arange(r1 - r0, device=device), idx] += peak[b, r0:r1].to(device)
            logits[b, r0:r1] = t.to(torch.bfloat16)
    return logits, mask.to(device), planted.to(torch.int32).to(device), agree.to(device), \
        other.to(torch.int32).to(device)
