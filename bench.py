"""Benchmark of the denoising step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload llada8b]

A "step" is one pass of the whole hot path (forward over all positions, row
phase, selection, transition) through dllm_step on a synthetic batch that is
resident in HBM.  Prints ONE JSON line.  The headline value is tokens processed
per denoising step per second, B * L / t_step, on the LLaDA-8B-shaped workload
(batch 1, 256 prompt + 256 masked positions).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0     # MI355X dense bf16
HBM_PEAK_GBS = 8000.0              # MI355X HBM3E


def step_flops(cfg, B, L, vocab_rows):
    """Executed flops of one step: layer GEMMs 2*M*nL*(4d^2 + 3df), attention 4*nL*B*L^2*d, and the
    vocabulary projection 2*rows*d*V over the rows the selector reads (the windows)."""
    d, f, V, nl = cfg["d_model"], cfg["d_ffn"], cfg["vocab"], cfg["n_layers"]
    M = B * L
    return 2.0 * M * nl * (4 * d * d + 3 * d * f) + 2.0 * vocab_rows * d * V + 4.0 * nl * B * L * L * d


def gemm_kernel_name(b, epi, M, N, K, what):
    p = b.gemm_plan(epi, M, N, K)
    kern = "gemm_il_kernel" if p["async_copy"] else "gemm_reg_kernel"
    return (f"{kern}<{p['bm']}x{p['bn']} tile, {p['waves_m']}x{p['waves_n']} waves, BK {p['bk']}, {p['stages']} stages, "
            f"{p['splits']} K split(s), {what}>")


def sustained_mfma(b, torch):
    """dllm_debug_mfma_rate: 256 workgroups x 4 waves x 40000 x 8 MFMAs (about 6 ms), best of 3, per operand kind."""
    g = torch.Generator(device="cuda"); g.manual_seed(7)
    sink = torch.empty(256 * 256, dtype=torch.float32, device="cuda")
    out = {"kernel": "v_mfma_f32_32x32x16_bf16 on register operands, 8 independent accumulator tiles per wave, "
                     "256 workgroups of 4 waves, 40000 iterations"}
    for name, ops in (("random_operands_TFLOPs", torch.randn(1 << 19, device="cuda", generator=g).to(torch.bfloat16)),
                      ("zero_operands_TFLOPs", torch.zeros(1 << 19, dtype=torch.bfloat16, device="cuda"))):
        best = None
        for _ in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            flop = b.debug_mfma_rate(ops, sink, 256, 40000)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1)
            best = ms if best is None or ms < best else best
        out[name] = flop / (best * 1e-3) / 1e12
    return out


def long_batch_extra(b, synth, torch, weights, mc):
    """B = 8, L = 512 + 1024 on the same LLaDA-8B-shaped weights: one timed step (slow stage over the whole
    generated region) and a SlowFast decode capped at a stated number of steps with thresholds at quantiles
    of the first step's confidences, reporting per-stage step time and tokens committed per step."""
    cfg = synth.CONFIGS["llada8b_long"]
    B, P, G = cfg["batch"], cfg["prompt"], cfg["gen"]
    L = P + G
    tokens0, mask0, prev0 = synth.make_state(cfg, device="cuda")
    model = b.Model(mc, weights, B, L)
    out = b.CommitList(B, L)
    sps = [b.stage_params(b.STAGE_SLOW, P, L - 1, 1, 0.1, 0.9, 1, P, L) for _ in range(B)]
    tokens, mask, prev = tokens0.clone(), mask0.clone(), prev0.clone()
    model.step(tokens, mask, prev, sps, out)                      # warm-up
    n = 3
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
    torch.cuda.synchronize()
    evs[0].record()
    for i in range(n):
        model.step(tokens, mask, prev, sps, out)
        evs[i + 1].record()
    torch.cuda.synchronize()
    step_ms = sorted(evs[i].elapsed_time(evs[i + 1]) for i in range(n))[n // 2]
    flops = step_flops(mc, B, L, vocab_rows=B * G)
    conf0 = model.debug_rows(B * L)[1].view(B, L)[mask.bool()].float()
    tau_min_q, tau_high_q = float(conf0.quantile(0.5)), float(conf0.quantile(0.9))
    cap = 24
    tokens, mask = tokens0.clone(), mask0.clone()
    dp = b.DecodeParams(cap, 8, 2, 1, 1, 0, 1.0, tau_min_q, tau_high_q)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    steps, st = model.decode(tokens, mask, P, dp, stats_capacity=cap)
    t_dec = time.perf_counter() - t0
    committed = B * G - int(mask.sum())
    slow = [s for s in st if s[0] > 0 and s[1] == 0]
    fast = [s for s in st if s[1] > 0 and s[0] == 0]
    mixed = [s for s in st if s[0] > 0 and s[1] > 0]
    mean = lambda xs: sum(xs) / max(len(xs), 1)
    res = {"workload": f"llada8b_long: batch {B}, {P} prompt + {G} masked (L={L}), same weights",
           "step_ms_median_of_3": step_ms, "tokens_per_s": B * L / (step_ms * 1e-3), "step_tflops": flops / 1e12,
           "step_mfma_frac": flops / (step_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
           "gate_up_kernel": gemm_kernel_name(b, 1, B * L, 2 * mc["d_ffn"], mc["d_model"], "SwiGLU"),
           "decode_capped": {
               "max_steps": cap, "steps": steps, "seconds": t_dec, "tokens_committed": committed,
               "committed_tokens_per_s": committed / t_dec,
               "slow_only_steps": len(slow), "fast_only_steps": len(fast), "mixed_steps": len(mixed),
               "slow_step_ms": mean([s[4] for s in slow]), "fast_step_ms": mean([s[4] for s in fast]),
               "mixed_step_ms": mean([s[4] for s in mixed]),
               "tokens_per_slow_step": mean([s[3] for s in slow]), "tokens_per_fast_step": mean([s[3] for s in fast]),
               "tokens_per_mixed_step": mean([s[3] for s in mixed]),
               "params": f"N capped at {cap} steps; tau_min = median ({tau_min_q:.3e}), tau_high = 90th percentile "
                         f"({tau_high_q:.3e}) of the first step's confidences, K_max 8, W_hist 2, sigma2 1.0, "
                         "k_slow=k_fast=1, conv_mode 0; a step is 'slow only' / 'fast only' / 'mixed' by the stages "
                         "of the 8 sequences during it"}}
    model.close()
    return res


def to_bits(t):
    import torch
    return t.detach().cpu().contiguous().view(torch.uint16).numpy()


def cpu_baseline_step(cfg, weights, tokens):
    """The oracle, as it stands, on a bounded sample of the same step: 1 of the
    n_layers layers plus the vocabulary projection and row phase of 128 of the
    B*L rows; scaled linearly to the whole step."""
    import numpy as np
    import oracle
    from paper_2506_10848_amd import synth
    B, L = tokens.shape
    M = B * L
    n_rows = min(128, M)
    rows = np.linspace(0, M - 1, n_rows).astype(np.int32)
    nl = cfg["n_layers"]
    tok = tokens.cpu().numpy()

    def weights_for(layers):
        w = {k: to_bits(weights[k]) for k in ("embed", "lm_head", "final_norm")}
        for k in ("attn_norm", "wqkv", "wo", "ffn_norm", "w_gate_up", "w_down"):
            w[k] = [to_bits(weights[k][l]) for l in range(layers)]
        return w

    mc = synth.model_config(cfg)
    n_sample = min(4, nl)                    # layers in the sample
    w1 = weights_for(n_sample)
    t0 = time.perf_counter()
    lg = oracle.forward(dict(mc, n_layers=0), dict(w1, **{k: [] for k in
                        ("attn_norm", "wqkv", "wo", "ffn_norm", "w_gate_up", "w_down")}), tok, rows=rows)
    oracle.row_phase(oracle.round_to_bf16(lg), mc["mask_id"])
    t_head = time.perf_counter() - t0
    t0 = time.perf_counter()
    oracle.forward(dict(mc, n_layers=n_sample), w1, tok, rows=rows)
    t_one = time.perf_counter() - t0
    t_layer = max(t_one - t_head, 0.0) / max(n_sample, 1)
    t_step = nl * t_layer + t_head * (M / n_rows)
    return dict(value=M / t_step, unit="tokens/s", cores=oracle.threads(), kind="oracle",
                sample=f"{n_sample} of {nl} layers over all {M} rows ({t_layer:.2f} s each) + vocabulary projection and row phase "
                       f"of {n_rows} of {M} rows ({t_head:.2f} s), scaled linearly to a whole step ({t_step:.1f} s)")


def cpu_baseline_selector(sample):
    """The oracle's row phase on the sampled rows of the selector workload: its rate on the host cores,
    and the check of the library's predictions and confidences for those rows."""
    import numpy as np
    import oracle
    t0 = time.perf_counter()
    o_pred, o_conf = oracle.row_phase(sample["logits_bits"], sample["mask_id"])
    dt = time.perf_counter() - t0
    same = bool(np.array_equal(o_pred, sample["pred"]))
    rel = float((np.abs(sample["conf"].astype(np.float64) - o_conf) / o_conf).max())
    assert same and rel <= 1e-3, f"selector rows differ from the oracle: predictions equal {same}, confidence error {rel}"
    n = len(o_pred)
    return dict(rows_per_s=n / dt, cores=oracle.threads(), kind="oracle", sample=f"{n} seeded rows of the workload ({dt:.3f} s)",
                check=f"{n} sampled rows: predictions identical to the oracle's, confidences within {rel:.1e} (bar 1e-3)")


def selector_extra(b, synth, torch):
    """Selector microbenchmark (16 x 2048 x 126464 bf16 logits, 50 % masked rows):
    achieved HBM bandwidth on the algorithmic bytes (masked rows only)."""
    cfg = synth.CONFIGS["selector"]
    B, L, V = cfg["batch"], cfg["seq"], cfg["vocab"]
    logits, mask, planted, agree, other = synth.make_selector_inputs(cfg, "cuda")
    tokens = torch.full((B, L), cfg["mask_id"], dtype=torch.int32, device="cuda")
    prev = torch.where(agree, planted, other).to(torch.int32)
    pred = torch.empty((B, L), dtype=torch.int32, device="cuda")
    conf = torch.empty((B, L), dtype=torch.float32, device="cuda")
    out = b.CommitList(B, L)
    sps = [b.stage_params(b.STAGE_SLOW, 0, L - 1, 1, 0.1, 0.9, 1, 0, L) for _ in range(B)]
    n_masked = int(mask.sum())
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    times = []
    for it in range(8):
        m = mask.clone(); p = prev.clone(); t = tokens.clone()
        torch.cuda.synchronize()
        ev[0].record()
        b.select(logits, t, m, p, sps, cfg["mask_id"], pred, conf, out)
        ev[1].record()
        torch.cuda.synchronize()
        times.append(ev[0].elapsed_time(ev[1]))
    ms = sorted(times[2:])[len(times[2:]) // 2]
    bytes_alg = n_masked * V * 2.0

    def timed(sp_list, mask_src):
        ts = []
        for it in range(5):
            m = mask_src.clone(); p = prev.clone(); t = tokens.clone()
            torch.cuda.synchronize()
            ev[0].record()
            b.select(logits, t, m, p, sp_list, cfg["mask_id"], pred, conf, out)
            ev[1].record()
            torch.cuda.synchronize()
            ts.append(ev[0].elapsed_time(ev[1]))
        return sorted(ts[1:])[len(ts[1:]) // 2]

    # fast stage over the first half of every sequence; and the slow stage with every row masked
    fast = [b.stage_params(b.STAGE_FAST, 0, L // 2 - 1, 1, 0.1, 0.9, 1, 0, L) for _ in range(B)]
    fast_ms = timed(fast, mask)
    fast_rows = int(mask[:, :L // 2].sum())
    all_ms = timed(sps, torch.ones_like(mask))
    # a sample of the rated rows (their logits, and what the last timed call left for them) for the check
    # against the oracle, which the CPU-baseline leg runs and times
    idx = torch.nonzero(torch.ones_like(mask).view(-1)).view(-1)
    idx = idx[torch.randperm(idx.numel(), generator=torch.Generator().manual_seed(7))[:256].to(idx.device)]
    sample = dict(rows=idx.cpu().numpy(), logits_bits=logits.view(B * L, V)[idx].cpu().view(torch.uint16).numpy(),
                  pred=pred.view(-1)[idx].cpu().numpy(), conf=conf.view(-1)[idx].cpu().numpy(), mask_id=cfg["mask_id"])
    del logits
    return dict(sample=sample, workload="selector 16x2048x126464 bf16, 50% masked, slow stage k=1", ms=ms,
                masked_rows=n_masked, achieved_GBs=bytes_alg / ms / 1e6, frac_hbm=bytes_alg / ms / 1e6 / HBM_PEAK_GBS,
                fast_stage_first_half={"ms": fast_ms, "masked_rows": fast_rows,
                                       "achieved_GBs": fast_rows * V * 2.0 / fast_ms / 1e6},
                all_rows_masked={"ms": all_ms, "rows": B * L, "achieved_GBs": B * L * V * 2.0 / all_ms / 1e6})


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="llada8b", choices=["llada8b", "llada8b_long", "medium", "tiny"])
    ap.add_argument("--no-extras", action="store_true", help="skip decode / selector / cpu baseline legs")
    ap.add_argument("--selector-only", action="store_true",
                    help="run only the selector workload (16 x 2048 x 126464 logits) and print its line")
    ap.add_argument("--pmc-copy", action="store_true",
                    help="also launch one plain elementwise copy of 1 GiB (calibrates HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no sharding, no collectives); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2506_10848_amd import binding as b
    from paper_2506_10848_amd import synth

    b.lib()  # fails loudly if the HIP library is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.selector_only:
        sel = selector_extra(b, synth, torch)
        if args.pmc_copy:
            src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
            dst = torch.empty_like(src)
            torch.mul(src, 1.0, out=dst)
            torch.cuda.synchronize()
        sample = sel.pop("sample")
        sel["cpu_baseline"] = cpu_baseline_selector(sample)
        print(json.dumps({"metric": "selector rows/s (fused softmax max/argmax + SlowFast commit)",
                          "value": sel["masked_rows"] / (sel["ms"] * 1e-3), "unit": "masked rows/s", "n_gpus": 1,
                          "dtype": "bf16 logits, fp32 arithmetic", "data": "synthetic",
                          "config": {"workload": sel["workload"]},
                          "roofline": {"kernel": "row_phase_kernel", "bound": "hbm", "achieved": sel["achieved_GBs"],
                                       "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": sel["frac_hbm"], "traffic": None},
                          "ms": sel["ms"], "fast_stage_first_half": sel["fast_stage_first_half"],
                          "all_rows_masked": sel["all_rows_masked"], "cpu_baseline": sel["cpu_baseline"]}))
        return
    cfg = synth.CONFIGS[args.workload]
    mc = synth.model_config(cfg)
    B, P, G = cfg["batch"], cfg["prompt"], cfg["gen"]
    L = P + G
    weights = synth.make_weights(cfg, device="cuda")
    tokens0, mask0, prev0 = synth.make_state(cfg, device="cuda")
    model = b.Model(mc, weights, B, L)
    out = b.CommitList(B, L)
    # first steps of a decode: slow stage over the whole generated region, k_slow = 1
    sps = [b.stage_params(b.STAGE_SLOW, P, L - 1, 1, 0.1, 0.9, 1, P, L) for _ in range(B)]
    # Every step commits one token per sequence, so after G steps nothing is masked: the state is put back to the
    # initial one before that happens (three device copies of B * L elements; only runs longer than G steps do it).
    tokens, mask, prev = tokens0.clone(), mask0.clone(), prev0.clone()
    since_reset, state_resets = 0, 0

    def next_step():
        nonlocal since_reset, state_resets
        if since_reset == G:
            tokens.copy_(tokens0); mask.copy_(mask0); prev.copy_(prev0)
            since_reset, state_resets = 0, state_resets + 1
        model.step(tokens, mask, prev, sps, out)
        since_reset += 1

    for _ in range(args.warmup):
        next_step()
    torch.cuda.synchronize()
    model.profile_begin(args.steps * mc["n_layers"])
    # the library works on the stream that is current here, so these events bracket its steps
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    evs[0].record()
    for i in range(args.steps):
        next_step()
        evs[i + 1].record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    k_ms, k_launches = model.profile_end()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    per_step = sorted(evs[i].elapsed_time(evs[i + 1]) for i in range(args.steps))
    ms_median = per_step[len(per_step) // 2]
    assert int(mask.sum()) == B * G - B * since_reset, "every step must commit one token per sequence"

    flops = step_flops(mc, B, L, vocab_rows=B * G)          # slow-stage window = the whole generated region
    k_flops = 2.0 * B * L * mc["d_model"] * 2 * mc["d_ffn"]          # one gate/up GEMM launch
    k_avg_ms = k_ms / max(k_launches, 1)
    achieved = k_flops / (k_avg_ms * 1e-3) / 1e12
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "traffic_gateup_gemm.json")
    if args.workload == "llada8b" and os.path.exists(tpath):
        traffic = json.load(open(tpath)).get("traffic_bytes_per_launch")

    result = {
        "metric": "tokens/s per denoising step (B*L/t_step), LLaDA-8B shape L=512" if args.workload == "llada8b"
                  else f"tokens/s per denoising step (B*L/t_step), workload {args.workload}",
        "value": B * L / (ms_per_step * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{args.workload}: {mc['n_layers']} layers d={mc['d_model']} H={mc['n_heads']}x"
                               f"{mc['head_dim']} ffn={mc['d_ffn']} V={mc['vocab']}, batch {B}, {P} prompt + {G} "
                               f"masked (L={L}), seeded N(0,0.02) bf16 weights, slow stage k_slow=1",
                   "global_batch": B, "seq_len": L},
        "ms_per_step_median_hip_events": ms_median,
        "state_resets": state_resets,
        "step_tflops": flops / 1e12,
        "step_mfma_frac": flops / (ms_per_step * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
        "roofline": {"kernel": gemm_kernel_name(b, 1, B * L, 2 * mc["d_ffn"], mc["d_model"], "SwiGLU")
                               + " (gate/up projection, one launch per layer; the plan the library reports for this shape)",
                     "bound": "mfma", "achieved": achieved, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / MFMA_BF16_PEAK_TFLOPS, "traffic": traffic,
                     "traffic_source": None if traffic is None else
                     "profiles/step_llada8b_hbm_traffic.txt (rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE runs of this "
                     "command, scaled by a 1 GiB copy); not measured in this run",
                     "avg_launch_ms": k_avg_ms, "launches": k_launches, "flops_per_launch": k_flops},
        "gemm_plans": {name: b.gemm_plan(epi, m, n, k) for name, epi, m, n, k in [
            ("qkv_rope", 4 if mc["head_dim"] == 128 else 3, B * L, 3 * mc["d_model"], mc["d_model"]),
            ("o_proj", 2, B * L, mc["d_model"], mc["d_model"]),
            ("gate_up_swiglu", 1, B * L, 2 * mc["d_ffn"], mc["d_model"]),
            ("down", 2, B * L, mc["d_model"], mc["d_ffn"]),
            ("vocab_rowstats", 5, B * G, mc["vocab"], mc["d_model"])]},
    }

    # What the matrix cores sustain when nothing else runs (registers only, one wave per SIMD on every CU): with
    # random operands the power limit sets it well below the nominal peak; all-zero operands reach the peak.
    result["roofline"]["sustained_mfma"] = sustained_mfma(b, torch)
    result["roofline"]["frac_of_sustained_random"] = achieved / result["roofline"]["sustained_mfma"]["random_operands_TFLOPs"]

    if args.pmc_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")          # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        torch.mul(src, 1.0, out=dst)
        torch.cuda.synchronize()
        del src, dst

    if not args.no_extras:
        # end-to-end generated tokens/s of a full SlowFast decode (paper's TPS definition)
        tokens, mask = tokens0.clone(), mask0.clone()
        dp = b.DecodeParams(10 ** 6, 8, 2, 1, 1, 1, 1.0, 0.1, 0.9)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        steps, _ = model.decode(tokens, mask, P, dp)
        t_dec = time.perf_counter() - t0
        result["decode"] = {"generated_tokens_per_s": B * G / t_dec, "steps": steps, "seconds": t_dec,
                            "params": "tau_min 0.1, tau_high 0.9, K_max 8, W_hist 2, sigma2 1.0, k_slow=k_fast=1, conv_mode 1"}
        # the baseline sampler (low-confidence remasking, one step per generated token), same kernels
        tokens, mask = tokens0.clone(), mask0.clone()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        steps_lc, _ = model.decode_low_confidence(tokens, mask, P, G, 0)
        t_lc = time.perf_counter() - t0
        result["decode_low_confidence"] = {"generated_tokens_per_s": B * G / t_lc, "steps": steps_lc, "seconds": t_lc,
                                           "params": f"N = {G} steps, one block"}
        # random-init confidences sit near 1/V, far below the paper's thresholds; to see the fast stage
        # commit spans, the thresholds are put at quantiles of the first step's confidences (labelled run)
        tokens, mask, prev = tokens0.clone(), mask0.clone(), prev0.clone()
        model.step(tokens, mask, prev, sps, out)
        torch.cuda.synchronize()
        conf0 = model.debug_rows(B * L)[1].view(B, L)[mask0.bool()].float()
        tau_min_q, tau_high_q = float(conf0.quantile(0.5)), float(conf0.quantile(0.9))
        tokens, mask = tokens0.clone(), mask0.clone()
        dpq = b.DecodeParams(10 ** 6, 8, 2, 1, 1, 0, 1.0, tau_min_q, tau_high_q)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        steps_q, st_q = model.decode(tokens, mask, P, dpq, stats_capacity=B * G)
        t_q = time.perf_counter() - t0
        slow_ms = [s[4] for s in st_q if s[0] > 0 and s[1] == 0]
        fast_ms = [s[4] for s in st_q if s[1] > 0 and s[0] == 0]
        fast_commits = [s[3] for s in st_q if s[1] > 0 and s[0] == 0]
        result["decode_quantile_thresholds"] = {
            "generated_tokens_per_s": B * G / t_q, "steps": steps_q, "seconds": t_q,
            "steps_vs_low_confidence": steps_q / max(steps_lc, 1),
            "slow_steps": len(slow_ms), "fast_steps": len(fast_ms),
            "slow_step_ms": sum(slow_ms) / max(len(slow_ms), 1), "fast_step_ms": sum(fast_ms) / max(len(fast_ms), 1),
            "tokens_per_fast_step": sum(fast_commits) / max(len(fast_commits), 1),
            "params": f"tau_min = median ({tau_min_q:.3e}), tau_high = 90th percentile ({tau_high_q:.3e}) of the first "
                      "step's confidences, K_max 8, W_hist 2, sigma2 1.0, k_slow=k_fast=1, conv_mode 0"}
        # fast-stage steps over a 32-token span, without and with out-of-span caching: every masked
        # position right of the span is cached (random-init confidences are all below tau_min = 0.1)
        span = min(32, G)
        fsp = [b.stage_params(b.STAGE_FAST, P, P + span - 1, 1, 0.1, 0.9, 0, P, L) for _ in range(B)]
        import numpy as np
        skip = np.zeros((B, L), np.uint8)
        skip[:, P + span:] = 1

        def timed_steps(fn, n=6):
            tk, mk, pv = tokens0.clone(), mask0.clone(), prev0.clone()
            fn(tk, mk, pv)                       # warm-up (and, for the cached variants, the cache fill)
            torch.cuda.synchronize()
            t = time.perf_counter()
            for _ in range(n):
                fn(tk, mk, pv)
            torch.cuda.synchronize()
            return (time.perf_counter() - t) * 1e3 / n

        plain_ms = timed_steps(lambda tk, mk, pv: model.step(tk, mk, pv, fsp, out))
        refresh_ms = timed_steps(lambda tk, mk, pv: model.step_cached(tk, mk, pv, fsp, [b.CACHE_REFRESH] * B, None, out))
        reuse_ms = timed_steps(lambda tk, mk, pv: model.step_cached(tk, mk, pv, fsp, [b.CACHE_REUSE] * B, skip, out))
        # with the prompt cached as well (prompt caching between refresh steps) only the span is recomputed
        skip_all = skip.copy()
        skip_all[:, :P] = 1
        span_only_ms = timed_steps(lambda tk, mk, pv: model.step_cached(tk, mk, pv, fsp, [b.CACHE_REUSE] * B, skip_all, out))
        # a slow-stage step that leaves the prompt out (rates the whole generated region)
        pskip = np.zeros((B, L), np.uint8)
        pskip[:, :P] = 1
        slow_prompt_cached_ms = timed_steps(lambda tk, mk, pv: model.step_cached(tk, mk, pv, sps, [b.CACHE_REUSE] * B, pskip, out))
        result["fast_step_out_of_span_cache"] = {
            "span": span, "rows_total": B * L, "rows_recomputed_in_reuse_step": int(B * L - skip.sum()),
            "plain_fast_step_ms": plain_ms, "refresh_step_ms": refresh_ms, "reuse_step_ms": reuse_ms,
            "reuse_step_prompt_cached_ms": span_only_ms, "rows_recomputed_prompt_cached": int(B * L - skip_all.sum()),
            "slow_step_prompt_cached_ms": slow_prompt_cached_ms, "slow_step_rows_recomputed": int(B * L - pskip.sum()),
            "note": "reuse steps read cached keys/values for the positions they leave out; the first timed call of "
                    "each variant follows a cache-filling call"}
        # the timed step takes the greedy decode inside the vocabulary projection; the same step through
        # bf16 logits and the separate row kernel, for comparison
        model.set_fused_selector(False)
        logits_path_ms = timed_steps(lambda tk, mk, pv: model.step(tk, mk, pv, sps, out))
        model.set_fused_selector(True)
        fused_ms = timed_steps(lambda tk, mk, pv: model.step(tk, mk, pv, sps, out))
        result["slow_step_selector_paths"] = {"fused_into_vocab_projection_ms": fused_ms,
                                              "through_bf16_logits_ms": logits_path_ms, "rows_rated": B * G}
        # SlowFast decode with both caches on (thresholds as in decode_quantile_thresholds)
        tokens, mask = tokens0.clone(), mask0.clone()
        dpc = b.DecodeParams(10 ** 6, 8, 2, 1, 1, 0, 1.0, tau_min_q, tau_high_q, 1, 8)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        steps_c, st_c = model.decode(tokens, mask, P, dpc, stats_capacity=B * G)
        t_c = time.perf_counter() - t0
        result["decode_quantile_thresholds_cached"] = {
            "generated_tokens_per_s": B * G / t_c, "steps": steps_c, "seconds": t_c,
            "mean_step_ms": sum(x[4] for x in st_c) / max(len(st_c), 1),
            "params": "as decode_quantile_thresholds, plus out_of_span_cache = 1 and prompt_cache_interval = 8"}
        # all three caches, intervals as in the paper's Table 4 (K_p = 100, K_r = 5)
        tokens, mask = tokens0.clone(), mask0.clone()
        dpa = b.DecodeParams(10 ** 6, 8, 2, 1, 1, 0, 1.0, tau_min_q, tau_high_q, 1, 100, 5)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        steps_a, st_a = model.decode(tokens, mask, P, dpa, stats_capacity=B * G)
        t_a = time.perf_counter() - t0
        result["decode_quantile_thresholds_all_caches"] = {
            "generated_tokens_per_s": B * G / t_a, "steps": steps_a, "seconds": t_a,
            "mean_step_ms": sum(x[4] for x in st_a) / max(len(st_a), 1),
            "params": "as decode_quantile_thresholds, plus out_of_span_cache = 1, prompt_cache_interval = 100, "
                      "response_cache_interval = 5"}
        result["cpu_baseline"] = cpu_baseline_step(mc, weights, tokens0)
        model.close()
        del model
        torch.cuda.empty_cache()
        if args.workload == "llada8b":
            result["long_batch"] = long_batch_extra(b, synth, torch, weights, mc)
        del weights
        torch.cuda.empty_cache()
        result["selector"] = selector_extra(b, synth, torch)
        result["selector"]["cpu_baseline"] = cpu_baseline_selector(result["selector"].pop("sample"))
    print(json.dumps(result))


if __name__ == "__main__":
    main()
