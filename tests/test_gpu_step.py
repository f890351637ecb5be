"""GPU parity of the whole denoising step (dllm_step) and of the decode loop
(dllm_decode) against the oracle.

Lock-step protocol: the oracle free-runs a SlowFast decode; before every one of
its steps the oracle's own state (tokens, mask, prev_pred, stage parameters) is
uploaded and the library takes one step from it.  Both sides therefore start
every step from identical bytes that come from the oracle side only.

Every step is checked twice.

(i) Against the oracle's own prediction.  The two sides compute their logits
independently (fp64 vs bf16 MFMA), so a decision is compared bit-exactly only
where the oracle's decision survives the confidence perturbation MEASURED in
that step (the largest relative difference between the library's and the
oracle's confidences over the rated rows) and, for a prediction, where the
oracle's top-2 logit gap exceeds twice the logit error measured in that step;
everything else is checked for validity, and the share of decisions that end
up exempt is bounded by every test.

(ii) Against the oracle's rule on the library's own numbers.  The library's
bf16 logits go through the oracle's row phase (predictions bit-exact,
confidences to 2e-5), and the library's predictions and confidences go
through the oracle's selection rule: commit list, committed tokens, e_cand,
first_masked, masks left, and the whole state after the transition must be
identical, with no exemption."""
import math

import numpy as np
import pytest
import torch

import oracle
from oracle import slowfast as sf
from paper_2506_10848_amd import synth
from util import OraclePredictor, bits, weights_bits

pytestmark = pytest.mark.gpu
DEV = "cuda"

LOGIT_NORMWISE = 1e-2     # asserted here; inside the 2e-2 bar


def binding():
    from paper_2506_10848_amd import binding as b
    b.lib()
    b.reload_env()          # the environment switches a test may have set (or a finished test has restored)
    return b


class Robust:
    """Which decisions of the oracle are safe against confidence errors of
    +-delta (relative) and against the predictions that came out differently
    (same[i] false; each such difference is checked separately to sit on a near-tie)."""

    def __init__(self, sp, mask, conf, pred, prev, same, delta):
        lo, hi = sp.window()
        self.sp = sp
        self.cands = [i for i in range(max(lo, 0), min(hi, len(mask) - 1) + 1) if mask[i]]
        self.c = {i: float(conf[i]) for i in self.cands}
        self.pred_ok = {i: bool(same[i]) for i in self.cands}
        self.conv = {i: int(pred[i]) == int(prev[i]) for i in self.cands}
        self.d = delta

    def topk_sets(self, k):
        must, never = set(), set()
        for i in self.cands:
            beat_me = sum(1 for j in self.cands if j != i and self.c[j] * (1 + self.d) >= self.c[i] * (1 - self.d))
            surely_above = sum(1 for j in self.cands if j != i and self.c[j] * (1 - self.d) > self.c[i] * (1 + self.d))
            if beat_me < k:
                must.add(i)
            if surely_above >= k:
                never.add(i)
        return must, never, min(k, len(self.cands))

    def decide(self):
        """Returns (must_commit, never_commit, exact_count or None)."""
        sp, d = self.sp, self.d
        if sp.stage == sf.IDLE or not self.cands:
            return set(), set(self.cands), 0
        if sp.stage == sf.SLOW:
            return self.topk_sets(sp.top_k)
        conv_sure = lambda i: sp.conv_mode == 0 or (self.pred_ok[i] and self.conv[i])
        conv_never = lambda i: sp.conv_mode == 1 and self.pred_ok[i] and not self.conv[i]
        sure = {i for i in self.cands if self.c[i] * (1 - d) > sp.tau_high_conf and conv_sure(i)}
        maybe = {i for i in self.cands if self.c[i] * (1 + d) > sp.tau_high_conf and not conv_never(i)}
        if sure:
            return sure, set(self.cands) - maybe, None
        if not maybe:
            return self.topk_sets(sp.top_k)
        return set(), set(), None

    def e_cand(self):
        """(value, robust?)"""
        above = [i for i in self.cands if self.c[i] > self.sp.tau_min_conf]
        val = max(above) if above else -1
        right = [i for i in self.cands if i >= (val if val >= 0 else -1)]
        robust = all(abs(self.c[i] - self.sp.tau_min_conf) > self.d * self.sp.tau_min_conf for i in right)
        return val, robust


class SlowFastDriver:
    """Stage parameters of every step from the oracle's Algorithm 1 controllers."""

    def __init__(self, B, P, L, params):
        self.ctl = [sf.Controller(P, L, params) for _ in range(B)]
        self.P, self.L, self.p = P, L, params
        self.n = 0

    def also(self):
        """Prompt / response caching: positions the sequences leave out in the coming step (None: both off)."""
        return sf.interval_skip(self.p, self.n, self.sps, self.P, self.L, self.L)

    def next(self, mask):
        sps = []
        for s, c in enumerate(self.ctl):
            sp = c.next_params(mask[s])
            sps.append(sp if sp is not None else
                       sf.StageParams(sf.IDLE, 0, -1, 1, self.p.tau_min_conf, self.p.tau_high_conf, self.p.conv_mode,
                                      self.P, self.L))
        self.sps = sps
        return sps

    def observe(self, sps, res, mask):
        self.n += 1
        for s, c in enumerate(self.ctl):
            if sps[s].stage != sf.IDLE:
                c.observe(res[s][3], res[s][4], mask[s], res[s][6])

    def skip(self):
        return [c.skip for c in self.ctl]


class LowConfidenceDriver:
    """Stage parameters of the baseline sampler (Section 3.1): block by block, the
    schedule's number of new tokens per step, taken from the oracle's schedule function."""

    def __init__(self, B, P, L, n_steps, block_len):
        G = L - P
        self.blocks = [(P + i * block_len, P + (i + 1) * block_len) for i in range(G // block_len)]
        self.per_block = n_steps // len(self.blocks)
        self.plan = [(lo, hi, j) for lo, hi in self.blocks for j in range(1, self.per_block + 1)]
        self.P, self.at = P, 0

    def next(self, mask):
        while self.at < len(self.plan):
            lo, hi, j = self.plan[self.at]
            self.at += 1
            target = sf.n_unmasked_target(hi - lo, self.per_block, j)
            sps = []
            for s in range(mask.shape[0]):
                k = target - ((hi - lo) - int(mask[s, lo:hi].sum()))
                sps.append(sf.StageParams(sf.SLOW, lo, hi - 1, k, 0.0, 1.0, 0, self.P, hi) if k >= 1 else
                           sf.StageParams(sf.IDLE, 0, -1, 1, 0.0, 1.0, 0, self.P, hi))
            if any(sp.stage != sf.IDLE for sp in sps):
                return sps
        return [sf.StageParams(sf.IDLE, 0, -1, 1, 0.0, 1.0, 0, self.P, self.P)] * mask.shape[0]

    def observe(self, sps, res, mask):
        pass


class CachedSpanDriver:
    """Fast stages over consecutive spans of `span` positions with out-of-span caching: a refresh
    step, then reuse steps (one token per step: tau_high is out of reach) until the span is clean.
    The cached set follows the paper's rule on the oracle's confidences of the refresh step."""

    def __init__(self, B, P, L, span, tau_min):
        self.P, self.L, self.span, self.tau_min = P, L, span, tau_min
        self.s, self.fresh = P, True
        self._skip = [np.zeros(L, np.uint8) for _ in range(B)]

    def _params(self, stage, mode):
        e = min(self.s + self.span, self.L) - 1
        return sf.StageParams(stage, self.s, e, 1, self.tau_min, 2.0, 0, self.P, self.L, mode)

    def next(self, mask):
        while self.s < self.L and not mask[:, self.s:self.s + self.span].any():
            self.s += self.span
            self.fresh = True
        if self.s >= self.L:
            return [sf.StageParams(sf.IDLE, 0, -1, 1, self.tau_min, 2.0, 0, self.P, self.L)] * mask.shape[0]
        mode = sf.CACHE_REFRESH if self.fresh else sf.CACHE_REUSE
        e = min(self.s + self.span, self.L) - 1
        return [self._params(sf.FAST, mode) if mask[b, self.s:e + 1].any() else
                sf.StageParams(sf.IDLE, 0, -1, 1, self.tau_min, 2.0, 0, self.P, self.L) for b in range(mask.shape[0])]

    def observe(self, sps, res, mask):
        if self.fresh:
            for b, sp in enumerate(sps):
                self._skip[b][:] = 0
                if sp.stage == sf.IDLE:
                    continue
                conf = res[b][6]
                for i in range(sp.e_cycle + 1, self.L):
                    if mask[b, i] and np.float32(conf[i]) < np.float32(self.tau_min):
                        self._skip[b][i] = 1
            self.fresh = False

    def skip(self):
        return self._skip


FUSED = pytest.mark.parametrize("fused", [False, True], ids=["logits", "fused"])


def lockstep(cfg, batch, params, final_gain=1.0, max_checked_steps=10 ** 9, driver=None, fused=False):
    """fused: the greedy decode runs inside the vocabulary projection and leaves no logits, so the
    logits comparison is the unfused run's; every decision is checked the same way in both."""
    b = binding()
    w = synth.make_weights(cfg)
    if final_gain != 1.0:
        w["final_norm"] = torch.full_like(w["final_norm"], final_gain)
    wb = weights_bits(w)
    wd = {k: ([t.to(DEV) for t in v] if isinstance(v, list) else v.to(DEV)) for k, v in w.items()}
    mc = synth.model_config(cfg)
    tokens, mask, prev = (t.numpy().copy() for t in synth.make_state(cfg, batch=batch))
    B, L = tokens.shape
    P = cfg["prompt"]
    model = b.Model(mc, wd, B, L)
    model.set_fused_selector(fused)
    out = b.CommitList(B, L)
    stats = dict(steps=0, exact=0, loose=0, max_logit_err=0.0, max_conf_rel_err=0.0, own_numbers_checked=0,
                 pred_checked=0, pred_differs=0, decisions=0, decisions_exempt=0)

    predict = OraclePredictor(mc, wb, B, L)

    drv = driver(B, P, L) if driver is not None else SlowFastDriver(B, P, L, params)
    prev_pred = prev
    while stats["steps"] < max_checked_steps:
        sps = drv.next(mask)
        if all(sp.stage == sf.IDLE for sp in sps):
            break
        # the library steps from the oracle's pre-step state
        g_tok = torch.from_numpy(tokens).to(DEV); g_mask = torch.from_numpy(mask).to(DEV)
        g_prev = torch.from_numpy(prev_pred).to(DEV)
        csp = [b.stage_params(p.stage, p.s_cycle, p.e_cycle, p.top_k, p.tau_min_conf, p.tau_high_conf, p.conv_mode,
                              p.gen_start, p.gen_end) for p in sps]
        modes = [p.cache_mode for p in sps]
        skip = drv.skip() if hasattr(drv, "skip") else None
        also = drv.also() if hasattr(drv, "also") else None
        if any(modes) or also is not None:
            sk = np.zeros((B, L), np.uint8)
            for s_ in range(B):
                if modes[s_] == sf.CACHE_REUSE:
                    sk[s_] = skip[s_]
                if also is not None and modes[s_] != sf.CACHE_REFRESH:
                    sk[s_] |= also[s_]
                    modes[s_] = sf.CACHE_REUSE      # an all-zero skip set = a complete forward that refreshes the cache
            model.step_cached(g_tok, g_mask, g_prev, csp, modes, sk, out)
            stats["cached_steps"] = stats.get("cached_steps", 0) + 1
            stats["rows_skipped"] = stats.get("rows_skipped", 0) + int(sk.sum())
        else:
            model.step(g_tok, g_mask, g_prev, csp, out)
        torch.cuda.synchronize()
        got = out.to_host()
        mask_before, prev_before, tok_before = mask.copy(), prev_pred.copy(), tokens.copy()
        res = sf.step(predict, tokens, mask, prev_pred, sps, skip, also)
        last = predict.last

        ref = last["logits"]
        # the step projects only the rows inside each window onto the vocabulary
        wrows = [s * L + i for s in range(B) for i in range(sps[s].eval_window()[0], sps[s].eval_window()[1] + 1)]
        assert not np.isnan(ref[wrows]).any()
        top = np.nanmax(np.abs(ref))
        g_pred, g_conf = (x.cpu().numpy().reshape(B, L) for x in model.debug_rows(B * L))
        active = np.stack([sf.active_rows(sps[s], mask_before[s]) for s in range(B)]).astype(bool)

        # ---- (ii) the oracle's rule on the library's own numbers: no exemptions
        if not fused:
            # row phase of the oracle on the library's bf16 logits
            lb = bits(model.debug_logits(B * L))
            o2_pred, o2_conf = oracle.row_phase(lb, mc["mask_id"], active.reshape(-1).astype(np.uint8))
            o2_pred, o2_conf = o2_pred.reshape(B, L), o2_conf.reshape(B, L)
            assert np.array_equal(g_pred[active], o2_pred[active])
            if active.any():
                assert (np.abs(g_conf[active] - o2_conf[active]) / o2_conf[active]).max() <= 2e-5
        g_tok, g_mask, g_prev = g_tok.cpu().numpy(), g_mask.cpu().numpy(), g_prev.cpu().numpy()
        for s in range(B):
            commit2, e2, first2 = sf.select(sps[s], mask_before[s], g_pred[s], g_conf[s], prev_before[s])
            g_pos, g_toks, g_cfs, g_e, g_first, g_left = got[s]
            assert g_pos == commit2 and g_e == e2 and g_first == first2, (stats["steps"], s)
            assert g_toks == [int(g_pred[s, i]) for i in commit2]
            assert np.array_equal(np.asarray(g_cfs, np.float32), g_conf[s][commit2].astype(np.float32))
            assert g_left == int(mask_before[s].sum()) - len(commit2)
            want_tok, want_mask, want_prev = tok_before[s].copy(), mask_before[s].copy(), prev_before[s].copy()
            want_tok[commit2] = g_pred[s][commit2]; want_mask[commit2] = 0
            want_prev[active[s]] = g_pred[s][active[s]]
            assert np.array_equal(g_tok[s], want_tok) and np.array_equal(g_mask[s], want_mask)
            assert np.array_equal(g_prev[s], want_prev)
            assert all(t != mc["mask_id"] for t in g_toks)
            stats["own_numbers_checked"] += 1

        # ---- (i) against the oracle's own prediction
        # logits: the stated bar; the measured error of this step bounds what a prediction may hang on
        if not fused:
            g_logits = oracle.bf16_to_f64(lb)
            eps_abs = np.abs(g_logits[wrows] - ref[wrows]).max()
            err = eps_abs / top
            stats["max_logit_err"] = max(stats["max_logit_err"], err)
            assert err <= 2e-2 and err <= LOGIT_NORMWISE
        else:
            eps_abs = LOGIT_NORMWISE * top          # no logits in this mode: the bound the other mode asserts
        o_conf, o_pred = last["conf"], last["pred"]
        # confidences: 1e-3 absolute end to end; their measured relative error is the perturbation the
        # decisions below have to survive to be compared
        delta = 0.0
        if active.any():
            # every logit within eps_abs moves a confidence by a factor inside exp(+-2 eps_abs)
            assert (np.abs(g_conf[active] - o_conf[active]) <= 1e-3 + (math.exp(2 * eps_abs) - 1) * o_conf[active]).all()
            delta = float((np.abs(g_conf[active] - o_conf[active]) / o_conf[active]).max()) * 1.0001 + 1e-7
        stats["max_conf_rel_err"] = max(stats["max_conf_rel_err"], delta)
        srt = np.sort(np.where(np.arange(ref.shape[1]) == mc["mask_id"], -np.inf, np.nan_to_num(ref)), axis=1)
        gap = (srt[:, -1] - srt[:, -2]).reshape(B, L)
        # a prediction may differ from the oracle's only where the oracle's top two logits are closer than
        # twice the logit error plus one bf16 rounding step of the larger one
        flip_ok = 2 * eps_abs + 2.0 ** -7 * np.abs(srt[:, -1]).reshape(B, L)
        differs = active & (g_pred != o_pred)
        assert not (differs & (gap > flip_ok)).any()
        stats["pred_checked"] += int(active.sum()); stats["pred_differs"] += int(differs.sum())

        for s in range(B):
            commit, toks, cfs, e_cand, first, left = res[s][:6]
            g_pos, g_toks, g_cfs, g_e, g_first, g_left = got[s]
            rb = Robust(sps[s], mask_before[s], o_conf[s], o_pred[s], prev_before[s], ~differs[s], delta)
            must, never, count = rb.decide()
            assert must <= set(g_pos) and not (never & set(g_pos)), (stats["steps"], s)
            if count is not None:
                assert len(g_pos) == count
            if sps[s].stage != sf.IDLE and rb.cands:
                assert len(g_pos) >= 1                                  # steady progress
                stats["decisions"] += 1
                stats["decisions_exempt"] += int(not (must | never == set(rb.cands) and count in (None, len(must))))
            assert g_pos == sorted(g_pos) and all(mask_before[s, i] for i in g_pos)
            assert g_first == first
            ev, e_robust = rb.e_cand()
            if e_robust:
                assert g_e == ev == e_cand
            if set(g_pos) == set(commit) and g_toks == toks:
                stats["exact"] += 1
            else:
                stats["loose"] += 1
        drv.observe(sps, res, mask)
        stats["steps"] += 1
    model.close()
    # What the exemptions of (i) rest on, bounded: the confidence perturbation (it scales with the logit
    # scale: measured 0.8e-2 at gain 1, 7e-2 at gain 10), the share of predictions that differ from the
    # oracle's (each one checked above to sit on a near-tie; measured <= 4 %), and the share of decisions
    # that such a perturbation leaves open.  Check (ii) has no exemptions.
    assert stats["own_numbers_checked"] == stats["steps"] * B
    assert stats["max_conf_rel_err"] <= 1.2e-2 * max(final_gain, 1.0) + 1e-2
    assert stats["pred_differs"] <= 0.06 * stats["pred_checked"] + 1
    assert stats["decisions_exempt"] <= 0.97 * stats["decisions"] + 1
    assert stats["loose"] <= 0.9 * (stats["exact"] + stats["loose"]) + 1
    return stats


@FUSED
def test_lockstep_tiny_config_full_decode(fused):
    """Random-init tiny config, the paper's default hyper-parameters (threshold
    0.9): confidences are ~1/V everywhere, so only top-k / empty-e_cand paths run."""
    cfg = synth.CONFIGS["tiny"]
    p = sf.DecodeParams(max_steps=10 ** 6, tau_min_conf=0.1, tau_high_conf=0.9, conv_mode=1)
    st = lockstep(cfg, cfg["batch"], p, fused=fused)
    assert st["steps"] == cfg["gen"]                # one token per step under random init
    print("lockstep tiny:", st)


@FUSED
def test_lockstep_tiny_config_peaked_logits(fused):
    """Same model with the final norm gain raised so that confidences spread
    over (0, 1): threshold, convergence-gate and e_cand paths run end to end."""
    cfg = synth.CONFIGS["tiny"]
    p = sf.DecodeParams(max_steps=10 ** 6, tau_min_conf=0.2, tau_high_conf=0.3, conv_mode=1, k_slow=2)
    st = lockstep(cfg, 2, p, final_gain=10.0, fused=fused)
    assert st["steps"] < cfg["gen"]                 # parallel commits happened
    assert st["exact"] >= st["loose"]
    print("lockstep tiny peaked:", st)


@FUSED
def test_lockstep_maximum_batch(fused):
    """64 sequences, the most one call takes (one window, one commit list slot, one row table entry each)."""
    cfg = synth.CONFIGS["tiny"]
    p = sf.DecodeParams(max_steps=10 ** 6, tau_min_conf=0.2, tau_high_conf=0.3, conv_mode=1, k_slow=2)
    st = lockstep(cfg, 64, p, final_gain=10.0, max_checked_steps=3, fused=fused)
    assert st["steps"] == 3 and st["pred_checked"] >= 64 and st["own_numbers_checked"] == 3 * 64
    print("lockstep 64 sequences:", st)


@FUSED
def test_lockstep_medium_config_first_steps(fused):
    cfg = synth.CONFIGS["medium"]
    p = sf.DecodeParams(max_steps=10 ** 6, tau_min_conf=0.1, tau_high_conf=0.9, conv_mode=1)
    st = lockstep(cfg, cfg["batch"], p, max_checked_steps=3, fused=fused)       # batch 4, as the config states
    print("lockstep medium:", st)


@FUSED
def test_lockstep_out_of_span_caching(fused):
    """SlowFast with out-of-span caching (Section 3.3): refresh and reuse steps of both sides start
    from the oracle's state and the oracle's cached set; the library's stale-feature forward must
    stay inside the same logit bound, and the decisions are compared as in the other lock-step runs."""
    cfg = synth.CONFIGS["tiny"]
    # a random-init model has no regional structure, so the spans are laid out by the driver; the
    # threshold for caching is the median confidence of the first prediction (about half is cached)
    w = synth.make_weights(cfg)
    w["final_norm"] = torch.full_like(w["final_norm"], 10.0)
    tokens, mask, _ = (t.numpy() for t in synth.make_state(cfg, batch=2))
    B, L = tokens.shape
    _, c0 = OraclePredictor(synth.model_config(cfg), weights_bits(w), B, L)(tokens, mask)
    tau_min = float(np.median(c0[mask == 1]))
    st = lockstep(cfg, 2, None, final_gain=10.0, max_checked_steps=40,
                  driver=lambda B, P, L: CachedSpanDriver(B, P, L, 8, tau_min), fused=fused)
    assert st["cached_steps"] == 40 and st["rows_skipped"] > 200
    print("lockstep cached:", st)


@FUSED
def test_lockstep_out_of_span_caching_random_init(fused):
    # confidences ~ 1/V < tau_min everywhere: every masked position right of the span is cached
    cfg = synth.CONFIGS["tiny"]
    # (spans are single positions here, so every fast stage is one refresh step: covers the wide
    # evaluation window of a refresh step and mixed slow / refresh batches under Algorithm 1's controller)
    p = sf.DecodeParams(max_steps=10 ** 6, tau_min_conf=0.1, tau_high_conf=0.9, conv_mode=0, k_fast=1, k_max=2,
                        out_of_span_cache=True)
    st = lockstep(cfg, 2, p, max_checked_steps=24, fused=fused)
    assert st.get("cached_steps", 0) >= 4
    print("lockstep cached, random init:", st)


@FUSED
def test_lockstep_prompt_caching(fused):
    """Prompt caching (K_p = 4) together with out-of-span caching under Algorithm 1's controller:
    three of four steps recompute the generated region only."""
    cfg = synth.CONFIGS["tiny"]
    p = sf.DecodeParams(max_steps=10 ** 6, tau_min_conf=0.2, tau_high_conf=0.3, conv_mode=1, k_slow=2,
                        out_of_span_cache=True, prompt_cache_interval=4)
    st = lockstep(cfg, 2, p, final_gain=10.0, fused=fused)
    assert st["cached_steps"] == st["steps"] and st["rows_skipped"] >= (st["steps"] // 2) * 2 * cfg["prompt"]
    print("lockstep prompt caching:", st)


@FUSED
def test_lockstep_prompt_caching_without_out_of_span_caching(fused):
    """K_p = 3 alone, with the convergence gate on: the steps that refresh the prompt go through the
    cached path but rate exactly the window of an uncached step (prev_pred outside it must not move)."""
    cfg = synth.CONFIGS["tiny"]
    p = sf.DecodeParams(max_steps=10 ** 6, tau_min_conf=0.2, tau_high_conf=0.3, conv_mode=1, k_slow=2,
                        prompt_cache_interval=3)
    st = lockstep(cfg, 2, p, final_gain=10.0, fused=fused)
    assert st["cached_steps"] == st["steps"] and st["rows_skipped"] >= (st["steps"] // 2) * 2 * cfg["prompt"]
    print("lockstep prompt caching only:", st)


@FUSED
@pytest.mark.parametrize("oos,kp,kr", [(False, 0, 3), (True, 4, 2)])
def test_lockstep_response_caching(oos, kp, kr, fused):
    """Response caching (K_r) alone and with the other two caches: between the K_r-th steps only the
    prompt (unless cached too) and each sequence's rated range are recomputed."""
    cfg = synth.CONFIGS["tiny"]
    p = sf.DecodeParams(max_steps=10 ** 6, tau_min_conf=0.2, tau_high_conf=0.3, conv_mode=1, k_slow=2, k_max=2, w_hist=1,
                        out_of_span_cache=oos, prompt_cache_interval=kp, response_cache_interval=kr)
    st = lockstep(cfg, 2, p, final_gain=10.0, fused=fused)
    assert st["cached_steps"] == st["steps"] and st["rows_skipped"] > 0
    print(f"lockstep response caching K_r={kr} K_p={kp} oos={oos}:", st)


@FUSED
def test_lockstep_low_confidence_baseline(fused):
    """The baseline sampler's steps (top-k of a block by confidence, k from the
    schedule) through the same lock-step protocol: 4 blocks, 2 tokens per step."""
    cfg = synth.CONFIGS["tiny"]
    G = cfg["gen"]
    st = lockstep(cfg, 2, None, final_gain=10.0,
                  driver=lambda B, P, L: LowConfidenceDriver(B, P, L, G // 2, G // 4), fused=fused)
    assert st["steps"] == G // 2
    print("lockstep low-confidence:", st)


def decode_params(b, p: sf.DecodeParams):
    return b.DecodeParams(p.max_steps, p.k_max, p.w_hist, p.k_slow, p.k_fast, p.conv_mode, p.sigma2_stable,
                          p.tau_min_conf, p.tau_high_conf, int(p.out_of_span_cache), int(p.prompt_cache_interval),
                          int(p.response_cache_interval))


@pytest.mark.parametrize("cache,kp,kr", [(False, 0, 0), (True, 0, 0), (True, 3, 0), (False, 5, 0), (False, 0, 3),
                                         (True, 4, 2), (False, 3, 1)])
@pytest.mark.parametrize("gain,tau_min,tau_high,k_max,w_hist", [(10.0, 0.2, 0.3, 8, 2), (10.0, 0.23, 0.999, 1, 1),
                                                               (1.0, None, None, 8, 2)])
def test_decode_follows_algorithm_1_on_the_librarys_own_predictions(cache, kp, kr, gain, tau_min, tau_high, k_max, w_hist):
    """dllm_decode (host controller + step kernels) against Algorithm 1 written as the listing's nested
    loops (oracle `alg1_sequence`, one generator per sequence).  Every "predict" line of a generator is
    answered with the predictions and confidences the library's own step leaves for exactly the stage
    parameters the generator asks for; the generator then applies the oracle's selection and transition.
    The library's state after every such step must equal the generators', and dllm_decode must take the
    same steps (stages, commits per step) and end in the same tokens.  Covers the stage transitions of
    Algorithm 1, the refresh / reuse protocol of out-of-span caching and the interval caches."""
    b = binding()
    cfg = synth.CONFIGS["tiny"]
    w = synth.make_weights(cfg)
    w["final_norm"] = torch.full_like(w["final_norm"], gain)
    wd = {k: ([t.to(DEV) for t in v] if isinstance(v, list) else v.to(DEV)) for k, v in w.items()}
    tokens, mask, _ = synth.make_state(cfg, batch=3)
    B, L = tokens.shape
    P, G = cfg["prompt"], cfg["gen"]
    model = b.Model(synth.model_config(cfg), wd, B, L)
    out = b.CommitList(B, L)
    if tau_min is None:            # thresholds at quantiles of the first prediction (random init: ~1/V)
        t, m, pv = tokens.to(DEV), mask.to(DEV), torch.full((B, L), -1, dtype=torch.int32, device=DEV)
        model.step(t, m, pv, [b.stage_params(b.STAGE_SLOW, P, L - 1, 1, 0.1, 0.9, 0, P, L)] * B, out)
        torch.cuda.synchronize()
        c0 = model.debug_rows(B * L)[1].view(B, L)[mask.bool().to(DEV)].float()
        tau_min, tau_high = float(c0.quantile(0.5)), float(c0.quantile(0.9))
    p = sf.DecodeParams(max_steps=10 ** 6, k_max=k_max, w_hist=w_hist, tau_min_conf=tau_min, tau_high_conf=tau_high,
                        conv_mode=1 if kr == 3 else 0, k_slow=1, k_fast=1, out_of_span_cache=cache,
                        prompt_cache_interval=kp, response_cache_interval=kr)
    g_tok, g_mask = tokens.to(DEV), mask.to(DEV)
    steps, stats = model.decode(g_tok, g_mask, P, decode_params(b, p), stats_capacity=4 * G)
    assert int(g_mask.sum()) == 0

    h_tok, h_mask = tokens.numpy().copy(), mask.numpy().copy()
    h_prev = np.full((B, L), -1, np.int32)
    logs = [[] for _ in range(B)]
    gens = [sf.alg1_sequence(h_tok[q], h_mask[q], h_prev[q], P, L, p, logs[q]) for q in range(B)]
    asks = [next(g, None) for g in gens]
    idle = sf.StageParams(sf.IDLE, 0, -1, 1, tau_min, tau_high, p.conv_mode, P, L)
    n, reuse_rows = 0, 0
    while any(a is not None for a in asks):
        sps = [a[0] if a is not None else idle for a in asks]
        s_tok, s_mask, s_prev = (torch.from_numpy(x).to(DEV) for x in (h_tok, h_mask, h_prev))
        csp = [b.stage_params(x.stage, x.s_cycle, x.e_cycle, x.top_k, x.tau_min_conf, x.tau_high_conf, x.conv_mode,
                              x.gen_start, x.gen_end) for x in sps]
        modes = [x.cache_mode for x in sps]
        also = sf.interval_skip(p, n, sps, P, L, L)
        if any(modes) or also is not None:
            sk = np.zeros((B, L), np.uint8)
            for q in range(B):
                if modes[q] == sf.CACHE_REUSE:
                    sk[q] = asks[q][1]
                if also is not None and modes[q] != sf.CACHE_REFRESH:
                    sk[q] |= also[q]
                    modes[q] = sf.CACHE_REUSE
            reuse_rows += int(sk.sum())
            model.step_cached(s_tok, s_mask, s_prev, csp, modes, sk, out)
        else:
            model.step(s_tok, s_mask, s_prev, csp, out)
        torch.cuda.synchronize()
        pred, conf = (x.cpu().numpy().reshape(B, L) for x in model.debug_rows(B * L))
        done = [len(lg) for lg in logs]
        for q in range(B):
            if asks[q] is not None:
                try:
                    asks[q] = gens[q].send((pred[q], conf[q]))
                except StopIteration:
                    asks[q] = None
        # the library's selection and transition on these numbers are the oracle's
        assert np.array_equal(s_tok.cpu().numpy(), h_tok) and np.array_equal(s_mask.cpu().numpy(), h_mask)
        assert np.array_equal(s_prev.cpu().numpy(), h_prev)
        # and dllm_decode took this very step
        assert n < steps
        new = [logs[q][done[q]] if len(logs[q]) > done[q] else None for q in range(B)]
        assert stats[n][:4] == (sum(sp.stage == sf.SLOW for sp in sps), sum(sp.stage == sf.FAST for sp in sps),
                                sum(sp.stage == sf.IDLE for sp in sps), sum(len(e[3]) for e in new if e is not None)), n
        n += 1
    assert n == steps and np.array_equal(h_tok, g_tok.cpu().numpy())
    print(f"decode cache={cache} K_p={kp} K_r={kr} gain={gain}: {steps} steps, rows skipped in reuse steps {reuse_rows}")
    if (cache and k_max == 1) or kp:       # (confidences sit in 0.20 .. 0.24 here: 0.23 ends the span mid-region)
        assert reuse_rows > 0
    model.close()


@pytest.mark.parametrize("gain,tau_high,k_slow", [(1.0, 0.9, 1), (10.0, 0.3, 2)])
def test_decode_runs_to_completion(gain, tau_high, k_slow):
    b = binding()
    cfg = synth.CONFIGS["tiny"]
    w = synth.make_weights(cfg)
    w["final_norm"] = torch.full_like(w["final_norm"], gain)
    wd = {k: ([t.to(DEV) for t in v] if isinstance(v, list) else v.to(DEV)) for k, v in w.items()}
    tokens, mask, _ = synth.make_state(cfg, batch=3)
    B, L = tokens.shape
    P, G = cfg["prompt"], cfg["gen"]
    model = b.Model(synth.model_config(cfg), wd, B, L)
    p = sf.DecodeParams(max_steps=10 ** 6, tau_min_conf=0.1, tau_high_conf=tau_high, conv_mode=1, k_slow=k_slow)
    g_tok, g_mask = tokens.to(DEV), mask.to(DEV)
    steps, stats = model.decode(g_tok, g_mask, P, decode_params(b, p), stats_capacity=4 * G)
    assert int(g_mask.sum()) == 0 and 1 <= steps <= G
    out = g_tok.cpu()
    assert torch.equal(out[:, :P], tokens[:, :P]) and not (out == cfg["mask_id"]).any()
    assert len(stats) == steps and sum(s[3] for s in stats) == B * G
    assert all(s[0] + s[1] + s[2] == B and s[3] >= 1 and s[4] > 0 for s in stats)
    # the oracle's free-running decode of the same problem, for the record
    o_tok, o_mask = tokens.numpy().copy(), mask.numpy().copy()
    wb = weights_bits(w)
    mc = synth.model_config(cfg)

    def predict(tok, active):
        lb = oracle.round_to_bf16(oracle.forward(mc, wb, tok))
        pr, cf = oracle.row_phase(lb, mc["mask_id"], active.reshape(-1))
        return pr.reshape(B, L), cf.reshape(B, L)

    o_steps = sf.decode(predict, o_tok, o_mask, P, L, p)
    same = float((out.numpy()[:, P:] == o_tok[:, P:]).mean())
    print(f"decode gain={gain}: gpu steps {steps}, oracle steps {o_steps}, equal generated tokens {same:.2f}")
    if gain == 1.0:
        assert steps == o_steps == G
    # max_steps stops the loop
    g_tok, g_mask = tokens.to(DEV), mask.to(DEV)
    p3 = sf.DecodeParams(max_steps=3, tau_min_conf=0.1, tau_high_conf=tau_high, conv_mode=1, k_slow=k_slow)
    steps3, _ = model.decode(g_tok, g_mask, P, decode_params(b, p3))
    assert steps3 == 3 and int(g_mask.sum()) > 0
    model.close()


@pytest.mark.parametrize("n_steps_div,n_blocks", [(1, 1), (2, 1), (2, 4), (4, 2)])
def test_decode_low_confidence(n_steps_div, n_blocks):
    """dllm_decode_low_confidence: the schedule of Section 3.1 (steps taken, tokens per
    step), the end state, and bit-equality with the same schedule driven step by step
    through dllm_step (same kernels, so the host loop is the only difference)."""
    b = binding()
    cfg = synth.CONFIGS["tiny"]
    w = synth.make_weights(cfg)
    w["final_norm"] = torch.full_like(w["final_norm"], 10.0)
    wd = {k: ([t.to(DEV) for t in v] if isinstance(v, list) else v.to(DEV)) for k, v in w.items()}
    tokens, mask, _ = synth.make_state(cfg, batch=3)
    B, L = tokens.shape
    P, G = cfg["prompt"], cfg["gen"]
    n_steps, block_len = G // n_steps_div, G // n_blocks
    model = b.Model(synth.model_config(cfg), wd, B, L)
    g_tok, g_mask = tokens.to(DEV), mask.to(DEV)
    steps, stats = model.decode_low_confidence(g_tok, g_mask, P, n_steps, block_len if n_blocks > 1 else 0,
                                               stats_capacity=2 * G)
    assert steps == n_steps and int(g_mask.sum()) == 0
    out = g_tok.cpu()
    assert torch.equal(out[:, :P], tokens[:, :P]) and not (out == cfg["mask_id"]).any()
    per_block = n_steps // n_blocks
    want = [B * (sf.n_unmasked_target(block_len, per_block, j) - sf.n_unmasked_target(block_len, per_block, j - 1))
            for _ in range(n_blocks) for j in range(1, per_block + 1)]
    assert [s[3] for s in stats] == want and all(s[0] == B and s[1] == 0 and s[2] == 0 for s in stats)

    # the same schedule, one dllm_step at a time
    s_tok, s_mask = tokens.to(DEV), mask.to(DEV)
    s_prev = torch.full((B, L), -1, dtype=torch.int32, device=DEV)
    cl = b.CommitList(B, L)
    drv = LowConfidenceDriver(B, P, L, n_steps, block_len)
    for _ in range(n_steps):
        sps = drv.next(s_mask.cpu().numpy())
        model.step(s_tok, s_mask, s_prev, [b.stage_params(p.stage, p.s_cycle, p.e_cycle, p.top_k, p.tau_min_conf,
                                                          p.tau_high_conf, p.conv_mode, p.gen_start, p.gen_end)
                                           for p in sps], cl)
    torch.cuda.synchronize()
    assert torch.equal(s_tok.cpu(), out) and int(s_mask.sum()) == 0

    # argument checks
    with pytest.raises(b.DllmError):
        model.decode_low_confidence(tokens.to(DEV), mask.to(DEV), P, n_steps, 5)       # 5 does not divide 64
    with pytest.raises(b.DllmError):
        model.decode_low_confidence(tokens.to(DEV), mask.to(DEV), P, 3, G // 2)        # 3 steps, 2 blocks
    model.close()


# ---- greedy decode fused into the vocabulary projection ----------------------------

@pytest.mark.parametrize("tile", [-1, 0, 1, 2, 3, 4, 7, 8, 9, "fallback"])
@pytest.mark.parametrize("cfg_name,n_layers,batch,stage", [("tiny", 2, 3, "slow"), ("tiny", 2, 3, "fast"),
                                                           ("medium", 2, 2, "fast"), ("llada8b", 1, 1, "slow"),
                                                           # vocabulary that ends inside an MFMA tile, [MASK] mid-tile
                                                           ("tiny_v2040", 2, 2, "slow")])
def test_fused_selector_matches_the_logits_path(cfg_name, n_layers, batch, stage, tile, monkeypatch):
    """The same step twice from the same state: with bf16 logits and the separate row kernel, and with
    the greedy decode taken on the projection's accumulators (every tile shape that epilogue is built
    for, and the register-staged kernel).  Predictions and commits must be identical, confidences
    equal up to the order of the fp32 sum; both are also checked against the oracle's row phase
    (Section 3.1 eq. 3: arg max and maximum of the softmax over the vocabulary without [MASK], in fp64)
    on the library's own logits, on every rated row.  llada8b: full widths and vocabulary (ragged last column tile, the
    [MASK] column inside a tile), one layer."""
    if tile == "fallback":
        monkeypatch.setenv("DLLM_GEMM_FALLBACK", "1")
    elif tile >= 0:
        monkeypatch.setenv("DLLM_GEMM_CFG_E5", str(tile))
    b = binding()
    if cfg_name == "tiny_v2040":
        cfg = dict(synth.CONFIGS["tiny"], n_layers=n_layers, vocab=2040, mask_id=1000)
    else:
        cfg = dict(synth.CONFIGS[cfg_name], n_layers=n_layers)
    dev = cfg_name == "llada8b"
    w = synth.make_weights(cfg, device=DEV) if dev else synth.make_weights(cfg)
    w["final_norm"] = torch.full_like(w["final_norm"], 10.0)      # confidences spread over (0, 1)
    wd = w if dev else {k: ([t.to(DEV) for t in v] if isinstance(v, list) else v.to(DEV)) for k, v in w.items()}
    mc = synth.model_config(cfg)
    tokens, mask, prev = synth.make_state(cfg, batch=batch)
    B, L = tokens.shape
    P = cfg["prompt"]
    if stage == "slow":
        sps = [b.stage_params(b.STAGE_SLOW, P, L - 1, 3, 0.1, 0.9, 1, P, L) for _ in range(B)]
        lo, hi = P, L - 1
    else:      # windows that do not touch: one projection per sequence
        lo, hi = P + 3, P + 3 + (L - P) // 2
        sps = [b.stage_params(b.STAGE_FAST, lo, hi, 2, 0.1, 0.5, 0, P, L) for _ in range(B)]
    model = b.Model(mc, wd, B, L)
    out = b.CommitList(B, L)
    res = []
    for fused in (False, True):
        model.set_fused_selector(fused)
        t, m, pv = tokens.to(DEV), mask.to(DEV), prev.to(DEV)
        model.step(t, m, pv, sps, out)
        torch.cuda.synchronize()
        pred, conf = (x.view(B, L).clone() for x in model.debug_rows(B * L))
        logits = model.debug_logits(B * L).view(B, L, -1)[:, lo:hi + 1].clone() if not fused else None
        res.append((pred, conf, out.to_host(), t.cpu(), m.cpu(), pv.cpu(), logits))
    rated = torch.zeros(B, L, dtype=torch.bool)
    rated[:, lo:hi + 1] = mask[:, lo:hi + 1].bool()
    assert int(rated.sum()) > 0
    rd = rated.to(DEV)
    (p0, c0, o0, t0, m0, v0, logits), (p1, c1, o1, t1, m1, v1, _) = res
    assert torch.equal(p0[rd], p1[rd])
    assert torch.allclose(c0[rd], c1[rd], rtol=2e-6, atol=0)
    assert torch.equal(t0, t1) and torch.equal(m0, m1) and torch.equal(v0, v1)
    for q in range(B):
        assert o0[q][0] == o1[q][0] and o0[q][1] == o1[q][1] and o0[q][3:] == o1[q][3:]
        assert np.allclose(o0[q][2], o1[q][2], rtol=2e-6, atol=0)
    # the oracle's row phase (Section 3.1 eq. 3 on fp64 softmax rows) on the library's own bf16 logits,
    # every rated row: predictions bit-exact (lowest id among equal maxima), confidences to 2e-5
    lg = bits(logits.cpu()).reshape(B * (hi - lo + 1), -1)
    act = rated[:, lo:hi + 1].reshape(-1).numpy().astype(np.uint8)
    o_pred, o_conf = oracle.row_phase(lg, mc["mask_id"], act)
    sel = act.astype(bool)
    for got_p, got_c in ((p0, c0), (p1, c1)):
        gp = got_p[:, lo:hi + 1].reshape(-1).cpu().numpy()
        gc = got_c[:, lo:hi + 1].reshape(-1).cpu().numpy()
        assert np.array_equal(gp[sel], o_pred[sel])
        assert (np.abs(gc[sel] - o_conf[sel]) / o_conf[sel]).max() <= 2e-5
    model.close()


def test_logits_exist_only_after_a_call_that_writes_them():
    """Steps with the fused selector never write logits (the buffer is not even allocated until
    dllm_forward or a step with the fused selector off needs it): reading them before is an error."""
    b = binding()
    cfg = synth.CONFIGS["tiny"]
    w = synth.make_weights(cfg)
    wd = {k: ([t.to(DEV) for t in v] if isinstance(v, list) else v.to(DEV)) for k, v in w.items()}
    tokens, mask, prev = (t.to(DEV) for t in synth.make_state(cfg, batch=1))
    B, L = tokens.shape
    P = cfg["prompt"]
    model = b.Model(synth.model_config(cfg), wd, B, L)
    out = b.CommitList(B, L)
    sp = [b.stage_params(b.STAGE_SLOW, P, L - 1, 1, 0.1, 0.9, 0, P, L)]
    model.step(tokens, mask, prev, sp, out)
    torch.cuda.synchronize()
    assert out.to_host()[0][5] == cfg["gen"] - 1
    with pytest.raises(b.DllmError) as e:
        model.debug_logits(B * L)
    assert e.value.code == b.ESTATE
    model.set_fused_selector(False)
    model.step(tokens, mask, prev, sp, out)
    torch.cuda.synchronize()
    assert model.debug_logits(B * L).shape == (B * L, cfg["vocab"]) and out.to_host()[0][5] == cfg["gen"] - 2
    model.close()


def test_token_id_outside_the_vocabulary_is_reported_and_never_used_as_an_index():
    """Token ids live on the device, so only the embedding kernel can check them: an id outside
    [0, vocab) becomes a row of zeros and a flag that dllm_sync_status and the decode calls report."""
    b = binding()
    cfg = synth.CONFIGS["tiny"]
    w = synth.make_weights(cfg)
    wd = {k: ([t.to(DEV) for t in v] if isinstance(v, list) else v.to(DEV)) for k, v in w.items()}
    tokens, mask, prev = (t.to(DEV) for t in synth.make_state(cfg, batch=2))
    B, L = tokens.shape
    P = cfg["prompt"]
    model = b.Model(synth.model_config(cfg), wd, B, L)
    out = b.CommitList(B, L)
    sp = [b.stage_params(b.STAGE_SLOW, P, L - 1, 1, 0.1, 0.9, 0, P, L)] * B
    model.step(tokens.clone(), mask.clone(), prev.clone(), sp, out)
    model.sync_status()                                        # clean input: nothing to report
    for bad_id in (cfg["vocab"], cfg["vocab"] + 12345, -1, -2 ** 31):
        t = tokens.clone()
        t[1, 3] = bad_id
        model.step(t, mask.clone(), prev.clone(), sp, out)
        with pytest.raises(b.DllmError) as e:
            model.sync_status()
        assert e.value.code == b.EINVAL and "token id" in str(e.value)
        model.sync_status()                                    # reporting cleared it
    # the decode loops report it after the step that met it
    t = tokens.clone()
    t[0, 0] = cfg["vocab"] + 1
    p = sf.DecodeParams(max_steps=10 ** 6)
    with pytest.raises(b.DllmError) as e:
        model.decode(t, mask.clone(), P, decode_params(b, p))
    assert e.value.code == b.EINVAL
    with pytest.raises(b.DllmError) as e:
        model.decode_low_confidence(t, mask.clone(), P, cfg["gen"], 0)
    assert e.value.code == b.EINVAL
    # and the handle still works
    steps, _ = model.decode(tokens.clone(), mask.clone(), P, decode_params(b, p))
    assert steps == cfg["gen"]
    model.close()
