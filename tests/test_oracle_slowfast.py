"""Pins for the oracle's SlowFast selection rule, controller and decode loop.

Hand-built cases that follow from Section 3.3 / Algorithm 1, the special case
that reduces to LLaDA's low-confidence remasking (Section 3.1), and the
invariants the method guarantees."""
import os

import numpy as np
import pytest

import oracle
from oracle import slowfast as sf
from paper_2506_10848_amd import synth
from util import weights_bits

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def load_cases():
    cases = []
    for line in open(os.path.join(GOLDEN, "commit_sets.txt")):
        if line.startswith("#") or not line.strip():
            continue
        f = [t.strip() for t in line.split("|")]
        cases.append(dict(name=f[0], stage=sf.SLOW if f[1] == "slow" else sf.FAST, s=int(f[2]), e=int(f[3]),
                          k=int(f[4]), conv=int(f[5]), conf=[float(t) for t in f[6].split()],
                          agree=[int(t) for t in f[7].split()], commit=[int(t) for t in f[8].split()],
                          e_cand=int(f[9])))
    return cases


@pytest.mark.parametrize("case", load_cases(), ids=lambda c: c["name"])
def test_hand_built_commit_sets(case):
    n = len(case["conf"])
    pred = np.arange(100, 100 + n, dtype=np.int32)
    prev = np.where(np.array(case["agree"]) == 1, pred, pred + 1).astype(np.int32)
    sp = sf.StageParams(case["stage"], case["s"], case["e"], case["k"], 0.1, 0.9, case["conv"], 0, n)
    commit, e_cand, first = sf.select(sp, np.ones(n, np.uint8), pred, np.array(case["conf"], np.float32), prev)
    assert commit == case["commit"]
    assert e_cand == case["e_cand"]
    assert first == case["s"]


def test_select_only_sees_masked_positions_in_the_window():
    conf = np.array([.99, .99, .99, .99, .99, .99], np.float32)
    mask = np.array([1, 0, 1, 0, 1, 1], np.uint8)
    pred = np.zeros(6, np.int32)
    sp = sf.StageParams(sf.FAST, 1, 4, 1, 0.1, 0.9, 0, 0, 6)
    commit, e_cand, first = sf.select(sp, mask, pred, conf, pred)
    assert commit == [2, 4] and e_cand == 4 and first == 2
    sp = sf.StageParams(sf.SLOW, 3, 0, 2, 0.1, 0.9, 0, 0, 6)          # slow ignores e_cycle
    commit, e_cand, first = sf.select(sp, mask, pred, conf, pred)
    assert commit == [4, 5] and e_cand == 5 and first == 4
    sp = sf.StageParams(sf.IDLE, 0, 5, 1, 0.1, 0.9, 0, 0, 6)
    assert sf.select(sp, mask, pred, conf, pred) == ([], -1, -1)
    # thresholds are strict
    conf = np.array([.9, .1], np.float32)
    sp = sf.StageParams(sf.FAST, 0, 1, 1, np.float32(.1), np.float32(.9), 0, 0, 2)
    commit, e_cand, _ = sf.select(sp, np.ones(2, np.uint8), pred[:2], conf, pred[:2])
    assert commit == [0] and e_cand == 0       # 0.9 is not > 0.9 -> fallback top-1; 0.1 is not > 0.1


def test_prev_pred_of_minus_one_is_not_converged():
    conf = np.array([.99, .99], np.float32)
    pred = np.array([5, 6], np.int32)
    prev = np.array([-1, 6], np.int32)
    sp = sf.StageParams(sf.FAST, 0, 1, 1, 0.1, 0.9, 1, 0, 2)
    assert sf.select(sp, np.ones(2, np.uint8), pred, conf, prev)[0] == [1]


# ---- controller -----------------------------------------------------------------

def run_slow(history, k_max=8, sigma2=1.0, w_hist=2, L=10):
    """Feed e_cand values to a fresh controller; return (stage, e_cycle, s_cycle)
    right after the last one."""
    p = sf.DecodeParams(max_steps=100, k_max=k_max, w_hist=w_hist, sigma2_stable=sigma2)
    c = sf.Controller(0, L, p)
    mask = np.ones(L, np.uint8)
    for e in history:
        assert c.stage == sf.SLOW
        c.observe(e, 0, mask)
    return c.stage, c.e_cycle, c.s_cycle


def test_stability_check_window_of_two():
    assert run_slow([3])[0] == sf.SLOW                       # needs W_hist samples
    assert run_slow([3, 3]) == (sf.FAST, 3, 0)               # var 0
    assert run_slow([3, 4]) == (sf.FAST, 3, 0)               # var .25, mean 3.5 -> 3
    assert run_slow([3, 5])[0] == sf.SLOW                    # var 1.0 is not < 1.0
    assert run_slow([3, 5], sigma2=1.0001)[:2] == (sf.FAST, 4)
    assert run_slow([9, 3, 5, 6]) == (sf.FAST, 5, 0)         # only the last W_hist count


def test_variance_is_strictly_below_threshold_as_in_fig3():
    # Fig. 3: the stage switch fires at "0.22 < 0.23"; equality must not fire.
    # window {0, 1, 1}: population variance 2/9 = 0.2222
    assert run_slow([0, 1, 1], sigma2=0.23, w_hist=3)[0] == sf.FAST
    assert run_slow([0, 1, 1], sigma2=2.0 / 9.0, w_hist=3)[0] == sf.SLOW
    # the sample variance of the same window is 1/3 and would not fire at 0.23
    assert run_slow([0, 1, 1], sigma2=0.3, w_hist=3)[0] == sf.FAST


def test_kmax_fallback_uses_last_candidate():
    stage, e, _ = run_slow([0, 2, 4, 7], k_max=4, L=10)
    assert (stage, e) == (sf.FAST, 7)
    assert run_slow([0, 2, 4], k_max=4)[0] == sf.SLOW


def test_empty_candidate_set_falls_back_to_leftmost_mask():
    p = sf.DecodeParams(max_steps=100)
    c = sf.Controller(2, 10, p)
    mask = np.zeros(10, np.uint8); mask[4:] = 1
    c.observe(-1, 4, mask)
    c.observe(-1, 4, mask)
    assert (c.stage, c.s_cycle, c.e_cycle) == (sf.FAST, 2, 4)
    # fast stage ends when [s, e] holds no mask: next cycle starts right after e
    mask[4] = 0
    c.observe(-1, -1, mask)
    assert (c.stage, c.s_cycle, c.history, c.step_count) == (sf.SLOW, 5, [], 0)


def test_span_that_is_already_clean_skips_the_fast_stage():
    p = sf.DecodeParams(max_steps=100)
    c = sf.Controller(0, 8, p)
    mask = np.ones(8, np.uint8)
    c.observe(0, 0, mask)
    mask[0] = 0                              # the second slow step committed position 0 itself
    c.observe(0, 0, mask)
    assert (c.stage, c.s_cycle) == (sf.SLOW, 1)


# ---- decode ---------------------------------------------------------------------

def fixed_conf_predictor(conf_map, pred_map):
    """A predictor whose confidences do not depend on the state."""
    def predict(tokens, active):
        return pred_map.copy(), np.where(active == 1, conf_map, 0).astype(np.float32)
    return predict


def test_reduces_to_low_confidence_remasking():
    # tau_high >= 1 never fires, tau_min < 0 makes e_cand the rightmost mask,
    # k_slow = k_fast = 1: every step commits the single most confident masked
    # position, i.e. low-confidence remasking with N = G (n_un grows by one per step).
    rng = np.random.default_rng(3)
    P, G = 3, 17
    L = P + G
    conf = rng.random((1, L)).astype(np.float32)
    pred = rng.integers(0, 50, (1, L)).astype(np.int32)
    tokens = np.full((1, L), 99, np.int32); mask = np.zeros((1, L), np.uint8); mask[:, P:] = 1
    trace = []
    p = sf.DecodeParams(max_steps=1000, tau_min_conf=-1.0, tau_high_conf=1.0, k_slow=1, k_fast=1)
    steps = sf.decode(fixed_conf_predictor(conf, pred), tokens, mask, P, L, p, trace)
    assert steps == G
    order = [res[0][0] for _, res in trace]
    assert all(len(o) == 1 for o in order)
    expected = sorted(range(P, L), key=lambda i: -conf[0, i])
    assert [o[0] for o in order] == expected
    assert np.array_equal(tokens[0, P:], pred[0, P:]) and not mask.any()


def test_decode_with_regional_confidences_commits_spans_in_parallel():
    # confident block at the left of the generated region, uncertain to its right
    P, L = 2, 14
    conf = np.full((1, L), 0.05, np.float32); conf[0, 2:8] = 0.95
    pred = np.arange(L, dtype=np.int32)[None] + 200
    tokens = np.full((1, L), 999, np.int32); mask = np.zeros((1, L), np.uint8); mask[:, P:] = 1
    trace = []
    p = sf.DecodeParams(max_steps=100, tau_min_conf=0.1, tau_high_conf=0.9, conv_mode=1)
    steps = sf.decode(fixed_conf_predictor(conf, pred), tokens, mask, P, L, p, trace)
    # slow, slow (e_cand = 7 twice -> stable, e_cycle = 7), then one fast step commits
    # the rest of [2, 7] at once (predictions repeat, so they count as converged)
    stages = [sps[0].stage for sps, _ in trace]
    assert stages[:3] == [sf.SLOW, sf.SLOW, sf.FAST]
    assert trace[0][1][0][3] == 7 and trace[1][1][0][3] == 7
    assert trace[2][0][0].s_cycle == 2 and trace[2][0][0].e_cycle == 7
    assert len(trace[2][1][0][0]) == 4
    assert not mask.any() and steps < L - P
    assert np.array_equal(tokens[0, P:], pred[0, P:])


def model_predictor(cfg, wbits):
    def predict(tokens, active):
        B, L = tokens.shape
        logits = oracle.forward(synth.model_config(cfg), wbits, tokens)
        pred, conf = oracle.row_phase(oracle.round_to_bf16(logits), cfg["mask_id"], active.reshape(-1))
        return pred.reshape(B, L), conf.reshape(B, L)
    return predict


@pytest.mark.parametrize("conv_mode,quantile", [(1, None), (0, 0.8)])
def test_decode_invariants_on_a_small_model(conv_mode, quantile):
    cfg = dict(synth.CONFIGS["tiny"], vocab=257, mask_id=256, prompt=6, gen=20, d_model=64, n_heads=2,
               head_dim=32, d_ffn=96, n_layers=1)
    w = synth.make_weights(cfg, std=0.25)            # wide init so that confidences spread out
    tokens, mask, _ = synth.make_state(cfg, batch=2)
    tokens, mask = tokens.numpy().copy(), mask.numpy().copy()
    predict = model_predictor(cfg, weights_bits(w))
    P, L = cfg["prompt"], cfg["prompt"] + cfg["gen"]
    tau_high, tau_min = 0.9, 0.1
    if quantile is not None:                         # thresholds at quantiles of the first step
        _, c0 = predict(tokens, mask)
        tau_high = float(np.quantile(c0[mask == 1], quantile)); tau_min = float(np.quantile(c0[mask == 1], 0.3))
    p = sf.DecodeParams(max_steps=10 ** 6, tau_min_conf=tau_min, tau_high_conf=tau_high, conv_mode=conv_mode)
    prompt = tokens[:, :P].copy()
    trace = []
    steps = sf.decode(predict, tokens, mask, P, L, p, trace)
    assert not mask.any() and steps <= cfg["gen"]
    assert np.array_equal(tokens[:, :P], prompt) and not (tokens == cfg["mask_id"]).any()
    committed = [dict() for _ in range(2)]
    for sps, res in trace:
        for b in range(2):
            commit, toks, cfs, e_cand, first, left = res[b][:6]
            if sps[b].stage == sf.IDLE:
                assert commit == []
                continue
            assert len(commit) >= 1                                     # steady progress
            lo, hi = sps[b].window()
            assert all(lo <= i <= hi and P <= i < L for i in commit)
            if sps[b].stage == sf.SLOW:
                assert len(commit) <= sps[b].top_k
            for i, t in zip(commit, toks):
                assert i not in committed[b]                             # never committed twice
                committed[b][i] = t
    for b in range(2):
        assert all(tokens[b, i] == t for i, t in committed[b].items())   # never changed afterwards
        assert len(committed[b]) == cfg["gen"]


def test_max_steps_stops_the_decode():
    P, L = 1, 9
    conf = np.linspace(0.01, 0.05, L, dtype=np.float32)[None]
    pred = np.zeros((1, L), np.int32)
    tokens = np.full((1, L), 7, np.int32); mask = np.zeros((1, L), np.uint8); mask[:, P:] = 1
    p = sf.DecodeParams(max_steps=3)
    assert sf.decode(fixed_conf_predictor(conf, pred), tokens, mask, P, L, p) == 3
    assert mask.sum() == L - P - 3


# ---- low-confidence remasking baseline (Section 3.1) ------------------------------

def test_low_confidence_schedule_values():
    # n_un = floor(L (1 - (k-1)/N)), k = N .. 1, worked by hand:
    # L = 10, N = 4: 10*1/4 = 2.5, 10*2/4 = 5, 10*3/4 = 7.5, 10 -> 2, 5, 7, 10
    assert [sf.n_unmasked_target(10, 4, j) for j in (1, 2, 3, 4)] == [2, 5, 7, 10]
    # L = N: one more token per step;  L = 7, N = 3: 2.33, 4.67, 7 -> 2, 4, 7
    assert [sf.n_unmasked_target(6, 6, j) for j in range(1, 7)] == [1, 2, 3, 4, 5, 6]
    assert [sf.n_unmasked_target(7, 3, j) for j in (1, 2, 3)] == [2, 4, 7]


def test_low_confidence_decode_commits_in_order_of_confidence():
    rng = np.random.default_rng(8)
    P, G = 2, 10
    L = P + G
    conf = rng.random((1, L)).astype(np.float32)
    pred = rng.integers(0, 50, (1, L)).astype(np.int32)
    ranked = sorted(range(P, L), key=lambda i: -conf[0, i])
    for n_steps, sizes in ((10, [1] * 10), (4, [2, 3, 2, 3]), (1, [10])):
        tokens = np.full((1, L), 99, np.int32); mask = np.zeros((1, L), np.uint8); mask[:, P:] = 1
        trace = []
        steps = sf.decode_low_confidence(fixed_conf_predictor(conf, pred), tokens, mask, P, L, n_steps, None, trace)
        assert steps == n_steps
        got = [res[0][0] for _, res in trace]
        assert [len(c) for c in got] == sizes
        at = 0
        for c in got:                                  # each step takes the next most confident ones
            assert sorted(c) == sorted(ranked[at:at + len(c)])
            at += len(c)
        assert not mask.any() and np.array_equal(tokens[0, P:], pred[0, P:])


def test_low_confidence_decode_equals_the_slowfast_special_case():
    # N = G: the reduction used by test_reduces_to_low_confidence_remasking must give the same trajectory
    rng = np.random.default_rng(9)
    P, G = 1, 12
    L = P + G
    conf = rng.random((2, L)).astype(np.float32)
    pred = rng.integers(0, 50, (2, L)).astype(np.int32)
    t1 = np.full((2, L), 99, np.int32); m1 = np.zeros((2, L), np.uint8); m1[:, P:] = 1
    t2, m2 = t1.copy(), m1.copy()
    tr1, tr2 = [], []
    sf.decode_low_confidence(fixed_conf_predictor(conf, pred), t1, m1, P, L, G, None, tr1)
    p = sf.DecodeParams(max_steps=1000, tau_min_conf=-1.0, tau_high_conf=1.0, k_slow=1, k_fast=1)
    sf.decode(fixed_conf_predictor(conf, pred), t2, m2, P, L, p, tr2)
    assert [[r[0] for r in res] for _, res in tr1] == [[r[0] for r in res] for _, res in tr2]
    assert np.array_equal(t1, t2)


def test_semi_autoregressive_blocks_go_left_to_right():
    P, G, Lb = 3, 12, 4
    L = P + G
    conf = np.linspace(0.1, 0.9, L, dtype=np.float32)[None]       # rightmost is the most confident
    pred = np.arange(L, dtype=np.int32)[None]
    tokens = np.full((1, L), 99, np.int32); mask = np.zeros((1, L), np.uint8); mask[:, P:] = 1
    trace = []
    steps = sf.decode_low_confidence(fixed_conf_predictor(conf, pred), tokens, mask, P, L, 6, Lb, trace)
    assert steps == 6                                              # 3 blocks x 2 steps x 2 tokens
    got = [res[0][0] for _, res in trace]
    assert got == [[5, 6], [3, 4], [9, 10], [7, 8], [13, 14], [11, 12]]
    with pytest.raises(ValueError):
        sf.decode_low_confidence(fixed_conf_predictor(conf, pred), tokens, mask, P, L, 6, 5)
    with pytest.raises(ValueError):
        sf.decode_low_confidence(fixed_conf_predictor(conf, pred), tokens, mask, P, L, 4, Lb)


def test_low_confidence_decode_skips_steps_whose_target_is_met():
    # half of the region is already unmasked: the first steps have nothing to add and run no forward
    P, G = 0, 8
    conf = np.linspace(0.9, 0.1, G, dtype=np.float32)[None]
    pred = np.arange(G, dtype=np.int32)[None]
    tokens = np.full((1, G), 99, np.int32); mask = np.ones((1, G), np.uint8); mask[0, :4] = 0
    calls = []
    def predict(tokens, active):
        calls.append(1)
        return pred.copy(), np.where(active == 1, conf, 0).astype(np.float32)
    steps = sf.decode_low_confidence(predict, tokens, mask, P, G, 8, None)
    assert steps == 4 == len(calls) and not mask.any()


# ---- out-of-span caching (Section 3.3) ----------------------------------------------

class RecordingPredictor:
    """State-independent confidences; records how it was called."""

    def __init__(self, conf, pred):
        self.conf, self.pred, self.calls = conf, pred, []

    def __call__(self, tokens, active):
        self.calls.append(("plain", active.copy(), None))
        return self.pred.copy(), np.where(active == 1, self.conf, 0).astype(np.float32)

    def cached(self, tokens, active, skip):
        self.calls.append(("cached", active.copy(), skip.copy()))
        return self.pred.copy(), np.where(active == 1, self.conf, 0).astype(np.float32)


def test_out_of_span_caching_protocol():
    # positions 2..7 confident, 8..13 not: slow, slow -> e_cycle = 7; the fast stage needs two steps
    # (top-1 fallback is avoided: 0.95 > tau_high, but convergence holds from the second look only)
    P, L = 2, 14
    conf = np.full((1, L), 0.05, np.float32); conf[0, 2:8] = 0.95; conf[0, 12] = 0.5
    pred = np.arange(L, dtype=np.int32)[None] + 200
    tokens = np.full((1, L), 999, np.int32); mask = np.zeros((1, L), np.uint8); mask[:, P:] = 1
    rp = RecordingPredictor(conf, pred)
    trace = []
    p = sf.DecodeParams(max_steps=100, tau_min_conf=0.1, tau_high_conf=0.9, conv_mode=0, k_fast=1,
                        out_of_span_cache=True)
    # make the fast stage last: only one position clears tau_high per step
    conf[0, 2:8] = [0.95, 0.5, 0.5, 0.5, 0.5, 0.5]
    steps = sf.decode(rp, tokens, mask, P, L, p, trace)
    assert not mask.any()
    modes = [(sps[0].stage, sps[0].cache_mode) for sps, _ in trace]
    # every fast stage starts with a refresh and continues with reuse steps; slow steps never cache
    for i, (stage, mode) in enumerate(modes):
        if stage == sf.SLOW:
            assert mode == sf.CACHE_OFF
        else:
            first = i == 0 or modes[i - 1][0] == sf.SLOW or trace[i][0][0].s_cycle != trace[i - 1][0][0].s_cycle
            assert mode == (sf.CACHE_REFRESH if first else sf.CACHE_REUSE)
    assert any(m == sf.CACHE_REUSE for _, m in modes)
    kinds = [c[0] for c in rp.calls]
    assert kinds == ["plain" if m == sf.CACHE_OFF else "cached" for _, m in modes]
    cur_mask = np.zeros(L, np.uint8); cur_mask[P:] = 1
    for (kind, active, skip), (sps, res) in zip(rp.calls, trace):
        sp = sps[0]
        mask_before = cur_mask.copy()
        cur_mask[res[0][0]] = 0
        if sp.cache_mode == sf.CACHE_REFRESH:
            # confidences right of the span are evaluated, nothing is skipped
            assert not skip.any()
            lo, hi = sp.eval_window()
            assert (lo, hi) == (sp.s_cycle, L - 1) and active[0, sp.e_cycle + 1:].sum() > 0
        if sp.cache_mode == sf.CACHE_REUSE:
            # skipped = masked, right of the span, confidence below tau_min at the refresh step
            want = np.zeros(L, np.uint8)
            for i in range(sp.e_cycle + 1, L):
                want[i] = 1 if conf[0, i] < 0.1 else 0
            assert np.array_equal(skip[0], want & mask_before) and skip[0].sum() > 0
            assert not (skip[0][:sp.e_cycle + 1]).any() and not (skip & active).any()
            assert skip[0, 12] == 0                          # 0.5 >= tau_min: recomputed
            assert all(sp.s_cycle <= i <= sp.e_cycle for i in res[0][0])


def test_caching_does_not_change_a_state_independent_trajectory():
    # when predictions do not depend on the state, stale features cannot matter:
    # the decode with caching must take exactly the steps of the decode without
    rng = np.random.default_rng(12)
    P, G = 3, 40
    L = P + G
    conf = (rng.random((2, L)) ** 3).astype(np.float32)
    pred = rng.integers(0, 50, (2, L)).astype(np.int32)
    outs = []
    for cache in (False, True):
        tokens = np.full((2, L), 99, np.int32); mask = np.zeros((2, L), np.uint8); mask[:, P:] = 1
        trace = []
        p = sf.DecodeParams(max_steps=10 ** 6, tau_min_conf=0.2, tau_high_conf=0.6, out_of_span_cache=cache)
        steps = sf.decode(RecordingPredictor(conf, pred), tokens, mask, P, L, p, trace)
        outs.append((steps, [[r[0] for r in res] for _, res in trace], tokens.copy()))
    assert outs[0][0] == outs[1][0] and outs[0][1] == outs[1][1] and np.array_equal(outs[0][2], outs[1][2])


def test_cached_decode_on_a_small_model_keeps_the_invariants():
    from util import OraclePredictor
    cfg = dict(synth.CONFIGS["tiny"], vocab=257, mask_id=256, prompt=6, gen=24, d_model=64, n_heads=2,
               head_dim=32, d_ffn=96, n_layers=2)
    w = synth.make_weights(cfg, std=0.25)
    tokens, mask, _ = synth.make_state(cfg, batch=2)
    tokens, mask = tokens.numpy().copy(), mask.numpy().copy()
    B, L = tokens.shape
    P = cfg["prompt"]
    predict = OraclePredictor(synth.model_config(cfg), weights_bits(w), B, L)
    _, c0 = predict(tokens, mask)
    tau_high = float(np.quantile(c0[mask == 1], 0.8)); tau_min = float(np.quantile(c0[mask == 1], 0.5))
    predict.recomputed.clear()
    p = sf.DecodeParams(max_steps=10 ** 6, tau_min_conf=tau_min, tau_high_conf=tau_high, out_of_span_cache=True)
    trace = []
    steps = sf.decode(predict, tokens, mask, P, L, p, trace)
    assert not mask.any() and steps <= B * cfg["gen"] and not (tokens == cfg["mask_id"]).any()
    reuse = [n for (sps, _), n in zip(trace, predict.recomputed) if any(sp.cache_mode == sf.CACHE_REUSE for sp in sps)]
    assert reuse and min(reuse) < B * L                   # some steps really skipped positions
    for sps, res in trace:
        for b in range(B):
            if sps[b].stage != sf.IDLE:
                assert len(res[b][0]) >= 1
                lo, hi = sps[b].window()
                assert all(lo <= i <= hi for i in res[b][0])


# ---- prompt caching (the long-interval half of dLLM-Cache, Section 4.2) -------------

def test_prompt_caching_protocol_and_state_independent_trajectory():
    rng = np.random.default_rng(21)
    P, G = 4, 30
    L = P + G
    conf = (rng.random((2, L)) ** 3).astype(np.float32)
    pred = rng.integers(0, 50, (2, L)).astype(np.int32)
    runs = []
    for kp, oos in ((0, False), (3, False), (3, True), (1, True)):
        tokens = np.full((2, L), 99, np.int32); mask = np.zeros((2, L), np.uint8); mask[:, P:] = 1
        rp = RecordingPredictor(conf, pred)
        trace = []
        p = sf.DecodeParams(max_steps=10 ** 6, tau_min_conf=0.2, tau_high_conf=0.6, out_of_span_cache=oos,
                            prompt_cache_interval=kp)
        steps = sf.decode(rp, tokens, mask, P, L, p, trace)
        runs.append((steps, [[r[0] for r in res] for _, res in trace], tokens.copy()))
        if kp:
            assert all(c[0] == "cached" for c in rp.calls)
            for n, ((kind, active, skip), (sps, _)) in enumerate(zip(rp.calls, trace)):
                # every K_p-th step recomputes the prompt, the others leave all of it out (a sequence in an
                # out-of-span refresh step recomputes everything)
                for q in range(2):
                    full = n % kp == 0 or sps[q].cache_mode == sf.CACHE_REFRESH
                    assert not skip[q, :P].any() if full else skip[q, :P].all()
                assert not (skip & active).any()
                if not oos:
                    assert not skip[:, P:].any()
    for r in runs[1:]:                                   # predictions do not depend on the state here
        assert r[0] == runs[0][0] and r[1] == runs[0][1] and np.array_equal(r[2], runs[0][2])


def test_prompt_caching_with_interval_one_is_the_plain_decode():
    from util import OraclePredictor
    cfg = dict(synth.CONFIGS["tiny"], vocab=257, mask_id=256, prompt=6, gen=16, d_model=64, n_heads=2,
               head_dim=32, d_ffn=96, n_layers=2)
    w = synth.make_weights(cfg, std=0.25)
    outs = []
    for kp in (0, 1, 4):
        tokens, mask, _ = synth.make_state(cfg, batch=2)
        tokens, mask = tokens.numpy().copy(), mask.numpy().copy()
        B, L = tokens.shape
        predict = OraclePredictor(synth.model_config(cfg), weights_bits(w), B, L)
        p = sf.DecodeParams(max_steps=10 ** 6, tau_min_conf=0.004, tau_high_conf=0.0045, prompt_cache_interval=kp)
        trace = []
        steps = sf.decode(predict, tokens, mask, cfg["prompt"], L, p, trace)
        assert not mask.any() and not (tokens == cfg["mask_id"]).any()
        outs.append((steps, tokens.copy(), list(predict.recomputed)))
    # K_p = 1: every step is a complete forward through the cached path = the plain decode, exactly
    assert outs[1][0] == outs[0][0] and np.array_equal(outs[1][1], outs[0][1])
    # K_p = 4: three of four steps leave the prompt out
    rec = outs[2][2]
    assert all(n == (B * L if i % 4 == 0 else B * (L - cfg["prompt"])) for i, n in enumerate(rec))


# ---- response caching (the short-interval half of dLLM-Cache, Section 4.2) ----------

def test_interval_skip_hand_worked():
    """P = 2, G = 6: K_p = 2, K_r = 3.  Step 0 refreshes both, step 1 leaves out the prompt and the
    response outside each rated range, step 2 only the response part, step 3 only the prompt, step 6 nothing."""
    P, L = 2, 8
    p = sf.DecodeParams(max_steps=99, prompt_cache_interval=2, response_cache_interval=3)
    slow = sf.StageParams(sf.SLOW, 4, L - 1, 1, 0.1, 0.9, 0, P, L)           # rates [4, 7]
    fast = sf.StageParams(sf.FAST, 3, 5, 1, 0.1, 0.9, 0, P, L)               # rates [3, 5]
    idle = sf.StageParams(sf.IDLE, 0, -1, 1, 0.1, 0.9, 0, P, L)              # rates nothing
    wide = sf.StageParams(sf.FAST, 3, 5, 1, 0.1, 0.9, 0, P, L, sf.CACHE_REFRESH)   # rates [3, 7]
    sps = [slow, fast, idle, wide]
    assert sf.interval_skip(sf.DecodeParams(max_steps=99), 1, sps, P, L, L) is None
    assert not sf.interval_skip(p, 0, sps, P, L, L).any() and not sf.interval_skip(p, 6, sps, P, L, L).any()
    assert sf.interval_skip(p, 1, sps, P, L, L).tolist() == [[1, 1, 1, 1, 0, 0, 0, 0], [1, 1, 1, 0, 0, 0, 1, 1],
                                                             [1, 1, 1, 1, 1, 1, 1, 1], [1, 1, 1, 0, 0, 0, 0, 0]]
    assert sf.interval_skip(p, 2, sps, P, L, L).tolist() == [[0, 0, 1, 1, 0, 0, 0, 0], [0, 0, 1, 0, 0, 0, 1, 1],
                                                             [0, 0, 1, 1, 1, 1, 1, 1], [0, 0, 1, 0, 0, 0, 0, 0]]
    assert sf.interval_skip(p, 3, sps, P, L, L).tolist() == [[1, 1, 0, 0, 0, 0, 0, 0]] * 4


def test_response_caching_protocol_and_state_independent_trajectory():
    rng = np.random.default_rng(22)
    P, G = 4, 30
    L = P + G
    conf = (rng.random((2, L)) ** 3).astype(np.float32)
    pred = rng.integers(0, 50, (2, L)).astype(np.int32)
    runs = []
    for kr, kp, oos in ((0, 0, False), (3, 0, False), (2, 5, True), (1, 0, True)):
        tokens = np.full((2, L), 99, np.int32); mask = np.zeros((2, L), np.uint8); mask[:, P:] = 1
        rp = RecordingPredictor(conf, pred)
        trace = []
        p = sf.DecodeParams(max_steps=10 ** 6, tau_min_conf=0.2, tau_high_conf=0.6, out_of_span_cache=oos,
                            prompt_cache_interval=kp, response_cache_interval=kr)
        steps = sf.decode(rp, tokens, mask, P, L, p, trace)
        runs.append((steps, [[r[0] for r in res] for _, res in trace], tokens.copy()))
        if kr:
            assert all(c[0] == "cached" for c in rp.calls)
            skipped = 0
            for n, ((kind, active, skip), (sps, _)) in enumerate(zip(rp.calls, trace)):
                assert not (skip & active).any()
                for q in range(2):
                    lo, hi = sps[q].eval_window()
                    outside = np.array([not (lo <= i <= hi) for i in range(P, L)])
                    if sps[q].cache_mode == sf.CACHE_REFRESH:
                        assert not skip[q].any()                 # first step of a fast stage: complete
                    elif n % kr:
                        assert np.array_equal(skip[q, P:] != 0, outside)
                        skipped += int(outside.sum())
                    elif sps[q].cache_mode != sf.CACHE_REUSE:
                        assert not skip[q, P:].any()             # every K_r-th step recomputes the response
                    if kp and sps[q].cache_mode != sf.CACHE_REFRESH:
                        assert skip[q, :P].all() if n % kp else not skip[q, :P].any()
            assert skipped > 0 or kr == 1
    for r in runs[1:]:                                   # predictions do not depend on the state here
        assert r[0] == runs[0][0] and r[1] == runs[0][1] and np.array_equal(r[2], runs[0][2])


def test_response_caching_with_interval_one_is_the_plain_decode():
    from util import OraclePredictor
    cfg = dict(synth.CONFIGS["tiny"], vocab=257, mask_id=256, prompt=6, gen=16, d_model=64, n_heads=2,
               head_dim=32, d_ffn=96, n_layers=2)
    w = synth.make_weights(cfg, std=0.25)
    outs = []
    for kr in (0, 1, 3):
        tokens, mask, _ = synth.make_state(cfg, batch=2)
        tokens, mask = tokens.numpy().copy(), mask.numpy().copy()
        B, L = tokens.shape
        predict = OraclePredictor(synth.model_config(cfg), weights_bits(w), B, L)
        # confidences of this model sit in 0.08 .. 0.26: spans of one to a few positions, many cycles
        p = sf.DecodeParams(max_steps=10 ** 6, tau_min_conf=0.3, tau_high_conf=0.95, k_max=2, w_hist=1,
                            response_cache_interval=kr)
        trace = []
        steps = sf.decode(predict, tokens, mask, cfg["prompt"], L, p, trace)
        assert not mask.any() and not (tokens == cfg["mask_id"]).any()
        outs.append((steps, tokens.copy(), list(predict.recomputed), [sps for sps, _ in trace]))
    # K_r = 1: every step is a complete forward through the cached path = the plain decode, exactly
    assert outs[1][0] == outs[0][0] and np.array_equal(outs[1][1], outs[0][1])
    # K_r = 3: two of three steps recompute the prompt and each sequence's rated range only
    rec, spss = outs[2][2], outs[2][3]
    for n, (cnt, sps) in enumerate(zip(rec, spss)):
        full = B * L
        part = sum(cfg["prompt"] + max(0, sp.eval_window()[1] - sp.eval_window()[0] + 1) for sp in sps)
        assert cnt == (full if n % 3 == 0 else part)
    assert any(c < B * L for c in rec)


# ---- Algorithm 1 as nested loops (alg1_sequence / decode_alg1) ---------------------
# Pinned by hand-worked runs, then held against the state-machine form (Controller / decode):
# the two are written in different shapes, so a misreading has to be made twice to go unseen.

def run_alg1(conf, pred, P, L, p):
    B = conf.shape[0]
    tokens = np.full((B, L), 999, np.int32); mask = np.zeros((B, L), np.uint8); mask[:, P:] = 1
    trace = []
    steps = sf.decode_alg1(RecordingPredictor(conf, pred), tokens, mask, P, L, p, trace)
    return steps, trace, tokens, mask


def test_alg1_hand_worked_stable_cycle():
    # confident block 2..7, the rest below tau_min; Section 3.3 step by step:
    #  slow: top-1 of [2, 13] is position 2 (ties -> lower position), e_cand = 7
    #  slow: commits 3, e_cand = 7 -> H = {7, 7}, variance 0 < 1 -> e_cycle = 7
    #  fast: masks 4..7 of [2, 7] all exceed 0.9 and repeat their prediction -> committed together
    #  then nothing exceeds tau_min: e_cand = leftmost mask; cycles of two slow steps whose spans are
    #  already clean when they end (H = {8, 9} -> floor(8.5) = 8, H = {10, 11} -> 10, H = {12, 13} -> 12)
    P, L = 2, 14
    conf = np.full((1, L), 0.05, np.float32); conf[0, 2:8] = 0.95
    pred = np.arange(L, dtype=np.int32)[None] + 200
    p = sf.DecodeParams(max_steps=100, tau_min_conf=0.1, tau_high_conf=0.9, conv_mode=1)
    steps, trace, tokens, mask = run_alg1(conf, pred, P, L, p)
    end = L - 1
    assert [t[0] for t in trace] == [
        (sf.SLOW, 2, end, [2]), (sf.SLOW, 2, end, [3]), (sf.FAST, 2, 7, [4, 5, 6, 7]),
        (sf.SLOW, 8, end, [8]), (sf.SLOW, 8, end, [9]),
        (sf.SLOW, 9, end, [10]), (sf.SLOW, 9, end, [11]),
        (sf.SLOW, 11, end, [12]), (sf.SLOW, 11, end, [13])]
    assert steps == 9 and not mask.any() and np.array_equal(tokens[0, P:], pred[0, P:])


def test_alg1_hand_worked_kmax_fallback_and_fast_fallback():
    # e_cand walks 9, 7, 5 (each is committed by the step that reports it): windows {9,7} and {7,5}
    # have variance 1, not < 1, so K_max = 3 ends the stage with the LAST candidate, e_cycle = 5;
    # nothing in [1, 5] reaches tau_high, so every fast step falls back to the top-1 of the span.
    P, L = 1, 10
    conf = np.full((1, L), 0.05, np.float32)
    conf[0, 9], conf[0, 7], conf[0, 5], conf[0, 3] = 0.5, 0.4, 0.3, 0.2
    pred = np.arange(L, dtype=np.int32)[None]
    p = sf.DecodeParams(max_steps=100, k_max=3, w_hist=2, sigma2_stable=1.0, tau_min_conf=0.1, tau_high_conf=0.9)
    steps, trace, tokens, mask = run_alg1(conf, pred, P, L, p)
    assert [t[0] for t in trace] == [
        (sf.SLOW, 1, 9, [9]), (sf.SLOW, 1, 9, [7]), (sf.SLOW, 1, 9, [5]),
        (sf.FAST, 1, 5, [3]), (sf.FAST, 1, 5, [1]), (sf.FAST, 1, 5, [2]), (sf.FAST, 1, 5, [4]),
        (sf.SLOW, 6, 9, [6]), (sf.SLOW, 6, 9, [8])]
    assert steps == 9 and not mask.any()
    # N = 4 stops after the first fast step
    p4 = sf.DecodeParams(max_steps=4, k_max=3, w_hist=2, sigma2_stable=1.0, tau_min_conf=0.1, tau_high_conf=0.9)
    steps, trace, tokens, mask = run_alg1(conf, pred, P, L, p4)
    assert steps == 4 and [t[0][0] for t in trace] == [sf.SLOW, sf.SLOW, sf.SLOW, sf.FAST] and mask.sum() == 5


def state_machine_trace(trace):
    """decode()'s trace in the shape of decode_alg1's."""
    out = []
    for sps, res in trace:
        out.append([None if sp.stage == sf.IDLE else (sp.stage, sp.s_cycle, sp.window()[1], r[0])
                    for sp, r in zip(sps, res)])
    return out


@pytest.mark.parametrize("k_max,w_hist,sigma2", [(8, 2, 1.0), (1, 1, 1.0), (3, 3, 0.23), (4, 2, 30.0), (2, 4, 1.0)])
@pytest.mark.parametrize("tau_min,tau_high,conv,k_slow,k_fast", [(0.2, 0.6, 0, 1, 1), (0.1, 0.9, 1, 2, 3),
                                                                 (-1.0, 1.0, 0, 1, 1), (0.5, 0.5, 1, 3, 1)])
@pytest.mark.parametrize("cache", [False, True])
def test_alg1_loops_and_state_machine_agree_on_state_independent_confidences(k_max, w_hist, sigma2, tau_min, tau_high,
                                                                             conv, k_slow, k_fast, cache):
    rng = np.random.default_rng(100 * k_max + w_hist)
    P, G, B = 3, 37, 3
    L = P + G
    conf = (rng.random((B, L)) ** 2).astype(np.float32)
    conf[1, P + 5:P + 20] = 0.97                       # a confident region in one sequence
    pred = rng.integers(0, 50, (B, L)).astype(np.int32)
    for max_steps in (10 ** 6, 7):
        p = sf.DecodeParams(max_steps=max_steps, k_max=k_max, w_hist=w_hist, sigma2_stable=sigma2, tau_min_conf=tau_min,
                            tau_high_conf=tau_high, k_slow=k_slow, k_fast=k_fast, conv_mode=conv, out_of_span_cache=cache)
        s1, t1, tok1, m1 = run_alg1(conf, pred, P, L, p)
        tok2 = np.full((B, L), 999, np.int32); m2 = np.zeros((B, L), np.uint8); m2[:, P:] = 1
        t2 = []
        rp = RecordingPredictor(conf, pred)
        s2 = sf.decode(rp, tok2, m2, P, L, p, t2)
        assert s1 == s2 and t1 == state_machine_trace(t2)
        assert np.array_equal(tok1, tok2) and np.array_equal(m1, m2)


@pytest.mark.parametrize("cache,kp,kr", [(False, 0, 0), (True, 0, 0), (True, 3, 2), (False, 0, 3)])
def test_alg1_loops_and_state_machine_agree_on_a_small_model(cache, kp, kr):
    """State-dependent predictions (and stale cached features): the two forms must ask the predictor
    for the same steps, with the same cached sets, and end in the same tokens."""
    cfg = dict(synth.CONFIGS["tiny"], vocab=257, mask_id=256, prompt=6, gen=20, d_model=64, n_heads=2,
               head_dim=32, d_ffn=96, n_layers=1)
    w = synth.make_weights(cfg, std=0.25)
    mc = synth.model_config(cfg)
    P, L = cfg["prompt"], cfg["prompt"] + cfg["gen"]
    tok0, mask0, _ = synth.make_state(cfg, batch=2)
    from util import OraclePredictor
    c0 = OraclePredictor(mc, weights_bits(w), 2, L)(tok0.numpy(), mask0.numpy())[1]
    tau_min, tau_high = float(np.quantile(c0[mask0.numpy() == 1], 0.4)), float(np.quantile(c0[mask0.numpy() == 1], 0.8))
    p = sf.DecodeParams(max_steps=10 ** 6, k_max=3, tau_min_conf=tau_min, tau_high_conf=tau_high, conv_mode=1,
                        out_of_span_cache=cache, prompt_cache_interval=kp, response_cache_interval=kr)
    runs = []
    for fn in (sf.decode_alg1, sf.decode):
        tokens, mask = tok0.numpy().copy(), mask0.numpy().copy()
        pr = OraclePredictor(mc, weights_bits(w), 2, L)
        trace = []
        steps = fn(pr, tokens, mask, P, L, p, trace)
        runs.append((steps, trace if fn is sf.decode_alg1 else state_machine_trace(trace), tokens, pr.recomputed))
    assert runs[0][0] == runs[1][0] and runs[0][1] == runs[1][1]
    assert np.array_equal(runs[0][2], runs[1][2]) and runs[0][3] == runs[1][3]
    assert not (runs[0][2] == cfg["mask_id"]).any()
    if cache or kp or kr:
        assert min(runs[0][3]) < 2 * L            # some step really left positions out
