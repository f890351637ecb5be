"""GPU parity of the selector (dllm_select) against the oracle, on identical
seeded bf16 logits: arg max ids bit-exact, confidences to 1e-3 relative (the
bar; the kernel is in fact much closer), commit sets / e_cand / state transition
bit-exact wherever the oracle's own decision is not within rounding of a
boundary."""
import numpy as np
import pytest
import torch

import oracle
from oracle import slowfast as sf
from paper_2506_10848_amd import synth
from util import bits

pytestmark = pytest.mark.gpu

CONF_RTOL = 1e-3          # the stated bar for fp32 confidences
TIE_RTOL = 2e-5           # decisions closer than this to a boundary are not compared bit-exactly


def binding():
    from paper_2506_10848_amd import binding as b
    b.lib()
    b.reload_env()          # the environment switches a test may have set (or a finished test has restored)
    return b


def oracle_step_on_logits(logits_bits, mask_id, tokens, mask, prev, sps):
    """Oracle: row phase on the given logits + selection + transition."""
    B, L, V = logits_bits.shape

    def predict(tok, active):
        pred, conf = oracle.row_phase(logits_bits.reshape(B * L, V), mask_id, active.reshape(-1))
        return pred.reshape(B, L), conf.reshape(B, L)

    cache = {}

    def predict_cached(tok, active):
        cache["out"] = predict(tok, active)
        cache["active"] = active
        return cache["out"]

    res = sf.step(predict_cached, tokens, mask, prev, sps)
    return res, cache["out"][0], cache["out"][1], cache["active"]


def ambiguous(sp, mask_before, conf, pred=None, prev=None):
    """True if a decision of the oracle sits within rounding of a boundary, so
    that a correct fp32 kernel may legitimately decide the other way.  With pred / prev
    given, the top-k boundary is only looked at when the step can reach the top-k rule at
    all (slow stage, or a fast stage without a position that is safely in S_high)."""
    lo, hi = sp.window()
    idx = [i for i in range(max(lo, 0), min(hi, len(conf) - 1) + 1) if mask_before[i]]
    c = np.array([conf[i] for i in idx], np.float64)
    if c.size == 0:
        return False
    near = lambda a, b: abs(a - b) <= TIE_RTOL * max(abs(a), abs(b))
    if any(near(x, sp.tau_min_conf) for x in c):
        return True
    if sp.stage == sf.FAST and any(near(x, sp.tau_high_conf) for x in c):
        return True
    if sp.stage == sf.FAST and pred is not None:
        safe_high = [i for i in idx if conf[i] > sp.tau_high_conf * (1 + TIE_RTOL)
                     and (sp.conv_mode == 0 or int(pred[i]) == int(prev[i]))]
        if safe_high:
            return False                      # S_high is not empty on either side: top-k is not consulted
    s = np.sort(c)[::-1]
    k = sp.top_k
    if k < s.size and near(s[k - 1], s[k]) and s[k - 1] != s[k]:
        return True
    return False


def run_case(B, L, V, mask_id, logits, mask, prev, sps, capacity=None):
    b = binding()
    dev = "cuda"
    tokens = torch.full((B, L), mask_id, dtype=torch.int32)
    tokens[mask == 0] = 5
    lg_bits = bits(logits)
    # oracle
    o_tok, o_mask, o_prev = tokens.numpy().copy(), mask.numpy().copy(), prev.numpy().copy()
    mask_before = o_mask.copy()
    res, o_pred, o_conf, active = oracle_step_on_logits(lg_bits, mask_id, o_tok, o_mask, o_prev, sps)
    # gpu
    g_tok, g_mask, g_prev = tokens.to(dev), mask.to(dev), prev.to(dev)
    pred = torch.full((B, L), -7, dtype=torch.int32, device=dev)
    conf = torch.full((B, L), -7.0, dtype=torch.float32, device=dev)
    cap = L if capacity is None else capacity
    out = b.CommitList(B, cap)
    csp = [b.stage_params(s.stage, s.s_cycle, s.e_cycle, s.top_k, s.tau_min_conf, s.tau_high_conf, s.conv_mode,
                          s.gen_start, s.gen_end) for s in sps]
    b.select(logits.to(dev), g_tok, g_mask, g_prev, csp, mask_id, pred, conf, out)
    torch.cuda.synchronize()
    pred, conf = pred.cpu().numpy(), conf.cpu().numpy()
    act = active.astype(bool)
    # row phase: ids bit-exact, confidences within the bar; inactive rows untouched
    assert np.array_equal(pred[act], o_pred[act])
    assert np.all(pred[~act] == -7) and np.all(conf[~act] == -7.0)
    if act.any():
        rel = np.abs(conf[act].astype(np.float64) - o_conf[act]) / o_conf[act]
        assert rel.max() <= CONF_RTOL
        assert rel.max() <= 2e-5, f"kernel confidence drifted: {rel.max()}"
    got = out.to_host()
    n_amb = 0
    for s in range(B):
        commit, toks, cfs, e_cand, first, left = res[s][:6]
        g_pos, g_toks, g_cfs, g_e, g_first, g_left = got[s]
        assert g_first == first
        if ambiguous(sps[s], mask_before[s], o_conf[s]):
            n_amb += 1
            lo, hi = sps[s].window()
            assert all(lo <= i <= hi and mask_before[s, i] for i in g_pos)
            assert g_pos == sorted(g_pos)
            continue
        assert g_pos == commit, f"sequence {s}"
        assert g_toks == toks
        assert np.allclose(g_cfs, cfs, rtol=CONF_RTOL)
        assert g_e == e_cand and g_left == left
        assert np.array_equal(g_tok[s].cpu().numpy(), o_tok[s])
        assert np.array_equal(g_mask[s].cpu().numpy(), o_mask[s])
        assert np.array_equal(g_prev[s].cpu().numpy(), o_prev[s])
    return n_amb, res


def make_inputs(name, B, L, V, seed_shift=0, quant=None):
    cfg = dict(synth.CONFIGS[name], seed=synth.CONFIGS[name]["seed"] + seed_shift)
    logits, mask, planted, agree, other = synth.make_selector_inputs(cfg, "cpu", batch=B, seq=L, vocab=V)
    if quant:                                   # coarse grid -> many exact ties for the arg max
        logits = (torch.round(logits.float() / quant) * quant).to(torch.bfloat16)
    mask_id = min(cfg["mask_id"], V - 1)
    # previous prediction: the current arg max where `agree`, a different seeded id elsewhere
    pred, _ = oracle.row_phase(bits(logits).reshape(B * L, V), mask_id)
    pred = torch.from_numpy(pred.reshape(B, L))
    prev = torch.where(agree, pred, torch.where(other == pred, (other + 1) % (V - 1), other)).to(torch.int32)
    return logits, mask, prev, mask_id


SHAPES = [  # B, L, V
    (2, 37, 2048),        # ragged L, one 4-chunk group per lane + nothing else
    (3, 96, 32000),       # tail chunks after the unrolled groups
    (1, 70, 126464),      # full vocabulary width
    (2, 19, 1003),        # V % 8 != 0: scalar row path
    (1, 5, 8),            # a single chunk
]


@pytest.mark.parametrize("B,L,V", SHAPES)
@pytest.mark.parametrize("peaked", ["selector", "selector_peaked"])
def test_selector_slow_and_fast(B, L, V, peaked):
    logits, mask, prev, mask_id = make_inputs(peaked, B, L, V)
    gs, ge = 2, L - 1                      # generated region inside the sequence
    mask[:, :gs] = 0; mask[:, ge:] = 0
    total_amb = 0
    for stage, s, e, k, conv in [(sf.SLOW, gs, 0, 1, 1), (sf.SLOW, gs + 1, 0, 3, 0), (sf.FAST, gs, (gs + ge) // 2, 1, 1),
                                 (sf.FAST, gs, ge - 1, 2, 0), (sf.SLOW, gs, 0, 10 ** 6, 0)]:
        tau_high = 0.9 if peaked == "selector_peaked" else 0.004
        tau_min = 0.1 if peaked == "selector_peaked" else 0.001
        sps = [sf.StageParams(stage, s, e, k, tau_min, tau_high, conv, gs, ge) for _ in range(B)]
        amb, res = run_case(B, L, V, mask_id, logits, mask.clone(), prev.clone(), sps)
        total_amb += amb
    assert total_amb <= 2


def test_threshold_paths_fire_on_peaked_logits():
    """Sanity of the workload itself: with +U(8,18) peaks both thresholds are
    crossed by some rows and missed by others, and the convergence gate bites."""
    B, L, V = 2, 128, 126464
    logits, mask, prev, mask_id = make_inputs("selector_peaked", B, L, V)
    sps = [sf.StageParams(sf.FAST, 0, L - 1, 1, 0.1, 0.9, 1, 0, L) for _ in range(B)]
    amb, res = run_case(B, L, V, mask_id, logits, mask.clone(), prev.clone(), sps)
    sps0 = [sf.StageParams(sf.FAST, 0, L - 1, 1, 0.1, 0.9, 0, 0, L) for _ in range(B)]
    amb0, res0 = run_case(B, L, V, mask_id, logits, mask.clone(), prev.clone(), sps0)
    for s in range(B):
        assert 1 < len(res[s][0]) < len(res0[s][0]) < int(mask[s].sum())
        assert res[s][3] >= 0


def test_exact_ties_pick_the_lowest_id():
    B, L, V = 2, 33, 4096
    logits, mask, prev, mask_id = make_inputs("selector", B, L, V, seed_shift=3, quant=1.0)
    # the planted peak may be unique: flatten it so that several ids share the max
    logits = torch.clamp(logits.float(), max=2.0).to(torch.bfloat16)
    flat = bits(logits).reshape(B * L, V)
    vals = oracle.bf16_to_f64(flat)
    assert ((vals == vals.max(axis=1, keepdims=True)).sum(axis=1) > 1).all()
    sps = [sf.StageParams(sf.SLOW, 0, 0, 2, 0.1, 0.9, 0, 0, L) for _ in range(B)]
    run_case(B, L, V, mask_id, logits, mask.clone(), prev.clone(), sps)


def test_mask_id_is_never_predicted():
    B, L, V = 1, 12, 2048
    logits, mask, prev, mask_id = make_inputs("selector", B, L, V, seed_shift=5)
    logits[:, :, mask_id] = 30.0                                   # would win every row
    mask[:] = 1
    sps = [sf.StageParams(sf.FAST, 0, L - 1, 1, 0.1, 0.9, 0, 0, L)]
    amb, res = run_case(B, L, V, mask_id, logits, mask.clone(), prev.clone(), sps)
    assert all(t != mask_id for t in res[0][1])


def test_degenerate_windows_and_states():
    B, L, V = 4, 24, 2048
    logits, mask, prev, mask_id = make_inputs("selector_peaked", B, L, V, seed_shift=9)
    mask[0] = 0                                                    # nothing masked at all
    mask[1] = 0; mask[1, 7] = 1                                    # one masked position, window of one
    sps = [sf.StageParams(sf.SLOW, 0, 0, 1, 0.1, 0.9, 1, 0, L),
           sf.StageParams(sf.FAST, 7, 7, 1, 0.1, 0.9, 1, 0, L),
           sf.StageParams(sf.IDLE, 0, -1, 1, 0.1, 0.9, 1, 0, L),   # rides along, nothing selected
           sf.StageParams(sf.FAST, 3, 3, 4, 0.1, 0.9, 0, 3, 4)]    # generated region of one position
    mask[3, 3] = 1
    amb, res = run_case(B, L, V, mask_id, logits, mask.clone(), prev.clone(), sps)
    assert res[0][0] == [] and res[0][3] == -1 and res[0][4] == -1
    assert res[1][0] == [7]
    assert res[2][0] == [] and res[2][5] == int(mask[2].sum())
    assert res[3][0] == [3]


def test_long_sequence_and_many_commits():
    # L spans several passes of the 512-thread sequence phase; large top-k uses rank counting
    B, L, V = 2, 1300, 512
    logits, mask, prev, mask_id = make_inputs("selector_peaked", B, L, V, seed_shift=11)
    for stage, k in [(sf.SLOW, 37), (sf.FAST, 5), (sf.SLOW, 1)]:
        sps = [sf.StageParams(stage, 10, L - 20, k, 0.1, 0.9, 1, 10, L - 3) for _ in range(B)]
        run_case(B, L, V, mask_id, logits, mask.clone(), prev.clone(), sps)


def test_top_k_among_thousands_of_candidates():
    """The longest sequence the library takes, every position masked: top-k with 1 < k < candidates over
    more than 1024 candidates goes through the bit-by-bit selection of the k-th largest key."""
    B, L, V = 2, 8192, 64
    logits, mask, prev, mask_id = make_inputs("selector", B, L, V, seed_shift=13)     # confidences spread over (0, 1)
    mask[:] = 1
    total_amb = 0
    for stage, lo, hi, k, tau_high in [(sf.SLOW, 0, L - 1, 32, 0.9), (sf.SLOW, 5, L - 1, 1500, 0.9),
                                       (sf.FAST, 100, 7000, 200, 2.0), (sf.SLOW, 0, L - 1, 8191, 0.9)]:
        sps = [sf.StageParams(stage, lo, hi, k, -1.0, tau_high, 0, 0, L) for _ in range(B)]
        amb, res = run_case(B, L, V, mask_id, logits, mask.clone(), prev.clone(), sps)
        total_amb += amb
        assert all(len(r[0]) == k for r in res)
    assert total_amb <= 4          # of 8 decisions; the rest were compared position by position


def test_error_paths_reach_the_caller():
    b = binding()
    B, L, V = 1, 8, 64
    logits = torch.zeros((B, L, V), dtype=torch.bfloat16, device="cuda")
    tok = torch.zeros((B, L), dtype=torch.int32, device="cuda")
    mask = torch.ones((B, L), dtype=torch.uint8, device="cuda")
    prev = torch.zeros((B, L), dtype=torch.int32, device="cuda")
    pred = torch.zeros((B, L), dtype=torch.int32, device="cuda")
    conf = torch.zeros((B, L), dtype=torch.float32, device="cuda")
    ok = dict(stage=0, s_cycle=0, e_cycle=7, top_k=1, tau_min_conf=.1, tau_high_conf=.9, conv_mode=0, gen_start=0,
              gen_end=8)

    def call(cap=8, mask_id=63, **kw):
        sp = b.stage_params(**dict(ok, **kw))
        b.select(logits, tok, mask, prev, [sp], mask_id, pred, conf, b.CommitList(B, cap))

    call()
    for kw, code in [(dict(top_k=0), b.EINVAL), (dict(stage=1, s_cycle=5, e_cycle=4), b.EINVAL),
                     (dict(stage=7), b.EINVAL), (dict(s_cycle=-1), b.EINVAL), (dict(gen_end=9), b.EINVAL),
                     (dict(stage=1, e_cycle=8), b.EINVAL), (dict(conv_mode=2), b.EINVAL),
                     (dict(cap=3), b.ECAPACITY), (dict(mask_id=64), b.EINVAL)]:
        with pytest.raises(b.DllmError) as ei:
            call(**kw)
        assert ei.value.code == code, kw
    torch.cuda.synchronize()
    assert int(mask.sum()) == 7                     # only the one good call committed anything


@pytest.mark.parametrize("workload", ["selector", "selector_peaked"])
def test_full_size_selector_workload_every_masked_row(workload):
    """The selector workload at its full size, 16 x 2048 x 126464 bf16 logits (8.3 GB, generated on the
    GPU), in the launch configuration the benchmark times: slow stage over whole sequences, then the fast
    stage over the first half of every sequence.  Every masked row of the windows goes through the oracle's
    row phase (logits copied to the host one sequence at a time): predictions bit-exact, confidences to
    the 1e-3 bar (and 2e-5 in fact); the 16 commit lists, e_cand, first_masked and the state after the
    transition against the oracle's selection rule on the oracle's confidences.  `selector` (+U(2,8)
    peaks) stays below tau_high everywhere and only rarely above tau_min: arg max / top-k fallback /
    sparse e_cand; `selector_peaked` (+U(8,18)) crosses both thresholds and the convergence gate."""
    b = binding()
    dev = "cuda"
    cfg = synth.CONFIGS[workload]
    B, L, V, mask_id = cfg["batch"], cfg["seq"], cfg["vocab"], cfg["mask_id"]
    logits, mask, planted, agree, other = synth.make_selector_inputs(cfg, dev)
    h_mask = mask.cpu().numpy()
    # the oracle's row phase over every masked row, one sequence of logits on the host at a time
    o_pred = np.full((B, L), -1, np.int32); o_conf = np.zeros((B, L), np.float32)
    for q in range(B):
        o_pred[q], o_conf[q] = oracle.row_phase(bits(logits[q]), mask_id, h_mask[q])
    # previous prediction: the current arg max on the seeded 70 %, another seeded id elsewhere
    pred_t = torch.from_numpy(o_pred)
    oth = other.cpu()
    prev = torch.where(agree.cpu(), pred_t, torch.where(oth == pred_t, (oth + 1) % (V - 1), oth)).to(torch.int32)
    tokens = torch.full((B, L), mask_id, dtype=torch.int32)
    tokens[mask.cpu() == 0] = 5
    n_amb = n_cmp = 0
    for stage, lo, hi, k, conv in [(sf.SLOW, 0, L - 1, 1, 1), (sf.FAST, 0, L // 2 - 1, 1, 1), (sf.FAST, 7, L - 9, 3, 0)]:
        sps = [sf.StageParams(stage, lo, hi, k, 0.1, 0.9, conv, 0, L) for _ in range(B)]
        g_tok, g_mask, g_prev = tokens.to(dev), mask.clone(), prev.to(dev)
        pred = torch.full((B, L), -7, dtype=torch.int32, device=dev)
        conf = torch.full((B, L), -7.0, dtype=torch.float32, device=dev)
        out = b.CommitList(B, L)
        csp = [b.stage_params(s.stage, s.s_cycle, s.e_cycle, s.top_k, s.tau_min_conf, s.tau_high_conf, s.conv_mode,
                              s.gen_start, s.gen_end) for s in sps]
        b.select(logits, g_tok, g_mask, g_prev, csp, mask_id, pred, conf, out)
        torch.cuda.synchronize()
        got = out.to_host()
        g_pred, g_conf = pred.cpu().numpy(), conf.cpu().numpy()
        act = np.stack([sf.active_rows(sps[q], h_mask[q]) for q in range(B)]).astype(bool)
        assert act.sum() > 4000
        assert np.array_equal(g_pred[act], o_pred[act])
        assert np.all(g_pred[~act] == -7) and np.all(g_conf[~act] == -7.0)        # other rows never touched
        rel = np.abs(g_conf[act].astype(np.float64) - o_conf[act]) / o_conf[act]
        assert rel.max() <= CONF_RTOL and rel.max() <= 2e-5
        g_tok, g_mask, g_prev = g_tok.cpu().numpy(), g_mask.cpu().numpy(), g_prev.cpu().numpy()
        n_multi = 0
        for q in range(B):
            commit, e_cand, first = sf.select(sps[q], h_mask[q], o_pred[q], o_conf[q], prev[q].numpy())
            g_pos, g_toks, g_cfs, g_e, g_first, g_left = got[q]
            assert g_first == first
            if ambiguous(sps[q], h_mask[q], o_conf[q], o_pred[q], prev[q].numpy()):
                n_amb += 1
                assert all(lo <= i <= hi and h_mask[q, i] for i in g_pos) and g_pos == sorted(g_pos)
                continue
            n_cmp += 1
            assert g_pos == commit and g_e == e_cand and g_left == int(h_mask[q].sum()) - len(commit)
            assert g_toks == [int(o_pred[q, i]) for i in commit]
            want_tok = tokens[q].numpy().copy(); want_tok[commit] = o_pred[q][commit]
            want_mask = h_mask[q].copy(); want_mask[commit] = 0
            want_prev = prev[q].numpy().copy(); want_prev[act[q]] = o_pred[q][act[q]]
            assert np.array_equal(g_tok[q], want_tok) and np.array_equal(g_mask[q], want_mask)
            assert np.array_equal(g_prev[q], want_prev)
            n_multi += len(commit) > 1
        if workload == "selector_peaked" and stage == sf.FAST:
            assert n_multi >= B - 3                    # the threshold path really fired
        print(f"{workload} stage {stage} k {k}: {n_cmp} sequences compared so far, {n_amb} within rounding of a boundary")
    # (peaked rows saturate near confidence 1, so the slow stage's top-1 often has a runner-up within 2e-5)
    assert n_cmp >= (2 * B - 3 if workload == "selector_peaked" else 3 * B - 3)
