"""SlowFast selection rule, stage controller and decode loop -- CPU oracle.

TEST INFRASTRUCTURE: plain Python over small arrays, written from Section 3.3
("SlowFast Sampling") and Algorithm 1 of the paper.  It imports nothing from
the HIP library.

Algorithm 1 appears twice, in two shapes that are checked against each other:
`alg1_sequence` / `decode_alg1` take its steps in the paper's order, as the
nested loops of the listing (outer cycle loop, exploratory loop, accelerated
loop) for one sequence; `Controller` / `decode` is the same method turned
inside out into a per-sequence state machine, which is what a batch that shares
one forward pass per step needs.

Positions are absolute and 0-based; a span [s, e] is inclusive at both ends.
The generated region is [gen_start, gen_end) and the prompt is never masked.

Readings taken where the paper is silent or at odds with itself:

* Candidates are masked positions only: a committed token is never revisited
  (one-way "unmask" wording of the cautious-decoding and in-span bullets).
* The [MASK] id is not a legal prediction (handled in the row phase).
* e_cand of a step whose confidences all fail tau_min is reported as -1; the
  controller then uses the leftmost masked position of the window.
* A step's commit set and its e_cand come from the same, pre-commit state.
* Ties: top-k ranks by (higher confidence, lower position); thresholds are
  strict ">" (eq. 6, eq. 9, and the "0.22 < 0.23" example of Fig. 3).
* The Convergence Principle at token level ("stable identity over recent
  steps"): with conv_mode = 1 a position joins S_high only if its prediction
  equals the previous step's prediction; conv_mode = 0 is Algorithm 1 as printed.
* The history H_W is reset at the start of every exploratory stage, the
  variance is the population variance, and the mean is floored.
* When K_max is reached without stability, e_cycle is the last e_cand
  (Algorithm 1's fallback branch).
* The fast stage repeats until no mask is left in [s_cycle, e_cycle]; then
  s_cycle <- e_cycle + 1.
* Every decision on a confidence is taken on its binary32 value.
* Out-of-span caching (optional, DecodeParams.out_of_span_cache): the first
  step of a fast stage is a complete prediction whose confidences cover
  [s_cycle, gen_end); the masked positions i > e_cycle with confidence below
  tau_min form the stage's cached set.  Their "features" are their keys and
  values in every layer as computed in that step.  The later steps of the
  stage do not recompute them: all other positions are recomputed from the
  current tokens and attend to those cached keys/values.  The set is dropped
  when the stage ends.  Committed positions are always recomputed, and so is
  the prompt unless prompt caching is on.
* Prompt caching (optional, DecodeParams.prompt_cache_interval = K_p > 0), the
  long-interval half of the dLLM-Cache scheme the paper combines its sampler
  with (Section 4.2, "Compatibility with dLLM-Cache"), in the simplest form
  that fits the same cache: every K_p-th step of a decode (counting from 0) is
  a complete forward that refreshes the keys/values of every position; in the
  steps between, the prompt positions are not recomputed and everyone attends
  to their cached keys/values.
* Response caching (optional, DecodeParams.response_cache_interval = K_r > 0),
  the short-interval half of that scheme, in the same simplest form: every
  K_r-th step of a decode (counting from 0) recomputes the whole response;
  in the steps between, the response positions outside the range the step
  rates ([s_cycle, end] in the slow stage, [s_cycle, e_cycle] in the fast
  stage) are not recomputed.  The first step of a fast stage with out-of-span
  caching stays a complete forward.  The cited scheme's value-based choice of
  response positions to refresh between the K_r-th steps is defined outside
  the paper and is not modelled.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Callable, List, Optional, Sequence, Tuple

import numpy as np

SLOW, FAST, IDLE = 0, 1, 2
CACHE_OFF, CACHE_REFRESH, CACHE_REUSE = 0, 1, 2


@dataclass
class StageParams:
    """What one denoising step needs to know about one sequence."""
    stage: int
    s_cycle: int
    e_cycle: int          # used by the fast stage only
    top_k: int            # k_slow or k_fast
    tau_min_conf: float
    tau_high_conf: float
    conv_mode: int
    gen_start: int
    gen_end: int
    cache_mode: int = 0   # CACHE_OFF, CACHE_REFRESH (first fast step of a stage) or CACHE_REUSE

    def eval_window(self) -> Tuple[int, int]:
        """Inclusive span whose masked positions get a prediction and a confidence:
        the decision window, widened to the end of the sequence in a refresh step
        (the confidences right of the span decide what is cached)."""
        if self.stage == FAST and self.cache_mode == CACHE_REFRESH:
            return self.s_cycle, self.gen_end - 1
        return self.window()

    def window(self) -> Tuple[int, int]:
        """Inclusive span the step looks at: [s_cycle, end of sequence] in the
        slow stage, [s_cycle, e_cycle] in the fast stage; empty when idle."""
        if self.stage == SLOW:
            return self.s_cycle, self.gen_end - 1
        if self.stage == FAST:
            return self.s_cycle, self.e_cycle
        return 0, -1


@dataclass
class DecodeParams:
    max_steps: int                 # N
    k_max: int = 8
    w_hist: int = 2
    sigma2_stable: float = 1.0
    tau_min_conf: float = 0.1
    tau_high_conf: float = 0.85
    k_slow: int = 1
    k_fast: int = 1
    conv_mode: int = 0
    out_of_span_cache: bool = False
    prompt_cache_interval: int = 0     # K_p; 0 = the prompt is recomputed in every step
    response_cache_interval: int = 0   # K_r; 0 = no response position is left out on this account


def active_rows(sp: StageParams, mask: np.ndarray) -> np.ndarray:
    """Positions whose prediction the step needs: masked and inside the window."""
    lo, hi = sp.eval_window()
    act = np.zeros(mask.shape[0], dtype=np.uint8)
    for i in range(max(lo, 0), min(hi, mask.shape[0] - 1) + 1):
        if mask[i]:
            act[i] = 1
    return act


def top_k(cands: Sequence[int], conf: np.ndarray, k: int) -> List[int]:
    order = sorted(cands, key=lambda i: (-float(conf[i]), i))
    return sorted(order[:k])


def select(sp: StageParams, mask, pred, conf, prev_pred):
    """The per-step rule of one sequence.  Returns (commit positions in
    ascending order, e_cand or -1, leftmost masked position of the window or -1)."""
    conf = np.asarray(conf, dtype=np.float32)
    lo, hi = sp.window()
    cands = [i for i in range(max(lo, 0), min(hi, len(mask) - 1) + 1) if mask[i]]
    first_masked = cands[0] if cands else -1

    # End point of convergence (eq. 6): the furthest position above tau_min.
    above = [i for i in cands if conf[i] > np.float32(sp.tau_min_conf)]
    e_cand = max(above) if above else -1

    if sp.stage == SLOW:
        # Cautious decoding: the top-k_slow confidences of the window.
        commit = top_k(cands, conf, sp.top_k)
    elif sp.stage == FAST:
        # In-span parallel decoding (eq. 9) ...
        s_high = [i for i in cands
                  if conf[i] > np.float32(sp.tau_high_conf)
                  and (sp.conv_mode == 0 or int(pred[i]) == int(prev_pred[i]))]
        # ... else the fallback top-k_fast refinement.
        commit = s_high if len(s_high) >= 1 else top_k(cands, conf, sp.top_k)
    else:
        commit = []
    return commit, e_cand, first_masked


Predictor = Callable[[np.ndarray, np.ndarray], Tuple[np.ndarray, np.ndarray]]
"""predict(tokens[B, L], active[B, L]) -> (pred int32 [B, L], conf float32 [B, L]):
the greedy estimate and its confidence at the active positions."""


def step(predict: Predictor, tokens, mask, prev_pred, sps: Sequence[StageParams], skip=None, also_skip=None):
    """One denoising step on a batch, in place.  Returns, per sequence,
    (commit positions, committed tokens, their confidences, e_cand,
    first_masked, masks left in the sequence, the step's confidences).

    With caching the predictor must offer predict.cached(tokens, active, skip),
    where skip[b, i] != 0 marks the positions that are not recomputed (it
    refreshes the cached features of every other position).  skip[b]: the
    out-of-span set of a CACHE_REUSE sequence.  also_skip [B, L] (prompt
    caching): further positions to leave out in this step; an all-zero array
    asks for a complete forward through the cached path (a refresh)."""
    B, L = tokens.shape
    active = np.stack([active_rows(sps[b], mask[b]) for b in range(B)])
    if any(sp.cache_mode != CACHE_OFF for sp in sps) or also_skip is not None:
        sk = np.zeros((B, L), dtype=np.uint8)
        for b in range(B):
            if sps[b].cache_mode == CACHE_REUSE:
                sk[b] = skip[b]
            if also_skip is not None and sps[b].cache_mode != CACHE_REFRESH:
                sk[b] |= np.asarray(also_skip[b], dtype=np.uint8)
            assert not np.any(sk[b] & active[b]), "a skipped position has no prediction"
        pred, conf = predict.cached(tokens, active, sk)
    else:
        pred, conf = predict(tokens, active)
    out = []
    for b in range(B):
        commit, e_cand, first_masked = select(sps[b], mask[b], pred[b], conf[b], prev_pred[b])
        toks = [int(pred[b, i]) for i in commit]
        cfs = [float(conf[b, i]) for i in commit]
        for i in commit:                       # transition: unmask, never re-mask
            tokens[b, i] = pred[b, i]
            mask[b, i] = 0
        for i in range(L):                     # remember this step's estimate
            if active[b, i]:
                prev_pred[b, i] = pred[b, i]
        out.append((commit, toks, cfs, e_cand, first_masked, int(mask[b].sum()), np.asarray(conf[b], dtype=np.float32)))
    return out


@dataclass
class Controller:
    """Stage controller of one sequence (Algorithm 1's outer loop as a state
    machine: ask `next_params`, run the step, report back with `observe`)."""
    gen_start: int
    gen_end: int
    p: DecodeParams
    s_cycle: int = field(init=False)
    e_cycle: int = field(init=False)
    stage: int = field(init=False, default=SLOW)
    history: List[int] = field(init=False, default_factory=list)
    step_count: int = field(init=False, default=0)   # steps of this slow stage
    steps: int = field(init=False, default=0)        # N - k
    log: List[Tuple[int, int, int]] = field(init=False, default_factory=list)
    fast_steps: int = field(init=False, default=0)   # steps of this fast stage
    skip: Optional[np.ndarray] = field(init=False, default=None)   # cached set of this fast stage

    def __post_init__(self):
        self.s_cycle = self.gen_start
        self.e_cycle = self.gen_end - 1

    def next_params(self, mask) -> Optional[StageParams]:
        if not np.any(mask) or self.steps >= self.p.max_steps:
            return None
        slow = self.stage == SLOW
        cache = CACHE_OFF
        if not slow and self.p.out_of_span_cache:
            cache = CACHE_REFRESH if self.fast_steps == 0 else CACHE_REUSE
        return StageParams(self.stage, self.s_cycle, self.e_cycle if not slow else self.gen_end - 1,
                           self.p.k_slow if slow else self.p.k_fast,
                           self.p.tau_min_conf, self.p.tau_high_conf, self.p.conv_mode,
                           self.gen_start, self.gen_end, cache)

    def _start_slow(self):
        self.stage, self.history, self.step_count = SLOW, [], 0
        self.fast_steps, self.skip = 0, None

    def _enter_fast(self, e, mask):
        e = min(max(e, self.s_cycle), self.gen_end - 1)
        self.e_cycle = e
        if np.any(mask[self.s_cycle:e + 1]):
            self.stage, self.fast_steps, self.skip = FAST, 0, None
        else:                                   # span already clean: next cycle
            self.s_cycle = e + 1
            self._start_slow()

    def observe(self, e_cand: int, first_masked: int, mask_after, conf=None) -> None:
        """conf: the step's confidences (needed after a refresh step only)."""
        self.steps += 1
        self.log.append((self.stage, self.s_cycle, self.e_cycle))
        if self.stage == SLOW:
            self.step_count += 1
            e_k = e_cand if e_cand >= 0 else first_masked
            self.history = (self.history + [e_k])[-self.p.w_hist:]
            var = float(np.var(np.asarray(self.history, dtype=np.float64)))   # population
            if len(self.history) >= self.p.w_hist and var < self.p.sigma2_stable:
                self._enter_fast(sum(self.history) // len(self.history), mask_after)
            elif self.step_count >= self.p.k_max:
                self._enter_fast(e_k, mask_after)
        else:
            if self.p.out_of_span_cache and self.fast_steps == 0:
                # Out-of-span caching: masked positions right of the span whose confidence in
                # this (complete) step is below tau_min are not recomputed for the rest of the stage
                L = len(mask_after)
                self.skip = np.zeros(L, dtype=np.uint8)
                for i in range(self.e_cycle + 1, self.gen_end):
                    if mask_after[i] and np.float32(conf[i]) < np.float32(self.p.tau_min_conf):
                        self.skip[i] = 1
            self.fast_steps += 1
            if not np.any(mask_after[self.s_cycle:self.e_cycle + 1]):
                self.s_cycle = self.e_cycle + 1
                self._start_slow()


def interval_skip(p: DecodeParams, steps: int, sps: Sequence[StageParams], gen_start: int, gen_end: int, L: int):
    """Positions the interval caches leave out in step number `steps` (from 0):
    the prompt unless K_p divides the step number, the response outside each
    sequence's rated range unless K_r does.  None when both caches are off; an
    all-zero array (a complete forward that refreshes the cache) on a common
    multiple."""
    if p.prompt_cache_interval <= 0 and p.response_cache_interval <= 0:
        return None
    also = np.zeros((len(sps), L), dtype=np.uint8)
    if p.prompt_cache_interval > 0 and steps % p.prompt_cache_interval != 0:
        also[:, :gen_start] = 1
    if p.response_cache_interval > 0 and steps % p.response_cache_interval != 0:
        for b, sp in enumerate(sps):
            lo, hi = sp.eval_window()
            for i in range(gen_start, gen_end):
                if i < lo or i > hi:
                    also[b, i] = 1
    return also


def decode(predict: Predictor, tokens, mask, gen_start: int, gen_end: int, p: DecodeParams,
           trace: Optional[list] = None) -> int:
    """Full SlowFast decode of a batch, in place; returns the number of
    denoising steps (forward passes) taken.  Sequences are independent; one
    shared forward serves every sequence that still has work."""
    B, L = tokens.shape
    prev_pred = np.full((B, L), -1, dtype=np.int32)
    ctl = [Controller(gen_start, gen_end, p) for _ in range(B)]
    steps = 0
    while True:
        sps, live = [], False
        for b in range(B):
            sp = ctl[b].next_params(mask[b])
            if sp is None:
                sp = StageParams(IDLE, 0, -1, 1, p.tau_min_conf, p.tau_high_conf, p.conv_mode,
                                 gen_start, gen_end)
            else:
                live = True
            sps.append(sp)
        if not live:
            return steps
        skip = [ctl[b].skip for b in range(B)]
        also = interval_skip(p, steps, sps, gen_start, gen_end, L)
        res = step(predict, tokens, mask, prev_pred, sps, skip, also)
        steps += 1
        for b in range(B):
            if sps[b].stage != IDLE:
                ctl[b].observe(res[b][3], res[b][4], mask[b], res[b][6])
        if trace is not None:
            trace.append((sps, res))


def alg1_sequence(tokens, mask, prev_pred, gen_start: int, gen_end: int, p: DecodeParams, log: Optional[list] = None):
    """Algorithm 1 for ONE sequence, as the listing's nested loops, in place on
    tokens / mask / prev_pred (1-D arrays over the L positions).

    A generator: every "Predict r_0 and confidence" line of the listing is a
    `yield (stage params, cached set or None)` that must be answered (`send`)
    with (pred [L], conf [L]) valid at the masked positions of the step's
    evaluation window.  Everything else -- cautious decoding, end-point
    prediction, stability check, fallback, in-span decoding, out-of-span
    caching, cycle advance -- is written out below in the listing's order,
    with the readings of the module docstring marked where they enter.
    log (optional) receives one (stage, s_cycle, e_cycle, commit positions) per step."""
    L = len(mask)
    k = p.max_steps                                   # k <- N
    s_cycle = gen_start                               # s_cycle <- first generated position
    tau_min, tau_high = np.float32(p.tau_min_conf), np.float32(p.tau_high_conf)

    def masked(lo, hi):                               # masked positions of [lo, hi]
        return [i for i in range(max(lo, 0), min(hi, L - 1) + 1) if mask[i]]

    def unmask(commit, pred, rated):
        for i in commit:                              # transition: unmask, never re-mask
            tokens[i] = pred[i]
            mask[i] = 0
        for i in rated:                               # this step's estimate, for the convergence gate
            prev_pred[i] = pred[i]

    # "while k > 0 and s_cycle < L": every mask lies in [s_cycle, gen_end), so "a mask is left" is the same test
    while k > 0 and masked(s_cycle, gen_end - 1):
        # ---- Phase 1: exploratory stage (slow) ----
        H_W: List[int] = []                           # reading: the history starts empty in every exploratory stage
        step_count = 0
        is_stable = False
        e_cycle = e_k = None
        while step_count < p.k_max and k > 0 and masked(s_cycle, gen_end - 1):
            sp = StageParams(SLOW, s_cycle, gen_end - 1, p.k_slow, p.tau_min_conf, p.tau_high_conf, p.conv_mode,
                             gen_start, gen_end)
            pred, conf = yield sp, None               # predict r_0 and its confidence
            conf = np.asarray(conf, dtype=np.float32)
            window = masked(s_cycle, gen_end - 1)     # the state before this step's commits
            # cautious decoding: the k_slow most confident positions of [s_cycle, end] (ties: lower position)
            commit = sorted(sorted(window, key=lambda i: (-float(conf[i]), i))[:p.k_slow])
            # end point prediction (eq. 6); reading: nothing above tau_min -> the leftmost mask of the window
            above = [i for i in window if conf[i] > tau_min]
            e_k = max(above) if above else window[0]
            H_W = (H_W + [e_k])[-p.w_hist:]           # sliding window of the last W_hist candidates
            unmask(commit, pred, window)
            if log is not None:
                log.append((SLOW, s_cycle, gen_end - 1, commit))
            k -= 1
            step_count += 1
            # stability check (eq. 7): population variance, strictly below the threshold
            mean = sum(H_W) / len(H_W)
            var = sum((h - mean) ** 2 for h in H_W) / len(H_W)
            if len(H_W) >= p.w_hist and var < p.sigma2_stable:
                is_stable = True
                e_cycle = sum(H_W) // len(H_W)        # eq. 8, floored
                break
        if e_k is None:                               # no exploratory step ran (k exhausted)
            break
        if not is_stable:
            e_cycle = e_k                             # fallback if no convergence: the last candidate
        e_cycle = min(max(e_cycle, s_cycle), gen_end - 1)

        # ---- Phase 2: accelerated decoding stage (fast) ----
        # reading: repeated until no mask is left in [s_cycle, e_cycle] (a span that the slow steps
        # already emptied costs no forward pass)
        cached = None
        first_of_stage = True
        while k > 0 and masked(s_cycle, e_cycle):
            mode = CACHE_OFF
            if p.out_of_span_cache:
                mode = CACHE_REFRESH if first_of_stage else CACHE_REUSE
            sp = StageParams(FAST, s_cycle, e_cycle, p.k_fast, p.tau_min_conf, p.tau_high_conf, p.conv_mode,
                             gen_start, gen_end, mode)
            pred, conf = yield sp, cached             # predict r_0 and its confidence
            conf = np.asarray(conf, dtype=np.float32)
            span = masked(s_cycle, e_cycle)
            if p.out_of_span_cache and first_of_stage:
                # out-of-span caching: masked positions right of the span whose confidence in this
                # complete prediction is below tau_min keep their features for the rest of the stage
                cached = np.zeros(L, dtype=np.uint8)
                for i in masked(e_cycle + 1, gen_end - 1):
                    if conf[i] < tau_min:
                        cached[i] = 1
            # in-span parallel decoding (eq. 9), with the token-level convergence gate when conv_mode = 1
            s_high = [i for i in span if conf[i] > tau_high
                      and (p.conv_mode == 0 or int(pred[i]) == int(prev_pred[i]))]
            if s_high:
                commit = s_high                       # aggressive unmasking
            else:                                     # fallback refinement: top-k_fast of the span
                commit = sorted(sorted(span, key=lambda i: (-float(conf[i]), i))[:p.k_fast])
            lo, hi = sp.eval_window()
            unmask(commit, pred, masked(lo, hi))
            if log is not None:
                log.append((FAST, s_cycle, e_cycle, commit))
            k -= 1
            first_of_stage = False
        s_cycle = e_cycle + 1                         # advance the stable region start


def decode_alg1(predict: Predictor, tokens, mask, gen_start: int, gen_end: int, p: DecodeParams,
                trace: Optional[list] = None) -> int:
    """Full decode of a batch by running `alg1_sequence` once per sequence; the
    sequences whose generators ask for a prediction share one forward pass per
    step, the finished ones ride along idle.  In place; returns the number of
    forward passes.  trace (optional) receives one list per step with, per
    sequence, (stage, s_cycle, e_cycle, commit positions) or None when idle.
    The interval caches of DecodeParams (K_p, K_r) act on the forward pass only
    and are applied here, outside Algorithm 1, exactly as `decode` applies them."""
    B, L = tokens.shape
    prev_pred = np.full((B, L), -1, dtype=np.int32)
    logs: List[list] = [[] for _ in range(B)]
    gens = [alg1_sequence(tokens[b], mask[b], prev_pred[b], gen_start, gen_end, p, logs[b]) for b in range(B)]
    asks: List[Optional[tuple]] = []
    for g in gens:                                    # run every sequence up to its first prediction
        try:
            asks.append(next(g))
        except StopIteration:
            asks.append(None)
    idle = StageParams(IDLE, 0, -1, 1, p.tau_min_conf, p.tau_high_conf, p.conv_mode, gen_start, gen_end)
    steps = 0
    while any(a is not None for a in asks):
        sps = [a[0] if a is not None else idle for a in asks]
        active = np.stack([active_rows(sps[b], mask[b]) for b in range(B)])
        also = interval_skip(p, steps, sps, gen_start, gen_end, L)
        if any(sp.cache_mode != CACHE_OFF for sp in sps) or also is not None:
            sk = np.zeros((B, L), dtype=np.uint8)
            for b in range(B):
                if sps[b].cache_mode == CACHE_REUSE:
                    sk[b] = asks[b][1]
                if also is not None and sps[b].cache_mode != CACHE_REFRESH:
                    sk[b] |= also[b]
            pred, conf = predict.cached(tokens, active, sk)
        else:
            pred, conf = predict(tokens, active)
        steps += 1
        done_before = [len(lg) for lg in logs]
        for b in range(B):
            if asks[b] is None:
                continue
            try:
                asks[b] = gens[b].send((pred[b], conf[b]))
            except StopIteration:
                asks[b] = None
        if trace is not None:
            trace.append([logs[b][done_before[b]] if len(logs[b]) > done_before[b] else None for b in range(B)])
    return steps


def n_unmasked_target(length: int, n_steps: int, j: int) -> int:
    """Low-confidence remasking schedule (Section 3.1): after the j-th of n_steps
    steps (the paper's k = n_steps - j + 1, t_{k-1} = (k - 1) / n_steps) the state
    holds floor(length * (1 - t_{k-1})) = floor(length * j / n_steps) unmasked tokens."""
    return (length * j) // n_steps


def decode_low_confidence(predict: Predictor, tokens, mask, gen_start: int, gen_end: int, n_steps: int,
                          block_len: Optional[int] = None, trace: Optional[list] = None) -> int:
    """The baseline sampler the paper starts from (Section 3.1): low-confidence
    remasking, optionally semi-autoregressive over blocks of block_len positions
    that are denoised left to right with n_steps / n_blocks steps each.

    Every step predicts all masked positions of the current block; committed
    positions have confidence 1 and stay, so "keep the n_un most confident" means:
    unmask the (n_un - already unmasked) most confident masked positions of the
    block (ties: lower position).  A step whose target is already met commits
    nothing and is skipped without a forward pass.  Returns the forward passes run."""
    B, L = tokens.shape
    G = gen_end - gen_start
    block_len = G if block_len is None else block_len
    if G <= 0:
        return 0
    if block_len < 1 or G % block_len:
        raise ValueError("block_len must divide the generated length")
    n_blocks = G // block_len
    if n_steps < n_blocks or n_steps % n_blocks:
        raise ValueError("n_steps must be a positive multiple of the number of blocks")
    per_block = n_steps // n_blocks
    prev_pred = np.full((B, L), -1, dtype=np.int32)
    steps = 0
    for blk in range(n_blocks):
        lo = gen_start + blk * block_len
        hi = lo + block_len                      # exclusive
        for j in range(1, per_block + 1):
            target = n_unmasked_target(block_len, per_block, j)
            sps = []
            for b in range(B):
                unmasked = block_len - int(mask[b, lo:hi].sum())
                k = target - unmasked
                if k >= 1:
                    # the slow-stage rule on the window [lo, hi): top-k by confidence
                    sps.append(StageParams(SLOW, lo, hi - 1, k, 0.0, 1.0, 0, gen_start, hi))
                else:
                    sps.append(StageParams(IDLE, 0, -1, 1, 0.0, 1.0, 0, gen_start, hi))
            if all(sp.stage == IDLE for sp in sps):
                continue
            res = step(predict, tokens, mask, prev_pred, sps)
            steps += 1
            if trace is not None:
                trace.append((sps, res))
    return steps
