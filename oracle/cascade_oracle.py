"""Plain-Python statement of the paper's host-side policy — TEST INFRASTRUCTURE, not a product path.

Follows the paper's Section 4 (speculation utility, Theorem 1) and Section 5
(test-and-set, disabling speculation, adaptive back-off, hill-climbing search),
with the hyper-parameters of Section 6 (t = 4, T = 16 i.e. up to M = 4 trials,
S = 16) and K_start = 3 (Section 7.4).  Only tests/ and the smoke check may import
this; the C controller in the product library is written separately and is
compared with this one by replaying identical (tokens, time) traces.

Where the paper is silent (its hill-climbing flow chart is a figure), the reading
taken is stated next to the code.  PARITY UNPINNED for: the exact hill-climb
step rule, the first back-off length, the baseline-refresh policy and the
K_start history window — nothing printed in the paper fixes them; the pins in
tests/test_cascade_pins.py cover utility, Theorem 1, the test-cost and back-off
worked examples, the interval lengths and the invariants.
"""
from __future__ import annotations

import math
from dataclasses import dataclass


def utility(tokens_per_iter: float, t_verify: float, t_base: float) -> float:
    """Speculation utility (Section 4, Definition + Eq. 3): benefit / cost =
    ETR / (t_iter,spec / t_iter,base).  tokens_per_iter counts the always-emitted
    token (ETR_base = 1), so K = 0 gives exactly 1.  NaN for non-positive times."""
    if not (t_verify > 0.0) or not (t_base > 0.0):
        return math.nan
    return tokens_per_iter / (t_verify / t_base)


@dataclass
class Params:
    t_trial: int = 4          # iterations per trial (Section 5.3, "t = 4")
    max_trials: int = 4       # M (Section 5.3)
    s_set: int = 16           # S (Section 5.3 / 6)
    k_max: int = 8            # largest speculation length considered
    k_start: int = 3          # first K_start of a request (Section 7.4)
    base_iters: int = 4       # no-speculation iterations used to measure t_base (Section 5.3)
    base_refresh: int = 100   # refresh t_base about this often (Section 5.3)
    s_max: int = 0            # cap on the backed-off set length; 0 = none
    converge_frac: float = 0.10  # early exit (3) of Section 5.6
    backoff: int = 1          # adaptive back-off (Section 5.5): 0 off (ablation); 1 the first disabled set phase keeps S
                              # and every further consecutive one doubles (the section's figure: "persistently" below
                              # 1); 2 every drop to K = 0 doubles S, the first included (the section's sentence)
    hillclimb: int = 1        # 0: test only K_start (Section 7.4 ablation)


BASELINE, TEST, SET = 0, 1, 2


class Controller:
    def __init__(self, p: Params | None = None):
        self.p = p or Params()
        p = self.p
        if min(p.t_trial, p.max_trials, p.s_set, p.k_max, p.base_iters, p.base_refresh) < 1 \
                or not (1 <= p.k_start <= p.k_max) or p.s_max < 0 or not (p.converge_frac >= 0.0) \
                or p.backoff not in (0, 1, 2):
            raise ValueError("bad parameters")
        self.iters = 0
        self.t_base = math.nan
        self.s_cur = p.s_set
        self.prev_set_k = -1            # -1: no set phase yet (request start)
        self.cycles = []                # records [(K, U), ...] of the last two cycles
        self.cur_cycle = []
        self.last_refresh = 0
        self.spec_trial_iters = 0       # bookkeeping for reports
        self._enter_baseline()

    # ---- phases ---------------------------------------------------------
    def _enter_baseline(self):
        self.phase = BASELINE
        self.left = self.p.base_iters
        self.acc_time = 0.0

    def _k_start(self) -> int:
        # Section 5.4: after a disabled set phase every cycle begins with K = 1.
        if self.prev_set_k == 0:
            return 1
        # Section 5.3: scan recent history for the non-zero K with the highest utility.
        best_k, best_u = None, None
        for cyc in self.cycles:
            for k, u in cyc:
                if k > 0 and (best_u is None or u > best_u or (u == best_u and k < best_k)):
                    best_k, best_u = k, u
        if best_k is None:
            best_k = self.p.k_start
        return max(1, min(self.p.k_max, best_k))

    def _enter_test(self):
        self.phase = TEST
        self.cur_cycle = []
        self.trials = []                # [(K, U)] of this test phase in order
        self.best_k, self.best_u = None, None
        self._begin_trial(self._k_start())

    def _begin_trial(self, k: int):
        self.cur_k = k
        self.left = self.p.t_trial
        self.acc_tokens = 0
        self.acc_time = 0.0

    def _enter_set(self, k_set: int):
        p = self.p
        if k_set == 0:
            # Section 5.5: "double the set phase length S whenever K drops to 0" (backoff = 2: every drop, the
            # first included; backoff = 1: the first disabled phase keeps S, further consecutive ones double).
            if p.backoff == 2 or (p.backoff == 1 and self.prev_set_k == 0):
                self.s_cur = self.s_cur * 2
                if p.s_max > 0 and self.s_cur > p.s_max:
                    self.s_cur = p.s_max
            else:
                self.s_cur = p.s_set
        else:
            self.s_cur = p.s_set
        self.phase = SET
        self.cur_k = k_set
        self.left = self.s_cur
        self.acc_tokens = 0
        self.acc_time = 0.0
        self.tail = []                  # last base_iters iteration times (free t_base refresh at K = 0)

    # ---- per-iteration interface ------------------------------------------
    def next_k(self) -> int:
        return 0 if self.phase == BASELINE else self.cur_k

    def observe(self, k_used: int, tokens: int, t_iter: float) -> None:
        if k_used != self.next_k() or not (1 <= tokens <= k_used + 1) or not (t_iter > 0.0) or math.isinf(t_iter):
            raise ValueError("bad observation")
        self.iters += 1
        if self.phase == BASELINE:
            self.acc_time += t_iter
            self.left -= 1
            if self.left == 0:
                self.t_base = self.acc_time / self.p.base_iters
                self.last_refresh = self.iters
                self._enter_test()
        elif self.phase == TEST:
            self.spec_trial_iters += 1
            self.acc_tokens += tokens
            self.acc_time += t_iter
            self.left -= 1
            if self.left == 0:
                self._end_trial()
        else:
            self.acc_tokens += tokens
            self.acc_time += t_iter
            self.tail.append(t_iter)
            if len(self.tail) > self.p.base_iters:
                self.tail.pop(0)
            self.left -= 1
            if self.left == 0:
                self._end_set()

    # ---- transitions ----------------------------------------------------
    def _phase_utility(self, n: int) -> float:
        # ratio of means over the n iterations of the trial / phase (Section 5.4: utility
        # is computed at the end of each trial)
        return utility(self.acc_tokens / n, self.acc_time / n, self.t_base)

    def _end_trial(self):
        p = self.p
        u = self._phase_utility(p.t_trial)
        k = self.cur_k
        self.trials.append((k, u))
        self.cur_cycle.append((k, u))
        if self.best_u is None or u > self.best_u or (u == self.best_u and k < self.best_k):
            self.best_k, self.best_u = k, u
        j = len(self.trials)
        done = j >= p.max_trials or not p.hillclimb
        # Section 5.4: already at the most conservative K and still unprofitable -> stop testing.
        if k == 1 and u < 1.0:
            done = True
        # Section 5.6 exit (1): utility fell on two successive steps -> the maximum was passed.
        if j >= 3 and self.trials[-1][1] < self.trials[-2][1] < self.trials[-3][1]:
            done = True
        # Section 5.6 exit (3): successive utilities within 10 %.
        if j >= 2 and abs(u - self.trials[-2][1]) <= p.converge_frac * self.trials[-2][1]:
            done = True
        nxt = None
        if not done:
            # Section 5.6: the direction in which utility grows, from (prev-K, prev-U, curr-K, curr-U).
            if j == 1:
                nxt = k + (1 if u >= 1.0 else -1)
            else:
                pk, pu = self.trials[-2]
                step = 1 if k > pk else -1
                if u > pu:
                    nxt = k + step          # still climbing: keep going the same way
                else:
                    nxt = pk - step         # got worse: backtrack to the other side of prev-K
            # exit (2) of Section 5.6 (K reaches 0), range end, or nothing new to learn
            if nxt < 1 or nxt > p.k_max or any(nxt == tk for tk, _ in self.trials):
                done = True
        if done:
            # Section 5.1 / 5.4: speculate only if the best utility seen does not fall below one.
            self._enter_set(self.best_k if self.best_u >= 1.0 else 0)
        else:
            self._begin_trial(nxt)

    def _end_set(self):
        p = self.p
        k = self.cur_k
        if k > 0:
            self.cur_cycle.append((k, self._phase_utility(self.s_cur)))
        elif len(self.tail) == p.base_iters:
            # a disabled set phase IS a no-speculation measurement: refresh t_base for free
            acc = 0.0
            for v in self.tail:         # plain left-to-right sum
                acc += v
            self.t_base = acc / p.base_iters
            self.last_refresh = self.iters
        self.cycles.append(self.cur_cycle)
        self.cycles = self.cycles[-2:]
        self.prev_set_k = k
        if self.iters - self.last_refresh >= p.base_refresh:
            self._enter_baseline()      # Section 5.3: infrequent refresh of the baseline time
        else:
            self._enter_test()
