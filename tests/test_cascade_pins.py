"""Pins for the host-side policy oracle (utility + test-and-set loop).  No GPU.

Values come from the paper's worked examples (tests/golden) and from Theorem 1;
traces are synthetic (cost of K from the balls-and-bins model of Section 2.4,
acceptance from the seeded chain in synth).
"""
import math
import os

import numpy as np
import pytest

from oracle import cascade_oracle as co
from paper_2506_20675_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _golden_rows(name):
    rows = []
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                rows.append([float(v) for v in line.split()])
    return rows


def bins_cost(K, E=8, top_k=2):
    """Verification cost of K drafts relative to K = 0 under uniform routing (Section 2.4)."""
    return (E * (1 - (1 - top_k / E) ** (K + 1))) / top_k


def run_trace(ctrl, n_iter, cost_of_k, p_of_iter, seed_field=0, t0=1.0):
    """Drive a controller with synthetic (tokens, time) observations; returns arrays K, tokens, time, phase."""
    u = synth.acceptance_uniforms(n_iter, seed_field)
    Ks, toks, times, phases = [], [], [], []
    for i in range(n_iter):
        k = ctrl.next_k()
        assert 0 <= k <= ctrl.p.k_max
        tok = synth.tokens_emitted(u[i], p_of_iter(i), k)
        t = t0 * cost_of_k(k)
        phases.append(ctrl.phase)
        ctrl.observe(k, tok, t)
        Ks.append(k)
        toks.append(tok)
        times.append(t)
    return np.array(Ks), np.array(toks), np.array(times), np.array(phases)


# ------------------------------------------------------------------ utility
def test_utility_paper_examples():
    for etr, cost, u in _golden_rows("utility_examples.txt"):
        assert co.utility(etr, cost * 7.0, 7.0) == pytest.approx(u, rel=1e-15)
    assert co.utility(1.0, 3.0, 3.0) == 1.0
    for bad in ((1.0, 0.0, 1.0), (1.0, 1.0, 0.0), (1.0, -1.0, 1.0), (1.0, math.nan, 1.0)):
        assert math.isnan(co.utility(*bad))


def test_theorem_1_tpot_equals_base_over_utility():
    """Static K on a synthetic trace: measured time per output token == t_base / U (Section 4, Theorem 1)."""
    n = 400
    u = synth.acceptance_uniforms(n, 3)
    t_base = 0.7
    for K in (1, 3, 7):
        toks = np.array([synth.tokens_emitted(u[i], 0.6, K) for i in range(n)])
        t_iter = t_base * bins_cost(K) * (1.0 + 0.1 * np.sin(np.arange(n)))      # varying iteration times
        tpot = t_iter.sum() / toks.sum()
        U = co.utility(toks.mean(), t_iter.mean(), t_base)
        assert tpot == pytest.approx(t_base / U, rel=1e-12)


# ------------------------------------------------------------------ test-and-set loop
def test_request_start_measures_baseline_then_tests_k_start():
    c = co.Controller()
    Ks, _, _, ph = run_trace(c, 8, bins_cost, lambda i: 0.9)
    assert list(Ks[:4]) == [0, 0, 0, 0] and list(ph[:4]) == [co.BASELINE] * 4
    assert list(Ks[4:8]) == [3, 3, 3, 3] and list(ph[4:8]) == [co.TEST] * 4
    assert c.t_base == pytest.approx(1.0)


def test_test_cost_example_no_backoff():
    """t=4, S=16, cost 2x, ETR 1: every 20-iteration interval takes 8 + 16 = 24 time units (Section 5.5)."""
    (t, S, cost, test_units, interval_units, base_units), = _golden_rows("test_cost_example.txt")
    c = co.Controller(co.Params(t_trial=int(t), s_set=int(S), backoff=0))
    Ks, toks, times, ph = run_trace(c, 400, lambda k: cost if k > 0 else 1.0, lambda i: 0.0)
    # steady state: after the first disabled set phase every cycle is one K=1 trial + S iterations at K=0
    first_set0 = next(i for i in range(len(Ks)) if ph[i] == co.SET and Ks[i] == 0)
    start = first_set0 + int(S)
    for cyc in range(5):
        a = start + cyc * int(t + S)
        seg_k, seg_t = Ks[a:a + int(t + S)], times[a:a + int(t + S)]
        assert list(seg_k) == [1] * int(t) + [0] * int(S)
        assert seg_t[:int(t)].sum() == test_units
        assert seg_t.sum() == interval_units
        assert len(seg_k) * 1.0 == base_units


@pytest.mark.parametrize("variant", [1, 2])
def test_backoff_example_trial_iterations_in_250(variant):
    """Both readings of "double S whenever K drops to 0" (first disabled phase keeps S / already doubles) give the
    same count over the paper's 250-iteration window of steady-state cycles."""
    (window, no_bo, with_bo, slow_no, slow_bo), = _golden_rows("backoff_example.txt")
    window = int(window)
    res = {}
    for bo in (0, variant):
        c = co.Controller(co.Params(backoff=bo))
        Ks, toks, times, ph = run_trace(c, 800, bins_cost, lambda i: 0.0)
        first_set0 = next(i for i in range(len(Ks)) if ph[i] == co.SET and Ks[i] == 0)
        # window = whole steady-state cycles: it opens with the K = 1 trial that precedes the first disabled phase
        w = slice(first_set0 - c.p.t_trial, first_set0 - c.p.t_trial + window)
        res[bo] = (int((Ks[w] > 0).sum()), times[w].sum() / window - 1.0)
    # without back-off: 4 of every 20 iterations -> 48..52 ("nearly 50"), slowdown ~ 4*0.75/20 = 15 % (paper: 14 %)
    assert abs(res[0][0] - no_bo) <= 2
    assert abs(res[0][1] - slow_no) < 0.02
    # with back-off: set lengths 16, 32, 64, 128 (or 32, 64, 128) -> 16 trial iterations in the window (paper: 18),
    # slowdown ~ 5 %
    assert abs(res[variant][0] - with_bo) <= 2
    assert abs(res[variant][1] - slow_bo) < 0.015


@pytest.mark.parametrize("variant,first", [(1, 16), (2, 32)])
def test_backoff_doubles_and_resets(variant, first):
    c = co.Controller(co.Params(backoff=variant))
    # unprofitable for 300 iterations, then very profitable
    Ks, toks, times, ph = run_trace(c, 600, lambda k: 1.0 + 0.9 * k if k else 1.0, lambda i: 0.0 if i < 300 else 1.0)
    # lengths of maximal runs of SET phases at K = 0
    runs, i = [], 0
    while i < len(Ks):
        if ph[i] == co.SET and Ks[i] == 0:
            j = i
            while j < len(Ks) and ph[j] == co.SET and Ks[j] == 0:
                j += 1
            runs.append(j - i)
            i = j
        else:
            i += 1
    assert runs[:4] == [first, 2 * first, 4 * first, 8 * first]
    # once speculation pays again (tokens = K+1, cost 1+0.9K -> U > 1 for K >= 1 ... ) the set length returns to S
    assert c.s_cur == 16 and c.cur_k > 0


def test_interval_is_at_most_32_and_trials_at_most_4():
    """Section 1: test-and-set interval of 32 iterations = 16 test (4 trials x 4) + 16 set."""
    # utility keeps rising with K by > 10 % per step -> all 4 trials are used
    c = co.Controller()
    Ks, toks, times, ph = run_trace(c, 200, lambda k: 1.0, lambda i: 1.0)
    t = 4
    tests = []
    while t < len(Ks):
        a = t
        while t < len(Ks) and ph[t] == co.TEST:
            t += 1
        b = t
        while t < len(Ks) and ph[t] == co.SET:
            t += 1
        if t < len(Ks) and ph[t] == co.BASELINE:
            t += 4
        tests.append((b - a, t - b))
    assert tests[0][0] == 16 and all(tl <= 16 and tl % 4 == 0 for tl, _ in tests[:-1])
    assert all(sl in (16, 20) for _, sl in tests[:-1])          # 20 = set + a 4-iteration baseline refresh
    assert list(Ks[4:20]) == [3] * 4 + [4] * 4 + [5] * 4 + [6] * 4
    assert list(Ks[20:36]) == [6] * 16                           # best K of the test phase is used in the set phase


@pytest.mark.parametrize("variant,first", [(1, 16), (2, 32)])
def test_disable_when_utility_below_one_at_k1(variant, first):
    c = co.Controller(co.Params(backoff=variant))
    Ks, toks, times, ph = run_trace(c, 60, bins_cost, lambda i: 0.0)
    # K_start = 3 -> utility < 1 -> step down 2, 1 -> still < 1 at K = 1 -> set phase at K = 0
    assert list(Ks[4:16]) == [3] * 4 + [2] * 4 + [1] * 4
    assert list(Ks[16:16 + first]) == [0] * first                # S, or already 2 S (the two back-off readings)
    assert list(Ks[16 + first:20 + first]) == [1] * 4            # retest begins with K = 1
    assert list(Ks[20 + first:24 + first]) == [0] * 4


def test_hill_climb_backtracks_over_a_peak():
    # utility peaks at K = 4: U = 2.0, 1.6 on both sides, falling by > 10 % per step
    table = {0: 1.0, 1: 0.9, 2: 1.2, 3: 1.6, 4: 2.0, 5: 1.6, 6: 1.2, 7: 0.9, 8: 0.7}
    c = co.Controller()
    # tokens fixed at 1 (p = 0) -> U = 1 / cost
    Ks, toks, times, ph = run_trace(c, 40, lambda k: 1.0 / table[k], lambda i: 0.0)
    assert list(Ks[4:20]) == [3] * 4 + [4] * 4 + [5] * 4 + [3] * 4 or list(Ks[4:16]) == [3] * 4 + [4] * 4 + [5] * 4
    sets = Ks[(ph == co.SET)]
    assert sets[0] == 4


def test_k_start_comes_from_recent_history():
    table = {0: 1.0, 1: 1.1, 2: 1.3, 3: 1.6, 4: 2.0, 5: 2.6, 6: 2.0, 7: 1.5, 8: 1.2}
    c = co.Controller()
    Ks, toks, times, ph = run_trace(c, 120, lambda k: 1.0 / table[k], lambda i: 0.0)
    # second test phase starts from the best K seen in the first cycle
    test_starts = [i for i in range(1, len(Ks)) if ph[i] == co.TEST and ph[i - 1] != co.TEST]
    assert Ks[test_starts[0]] == 3
    assert Ks[test_starts[1]] == 5


def test_baseline_refresh_about_every_100_iterations():
    c = co.Controller()
    Ks, toks, times, ph = run_trace(c, 500, lambda k: 1.0, lambda i: 1.0)
    base_iters = np.flatnonzero(ph == co.BASELINE)
    starts = [i for i in base_iters if i == 0 or ph[i - 1] != co.BASELINE]
    assert starts[0] == 0 and len(starts) >= 4
    gaps = np.diff(starts)
    assert gaps.min() >= 100 and gaps.max() <= 100 + 4 + 32 + 4


@pytest.mark.parametrize("seed", range(6))
def test_invariants_on_random_regimes(seed):
    rng = np.random.default_rng(seed)
    p = co.Params(t_trial=int(rng.integers(1, 6)), max_trials=int(rng.integers(1, 6)), s_set=int(rng.integers(1, 24)),
                  k_max=int(rng.integers(1, 9)), base_iters=int(rng.integers(1, 6)), base_refresh=int(rng.integers(5, 150)),
                  s_max=int(rng.choice([0, 64])), backoff=int(rng.integers(0, 3)), hillclimb=int(rng.integers(0, 2)))
    p.k_start = int(rng.integers(1, p.k_max + 1))
    c = co.Controller(p)
    regimes = synth.regime_sequence(1500, seed)
    noise = rng.uniform(0.9, 1.1, 1500)
    it = iter(range(10 ** 9))
    Ks, toks, times, ph = run_trace(c, 1500, lambda k: bins_cost(k) * noise[next(it) % 1500], lambda i: regimes[i], seed)
    assert Ks.min() >= 0 and Ks.max() <= p.k_max
    assert ((toks >= 1) & (toks <= Ks + 1)).all()
    # a test phase never exceeds M trials of t iterations
    run = 0
    for i in range(len(Ks)):
        run = run + 1 if ph[i] == co.TEST else 0
        assert run <= p.t_trial * p.max_trials
    if p.s_max:
        assert c.s_cur <= max(p.s_max, p.s_set)


def test_controller_tracks_regimes_and_beats_static_k():
    """Stand-in for the paper's comparison with static K (Section 7): switching acceptance regimes."""
    n = 3000
    regimes = synth.regime_sequence(n, 1)

    def total_time_per_token(policy_k):
        u = synth.acceptance_uniforms(n, 1)
        if policy_k is None:
            c = co.Controller()
            Ks, toks, times, _ = run_trace(c, n, bins_cost, lambda i: regimes[i], 1)
            return times.sum() / toks.sum()
        toks = sum(synth.tokens_emitted(u[i], regimes[i], policy_k) for i in range(n))
        return n * bins_cost(policy_k) / toks

    base = total_time_per_token(0)
    assert base == pytest.approx(1.0)
    cascade = total_time_per_token(None)
    statics = {k: total_time_per_token(k) for k in (1, 2, 3)}
    assert cascade < base * 1.05                      # never much worse than no speculation
    assert cascade < min(statics.values()) * 1.02     # and at least on par with the best static K


def test_bad_observations_rejected():
    c = co.Controller()
    with pytest.raises(ValueError):
        c.observe(1, 1, 1.0)        # controller asked for K = 0
    with pytest.raises(ValueError):
        c.observe(0, 2, 1.0)        # more tokens than K + 1
    with pytest.raises(ValueError):
        c.observe(0, 1, 0.0)
    with pytest.raises(ValueError):
        co.Controller(co.Params(k_start=9))
