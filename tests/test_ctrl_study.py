"""Controller studies (host only): the C controller driven by a cost table on seeded acceptance traces."""
import numpy as np
import pytest

from paper_2506_20675_amd import ctrl_study as cs


def test_cost_tables_and_closed_forms():
    c = cs.cost_table("mixtral-bf16-layer")
    assert len(c) == 9 and np.all(np.diff(c) >= 0) and 80.0 < c[0] < 200.0      # a measured table: about 120 us at K = 0
    assert np.array_equal(cs.monotone([1, 3, 2, 5, 4]), [1, 3, 3, 5, 5])
    m = cs.balls_in_bins(8, 2, 8)
    assert m[0] == 2.0 and 7.0 < m[7] < 7.3                     # 8 tokens x top-2 of 8: "over seven" experts (Section 2.4)
    assert cs.expected_tokens(0.5, 0) == 1.0 and cs.expected_tokens(0.5, 2) == 1.75 and cs.expected_tokens(1.0, 3) == 4.0
    assert cs.clairvoyant_k(0.1, c) == 0 and cs.clairvoyant_k(0.8, c) >= 3
    line = '{"by_K": {"0": {"latency_us": 10.0}, "1": {"latency_us": 15.0}, "2": {"latency_us": 14.0}}}'
    assert np.array_equal(cs.cost_table(cs.from_bench_json(line)), [10.0, 15.0, 15.0])


def test_static_and_clairvoyant_baselines():
    cost = cs.cost_table("mixtral-bf16-layer")
    tr = cs.Trace(3000, 1)
    s0 = cs.run_static(tr, cost, 0)
    assert s0["tokens"] == 3000 and abs(s0["tpot"] - cost[0]) < 1e-9        # Theorem 1 at K = 0: U = 1
    cv = cs.run_clairvoyant(tr, cost)
    statics = [cs.run_static(tr, cost, k) for k in range(len(cost))]
    assert cv["tpot"] <= min(s["tpot"] for s in statics)
    full = cs.run_cascade(tr, cost)
    assert cv["tpot"] <= full["tpot"]
    assert full["iters"] == 3000 and sum(full["K_histogram"].values()) == 3000
    again = cs.run_cascade(tr, cost)
    assert again["tpot"] == full["tpot"] and again["K_histogram"] == full["K_histogram"]     # deterministic


def test_low_acceptance_backoff_bounds_the_slowdown():
    """Section 5.5: when speculation never pays, testing again and again is the cost; backing off bounds it."""
    cost = cs.cost_table("mixtral-bf16-layer")
    tr = cs.Trace(4000, 2, rates=(0.1,))
    base = cs.run_static(tr, cost, 0)["tpot"]
    no_bo = cs.run_cascade(tr, cost, hillclimb=1, backoff=0)
    bo = cs.run_cascade(tr, cost, hillclimb=1, backoff=1)
    assert cs.run_cascade(tr, cost, hillclimb=1, backoff=2)["trial_iters"] <= bo["trial_iters"]   # the earlier start tests less
    assert bo["tpot"] < no_bo["tpot"]
    assert bo["trial_iters"] < no_bo["trial_iters"] / 3
    assert bo["tpot"] / base < 1.02                      # within 2 % of never speculating
    assert no_bo["tpot"] / base > 1.05
    assert cs.run_static(tr, cost, 3)["tpot"] / base > 1.5     # what a fixed K = 3 would have cost


def test_high_acceptance_hill_climbing_finds_a_longer_draft():
    cost = cs.cost_table("mixtral-bf16-layer")
    tr = cs.Trace(4000, 3, rates=(0.8,))
    base = cs.run_static(tr, cost, 0)["tpot"]
    start_only = cs.run_cascade(tr, cost, hillclimb=0)
    full = cs.run_cascade(tr, cost, hillclimb=1)
    assert base / full["tpot"] > 1.4
    assert full["tpot"] <= start_only["tpot"] * 1.01
    mean_k = lambda r: sum(int(k) * n for k, n in r["K_histogram"].items()) / r["iters"]
    assert mean_k(full) >= 3.0


def test_concurrent_requests_choose_their_own_k():
    cost = cs.cost_table("mixtral-bf16-layer")
    good, bad = cs.Trace(3000, 4, rates=(0.8,)), cs.Trace(3000, 5, rates=(0.1,))
    r = cs.run_concurrent([good, bad], cost)
    assert r["k_max_per_request"] == 3                      # 2 x (3 + 1) = 8 tokens <= the 9 the table covers
    assert r["mean_K_per_request"][0] > r["mean_K_per_request"][1] + 0.5
    assert r["tokens_per_request"][0] > r["tokens_per_request"][1]
    with pytest.raises(ValueError):
        cs.run_concurrent([good] * 5, cost)
