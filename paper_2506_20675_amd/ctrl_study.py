"""Controller studies on synthetic acceptance traces — host only, no GPU.

The K-selection policy (paper: Section 5.3 test-and-set, 5.4 disabling, 5.5 back-off, 5.6 hill-climbing)
is driven here by a verification-cost table t_verify(K) instead of live kernels, so that its parts can
be switched on one by one (the ablation of Section 7.4), its hyper-parameters swept (t, S; Section 7.5)
and its result put next to static-K and clairvoyant choices, all on the seeded acceptance traces of
synth.py.  The controller itself is the C one of the product library (cascade_ctrl_*); this module only
feeds it (tokens, time) pairs.

Cost tables: per-iteration verification latency for K = 0..8.  The built-in ones are latencies measured
with bench.py / stack_driver.py on an MI355X (see MEASURED below for the commands); `balls_in_bins`
builds one from the uniform-routing model of Section 2.4; `from_bench_json` reads the by_K table of a
bench.py line.  Tables are made non-decreasing in K (a larger K never verifies faster; measured tables
can dip where the sampled inputs happened to form a smaller expert union).

  python -m paper_2506_20675_amd.ctrl_study --cost mixtral-bf16-layer --iters 6000
"""
from __future__ import annotations

import argparse
import json
import os
import sys

import numpy as np

from . import binding, synth

# Verification-cost tables measured on an MI355X (rho = 0.5) live in measured_costs.json next to this module, each
# with the command that produced it; `--record NAME --bench-json FILE` (or --stack-json FILE) rewrites an entry from
# a fresh bench.py / stack_driver line, so the tables follow the kernels instead of being typed in.
_MEASURED_FILE = os.path.join(os.path.dirname(os.path.abspath(__file__)), "measured_costs.json")


def _load_measured() -> dict:
    with open(_MEASURED_FILE) as f:
        return {name: entry["cost"] for name, entry in json.load(f).items()}


MEASURED = _load_measured()


def record_measured(name: str, cost, unit: str, command: str) -> None:
    """Replace (or add) one table of measured_costs.json."""
    with open(_MEASURED_FILE) as f:
        data = json.load(f)
    data[name] = {"cost": [round(float(c), 4) for c in cost], "unit": unit, "command": command}
    with open(_MEASURED_FILE, "w") as f:
        json.dump(data, f, indent=1, sort_keys=True)
        f.write("\n")
    MEASURED[name] = data[name]["cost"]


def from_stack_json(line: str) -> np.ndarray:
    """t_verify per iteration for K = 0, 1, ... from a stack_driver line: the static-K runs first, then the K the
    controller run reached beyond them."""
    d = json.loads(line)
    cost, k = [], 0
    while True:
        v = d.get(f"static_{k}", {}).get("t_verify_ms_by_K", {}).get(str(k))
        if v is None:
            v = d.get("cascade", {}).get("t_verify_ms_by_K", {}).get(str(k))
        if v is None:
            break
        cost.append(v)
        k += 1
    return np.array(cost)


def monotone(cost) -> np.ndarray:
    return np.maximum.accumulate(np.asarray(cost, dtype=np.float64))


def balls_in_bins(n_experts=8, top_k=2, k_max=8, fixed=0.0) -> np.ndarray:
    """t(K) proportional to the expected number of unique experts of K+1 tokens under uniform routing
    (Section 2.4), plus a K-independent share `fixed` (attention and the like) in units of one expert."""
    T = np.arange(1, k_max + 2, dtype=np.float64)
    return fixed + n_experts * (1.0 - (1.0 - top_k / n_experts) ** T)


def from_bench_json(line: str) -> np.ndarray:
    d = json.loads(line)
    ks = sorted(int(k) for k in d["by_K"])
    assert ks == list(range(len(ks))), "by_K must cover K = 0..n without gaps"
    return np.array([d["by_K"][str(k)]["latency_us"] for k in ks])


def cost_table(name_or_list) -> np.ndarray:
    if isinstance(name_or_list, str):
        if name_or_list not in MEASURED:
            raise KeyError(f"unknown cost table {name_or_list}; have {sorted(MEASURED)}")
        return monotone(MEASURED[name_or_list])
    return monotone(name_or_list)


def expected_tokens(p: float, K: int) -> float:
    """Mean tokens per iteration with causal acceptance at per-draft rate p: 1 + p + ... + p^K."""
    return float(K + 1) if p >= 1.0 else (1.0 - p ** (K + 1)) / (1.0 - p)


def clairvoyant_k(p: float, cost: np.ndarray) -> int:
    """The K an all-knowing policy picks for acceptance rate p: arg-max of expected utility (Section 4)."""
    u = [expected_tokens(p, k) / (cost[k] / cost[0]) for k in range(len(cost))]
    return int(np.argmax(u))


class Trace:
    """Seeded acceptance trace (regime per iteration + one uniform per draft position)."""

    def __init__(self, iters: int, seed_field: int = 0, rates=synth.ACCEPT_RATES, period: int = synth.REGIME_PERIOD):
        self.iters = iters
        self.p = synth.regime_sequence(iters, seed_field, rates, period)
        self.u = synth.acceptance_uniforms(iters, seed_field)

    def tokens(self, i: int, K: int) -> int:
        return synth.tokens_emitted(self.u[i], self.p[i], K)


def _summary(name, ks, toks, times, extra=None):
    ks, toks, times = np.asarray(ks), np.asarray(toks), np.asarray(times, dtype=np.float64)
    out = {"policy": name, "iters": int(len(ks)), "tokens": int(toks.sum()), "time": float(times.sum()),
           "tpot": float(times.sum() / toks.sum()), "etr": float(toks.mean()),
           "K_histogram": {str(k): int((ks == k).sum()) for k in sorted(set(ks.tolist()))}}
    if extra:
        out.update(extra)
    return out


def run_static(trace: Trace, cost: np.ndarray, K: int):
    ks = [K] * trace.iters
    toks = [trace.tokens(i, K) for i in range(trace.iters)]
    return _summary(f"static K={K}", ks, toks, [cost[K]] * trace.iters)


def run_clairvoyant(trace: Trace, cost: np.ndarray):
    best = {p: clairvoyant_k(p, cost) for p in set(trace.p.tolist())}
    ks = [best[p] for p in trace.p.tolist()]
    toks = [trace.tokens(i, ks[i]) for i in range(trace.iters)]
    return _summary("clairvoyant", ks, toks, [cost[k] for k in ks], {"K_per_rate": {str(p): k for p, k in sorted(best.items())}})


def run_cascade(trace: Trace, cost: np.ndarray, name="cascade", **params):
    """The C controller on the trace.  params override cascade_default_params (k_max is capped by the table)."""
    params.setdefault("k_max", min(len(cost) - 1, synth.K_MAX))
    params.setdefault("k_start", min(3, params["k_max"]))
    ctrl = binding.CascadeController(**params)
    ks, toks, times = [], [], []
    for i in range(trace.iters):
        k = ctrl.next_k()
        tok = trace.tokens(i, k)
        ctrl.observe(k, tok, float(cost[k]))
        ks.append(k), toks.append(tok), times.append(cost[k])
    st = ctrl.state()
    out = _summary(name, ks, toks, times, {"trial_iters": int(st.trial_iters), "params": dict(params)})
    ctrl.close()
    return out


ABLATION = (  # Section 7.4: the parts of the policy added one at a time
    ("test K_start only, disable when U < 1", dict(hillclimb=0, backoff=0)),
    ("+ adaptive back-off", dict(hillclimb=0, backoff=1)),
    ("+ hill-climbing (full policy)", dict(hillclimb=1, backoff=1)),
)


def run_concurrent(traces, cost: np.ndarray, **params):
    """R requests decoded together, each with its own controller and K.  One iteration verifies all their tokens in
    one step, so its time is the table entry for the TOTAL number of in-flight tokens and every request observes that
    shared time with its own emitted tokens.  k_max per request keeps the total inside the table."""
    R = len(traces)
    k_cap = len(cost) // R - 1            # R * (k_cap + 1) tokens <= table length
    if k_cap < 1:
        raise ValueError("cost table too short for that many requests")
    params = dict(params)
    params["k_max"] = min(params.get("k_max", k_cap), k_cap)
    params.setdefault("k_start", min(3, params["k_max"]))
    ctrls = [binding.CascadeController(**params) for _ in range(R)]
    iters = min(t.iters for t in traces)
    ks = np.zeros((iters, R), dtype=np.int64)
    toks = np.zeros((iters, R), dtype=np.int64)
    times = np.zeros(iters)
    for i in range(iters):
        k = [c.next_k() for c in ctrls]
        t_joint = float(cost[sum(k) + R - 1])       # table index = total tokens - 1
        for r in range(R):
            toks[i, r] = traces[r].tokens(i, k[r])
            ctrls[r].observe(k[r], int(toks[i, r]), t_joint)
        ks[i], times[i] = k, t_joint
    for c in ctrls:
        c.close()
    base = float(cost[R - 1]) * iters / (iters * R)                  # every request at K = 0: R tokens per joint step
    return {"policy": f"cascade x{R} requests", "iters": iters, "tokens": int(toks.sum()), "time": float(times.sum()),
            "tpot": float(times.sum() / toks.sum()), "tpot_no_spec": base,
            "speedup_vs_no_spec": base / float(times.sum() / toks.sum()),
            "mean_K_per_request": [float(v) for v in ks.mean(axis=0)],
            "tokens_per_request": [int(v) for v in toks.sum(axis=0)], "k_max_per_request": params["k_max"]}


def backoff_example(window=250, cost_ratio=2.0):
    """The worked example of Section 5.5 from the start of a request: speculation never pays (no draft is ever
    accepted, every speculative iteration costs `cost_ratio` x a plain one), t = 4, S = 16.  For no back-off and for
    the two readings of "double S whenever K drops to 0": speculative-trial iterations among the first `window`
    iterations, and the slowdown over never speculating.  The paper quotes "nearly 50" against "only 18" and a
    worst-case slowdown of 14 % against 5 %."""
    out = {}
    for name, bo in (("no back-off", 0), ("first disabled phase keeps S", 1), ("every drop doubles S", 2)):
        ctrl = binding.CascadeController(backoff=bo)
        spec, t = 0, 0.0
        for _ in range(window):
            k = ctrl.next_k()
            dt = cost_ratio if k > 0 else 1.0
            ctrl.observe(k, 1, dt)
            spec += k > 0
            t += dt
        ctrl.close()
        out[name] = {"trial_iters": int(spec), "slowdown": round(t / window - 1.0, 4)}
    return out


def study(cost, iters=6000, seed_field=0, rates=synth.ACCEPT_RATES, period=synth.REGIME_PERIOD):
    cost = cost_table(cost)
    trace = Trace(iters, seed_field, rates, period)
    base = run_static(trace, cost, 0)
    res = {"cost_ratio": [round(float(c / cost[0]), 3) for c in cost], "regime_period": period, "static": [],
           "ablation": [], "sweep": [], "backoff_cap": []}

    def rel(r):
        r["speedup_vs_no_spec"] = round(base["tpot"] / r["tpot"], 4)
        return r

    for k in range(len(cost)):
        res["static"].append(rel(run_static(trace, cost, k)))
    res["clairvoyant"] = rel(run_clairvoyant(trace, cost))
    for name, flags in ABLATION:
        res["ablation"].append(rel(run_cascade(trace, cost, name, **flags)))
    for t in (2, 4, 8):
        for s in (8, 16, 32):
            res["sweep"].append(rel(run_cascade(trace, cost, f"t={t} S={s}", t_trial=t, s_set=s)))
    # the back-off doubles S without bound while speculation stays off; a cap trades test cost in long bad
    # stretches against the time it takes to notice that acceptance has recovered
    for cap in (0, 32, 64, 128):
        res["backoff_cap"].append(rel(run_cascade(trace, cost, f"s_max={cap}", s_max=cap)))
    # the two readings of the back-off rule on this trace, and on the paper's own worked example
    res["backoff_reading"] = [rel(run_cascade(trace, cost, f"backoff={bo}", backoff=bo)) for bo in (1, 2)]
    res["backoff_example_250"] = backoff_example()
    return res


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--cost", default="mixtral-bf16-layer", help=f"one of {sorted(MEASURED)}, or 'model' (balls in bins)")
    ap.add_argument("--bench-json", default=None, help="file holding a bench.py line; its by_K latencies are the table")
    ap.add_argument("--iters", type=int, default=6000)
    ap.add_argument("--requests", type=int, default=0, help="also run this many concurrent requests (0 = skip)")
    ap.add_argument("--period", type=int, default=synth.REGIME_PERIOD, help="iterations an acceptance regime lasts")
    ap.add_argument("--stack-json", default=None, help="file holding a stack_driver line; its t_verify per K is the table")
    ap.add_argument("--record", default=None, metavar="NAME",
                    help="store the table of --bench-json / --stack-json in measured_costs.json under NAME and exit")
    ap.add_argument("--command", default="", help="with --record: the command that produced the line")
    a = ap.parse_args(argv)
    if a.record:
        src = a.bench_json or a.stack_json
        line = [l for l in open(src) if l.startswith("{")][-1]
        cost = from_bench_json(line) if a.bench_json else from_stack_json(line)
        record_measured(a.record, cost, "us per layer-step" if a.bench_json else "ms per iteration", a.command)
        print(f"{a.record}: {list(MEASURED[a.record])}")
        return 0
    if a.stack_json:
        cost = from_stack_json([l for l in open(a.stack_json) if l.startswith("{")][-1])
    elif a.bench_json:
        cost = from_bench_json([l for l in open(a.bench_json) if l.startswith("{")][-1])
    elif a.cost == "model":
        cost = balls_in_bins()
    else:
        cost = a.cost
    res = study(cost, a.iters, period=a.period)
    if a.requests > 1:
        c = cost_table(cost)
        traces = [Trace(a.iters, 100 + r, period=a.period) for r in range(a.requests)]
        res["concurrent"] = run_concurrent(traces, c)
    print(json.dumps(res))
    return 0


if __name__ == "__main__":
    sys.exit(main())
