#!/usr/bin/env python3
"""Benchmark of the MoE verification path on one MI355X.

A "step" is one pass of the whole hot path (route -> group + gate/up -> down -> combine, i.e. one
moe_verify_layer call) over one batch of T = K+1 synthetic tokens on a Mixtral-8x7B-shaped layer.
Step i uses K = i mod 9 (so every sweep K = 0..8 is timed equally often) and layer i mod L of L
distinct resident layers, so consecutive steps never re-read weights that could still sit in the
256 MB last-level cache.  Inputs are resident in HBM before the timed region starts.

Prints ONE JSON line:  metric / value = unique-expert GB/s over the whole timed region (sum of
unique-expert weight bytes / wall time), per-K latency and GB/s tables, the roofline object for the
dominant kernel (gate/up projection, 2/3 of the bytes), and the CPU oracle timed beside it.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E peak
TRAFFIC_TAG = {"mixtral-8x7b-shaped": "mixtral", "olmoe-like": "olmoe", "deepseek-v2-lite-like": "deepseek"}
BY_K_STEPS = 20        # layer-steps per K in the latency-vs-K table (a sample of its own, independent of --steps)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None, help="timed steps (default 180; 36 with --stack)")
    ap.add_argument("--warmup", type=int, default=None, help="untimed warm-up steps (default 18; 9 with --stack)")
    ap.add_argument("--stack", type=int, default=0, metavar="L",
                    help="a step = ONE moe_verify_stack call over L distinct resident layers (32 = the 90 GB Mixtral-shaped "
                         "stack) instead of one moe_verify_layer call; latencies are still reported per layer")
    ap.add_argument("--rho", type=float, default=0.5)
    ap.add_argument("--layers", type=int, default=8, help="distinct resident layers rotated through")
    ap.add_argument("--config", default="mixtral-8x7b-shaped")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--fixed-k", type=int, default=-1, help="time a single K instead of cycling 0..8")
    ap.add_argument("--layout", choices=("tiled", "row"), default="tiled",
                    help="expert weight storage: tiled = re-ordered once at load time by moe_pack_weights")
    ap.add_argument("--weights", choices=("bf16", "fp8"), default="bf16",
                    help="expert weight type: bf16 (the headline workload) or fp8 = E4M3 codes + per-row scales")
    ap.add_argument("--tune", default="", help="tuning aid: gu_tiles,dn_tiles,dn_split_k,fused_down for moe_ctx_tune "
                                                 "(0,0,0,-1 = the automatic plan)")
    args = ap.parse_args()
    if args.gpus != 1:
        print(f"bench.py: this build is single-GPU (no sharding, no collectives); --gpus {args.gpus} is not supported",
              file=sys.stderr)
        sys.exit(2)

    if args.steps is None:
        args.steps = 36 if args.stack else 180
    if args.warmup is None:
        args.warmup = 9 if args.stack else 18
    fp8 = args.weights == "fp8"

    import torch
    from paper_2506_20675_amd import binding, synth

    if not os.path.exists(binding.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    cfg = synth.CONFIGS[args.config]
    expert_bytes = cfg.expert_bytes_fp8 if fp8 else cfg.expert_bytes
    S = args.stack                       # layers per step in stack mode, 0 = single-layer steps
    L, K_steps, W_steps = (S or args.layers), args.steps, args.warmup
    LS = S or 1
    by_k_steps = 4 if S else BY_K_STEPS  # a stack step is S layer-steps already
    T_MAX = 9

    # ---- resident inputs -------------------------------------------------------------------
    ctx = binding.MoeContext(cfg.d, cfg.ffn, cfg.n_experts, cfg.top_k, cfg.n_shared, T_MAX, cfg.gate_mode)
    if args.tune:
        ctx.moe_ctx_tune(*[int(v) for v in args.tune.split(",")])
    lw = []
    for l in range(L):
        # row-major, as the oracle sees them
        wd = synth.layer_weights_fp8_device(cfg, l) if fp8 else synth.layer_weights_device(cfg, l)
        w = ctx.weights(wd)
        if args.layout == "tiled":
            w = ctx.moe_pack_weights(w)                   # one-off static re-layout, same bytes
            torch.cuda.synchronize()
        lw.append(w)
        del wd
    total = W_steps + K_steps

    def k_of(i):
        return args.fixed_k if args.fixed_k >= 0 else i % T_MAX

    def hidden(layer, it, T):
        """Input of one step: [T, d] for layer `layer`, or in stack mode [S, T, d] for layers 0..S-1 (independent
        seeded per-layer inputs)."""
        if S:
            return torch.from_numpy(np.stack([synth.hidden_host(cfg, l, it, T, args.rho) for l in range(S)])).cuda()
        return torch.from_numpy(synth.hidden_host(cfg, layer, it, T, args.rho)).cuda()

    hid = [hidden(i % L, i, k_of(i) + 1) for i in range(total)]
    outs = [torch.empty((T_MAX, cfg.d), dtype=torch.float32, device="cuda") for _ in range(2)]
    outs_stack = {T: torch.empty((S, T, cfg.d), dtype=torch.float32, device="cuda") for T in range(1, T_MAX + 1)} if S else None
    nu = torch.zeros((total, LS), dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()

    def run(layer, x, nu_row, parity_slot):
        """One step of the path on input x: a single layer, or the whole stack in one call."""
        T = x.shape[-2]
        if S:
            ctx.moe_verify_stack(lw, x, outs_stack[T], nu_row)
        else:
            ctx.moe_verify_layer(lw[layer], x, outs[parity_slot][:T], n_unique=nu_row)

    def step(i):
        run(i % L, hid[i], nu[i], i & 1)

    # ---- warm-up, then the timed region: exactly K_steps steps, nothing else on the stream -----
    for i in range(W_steps):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for j in range(K_steps):
        step(W_steps + j)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    nu_h = nu.cpu().numpy()[W_steps:].reshape(-1)          # one entry per layer-step
    ubytes = (nu_h.astype(np.int64) + cfg.n_shared) * expert_bytes
    value = ubytes.sum() / wall / 1e9

    # ---- latency per layer vs K: a sample of its own, BY_K_STEPS steps per K whatever --steps is -----------
    # One event pair around each group of BY_K_STEPS steps (an event between every two steps would put an extra
    # packet into each kernel chain, and a pair around two or three steps would not amortise its own latency).
    k_list = [args.fixed_k] if args.fixed_k >= 0 else list(range(T_MAX))
    sample = {k: [(j % L, 50_000 + 100 * k + j) for j in range(by_k_steps)] for k in k_list}
    s_hid = {k: [hidden(l, it, k + 1) for l, it in sample[k]] for k in k_list}
    s_nu = torch.zeros((len(k_list), by_k_steps, LS), dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()

    def sample_step(ki, k, j):
        run(sample[k][j][0], s_hid[k][j], s_nu[ki, j], j & 1)

    by_k = {}
    for ki, k in enumerate(k_list):
        reps = []
        for _ in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            # lead-in: the group once untimed, so that the first timed step follows a busy GPU as every step of a
            # decode loop does (a launch into an idle GPU pays its wake-up, 10-20 us); the whole group, so that every
            # step of the sample is launched equally often (the counter summaries under profiles/ average over them)
            for j in range(by_k_steps):
                sample_step(ki, k, j)
            e0.record()
            for j in range(by_k_steps):
                sample_step(ki, k, j)
            e1.record()
            torch.cuda.synchronize()
            reps.append(e0.elapsed_time(e1) / (by_k_steps * LS))          # per layer-step
        lat_ms = float(np.median(reps))
        # spread of single steps: one event pair per step (each pair puts extra packets into the chain, so these
        # run a few us above the grouped figure; they are reported for the p10/p90 spread only)
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(by_k_steps)]
        for j in range(by_k_steps):
            evs[j][0].record()
            sample_step(ki, k, j)
            evs[j][1].record()
        torch.cuda.synchronize()
        single = np.array([a.elapsed_time(b) * 1e3 / LS for a, b in evs])
        nu_k = s_nu[ki].cpu().numpy().astype(np.int64).reshape(-1)
        gbs = float(((nu_k + cfg.n_shared) * expert_bytes).mean()) / (lat_ms * 1e-3) / 1e9
        by_k[str(k)] = {"latency_us": round(lat_ms * 1e3, 1), "mean_unique": round(float(nu_k.mean()), 2),
                        "unique_GBps": round(gbs, 1), "frac_hbm_peak": round(gbs / HBM_PEAK_GBS, 4),
                        "single_step_us_p10_p50_p90": [round(float(np.percentile(single, q)), 1) for q in (10, 50, 90)]}
    k0 = by_k.get("0", {}).get("latency_us")
    if k0:
        for k in by_k:
            by_k[k]["t_verify_over_t0"] = round(by_k[k]["latency_us"] / k0, 3)
    del s_hid

    # ---- roofline of the dominant kernel: same steps again with per-kernel events ------------
    ctx.moe_ctx_profile(True)
    for j in range(K_steps):
        step(W_steps + j)
    torch.cuda.synchronize()
    kms, n_prof = ctx.moe_ctx_profile_read()
    ctx.moe_ctx_profile(False)
    gu_bytes_per_launch = float((nu_h.astype(np.int64) + cfg.n_shared).mean()) * 2 * expert_bytes / 3
    gu_ms = kms["gateup"] / max(n_prof, 1)
    achieved = gu_bytes_per_launch / (gu_ms * 1e-3) / 1e9
    roofline = {"bound": "hbm", "kernel": "gateup_kernel", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": None,
                "avg_launch_us": round(gu_ms * 1e3, 2), "algorithmic_bytes_per_launch": int(gu_bytes_per_launch),
                "kernel_us_per_step": {k: round(v / max(n_prof, 1) * 1e3, 2) for k, v in kms.items()}}
    # HBM bytes per launch: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE cannot run inside this process, so the figure is
    # DERIVED from the committed counter run on this workload (profiles/): its measured traffic / algorithmic ratio
    # of the gate/up kernel times this run's algorithmic bytes per launch
    traffic_file = os.path.join("profiles", f"gateup_kernel_{TRAFFIC_TAG.get(cfg.name, cfg.name)}{'_fp8' if fp8 else ''}_hbm_traffic.txt")
    if args.layout == "tiled" and os.path.exists(os.path.join(ROOT, traffic_file)):
        t_b = a_b = None
        for line in open(os.path.join(ROOT, traffic_file)):
            if line.startswith("traffic_bytes_per_launch gateup_kernel"):
                t_b = int(line.split()[-1])
            elif line.startswith("algorithmic bytes per launch"):
                a_b = int(line.split("=")[-1])
        if t_b and a_b:
            roofline["traffic"] = int(round(t_b / a_b * gu_bytes_per_launch))
            roofline["traffic_source"] = (f"derived: traffic/algorithmic = {t_b / a_b:.4f} measured with rocprofv3 --pmc "
                                          f"FETCH_SIZE, WRITE_SIZE ({traffic_file}) x this run's algorithmic bytes per launch")
    dn_bytes = float((nu_h.astype(np.int64) + cfg.n_shared).mean()) * expert_bytes / 3
    roofline["down_kernel_GBps"] = round(dn_bytes / (kms["down"] / max(n_prof, 1) * 1e-3) / 1e9, 1)

    # ---- the box's plain read-stream rate, as a second denominator ---------------------------
    # one launch over 8 GB (so that the ~8 us a launch costs whatever it does are below 1 %), data that has not
    # been read before; best of three passes
    sink = torch.zeros(4096, dtype=torch.float32, device="cuda")
    probe = torch.empty(2 << 30, dtype=torch.int32, device="cuda")
    probe.random_()
    binding.moe_stream_read_probe(lw[0].tensors[1], sink)          # warm the kernel itself on other data
    torch.cuda.synchronize()
    stream_gbs = 0.0
    for _ in range(3):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        binding.moe_stream_read_probe(probe, sink)
        e1.record()
        torch.cuda.synchronize()
        stream_gbs = max(stream_gbs, probe.numel() * 4 / (e0.elapsed_time(e1) * 1e-3) / 1e9)
    del probe

    # ---- the gate/up kernel's weight loads alone (same grid, walk, loads and pipeline depth; no fragments, no
    # matrix-core instructions): what the bytes cost on this access pattern, next to the real kernel's time ------
    twin = None
    if not fp8 and args.layout == "tiled":
        n_list = sorted({min(n, cfg.n_experts) for n in (cfg.top_k, 2 * cfg.top_k, 3 * cfg.top_k, 4 * cfg.top_k)})
        us = {}
        for n in n_list:
            # as in the per-kernel pass above: one event pair around every launch, launches back to back on rotating
            # layers, one synchronisation at the end (a launch into an idle GPU would pay its wake-up as well)
            evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(9)]
            for rep, (e0, e1) in enumerate(evs):
                w = lw[(rep + n) % L]
                e0.record()
                binding.moe_weight_load_twin(w.tensors[1], w.tensors[2], n, cfg.ffn // 16, cfg.d // 32, sink)
                e1.record()
            torch.cuda.synchronize()
            us[n] = float(np.median([a.elapsed_time(b) * 1e3 for a, b in evs[1:]]))
        # time = a + b * slots (least squares), read at this run's mean number of live slots
        xs, ys = np.array(list(us.keys()), dtype=np.float64), np.array(list(us.values()))
        b_fit, a_fit = np.polyfit(xs, ys, 1) if len(xs) > 1 else (0.0, ys[0])
        mean_slots = float((nu_h.astype(np.int64) + cfg.n_shared).mean())
        twin = {"us_by_slots": {str(k): round(v, 2) for k, v in us.items()},
                "fit_us": [round(float(a_fit), 2), round(float(b_fit), 3)],
                "us_at_mean_live_slots": round(float(a_fit + b_fit * mean_slots), 2),
                "gateup_kernel_avg_launch_us": roofline["avg_launch_us"],
                "note": "one HIP event pair per launch in both figures"}

    # ---- CPU oracle beside it (bounded sample, single thread) ---------------------------------
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import moe_oracle as orc
        Wh = synth.layer_weights_fp8_host(cfg, 0) if fp8 else synth.layer_weights_host(cfg, 0)
        sample_T = tuple(range(1, T_MAX + 1)) + (T_MAX,)
        cbytes, csec = 0, 0.0
        max_err, err2, ref2, ids_equal = 0.0, 0.0, 0.0, True
        for n, T in enumerate(sample_T):
            x = synth.hidden_host(cfg, 0, 10_000 + n, T, args.rho)
            c0 = time.perf_counter()
            ref, rids, _ = (orc.layer_fp8 if fp8 else orc.layer)(x, Wh, cfg.top_k, cfg.n_shared, "f32", cfg.gate_mode)
            csec += time.perf_counter() - c0
            cbytes += (orc.union(rids, cfg.n_experts)["n_unique"] + cfg.n_shared) * expert_bytes
            # the same step through the library, in the launch configuration that was timed above
            ids_d = torch.full((T, cfg.top_k), -1, dtype=torch.int32, device="cuda")
            ctx.moe_verify_layer(lw[0], torch.from_numpy(x).cuda(), outs[0][:T], ids=ids_d)
            torch.cuda.synchronize()
            err = outs[0][:T].cpu().numpy().astype(np.float64) - ref
            max_err = max(max_err, float(np.abs(err).max()))
            err2 += float((err ** 2).sum())
            ref2 += float((ref.astype(np.float64) ** 2).sum())
            ids_equal = ids_equal and bool((ids_d.cpu().numpy() == rids).all())
        rel_rms = (err2 / ref2) ** 0.5
        cpu = {"value": round(cbytes / csec / 1e9, 3), "unit": "GB/s", "cores": 1, "kind": "oracle",
               "sample": f"fp32 oracle, layer 0, rho={args.rho}, one layer-step each at T in {list(sample_T)}; "
                         f"{csec:.1f} s of CPU time; host has {os.cpu_count()} logical cores",
               "ms_per_step": round(csec / len(sample_T) * 1e3, 1),
               "parity": {"steps": len(sample_T), "ids_equal": ids_equal, "max_abs_err": float(f"{max_err:.3e}"),
                          "rel_rms": float(f"{rel_rms:.3e}")}}
        if not (ids_equal and max_err <= 2e-2 and rel_rms <= 1e-2):
            print("bench.py: the library's output left the parity bar against the oracle: " + json.dumps(cpu["parity"]),
                  file=sys.stderr)
            sys.exit(1)

    res = {
        "metric": "unique-expert GB/s (MoE verify step, sum of unique-expert weight bytes / time); latency/layer vs K in by_K",
        "value": round(float(value), 1), "unit": "GB/s", "n_gpus": 1, "steps": K_steps, "warmup": W_steps,
        "ms_per_step": round(wall / K_steps * 1e3, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",   # MFMA operand type (FP8 codes are widened to bf16)
        "config": {"workload": f"{cfg.name} MoE layer d={cfg.d} E={cfg.n_experts} top{cfg.top_k} ffn={cfg.ffn} "
                               f"shared={cfg.n_shared}, {'FP8 E4M3 + per-row scale' if fp8 else 'bf16'} weights, T=K+1 with K "
                               + (f"= {args.fixed_k}" if args.fixed_k >= 0 else "cycling 0..8")
                               + f", rho={args.rho}, "
                               + (f"stack of {S} distinct resident layers with independent seeded inputs, one moe_verify_stack "
                                  f"call per step (latencies per layer)" if S else f"{L} rotating resident layers")
                               + f", {args.layout} weight layout"},
        "layer_steps_per_step": LS, "us_per_layer_step": round(wall / (K_steps * LS) * 1e6, 2),
        "frac_hbm_peak": round(float(value / HBM_PEAK_GBS), 4),
        "by_K": by_k, "roofline": roofline, "stream_read_GBps": round(stream_gbs, 1),
        "gateup_load_twin": twin, "cpu_baseline": cpu,
    }
    print(json.dumps(res))


if __name__ == "__main__":
    main()
