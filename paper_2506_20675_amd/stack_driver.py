"""Decode loop of the 32-layer MoE stack under the utility-driven choice of K.

Each iteration: K = cascade_next_k(); the K+1 in-flight tokens go through every MoE layer of the stack
(moe_verify_stack, one stream, no host synchronisation inside); HIP events give t_verify; the number of
emitted tokens comes from the seeded draft-acceptance trace (stand-in for drafter + rejection sampler,
see synth.py); cascade_observe() feeds both back (paper: Section 5.1 overview — speculation manager and
utility analyzer; Section 5.3 test-and-set; Section 6 telemetry).

Usage (needs a GPU):  python -m paper_2506_20675_amd.stack_driver --iters 600 --layers 32 --rho 0.5
Prints one JSON summary line; --log FILE also writes one JSON record per iteration.
"""
from __future__ import annotations

import argparse
import json
import sys
import time

import numpy as np

from . import binding, synth


class HiddenPool:
    """hidden[L, T, d] for iteration i, layer l.  Drawing 32 x 9 x 4096 normals per iteration on the host
    would dominate the loop, so a pool of `n_pool` distinct (layer, draw) inputs is generated once and
    iteration i uses draw (i mod n_pool); rows are nested in T (row t does not depend on T)."""

    def __init__(self, cfg, layers, rho, n_pool=8, t_max=9, device="cuda"):
        import torch
        self.t_max = t_max
        host = np.stack([np.stack([synth.hidden_host(cfg, l, j, t_max, rho) for l in range(layers)])
                         for j in range(n_pool)])                      # [pool, L, t_max, d]
        self.host = host
        # one contiguous [L, T, d] tensor per (draw, T) so that moe_verify_stack can take it as is
        self.dev = {}
        for j in range(n_pool):
            for T in range(1, t_max + 1):
                self.dev[(j, T)] = torch.from_numpy(np.ascontiguousarray(host[j, :, :T, :])).to(device)
        self.n_pool = n_pool

    def get(self, i, T):
        return self.dev[(i % self.n_pool, T)]


def build_stack(cfg, layers, ctx, layout="tiled", first_layer=0, weights="bf16"):
    """Generate `layers` layers of weights directly in HBM (and re-lay them out once if tiled).
    weights = "fp8": E4M3 codes + per-row scales (tiled layout only)."""
    import torch
    if weights == "fp8" and layout != "tiled":
        raise ValueError("FP8 weights are streamed in the tiled layout only")
    out = []
    for l in range(layers):
        wd = (synth.layer_weights_fp8_device if weights == "fp8" else synth.layer_weights_device)(cfg, first_layer + l)
        w = ctx.weights(wd)
        if layout == "tiled":
            w = ctx.moe_pack_weights(w)
            torch.cuda.synchronize()
        out.append(w)
    return out


def run(cfg=synth.MIXTRAL, layers=32, iters=600, rho=0.5, layout="tiled", seed_field=0, params=None,
        static_k=None, log=None, ctx=None, stack=None, pool=None, gammas=None, attn=None):
    """Runs the loop; static_k = None uses the controller, an int forces that K every iteration.
    gammas (one RMSNorm weight tensor per layer) switches to the chained stack: the layers feed each other
    through pre-norm residual blocks and only layer 0's pooled input is used.  attn (one AttnWeights per layer)
    adds the attention stub in front of every MoE block (moe_decoder_stack; the context must carry the geometry).
    Returns (summary dict, per-iteration records)."""
    import torch
    own = ctx is None
    if own:
        ctx = binding.MoeContext(cfg.d, cfg.ffn, cfg.n_experts, cfg.top_k, cfg.n_shared, synth.K_MAX + 1, cfg.gate_mode)
    if stack is None:
        stack = build_stack(cfg, layers, ctx, layout)
    if pool is None:
        pool = HiddenPool(cfg, layers, rho)
    ctrl = binding.CascadeController(params) if static_k is None else None
    regimes = synth.regime_sequence(iters, seed_field)
    uni = synth.acceptance_uniforms(iters, seed_field)
    out = torch.empty((layers, synth.K_MAX + 1, cfg.d), dtype=torch.float32, device="cuda")
    nu = torch.zeros((layers,), dtype=torch.int32, device="cuda")
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    # warm-up: touch every layer once at the largest T
    chain_out = torch.empty((synth.K_MAX + 1, cfg.d), dtype=torch.float32, device="cuda")

    def step(hid, o, T):
        if attn is not None:
            ctx.moe_decoder_stack(stack, attn, hid[0], chain_out[:T], 1e-5, None, nu)
        elif gammas is None:
            ctx.moe_verify_stack(stack, hid, o, nu)
        else:
            ctx.moe_chained_stack(stack, gammas, hid[0], chain_out[:T], 1e-5, None, nu)

    step(pool.get(0, pool.t_max), out[:, :pool.t_max].contiguous(), pool.t_max)
    torch.cuda.synchronize()
    recs = []
    t_wall = time.perf_counter()
    for i in range(iters):
        k = ctrl.next_k() if ctrl is not None else static_k
        T = k + 1
        hid = pool.get(i, T)
        o = out[:, :T].contiguous() if T != out.shape[1] else out
        e0.record()
        step(hid, o, T)
        e1.record()
        e1.synchronize()
        t_verify = e0.elapsed_time(e1) * 1e-3
        tokens = synth.tokens_emitted(uni[i], regimes[i], k)
        rec = {"iter": i, "K": k, "tokens": tokens, "t_verify_ms": t_verify * 1e3, "p": float(regimes[i]),
               "mean_unique": float(nu.float().mean().item())}
        if ctrl is not None:
            st = ctrl.state()
            rec.update(phase=int(st.phase), s_cur=int(st.s_cur))
            ctrl.observe(k, tokens, t_verify)
            st = ctrl.state()
            rec.update(t_base_ms=st.t_base * 1e3, last_utility=st.last_utility)
        recs.append(rec)
    t_wall = time.perf_counter() - t_wall
    tok = sum(r["tokens"] for r in recs)
    tv = sum(r["t_verify_ms"] for r in recs)
    by_k = {}
    for r in recs:
        by_k.setdefault(r["K"], []).append(r["t_verify_ms"])
    summary = {
        "policy": "cascade" if static_k is None else f"static K={static_k}", "layers": layers, "iters": iters,
        "chained": gammas is not None or attn is not None, "attention_stub": attn is not None,
        "rho": rho, "layout": layout, "tokens": tok, "t_verify_total_ms": round(tv, 3),
        "tpot_ms": round(tv / tok, 4), "etr": round(tok / iters, 4),
        "K_histogram": {str(k): len(v) for k, v in sorted(by_k.items())},
        "t_verify_ms_by_K": {str(k): round(float(np.median(v)), 4) for k, v in sorted(by_k.items())},
        "wall_s": round(t_wall, 2),
    }
    if ctrl is not None:
        summary["trial_iters"] = int(ctrl.state().trial_iters)
    if log:
        with open(log, "w") as f:
            for r in recs:
                f.write(json.dumps(r) + "\n")
    if own:
        ctx.close()
    return summary, recs


def run_concurrent(cfg=synth.MIXTRAL, layers=32, iters=600, rho=0.5, requests=2, static_k=None, ctx=None, stack=None,
                   pool=None, layout="tiled", weights="bf16"):
    """R requests decoded together, each with its own controller and its own acceptance trace (seed field r):
    every iteration verifies the in-flight tokens of all requests in ONE pass over the stack, T = sum(K_r + 1) <= 16,
    so a request that speculates also lengthens the others' iteration — every controller sees the joint t_verify
    (paper: Section 5.1, one speculation manager per request; Section 6, per-request K).
    static_k = None: controllers; an int: that K for every request.  Returns (summary, records)."""
    import torch
    t_cap = 16
    k_max = t_cap // requests - 1
    if requests < 1 or k_max < 1:
        raise ValueError("1 <= requests <= 8")
    own = ctx is None
    if own:
        ctx = binding.MoeContext(cfg.d, cfg.ffn, cfg.n_experts, cfg.top_k, cfg.n_shared, t_cap, cfg.gate_mode)
    if stack is None:
        stack = build_stack(cfg, layers, ctx, layout, weights=weights)
    if pool is None:
        pool = HiddenPool(cfg, layers, rho, t_max=t_cap)
    ctrls = None
    if static_k is None:
        ctrls = [binding.CascadeController(k_max=k_max, k_start=min(3, k_max)) for _ in range(requests)]
    elif not 0 <= static_k <= k_max:
        raise ValueError(f"static K must be in 0..{k_max} for {requests} requests")
    regimes = [synth.regime_sequence(iters, r) for r in range(requests)]
    uni = [synth.acceptance_uniforms(iters, r) for r in range(requests)]
    out = torch.empty((layers, t_cap, cfg.d), dtype=torch.float32, device="cuda")
    nu = torch.zeros((layers,), dtype=torch.int32, device="cuda")
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ctx.moe_verify_stack(stack, pool.get(0, t_cap), out, nu)   # warm-up: every layer once at the largest T
    torch.cuda.synchronize()
    recs = []
    for i in range(iters):
        ks = [c.next_k() for c in ctrls] if ctrls else [static_k] * requests
        T = sum(k + 1 for k in ks)
        o = out[:, :T].contiguous() if T != t_cap else out
        e0.record()
        ctx.moe_verify_stack(stack, pool.get(i, T), o, nu)
        e1.record()
        e1.synchronize()
        t_verify = e0.elapsed_time(e1) * 1e-3
        toks = [synth.tokens_emitted(uni[r][i], regimes[r][i], ks[r]) for r in range(requests)]
        if ctrls:
            for r in range(requests):
                ctrls[r].observe(ks[r], toks[r], t_verify)
        recs.append({"iter": i, "K": ks, "T": T, "tokens": toks, "t_verify_ms": t_verify * 1e3})
    tok = sum(sum(r["tokens"]) for r in recs)
    tv = sum(r["t_verify_ms"] for r in recs)
    summary = {"policy": "cascade" if static_k is None else f"static K={static_k}", "requests": requests, "k_max": k_max,
               "layers": layers, "iters": iters, "rho": rho, "tokens": tok, "t_verify_total_ms": round(tv, 3),
               "ms_per_token": round(tv / tok, 4), "tokens_per_s": round(tok / (tv * 1e-3), 1),
               "mean_T": round(float(np.mean([r["T"] for r in recs])), 3),
               "mean_K_per_request": [round(float(np.mean([r["K"][q] for r in recs])), 3) for q in range(requests)],
               "tokens_per_request": [sum(r["tokens"][q] for r in recs) for q in range(requests)]}
    if own:
        ctx.close()
    return summary, recs


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="mixtral-8x7b-shaped")
    ap.add_argument("--layers", type=int, default=32)
    ap.add_argument("--iters", type=int, default=600)
    ap.add_argument("--rho", type=float, default=0.5)
    ap.add_argument("--layout", choices=("tiled", "row"), default="tiled")
    ap.add_argument("--static", type=str, default="", help="comma list of static K baselines to run too, e.g. 0,1,2,3")
    ap.add_argument("--log", default=None)
    ap.add_argument("--weights", choices=("bf16", "fp8"), default="bf16")
    ap.add_argument("--decoder", action="store_true",
                    help="full decoder blocks: attention stub + MoE, each feeding the next (moe_decoder_stack)")
    ap.add_argument("--chained", action="store_true",
                    help="pre-norm residual blocks feeding each other (moe_chained_stack) instead of independent inputs")
    ap.add_argument("--requests", type=int, default=1,
                    help="decode this many requests together, one controller each (independent-input stack only)")
    a = ap.parse_args(argv)
    cfg = synth.CONFIGS[a.config]
    if a.requests > 1:
        if a.chained or a.decoder:
            ap.error("--requests runs the independent-input stack")
        ctx = binding.MoeContext(cfg.d, cfg.ffn, cfg.n_experts, cfg.top_k, cfg.n_shared, 16, cfg.gate_mode)
        stack = build_stack(cfg, a.layers, ctx, a.layout, weights=a.weights)
        pool = HiddenPool(cfg, a.layers, a.rho, t_max=16)
        res = {"cascade": run_concurrent(cfg, a.layers, a.iters, a.rho, a.requests, None, ctx, stack, pool)[0]}
        for k in [int(v) for v in a.static.split(",") if v != ""]:
            res[f"static_{k}"] = run_concurrent(cfg, a.layers, a.iters, a.rho, a.requests, k, ctx, stack, pool)[0]
        base = res.get("static_0")
        if base:
            for v in res.values():
                v["speedup_vs_no_spec"] = round(base["ms_per_token"] / v["ms_per_token"], 4)
        for v in res.values():
            v["weights"] = a.weights
        print(json.dumps(res))
        ctx.close()
        return 0
    H, Hkv, dh = synth.attn_geometry(cfg) if a.decoder else (0, 0, 0)
    ctx = binding.MoeContext(cfg.d, cfg.ffn, cfg.n_experts, cfg.top_k, cfg.n_shared, synth.K_MAX + 1, cfg.gate_mode,
                             H, Hkv, dh)
    stack = build_stack(cfg, a.layers, ctx, a.layout, weights=a.weights)
    pool = HiddenPool(cfg, a.layers, a.rho)
    gammas = None
    if a.chained:
        import torch
        gammas = [torch.from_numpy(synth.norm_gamma_host(cfg, l).view(np.int16)).cuda() for l in range(a.layers)]
    attn = None
    if a.decoder:
        import torch
        attn = []
        for l in range(a.layers):
            A = synth.attn_weights_host(cfg, l)
            attn.append(ctx.attn_weights({k: torch.from_numpy(v.view(np.int16)).cuda() for k, v in A.items()
                                          if isinstance(v, np.ndarray)}))
        torch.cuda.synchronize()
    res = {"cascade": run(cfg, a.layers, a.iters, a.rho, a.layout, log=a.log, ctx=ctx, stack=stack, pool=pool,
                          gammas=gammas, attn=attn)[0]}
    for k in [int(v) for v in a.static.split(",") if v != ""]:
        res[f"static_{k}"] = run(cfg, a.layers, a.iters, a.rho, a.layout, static_k=k, ctx=ctx, stack=stack,
                                 pool=pool, gammas=gammas, attn=attn)[0]
    base = res.get("static_0")
    if base:
        for v in res.values():
            v["speedup_vs_no_spec"] = round(base["tpot_ms"] / v["tpot_ms"], 4)
    for v in res.values():
        v["weights"] = a.weights
    print(json.dumps(res))
    ctx.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
