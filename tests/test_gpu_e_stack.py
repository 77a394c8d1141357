"""GPU parity, part 5: the 32-layer stack and the decode loop under the controller.
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from oracle import moe_oracle as orc
from paper_2506_20675_amd import binding, synth
from gpu_common import (_check_layer, _check_out, _dev, _run_layer, _tiled, _weights_dev)


from gpu_common import _attn_dev


def test_stack_full_size_sampled_layers_match_the_oracle():
    """The 32-layer Mixtral-shaped stack as the stack driver runs it (90 GB of device-generated weights, tiled,
    one moe_verify_stack call per T); the oracle regenerates the weights of layers 0, 15 and 31 from the seed and
    checks those layers' whole outputs and union sizes at T = 1, 4 and 9."""
    import torch
    from paper_2506_20675_amd import stack_driver
    cfg, L, sample = synth.MIXTRAL, 32, (0, 15, 31)
    free, _ = torch.cuda.mem_get_info()
    if free < 100 * 2**30:
        pytest.skip("needs 100 GB of free device memory")
    ctx = binding.MoeContext(cfg.d, cfg.ffn, cfg.n_experts, cfg.top_k, 0, 9)
    stack = stack_driver.build_stack(cfg, L, ctx, layout="tiled")
    x9 = np.stack([synth.hidden_host(cfg, l, 700, 9, 0.5) for l in range(L)])   # rows are nested in T
    outs = {}
    for T in (1, 4, 9):
        out = torch.full((L, T, cfg.d), float("nan"), dtype=torch.float32, device="cuda")
        nu = torch.full((L,), -7, dtype=torch.int32, device="cuda")
        ctx.moe_verify_stack(stack, _dev(np.ascontiguousarray(x9[:, :T])), out, nu)
        torch.cuda.synchronize()
        outs[T] = (out.cpu().numpy(), nu.cpu().numpy())
        assert np.isfinite(outs[T][0]).all()
    del stack
    ctx.close()
    torch.cuda.empty_cache()
    for l in sample:
        W = synth.layer_weights_host(cfg, l)
        for T in (1, 4, 9):
            x = np.ascontiguousarray(x9[l, :T])
            ref32, rids, _ = orc.layer(x, W, cfg.top_k, 0, "f32")
            ref64, _, _ = orc.layer(x, W, cfg.top_k, 0, "f64")
            _check_out(outs[T][0][l], ref32, ref64)
            assert int(outs[T][1][l]) == orc.union(rids, cfg.n_experts)["n_unique"]
    # every layer's union is possible for its T, not only the sampled ones
    for T in (1, 4, 9):
        assert ((outs[T][1] >= cfg.top_k) & (outs[T][1] <= min(cfg.n_experts, T * cfg.top_k))).all()


def test_stack_driver_decisions_replay_on_the_policy_oracle():
    """The decode loop on a small stack: measured t_verify feeds the C controller; replaying the recorded
    (K, tokens, time) trace through the Python policy oracle must give the same K at every iteration."""
    from oracle import cascade_oracle as co
    from paper_2506_20675_amd import stack_driver
    cfg = synth.TINY
    summary, recs = stack_driver.run(cfg, layers=4, iters=160, rho=0.5, layout="tiled")
    ref = co.Controller()
    for r in recs:
        assert ref.next_k() == r["K"], r
        assert 1 <= r["tokens"] <= r["K"] + 1
        ref.observe(r["K"], r["tokens"], r["t_verify_ms"] * 1e-3)
    assert summary["iters"] == 160 and summary["tokens"] >= 160
    assert [r["K"] for r in recs[:4]] == [0, 0, 0, 0] and recs[4]["K"] == 3
    assert all(2 <= r["mean_unique"] <= 8 for r in recs)
    # a static-K run uses the same trace
    s3, recs3 = stack_driver.run(cfg, layers=4, iters=40, rho=0.5, layout="row", static_k=3)
    assert s3["K_histogram"] == {"3": 40}


def test_stack_driver_chained_and_decoder_modes_run_under_the_controller():
    """The decode loop in its two chained forms on a small stack: every iteration gets a K from the C controller, a
    positive verification time and 1 .. K+1 tokens; the recorded trace replays on the policy oracle."""
    import torch
    from oracle import cascade_oracle as co
    from paper_2506_20675_amd import stack_driver
    cfg = synth.TINY
    H, Hkv, dh = synth.attn_geometry(cfg)
    L = 3
    ctx = binding.MoeContext(cfg.d, cfg.ffn, cfg.n_experts, cfg.top_k, 0, synth.K_MAX + 1, 0, H, Hkv, dh)
    stack = stack_driver.build_stack(cfg, L, ctx, "tiled")
    pool = stack_driver.HiddenPool(cfg, L, 0.5, n_pool=2)
    gammas = [_dev(synth.norm_gamma_host(cfg, l)) for l in range(L)]
    attn = [_attn_dev(ctx, synth.attn_weights_host(cfg, l)) for l in range(L)]
    for kw in (dict(gammas=gammas), dict(attn=attn)):
        summary, recs = stack_driver.run(cfg, layers=L, iters=60, ctx=ctx, stack=stack, pool=pool, **kw)
        assert summary["chained"] and summary["attention_stub"] == ("attn" in kw)
        ref = co.Controller()
        for r in recs:
            assert ref.next_k() == r["K"] and r["t_verify_ms"] > 0 and 1 <= r["tokens"] <= r["K"] + 1
            ref.observe(r["K"], r["tokens"], r["t_verify_ms"] * 1e-3)
    ctx.close()


def test_concurrent_requests_share_one_pass_and_keep_their_own_controllers():
    """Two and four requests decoded together on a small stack: the in-flight tokens of all requests go through one
    pass (T = sum(K_r + 1) <= 16), and every request's K sequence replays on the policy oracle fed with that request's
    own tokens and the joint iteration time."""
    from oracle import cascade_oracle as co
    from paper_2506_20675_amd import stack_driver
    cfg = synth.TINY
    for R in (2, 4):
        summary, recs = stack_driver.run_concurrent(cfg, layers=3, iters=120, rho=0.5, requests=R, layout="row")
        k_max = 16 // R - 1
        assert summary["k_max"] == k_max and summary["tokens"] >= 120 * R
        assert all(r["T"] == sum(k + 1 for k in r["K"]) <= 16 and max(r["K"]) <= k_max for r in recs)
        for q in range(R):
            ref = co.Controller(co.Params(k_max=k_max, k_start=min(3, k_max)))
            for r in recs:
                assert ref.next_k() == r["K"][q]
                assert 1 <= r["tokens"][q] <= r["K"][q] + 1
                ref.observe(r["K"][q], r["tokens"][q], r["t_verify_ms"] * 1e-3)
        assert [r["K"] for r in recs[:4]] == [[0] * R] * 4          # every request starts with its baseline window
    s0, _ = stack_driver.run_concurrent(cfg, layers=3, iters=20, rho=0.5, requests=2, static_k=2, layout="row")
    assert s0["mean_T"] == 6.0 and s0["mean_K_per_request"] == [2.0, 2.0]


