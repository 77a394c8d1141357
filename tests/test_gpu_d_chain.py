"""GPU parity, part 4: chained stack (pre-norm residual MoE blocks, each feeding the next) and decoder blocks with
the attention stub.
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from oracle import moe_oracle as orc
from paper_2506_20675_amd import binding, synth
from gpu_common import (_check_layer, _check_out, _dev, _run_layer, _tiled, _weights_dev)


from gpu_common import _attn_dev, _chain_block_check, _decoder_block_check


@pytest.mark.parametrize("T", [1, 5, 9])
def test_chained_block_parity_tiny(T):
    cfg = synth.TINY
    W = synth.layer_weights_host(cfg, 5)
    gam = synth.norm_gamma_host(cfg, 5)
    ctx = binding.MoeContext(cfg.d, cfg.ffn, cfg.n_experts, cfg.top_k, 0, 9)
    Wd = _weights_dev(W)
    x = (synth.hidden_host(cfg, 5, 70 + T, T, 0.5) * np.float32(3.0)).astype(np.float32)
    for lw in (ctx.weights(Wd), _tiled(ctx, Wd)):
        _chain_block_check(ctx, lw, W, gam, _dev(gam), x, cfg.top_k, 0)
    ctx.close()


@pytest.mark.parametrize("cfg,weights", [(synth.DEEPSEEK, "bf16"), (synth.QWEN15, "fp8"), (synth.OLMOE, "fp8")],
                         ids=lambda v: v if isinstance(v, str) else v.name)
def test_chained_block_parity_full_size_shapes(cfg, weights):
    W = synth.layer_weights_fp8_host(cfg, 2) if weights == "fp8" else synth.layer_weights_host(cfg, 2)
    gam = synth.norm_gamma_host(cfg, 2)
    ctx = binding.MoeContext(cfg.d, cfg.ffn, cfg.n_experts, cfg.top_k, cfg.n_shared, 9, gate_mode=cfg.gate_mode)
    Wd = _weights_dev(W)
    lw = _tiled(ctx, Wd)
    for it, T in enumerate((1, 6)):
        x = (synth.hidden_host(cfg, 2, 700 + it, T, 0.5) * np.float32(0.25)).astype(np.float32)
        _chain_block_check(ctx, lw, W, gam, _dev(gam), x, cfg.top_k, cfg.n_shared)
    ctx.close()


def test_chained_stack_teacher_forced_and_free_running():
    """Four blocks: every block reproduces the oracle's next stream from the oracle's current one (teacher-forced), and
    the free-running GPU chain ends where the oracle's chain ends (the routing agrees at every block on this seed)."""
    import torch
    cfg = synth.TINY
    L, T = 4, 5
    Ws = [synth.layer_weights_host(cfg, 30 + l) for l in range(L)]
    gs = [synth.norm_gamma_host(cfg, 30 + l) for l in range(L)]
    ctx = binding.MoeContext(cfg.d, cfg.ffn, cfg.n_experts, cfg.top_k, 0, 9)
    Wds = [_weights_dev(W) for W in Ws]
    lws = [ctx.moe_pack_weights(ctx.weights(w)) for w in Wds]
    gds = [_dev(g) for g in gs]
    x0 = synth.hidden_host(cfg, 30, 0, T, 0.5)
    xL, trace, ids = orc.chained_stack(x0, Ws, gs, cfg.top_k, 0, 1e-5, "f64")
    for l in range(L):
        nxt = _chain_block_check(ctx, lws[l], Ws[l], gs[l], gds[l], trace[l], cfg.top_k, 0)
        np.testing.assert_array_equal(nxt, trace[l + 1] if l + 1 < L else xL)
    out = torch.zeros((T, cfg.d), dtype=torch.float32, device="cuda")
    tr = torch.zeros((L, T, cfg.d), dtype=torch.float32, device="cuda")
    nu = torch.zeros((L,), dtype=torch.int32, device="cuda")
    ctx.moe_chained_stack(lws, gds, _dev(x0), out, 1e-5, tr, nu)
    torch.cuda.synchronize()
    for l in range(L):
        assert int(nu[l].item()) == orc.union(ids[l], cfg.n_experts)["n_unique"]
        e = tr[l].cpu().numpy().astype(np.float64) - trace[l]
        assert np.sqrt((e ** 2).sum() / (trace[l].astype(np.float64) ** 2).sum()) <= 1e-4
    e = out.cpu().numpy().astype(np.float64) - xL
    assert np.sqrt((e ** 2).sum() / (xL.astype(np.float64) ** 2).sum()) <= 1e-4
    # without a trace, and in place, the chain gives the same bits
    out2 = _dev(x0).clone()
    ctx.moe_chained_stack(lws, gds, out2, out2, 1e-5)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(out2.cpu().numpy(), out.cpu().numpy())
    ctx.close()


@pytest.mark.parametrize("d", [256, 16384], ids=["pass-in-the-logits-launch", "pass-in-its-own-launch"])
@pytest.mark.parametrize("fused", [1, 0], ids=["fused-down", "split-k-down"])
def test_chained_stack_with_a_wide_router(d, fused):
    """Three blocks behind a 40- or 32-expert router (logits + top-k kernels) with a shared expert: from the second block on
    the slab sum + residual + RMSNorm pass has a pending MoE term to add — slabs of the split-K down projection, or the
    fused kernel's summed term — and runs inside the logits launch (d <= 8192) or in front of it (d = 16384, the
    largest d the chained calls take).  Free-running chain against the oracle's chain, T = 1 and 5."""
    import torch
    E, k, ns, ffn, L = (40 if d == 256 else 32), 4, 1, 64, 3
    rng = np.random.default_rng(1000 + d + fused)
    bf = lambda a: synth.f32_to_bf16_bits(a.astype(np.float32))
    sw = 0.1 * (256 / d) ** 0.5                          # keeps the MoE term O(1) at both widths
    Ws = [dict(router_w=bf(rng.normal(0, 0.3, (E, d))), w1=bf(rng.normal(0, sw, (E, ffn, d))),
               w3=bf(rng.normal(0, sw, (E, ffn, d))), w2=bf(rng.normal(0, 0.1, (E, d, ffn))),
               sw1=bf(rng.normal(0, sw, (ns, ffn, d))), sw3=bf(rng.normal(0, sw, (ns, ffn, d))),
               sw2=bf(rng.normal(0, 0.1, (ns, d, ffn)))) for _ in range(L)]
    gs = [bf(1 + 0.1 * rng.normal(size=d)) for _ in range(L)]
    ctx = binding.MoeContext(d, ffn, E, k, ns, 9)
    ctx.moe_ctx_tune(fused_down=fused)
    Wds = [_weights_dev(W) for W in Ws]
    lws = [ctx.moe_pack_weights(ctx.weights(w)) for w in Wds]
    gds = [_dev(g) for g in gs]
    for T in (1, 5):
        x0 = rng.normal(size=(T, d)).astype(np.float32)
        xL, trace, ids = orc.chained_stack(x0, Ws, gs, k, ns, 1e-5, "f64")
        for l in range(L):                                # the routing must not hinge on the last bits of the stream
            n = orc.rmsnorm(trace[l].astype(np.float32), gs[l], 1e-5, "f64").astype(np.float32)
            _, _, logits = orc.route(n, Ws[l]["router_w"], k, "f64")
            srt = np.sort(logits, axis=1)[:, ::-1]
            assert (srt[:, k - 1] - srt[:, k]).min() > 1e-4, "seed produces a thin routing margin; pick another"
        out = torch.zeros((T, d), dtype=torch.float32, device="cuda")
        tr = torch.zeros((L, T, d), dtype=torch.float32, device="cuda")
        nu = torch.zeros((L,), dtype=torch.int32, device="cuda")
        ctx.moe_chained_stack(lws, gds, _dev(x0), out, 1e-5, tr, nu)
        torch.cuda.synchronize()
        for l in range(L):
            assert int(nu[l].item()) == orc.union(ids[l], E)["n_unique"]
            e = tr[l].cpu().numpy().astype(np.float64) - trace[l]
            assert np.sqrt((e ** 2).sum() / (trace[l].astype(np.float64) ** 2).sum()) <= 1e-4
        e = out.cpu().numpy().astype(np.float64) - xL
        assert np.sqrt((e ** 2).sum() / (xL.astype(np.float64) ** 2).sum()) <= 1e-4
    ctx.close()


@pytest.mark.parametrize("T", [1, 4, 9])
def test_decoder_block_parity_tiny(T):
    cfg = synth.TINY
    H, Hkv, dh = synth.attn_geometry(cfg)
    W = synth.layer_weights_host(cfg, 8)
    A = synth.attn_weights_host(cfg, 8)
    ctx = binding.MoeContext(cfg.d, cfg.ffn, cfg.n_experts, cfg.top_k, 0, 9, n_heads=H, n_kv_heads=Hkv, head_dim=dh)
    Wd = _weights_dev(W)
    x = (synth.hidden_host(cfg, 8, 80 + T, T, 0.5) * np.float32(2.0)).astype(np.float32)
    _decoder_block_check(ctx, _tiled(ctx, Wd), _attn_dev(ctx, A), W, A, x, cfg.top_k, 0)
    ctx.close()


def test_decoder_block_parity_other_geometries():
    """Several kv heads, head dims 32 and 96, T = 16, shared experts, FP8 experts."""
    rng = np.random.default_rng(91)
    bf = lambda a: synth.f32_to_bf16_bits(a.astype(np.float32))
    for (d, ffn, E, k, ns, T, H, Hkv, dh, fp8) in ((192, 128, 6, 2, 1, 16, 6, 3, 32, False), (384, 192, 5, 3, 0, 7, 4, 2, 96, True)):
        A = dict(wqkv=bf(rng.normal(0, 0.08, ((H + 2 * Hkv) * dh, d))), wo=bf(rng.normal(0, 0.08, (d, H * dh))),
                 gamma_attn=bf(1 + 0.1 * rng.normal(size=d)), gamma_moe=bf(1 + 0.1 * rng.normal(size=d)),
                 n_heads=H, n_kv_heads=Hkv, head_dim=dh)
        if fp8:
            finite = np.array([c for c in range(256) if c not in (0x7F, 0xFF)], dtype=np.uint8)
            W = dict(router_w=bf(rng.normal(0, 0.3, (E, d))))
            for q, s, shp in (("q1", "s1", (E, ffn, d)), ("q3", "s3", (E, ffn, d)), ("q2", "s2", (E, d, ffn))):
                W[q] = rng.choice(finite, shp)
                W[s] = (1e-4 * 10.0 ** rng.uniform(-0.5, 0.5, shp[:2])).astype(np.float32)
        else:
            W = dict(router_w=bf(rng.normal(0, 0.3, (E, d))), w1=bf(rng.normal(0, 0.1, (E, ffn, d))),
                     w3=bf(rng.normal(0, 0.1, (E, ffn, d))), w2=bf(rng.normal(0, 0.1, (E, d, ffn))),
                     sw1=bf(rng.normal(0, 0.1, (ns, ffn, d))), sw3=bf(rng.normal(0, 0.1, (ns, ffn, d))),
                     sw2=bf(rng.normal(0, 0.1, (ns, d, ffn))))
        x = rng.normal(size=(T, d)).astype(np.float32)
        ctx = binding.MoeContext(d, ffn, E, k, ns, 16, n_heads=H, n_kv_heads=Hkv, head_dim=dh)
        Wd = _weights_dev(W)
        _decoder_block_check(ctx, _tiled(ctx, Wd), _attn_dev(ctx, A), W, A, x, k, ns)
        ctx.close()


def test_decoder_stack_teacher_forced_and_free_running():
    import torch
    cfg = synth.TINY
    H, Hkv, dh = synth.attn_geometry(cfg)
    L, T = 3, 4
    Ws = [synth.layer_weights_host(cfg, 50 + l) for l in range(L)]
    As = [synth.attn_weights_host(cfg, 50 + l) for l in range(L)]
    ctx = binding.MoeContext(cfg.d, cfg.ffn, cfg.n_experts, cfg.top_k, 0, 9, n_heads=H, n_kv_heads=Hkv, head_dim=dh)
    Wds = [_weights_dev(W) for W in Ws]
    lws = [ctx.moe_pack_weights(ctx.weights(w)) for w in Wds]
    aws = [_attn_dev(ctx, A) for A in As]
    x0 = synth.hidden_host(cfg, 50, 0, T, 0.5)
    xL, trace, ids = orc.decoder_stack(x0, As, Ws, cfg.top_k, 0, 1e-5, "f64")
    for l in range(L):
        nxt = _decoder_block_check(ctx, lws[l], aws[l], Ws[l], As[l], trace[l], cfg.top_k, 0)
        np.testing.assert_array_equal(nxt, trace[l + 1] if l + 1 < L else xL)
    out = torch.zeros((T, cfg.d), dtype=torch.float32, device="cuda")
    tr = torch.zeros((L, T, cfg.d), dtype=torch.float32, device="cuda")
    nu = torch.zeros((L,), dtype=torch.int32, device="cuda")
    ctx.moe_decoder_stack(lws, aws, _dev(x0), out, 1e-5, tr, nu)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(tr[0].cpu().numpy(), x0)
    for l in range(L):
        assert int(nu[l].item()) == orc.union(ids[l], cfg.n_experts)["n_unique"]
        e = tr[l].cpu().numpy().astype(np.float64) - trace[l]
        assert np.sqrt((e ** 2).sum() / (trace[l].astype(np.float64) ** 2).sum()) <= 1e-4
    e = out.cpu().numpy().astype(np.float64) - xL
    assert np.sqrt((e ** 2).sum() / (xL.astype(np.float64) ** 2).sum()) <= 1e-4
    out2 = _dev(x0).clone()
    ctx.moe_decoder_stack(lws, aws, out2, out2, 1e-5)                # no trace, in place: same bits
    torch.cuda.synchronize()
    np.testing.assert_array_equal(out2.cpu().numpy(), out.cpu().numpy())
    plain = binding.MoeContext(cfg.d, cfg.ffn, cfg.n_experts, cfg.top_k, 0, 9)
    with pytest.raises(binding.MoeError) as err:                     # a context without the attention geometry refuses
        plain.moe_decoder_stack(lws[:1], aws[:1], out2, out2)
    assert err.value.status == -1
    plain.close()
    ctx.close()


