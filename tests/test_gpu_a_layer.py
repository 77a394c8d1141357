"""GPU parity, part 1: what the benchmark times comes first.  Router and grouping, then the full-size layers
(Mixtral-shaped bf16 in the launch configuration of bench.py, the fine-grained shapes, Mixtral-shaped FP8), then the small
cases that walk every kernel variant (both layouts, packed and split fragments, fused and split-K down projection).
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from oracle import moe_oracle as orc
from paper_2506_20675_amd import binding, synth
from gpu_common import (_check_layer, _check_layer_fp8, _check_out, _dev, _run_layer, _tiled, _weights_dev)


def test_device_weight_fill_is_bit_identical_to_host():
    import torch
    key = synth.stream_key(2, 5, synth.T_W1)
    for n, start in ((4096, 0), (1000, 4), (7, 0), (3, 8), (1 << 20, 1 << 22), (65537 * 4 + 2, 12)):
        t = torch.zeros(n, dtype=torch.int16, device="cuda")
        synth.fill_normal_bf16_device(t, key, 0.02, start)
        torch.cuda.synchronize()
        host = synth.normal_bf16(key, 0.02, n, start)
        assert (t.cpu().numpy().view(np.uint16) == host).all(), (n, start)
    Wd = synth.layer_weights_device(synth.TINY, 3)
    Wh = synth.layer_weights_host(synth.TINY, 3)
    torch.cuda.synchronize()
    for name in Wh:
        assert (Wd[name].cpu().numpy().view(np.uint16) == Wh[name]).all(), name


@pytest.mark.parametrize("cfg", [synth.TINY, synth.OLMOE, synth.DEEPSEEK, synth.MIXTRAL], ids=lambda c: c.name)
def test_route_parity(cfg):
    import torch
    W = synth.layer_weights_host(cfg, 0) if cfg is not synth.MIXTRAL else None
    if W is None:      # router only: no need to build 2.8 GB of expert weights
        rw = synth.normal_bf16(synth.weight_key(cfg, 0, synth.T_ROUTER), synth.SIGMA_ROUTER,
                               cfg.n_experts * cfg.d).reshape(cfg.n_experts, cfg.d)
    else:
        rw = W["router_w"]
    rwd = _dev(rw)
    ctx = binding.MoeContext(cfg.d, cfg.ffn, cfg.n_experts, cfg.top_k, cfg.n_shared, 9)
    for it, (T, rho) in enumerate(((1, 0.5), (2, 0.0), (5, 0.9), (9, 0.0), (9, 0.5), (9, 0.9))):
        x = synth.hidden_host(cfg, 0, 100 + it, T, rho)
        ids = torch.zeros((T, cfg.top_k), dtype=torch.int32, device="cuda")
        gates = torch.zeros((T, cfg.top_k), dtype=torch.float32, device="cuda")
        uniq = torch.zeros((cfg.n_experts,), dtype=torch.int32, device="cuda")
        nu = torch.zeros((1,), dtype=torch.int32, device="cuda")
        ctx.moe_route(_dev(x), rwd, ids, gates, uniq, nu)
        torch.cuda.synchronize()
        rids, rgates, logits = orc.route(x, rw, cfg.top_k, "f32")
        srt = np.sort(logits, axis=1)[:, ::-1]
        assert (srt[:, cfg.top_k - 1] - srt[:, cfg.top_k]).min() > 1e-9
        np.testing.assert_array_equal(ids.cpu().numpy(), rids)
        assert np.abs(gates.cpu().numpy() - rgates).max() <= 1e-5
        u = orc.union(rids, cfg.n_experts)
        assert int(nu.item()) == u["n_unique"]
        np.testing.assert_array_equal(uniq.cpu().numpy(), u["unique"])
        assert cfg.top_k <= u["n_unique"] <= min(cfg.n_experts, T * cfg.top_k)
    ctx.close()


def test_route_tie_rule_and_topk_equals_E():
    import torch
    d, E = 64, 8
    ctx = binding.MoeContext(d, 64, E, E, 0, 4)
    x = np.random.default_rng(0).normal(size=(3, d)).astype(np.float32)
    ids = torch.zeros((3, E), dtype=torch.int32, device="cuda")
    gates = torch.zeros((3, E), dtype=torch.float32, device="cuda")
    ctx.moe_route(_dev(x), _dev(np.zeros((E, d), np.uint16)), ids, gates)      # all logits equal -> index order
    torch.cuda.synchronize()
    assert (ids.cpu().numpy() == np.arange(E)[None]).all()
    np.testing.assert_allclose(gates.cpu().numpy(), 1.0 / E, rtol=1e-6)
    rw = synth.f32_to_bf16_bits(np.random.default_rng(1).normal(0, 0.5, (E, d)).astype(np.float32))
    rw[5] = rw[2]
    ctx.moe_route(_dev(x), _dev(rw), ids, gates)
    torch.cuda.synchronize()
    rids, rgates, _ = orc.route(x, rw, E)
    np.testing.assert_array_equal(ids.cpu().numpy(), rids)
    ctx.close()


def test_group_parity_random_routings():
    import torch
    rng = np.random.default_rng(2)
    for E, k, T in ((8, 2, 9), (64, 8, 9), (64, 6, 1), (256, 16, 16), (5, 5, 3), (1, 1, 4)):
        ctx = binding.MoeContext(64, 64, E, k, 0, T)
        ids = np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
        outs = dict(unique_experts=torch.full((E,), -9, dtype=torch.int32, device="cuda"),
                    n_unique=torch.full((1,), -9, dtype=torch.int32, device="cuda"),
                    expert_count=torch.full((E,), -9, dtype=torch.int32, device="cuda"),
                    expert_offset=torch.full((E + 1,), -9, dtype=torch.int32, device="cuda"),
                    assign=torch.full((T * k,), -9, dtype=torch.int32, device="cuda"))
        ctx.moe_group(_dev(ids), **outs)
        torch.cuda.synchronize()
        u = orc.union(ids, E)
        assert int(outs["n_unique"].item()) == u["n_unique"]
        np.testing.assert_array_equal(outs["unique_experts"].cpu().numpy(), u["unique"])
        np.testing.assert_array_equal(outs["expert_count"].cpu().numpy(), u["count"])
        np.testing.assert_array_equal(outs["expert_offset"].cpu().numpy(), u["offset"])
        np.testing.assert_array_equal(outs["assign"].cpu().numpy(), u["assign"])
        ctx.close()


def test_layer_parity_mixtral_full_size():
    """Full Mixtral-8x7B-shaped layer in the launch configuration the benchmark times; device-generated
    weights (bit-identical to the host generator) against the oracle on the whole output."""
    import torch
    cfg = synth.MIXTRAL
    W = synth.layer_weights_host(cfg, 0)
    Wd = synth.layer_weights_device(cfg, 0)
    torch.cuda.synchronize()
    assert (Wd["w2"][3, 100:200].cpu().numpy().view(np.uint16) == W["w2"][3, 100:200]).all()
    ctx = binding.MoeContext(cfg.d, cfg.ffn, cfg.n_experts, cfg.top_k, 0, 9)
    for it, (T, rho) in enumerate(((1, 0.5), (9, 0.0), (4, 0.5), (8, 0.9))):
        x = synth.hidden_host(cfg, 0, 300 + it, T, rho)
        _check_layer((cfg.d, cfg.ffn, cfg.n_experts, cfg.top_k, 0), W, x, ctx, Wd)
    ctx.close()


@pytest.mark.parametrize("cfg", [synth.OLMOE, synth.DEEPSEEK], ids=lambda c: c.name)
def test_layer_parity_fine_grained_full_size(cfg):
    W = synth.layer_weights_host(cfg, 1)
    ctx = binding.MoeContext(cfg.d, cfg.ffn, cfg.n_experts, cfg.top_k, cfg.n_shared, 9)
    Wd = _weights_dev(W)
    for it, (T, rho) in enumerate(((1, 0.5), (4, 0.0), (9, 0.9))):
        x = synth.hidden_host(cfg, 1, 200 + it, T, rho)
        _check_layer((cfg.d, cfg.ffn, cfg.n_experts, cfg.top_k, cfg.n_shared), W, x, ctx, Wd)
    ctx.close()


def test_fp8_layer_parity_mixtral_full_size():
    """Full Mixtral-8x7B-shaped FP8 layer in the launch configuration the benchmark times, device-generated codes
    (bit-identical to the host generator), whole output against the oracle."""
    import torch
    cfg = synth.MIXTRAL
    W = synth.layer_weights_fp8_host(cfg, 0)
    Wd = synth.layer_weights_fp8_device(cfg, 0)
    torch.cuda.synchronize()
    assert (Wd["q2"][3, 100:200].cpu().numpy() == W["q2"][3, 100:200]).all()
    assert (Wd["s1"].cpu().numpy() == W["s1"]).all()
    ctx = binding.MoeContext(cfg.d, cfg.ffn, cfg.n_experts, cfg.top_k, 0, 9)
    for it, (T, rho) in enumerate(((1, 0.5), (5, 0.0), (9, 0.5))):   # T = 9: split fragments, 8 row tiles per wave
        x = synth.hidden_host(cfg, 0, 500 + it, T, rho)
        _check_layer_fp8(ctx, W, Wd, x, cfg.top_k, 0, row_major=T < 9)
    ctx.close()



@pytest.mark.parametrize("T", [1, 2, 3, 5, 9])
def test_layer_parity_tiny(T):
    cfg = synth.TINY
    W = synth.layer_weights_host(cfg, 0)
    x = synth.hidden_host(cfg, 0, T, T, 0.5)
    _check_layer((cfg.d, cfg.ffn, cfg.n_experts, cfg.top_k, 0), W, x)


@pytest.mark.parametrize("shape", [
    # d, ffn, E, top_k, n_shared, T : ragged tile counts, odd k-step counts, shared experts, top_k == E, T = 16
    (96, 160, 5, 3, 1, 7), (32, 32, 1, 1, 0, 1), (64, 96, 4, 4, 2, 16), (160, 224, 12, 2, 0, 9), (1056, 544, 6, 2, 1, 4),
])
def test_layer_parity_ragged_shapes(shape):
    d, ffn, E, k, ns, T = shape
    rng = np.random.default_rng(sum(shape))
    bf = lambda a: synth.f32_to_bf16_bits(a.astype(np.float32))
    W = dict(router_w=bf(rng.normal(0, 0.3, (E, d))), w1=bf(rng.normal(0, 0.1, (E, ffn, d))),
             w3=bf(rng.normal(0, 0.1, (E, ffn, d))), w2=bf(rng.normal(0, 0.1, (E, d, ffn))))
    if ns:
        W.update(sw1=bf(rng.normal(0, 0.1, (ns, ffn, d))), sw3=bf(rng.normal(0, 0.1, (ns, ffn, d))),
                 sw2=bf(rng.normal(0, 0.1, (ns, d, ffn))))
    x = rng.normal(size=(T, d)).astype(np.float32)
    _check_layer((d, ffn, E, k, ns), W, x)


@pytest.mark.parametrize("shape", [(16384, 64, 4, 2, 1, 3), (16384, 32, 64, 8, 0, 2)], ids=["router-per-token", "wide-router"])
def test_layer_parity_widest_rows(shape):
    """d = 16384: 32 chunks of 512 per router row, 512 k-steps per gate/up wave, the largest row the chained calls and
    the slab sum take; both router kinds, both layouts."""
    d, ffn, E, k, ns, T = shape
    rng = np.random.default_rng(sum(shape))
    bf = lambda a: synth.f32_to_bf16_bits(a.astype(np.float32))
    W = dict(router_w=bf(rng.normal(0, 0.05, (E, d))), w1=bf(rng.normal(0, 0.0125, (E, ffn, d))),
             w3=bf(rng.normal(0, 0.0125, (E, ffn, d))), w2=bf(rng.normal(0, 0.1, (E, d, ffn))))
    if ns:
        W.update(sw1=bf(rng.normal(0, 0.0125, (ns, ffn, d))), sw3=bf(rng.normal(0, 0.0125, (ns, ffn, d))),
                 sw2=bf(rng.normal(0, 0.1, (ns, d, ffn))))
    x = rng.normal(size=(T, d)).astype(np.float32)
    _check_layer((d, ffn, E, k, ns), W, x)


def _small_layer(d, ffn, E, k, ns, seed):
    rng = np.random.default_rng(seed)
    bf = lambda a: synth.f32_to_bf16_bits(a.astype(np.float32))
    W = dict(router_w=bf(rng.normal(0, 0.3, (E, d))), w1=bf(rng.normal(0, 0.1, (E, ffn, d))),
             w3=bf(rng.normal(0, 0.1, (E, ffn, d))), w2=bf(rng.normal(0, 0.1, (E, d, ffn))))
    if ns:
        W.update(sw1=bf(rng.normal(0, 0.1, (ns, ffn, d))), sw3=bf(rng.normal(0, 0.1, (ns, ffn, d))),
                 sw2=bf(rng.normal(0, 0.1, (ns, d, ffn))))
    return W, rng


@pytest.mark.parametrize("T", [1, 5, 9, 16])
@pytest.mark.parametrize("fused", [False, True], ids=["splitk", "fused"])
def test_layer_parity_tiny_both_down_paths(T, fused):
    """The tiny layer with the down projection forced onto the split-K kernel + combine_kernel and onto the fused down
    + combine kernel (the two plans the benchmark's Mixtral-shaped layer runs at many and at few tokens in flight, here
    in a sub-second case), for packed (T <= 8; compact H fragments on the fused path) and split (T > 8) fragments.  The
    launch plan must say which of the two the automatic choice is."""
    cfg = synth.TINY
    W = synth.layer_weights_host(cfg, 0)
    x = synth.hidden_host(cfg, 0, 60 + T, T, 0.5)
    plan = binding.moe_plan_query(cfg.d, cfg.ffn, cfg.n_experts, cfg.top_k, 0, 16, T)
    assert (plan["dn_fused_chunks"] > 0) == (T <= 5) and plan["packed_fragments"] == (T <= 8)
    ctx = binding.MoeContext(cfg.d, cfg.ffn, cfg.n_experts, cfg.top_k, 0, 16)
    ctx.moe_ctx_tune(fused_down=1 if fused else 0)
    Wd = _weights_dev(W)
    _check_layer((cfg.d, cfg.ffn, cfg.n_experts, cfg.top_k, 0), W, x, ctx, Wd)
    if not fused:                      # the benchmark's instantiation (4 row tiles per wave; this small ffn caps the k-chunks at 2)
        ctx.moe_ctx_tune(dn_tiles=4, dn_split_k=4, fused_down=0)
        _check_layer((cfg.d, cfg.ffn, cfg.n_experts, cfg.top_k, 0), W, x, ctx, Wd)
    ctx.close()


@pytest.mark.parametrize("T", [1, 9])
def test_layer_parity_two_shared_experts(T):
    """A shared-plus-routed layer in miniature (two always-on experts beside 16 routed, top-6), both down paths."""
    d, ffn, E, k, ns = 256, 352, 16, 6, 2
    W, rng = _small_layer(d, ffn, E, k, ns, 4242)
    x = rng.normal(size=(T, d)).astype(np.float32)
    for fused in (True, False):
        ctx = binding.MoeContext(d, ffn, E, k, ns, 9)
        ctx.moe_ctx_tune(fused_down=1 if fused else 0)
        _check_layer((d, ffn, E, k, ns), W, x, ctx, _weights_dev(W))
        ctx.close()


def test_layer_parity_mid_size_takes_the_benchmarked_plans_by_itself():
    """A layer of 8 experts of 2048 x 8192 under the automatic plan, in a sub-second test: with 6 and 9 tokens in flight
    it picks the split-K down projection with 4 row tiles per wave and a slab sum, as the Mixtral-shaped layer does
    (T = 6: packed fragments, T = 9: split fragments); with 2 tokens the fused down + combine launch with compact H
    fragments."""
    d, ffn, E, k = 2048, 8192, 8, 2
    W, rng = _small_layer(d, ffn, E, k, 0, 77)
    ctx = binding.MoeContext(d, ffn, E, k, 0, 9)
    Wd = _weights_dev(W)
    for T in (6, 9, 2):
        plan = binding.moe_plan_query(d, ffn, E, k, 0, 9, T)
        if T > 5:
            assert plan["dn_fused_chunks"] == 0 and plan["dn_tiles"] == 4 and plan["dn_split_k"] >= 2, plan
        else:
            assert plan["dn_fused_chunks"] > 0, plan
        x = rng.normal(size=(T, d)).astype(np.float32)
        _check_layer((d, ffn, E, k, 0), W, x, ctx, Wd)
    ctx.close()


def test_pack_weights_layout_is_as_documented():
    """Block (i, s) of the tiled matrix is rows 16i..16i+15 x columns 32s..32s+31; 16-byte unit l = r + 16 g
    holds row 16i + r, columns 32s + 8g .. + 7."""
    import torch
    d, ffn, E = 64, 96, 3
    rng = np.random.default_rng(7)
    W = {n: rng.integers(0, 65536, size=shp, dtype=np.uint16) for n, shp in
         (("router_w", (E, d)), ("w1", (E, ffn, d)), ("w3", (E, ffn, d)), ("w2", (E, d, ffn)))}
    ctx = binding.MoeContext(d, ffn, E, 2, 0, 4)
    Wd = _weights_dev(W)
    packed = ctx.moe_pack_weights(ctx.weights(Wd))
    torch.cuda.synchronize()
    assert packed.c.layout == 1
    for idx, name, rows, K in ((1, "w1", E * ffn, d), (2, "w3", E * ffn, d), (3, "w2", E * d, ffn)):
        got = packed.tensors[idx].cpu().numpy().view(np.uint16).reshape(-1)
        src = W[name].reshape(rows, K)
        want = src.reshape(rows // 16, 16, K // 32, 4, 8).transpose(0, 2, 3, 1, 4).reshape(-1)   # [i][s][g][r][8]
        np.testing.assert_array_equal(got, want)
    ctx.close()


def test_batch_invariance_and_determinism_on_gpu():
    """Row t of a T-token step equals the T = 1 step on that token (verification == decoding), and
    reruns are bit-identical (fixed reduction order, no atomics)."""
    cfg = synth.TINY
    W = synth.layer_weights_host(cfg, 2)
    Wd = _weights_dev(W)
    ctx = binding.MoeContext(cfg.d, cfg.ffn, cfg.n_experts, cfg.top_k, 0, 9)
    x = synth.hidden_host(cfg, 2, 5, 9, 0.5)
    for tiled in (False, True):
        out9, ids9, *_ = _run_layer(ctx, Wd, x, tiled)
        again, *_ = _run_layer(ctx, Wd, x, tiled)
        np.testing.assert_array_equal(out9, again)
        for t in (0, 4, 8):
            o1, i1, *_ = _run_layer(ctx, Wd, x[t:t + 1], tiled)
            np.testing.assert_array_equal(i1[0], ids9[t])
            # T = 1 may use another split-K factor than T = 9, hence a tolerance and not bit equality
            np.testing.assert_allclose(o1[0], out9[t], rtol=0, atol=2e-6 * np.abs(out9).max())
    ctx.close()


@pytest.mark.parametrize("T", [1, 4, 9])
@pytest.mark.parametrize("wide", [False, True], ids=["router-per-token", "wide-router"])
def test_stack_matches_per_layer_oracle(T, wide):
    """moe_verify_stack on independent per-layer inputs: routing runs ahead for batches of 16 layers (19 layers here:
    a full batch and a ragged one) and, with the split-K down projection, the slab sum of layer l rides in the
    gate/up launch of layer l + 1 (a launch of its own only at a batch boundary and after the last layer); with the
    fused down projection every layer writes its own output.  Automatic plan and both plans forced, both layouts, both router kinds (8 experts: one
    workgroup per token; 40 experts top-4 with a shared expert: logits + top-k kernels); every layer against the
    oracle, and the stack call against single-layer calls, bit for bit."""
    import torch
    L = 19
    if wide:
        d, ffn, E, k, ns = 128, 96, 40, 4, 1
        rng = np.random.default_rng(77)
        bf = lambda a: synth.f32_to_bf16_bits(a.astype(np.float32))
        Ws = []
        for l in range(L):
            Ws.append(dict(router_w=bf(rng.normal(0, 0.3, (E, d))), w1=bf(rng.normal(0, 0.1, (E, ffn, d))),
                           w3=bf(rng.normal(0, 0.1, (E, ffn, d))), w2=bf(rng.normal(0, 0.1, (E, d, ffn))),
                           sw1=bf(rng.normal(0, 0.1, (ns, ffn, d))), sw3=bf(rng.normal(0, 0.1, (ns, ffn, d))),
                           sw2=bf(rng.normal(0, 0.1, (ns, d, ffn)))))
        x = rng.normal(size=(L, T, d)).astype(np.float32)
    else:
        cfg = synth.TINY
        d, ffn, E, k, ns = cfg.d, cfg.ffn, cfg.n_experts, cfg.top_k, 0
        Ws = [synth.layer_weights_host(cfg, 10 + l) for l in range(L)]
        x = np.stack([synth.hidden_host(cfg, 10 + l, 0, T, 0.5) for l in range(L)])
    Wds = [_weights_dev(W) for W in Ws]
    refs = [(orc.layer(x[l], Ws[l], k, ns, "f32"), orc.layer(x[l], Ws[l], k, ns, "f64")) for l in range(L)]
    for l in range(L):
        _, _, logits = orc.route(x[l], Ws[l]["router_w"], k, "f64")
        srt = np.sort(logits, axis=1)[:, ::-1]
        assert (srt[:, k - 1] - srt[:, k]).min() > 1e-9, "seed produces a routing near-tie; pick another"
    for fused in (-1, 0, 1):
        for tiled in (False, True):
            ctx = binding.MoeContext(d, ffn, E, k, ns, 9)
            ctx.moe_ctx_tune(fused_down=fused)
            layers = [_tiled(ctx, w) if tiled else ctx.weights(w) for w in Wds]
            out = torch.full((L, T, d), float("nan"), dtype=torch.float32, device="cuda")
            nu = torch.zeros((L,), dtype=torch.int32, device="cuda")
            for rep in range(2):          # twice: the second pass meets the first one's slabs and tables
                ctx.moe_verify_stack(layers, _dev(x), out, nu)
            torch.cuda.synchronize()
            for l in range(L):
                (ref32, rids, _), (ref64, _, _) = refs[l]
                _check_out(out[l].cpu().numpy(), ref32, ref64)
                assert int(nu[l].item()) == orc.union(rids, E)["n_unique"]
            # under one down-projection plan the stack call gives what L single-layer calls give, bit for bit (left
            # to itself it may pick another plan than a single call: its slab sums cost no launch)
            for l in range(L if fused >= 0 else 0):
                one = torch.zeros((T, d), dtype=torch.float32, device="cuda")
                ctx.moe_verify_layer(layers[l], _dev(x[l]), one)
                torch.cuda.synchronize()
                np.testing.assert_array_equal(one.cpu().numpy(), out[l].cpu().numpy())
            ctx.close()


def test_stack_with_mixed_layer_formats():
    """Every layer of a stack brings its own weight struct: bf16 and FP8, row-major and tiled, mixed in one call.  Each
    layer against the oracle of its own format, and against a single-layer call bit for bit."""
    import torch
    cfg = synth.TINY
    T, L = 5, 8
    ctx = binding.MoeContext(cfg.d, cfg.ffn, cfg.n_experts, cfg.top_k, 0, 9)
    Ws, layers, keep = [], [], []
    for l in range(L):
        fp8, tiled = bool(l & 1), bool(l & 2)
        W = synth.layer_weights_fp8_host(cfg, 30 + l) if fp8 else synth.layer_weights_host(cfg, 30 + l)
        Wd = _weights_dev(W)
        keep.append(Wd)
        Ws.append((W, fp8))
        layers.append(_tiled(ctx, Wd) if tiled else ctx.weights(Wd))
    x = np.stack([synth.hidden_host(cfg, 30 + l, 1, T, 0.5) for l in range(L)])
    out = torch.full((L, T, cfg.d), float("nan"), dtype=torch.float32, device="cuda")
    nu = torch.zeros((L,), dtype=torch.int32, device="cuda")
    ctx.moe_ctx_tune(fused_down=0)                # split-K: the slab sums ride in the next layer's gate/up launch
    ctx.moe_verify_stack(layers, _dev(x), out, nu)
    torch.cuda.synchronize()
    for l, (W, fp8) in enumerate(Ws):
        lay = orc.layer_fp8 if fp8 else orc.layer
        ref32, rids, _ = lay(x[l], W, cfg.top_k, 0, "f32")
        ref64, _, _ = lay(x[l], W, cfg.top_k, 0, "f64")
        _check_out(out[l].cpu().numpy(), ref32, ref64)
        assert int(nu[l].item()) == orc.union(rids, cfg.n_experts)["n_unique"]
        one = torch.zeros((T, cfg.d), dtype=torch.float32, device="cuda")
        ctx.moe_verify_layer(layers[l], _dev(x[l]), one)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(one.cpu().numpy(), out[l].cpu().numpy())
    ctx.close()


def test_argument_errors_are_reported_not_launched():
    import torch
    ctx = binding.MoeContext(64, 64, 4, 2, 0, 4)
    x = torch.zeros((5, 64), dtype=torch.float32, device="cuda")
    rw = torch.zeros((4, 64), dtype=torch.int16, device="cuda")
    with pytest.raises(binding.MoeError) as e:
        ctx.moe_route(x, rw)                       # T = 5 > max_tokens
    assert e.value.status == -1
    with pytest.raises(ValueError):
        ctx.moe_route(x[:2, :32].contiguous(), rw)
    with pytest.raises(binding.MoeError) as e:       # an empty batch (T = 0) is refused, nothing is launched
        ctx.moe_verify_layer(ctx.weights({"router_w": rw, "w1": torch.zeros((4, 64, 64), dtype=torch.int16, device="cuda"),
                                          "w3": torch.zeros((4, 64, 64), dtype=torch.int16, device="cuda"),
                                          "w2": torch.zeros((4, 64, 64), dtype=torch.int16, device="cuda")}),
                             x[:0].contiguous(), torch.zeros((0, 64), device="cuda"))
    assert e.value.status == -1
    # the tuning aid takes 0 / 1 / 2 / 4 tiles, a power-of-two split up to 16, and -1 / 0 / 1 for the fused down kernel
    for bad in ((3, 0, 0, -1), (0, 8, 0, -1), (0, 0, 3, -1), (0, 0, 32, -1), (0, 0, 0, 2), (0, 0, 0, -2)):
        with pytest.raises(binding.MoeError) as e:
            ctx.moe_ctx_tune(*bad)
        assert e.value.status == -1
    ctx.moe_ctx_tune(1, 4, 16, 0)                   # accepted; the split is clamped to what this shape allows
    ctx.moe_ctx_tune()                              # back to automatic
    # weights built for another geometry are refused by the binding before the library sees a pointer
    other = binding.MoeContext(64, 128, 4, 2, 0, 4)
    Wd = {n: torch.zeros(shp, dtype=torch.int16, device="cuda") for n, shp in
          (("router_w", (4, 64)), ("w1", (4, 128, 64)), ("w3", (4, 128, 64)), ("w2", (4, 64, 128)))}
    with pytest.raises(ValueError):
        ctx.moe_verify_layer(other.weights(Wd), x[:2].contiguous(), torch.zeros((2, 64), device="cuda"))
    # a stream that lives on this device is accepted explicitly
    st = torch.cuda.Stream()
    ok = binding.MoeContext(64, 128, 4, 2, 0, 4)
    ok.moe_route(x[:2].contiguous(), rw, stream=st)
    st.synchronize()
    ok.close()
    other.close()
    ctx.close()


