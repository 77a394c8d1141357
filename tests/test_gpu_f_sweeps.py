"""GPU parity, part 6: HIP-graph replay, degenerate routings, seeded random sweeps, workspace leftovers, measurement aids.
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from oracle import moe_oracle as orc
from paper_2506_20675_amd import binding, synth
from gpu_common import (_check_layer, _check_out, _dev, _run_layer, _tiled, _weights_dev)


from gpu_common import _attn_dev, _chain_block_check, _decoder_block_check


def test_layer_and_chain_replay_from_a_hip_graph():
    """The device calls only enqueue kernels (no allocation, no host copies, no memset nodes), so a caller may capture
    them in a HIP graph.  Replays — with eager work and synchronisation between them — must give the eager bits."""
    import torch
    cfg = synth.TINY
    T, L = 3, 2
    ctx = binding.MoeContext(cfg.d, cfg.ffn, cfg.n_experts, cfg.top_k, 0, 9)
    Wds = [_weights_dev(synth.layer_weights_host(cfg, 40 + l)) for l in range(L)]
    lws = [ctx.moe_pack_weights(ctx.weights(w)) for w in Wds]
    gds = [_dev(synth.norm_gamma_host(cfg, 40 + l)) for l in range(L)]
    xs = [_dev(synth.hidden_host(cfg, 40, it, T, 0.5)) for it in range(3)]
    x_static = xs[0].clone()
    out_layer = torch.zeros((T, cfg.d), dtype=torch.float32, device="cuda")
    out_chain = torch.zeros((T, cfg.d), dtype=torch.float32, device="cuda")
    eager = []
    for x in xs:
        a = torch.zeros_like(out_layer)
        b = torch.zeros_like(out_chain)
        ctx.moe_verify_layer(lws[0], x, a)
        ctx.moe_chained_stack(lws, gds, x, b)
        torch.cuda.synchronize()
        eager.append((a.clone(), b.clone()))
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        ctx.moe_verify_layer(lws[0], x_static, out_layer)          # warm-up on the capture stream
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            ctx.moe_verify_layer(lws[0], x_static, out_layer)
            ctx.moe_chained_stack(lws, gds, x_static, out_chain)
    torch.cuda.synchronize()
    for rep in range(2):
        for x, (a, b) in zip(xs, eager):
            x_static.copy_(x)
            out_layer.fill_(-1.0)
            out_chain.fill_(-1.0)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(out_layer, a) and torch.equal(out_chain, b)
    ctx.close()


def test_degenerate_routings_identical_tokens_and_largest_supported_shape():
    """All in-flight tokens identical (the limit of perfect expert affinity): the union is one token's picks, every
    pick is shared by all tokens, all rows of the output agree.  And the largest routing the library accepts
    (256 experts, top-16, 16 tokens: up to 256 live slots) against the oracle."""
    cfg = synth.TINY
    W = synth.layer_weights_host(cfg, 6)
    x1 = synth.hidden_host(cfg, 6, 0, 1, 0.5)
    x = np.repeat(x1, 9, axis=0)
    ctx = binding.MoeContext(cfg.d, cfg.ffn, cfg.n_experts, cfg.top_k, 0, 9)
    Wd = _weights_dev(W)
    for tiled in (False, True):
        out, ids, gates, uniq, nu = _run_layer(ctx, Wd, x, tiled)
        assert nu == cfg.top_k and (ids == ids[0]).all() and (gates == gates[0]).all()
        assert sorted(uniq[:nu].tolist()) == sorted(ids[0].tolist())
        np.testing.assert_array_equal(out, np.repeat(out[:1], 9, axis=0))
        ref64, _, _ = orc.layer(x1, W, cfg.top_k, 0, "f64")
        assert np.sqrt(((out[0] - ref64[0]) ** 2).sum() / (ref64[0] ** 2).sum()) <= 5e-5
    ctx.close()
    d, ffn, E, k, T = 128, 64, 256, 16, 16
    rng = np.random.default_rng(77)
    bf = lambda a: synth.f32_to_bf16_bits(a.astype(np.float32))
    Wb = dict(router_w=bf(rng.normal(0, 0.3, (E, d))), w1=bf(rng.normal(0, 0.1, (E, ffn, d))),
              w3=bf(rng.normal(0, 0.1, (E, ffn, d))), w2=bf(rng.normal(0, 0.1, (E, d, ffn))))
    xb = rng.normal(size=(T, d)).astype(np.float32)
    ctx = binding.MoeContext(d, ffn, E, k, 0, 16)
    assert ctx.workspace_bytes > 0
    _check_layer((d, ffn, E, k, 0), Wb, xb, ctx, _weights_dev(Wb))
    ctx.close()


def test_gate_that_underflows_to_zero_still_counts_as_routed():
    """Hidden states far from unit scale make the router's logit gaps so large that the weaker picks' gates underflow
    to exactly 0.  Such a pick is still a pick: its expert is in the union, and it contributes 0 * FFN = 0 — not
    whatever an unwritten buffer holds.  Checked on the fused and on the split-K down path."""
    cfg = synth.TINY
    W = synth.layer_weights_host(cfg, 9)
    x = (synth.hidden_host(cfg, 9, 0, 5, 0.5) * np.float32(300.0)).astype(np.float32)
    ref64, rids, rgates = orc.layer(x, W, cfg.top_k, 0, "f64")
    assert (rgates[:, 1] == 0.0).any(), "the case is meant to have underflowed gates"
    Wd = _weights_dev(W)
    for no_fused in (False, True):
        ctx = binding.MoeContext(cfg.d, cfg.ffn, cfg.n_experts, cfg.top_k, 0, 9)
        ctx.moe_ctx_tune(fused_down=0 if no_fused else 1)
        for tiled in (False, True):
            for rep in range(2):      # twice: the second run meets the first one's leftovers in the workspace
                out, ids, gates, uniq, nu = _run_layer(ctx, Wd, x if rep == 0 else x[::-1].copy(), tiled)
            want = ref64[::-1]
            np.testing.assert_array_equal(ids, rids[::-1])
            assert nu == orc.union(rids, cfg.n_experts)["n_unique"]
            assert np.isfinite(out).all()
            err = out.astype(np.float64) - want
            assert np.sqrt((err ** 2).sum() / (want ** 2).sum()) <= 5e-5
        ctx.close()


@pytest.mark.parametrize("block", range(4))
def test_random_valid_configurations_match_the_oracle(block):
    """48 seeded random draws over everything a caller may legally combine: d and ffn at the granularity of the
    weight type, 1 .. 256 experts (narrow and wide routers, top_k up to 16), 0 .. 8 shared experts, 1 .. 16 tokens,
    both gate rules, bf16 or FP8 in both layouts, token correlation 0 / 0.5 / 1.  Each is run twice on one context
    (the second run meets the first one's workspace) and compared with the fp64 oracle: ids, gates, union, output.
    (The same generator passed 1200 draws when this test was written.)"""
    import torch
    codes = synth.code_table_e4m3()
    for seed in range(12 * block, 12 * block + 12):
        rng = np.random.default_rng(seed)
        fp8 = bool(rng.integers(0, 2))
        q = 64 if fp8 else 32
        d, ffn = int(rng.integers(1, 9)) * q, int(rng.integers(1, 13)) * q
        E = int(rng.choice([1, 2, 3, 5, 8, 16, 31, 32, 33, 60, 64, 100, 256]))
        k = int(rng.integers(1, min(E, 16) + 1))
        if rng.random() < 0.5:
            k = min(k, 4)
        ns, T, gm = int(rng.choice([0, 0, 1, 2, 8])), int(rng.integers(1, 17)), int(rng.integers(0, 2))
        tiled = bool(seed & 1) if fp8 else bool(rng.integers(0, 2))   # FP8: by seed parity, no draw (keeps the screened streams)
        rho = float(rng.choice([0.0, 0.5, 1.0]))
        case = f"seed={seed} fp8={fp8} d={d} ffn={ffn} E={E} k={k} ns={ns} T={T} gate_mode={gm} tiled={tiled} rho={rho}"
        bf = lambda a: synth.f32_to_bf16_bits(a.astype(np.float32))
        qm = lambda shape: codes[rng.integers(0, len(codes), shape)]
        sc = lambda shape: (rng.uniform(0.5, 1.5, shape) * 2e-3).astype(np.float32)
        W = dict(router_w=bf(rng.normal(0, 0.3, (E, d))))
        if fp8:
            W.update(q1=qm((E, ffn, d)), q3=qm((E, ffn, d)), q2=qm((E, d, ffn)), s1=sc((E, ffn)), s3=sc((E, ffn)), s2=sc((E, d)))
            if ns:
                W.update(sq1=qm((ns, ffn, d)), sq3=qm((ns, ffn, d)), sq2=qm((ns, d, ffn)),
                         ss1=sc((ns, ffn)), ss3=sc((ns, ffn)), ss2=sc((ns, d)))
        else:
            W.update(w1=bf(rng.normal(0, 0.1, (E, ffn, d))), w3=bf(rng.normal(0, 0.1, (E, ffn, d))),
                     w2=bf(rng.normal(0, 0.1, (E, d, ffn))))
            if ns:
                W.update(sw1=bf(rng.normal(0, 0.1, (ns, ffn, d))), sw3=bf(rng.normal(0, 0.1, (ns, ffn, d))),
                         sw2=bf(rng.normal(0, 0.1, (ns, d, ffn))))
        x = (np.sqrt(rho) * rng.normal(size=(1, d)) + np.sqrt(1 - rho) * rng.normal(size=(T, d))).astype(np.float32)
        ref64, rids, rgates = (orc.layer_fp8 if fp8 else orc.layer)(x, W, k, ns, "f64", gm)
        _, _, logits = orc.route(x, W["router_w"], k, "f64")
        srt = np.sort(logits, axis=1)[:, ::-1][:, :min(k + 1, E)]
        assert srt.shape[1] < 2 or np.abs(np.diff(srt, axis=1)).min() > 1e-9, case + ": routing near-tie, change the seed"
        ctx = binding.MoeContext(d, ffn, E, k, ns, max_tokens=16, gate_mode=gm)
        lw = ctx.weights({n: torch.from_numpy(v.view(np.int16) if v.dtype == np.uint16 else v).cuda() for n, v in W.items()})
        if tiled:
            lw = ctx.moe_pack_weights(lw)
        out = torch.full((T, d), float("nan"), dtype=torch.float32, device="cuda")
        ids = torch.full((T, k), -7, dtype=torch.int32, device="cuda")
        gates = torch.zeros((T, k), dtype=torch.float32, device="cuda")
        uniq = torch.full((E,), -7, dtype=torch.int32, device="cuda")
        nu = torch.full((1,), -7, dtype=torch.int32, device="cuda")
        for _ in range(2):
            ctx.moe_verify_layer(lw, _dev(x), out, ids, gates, uniq, nu)
        torch.cuda.synchronize()
        o, u = out.cpu().numpy(), orc.union(rids, E)
        assert np.isfinite(o).all(), case
        np.testing.assert_array_equal(ids.cpu().numpy(), rids, err_msg=case)
        assert int(nu.item()) == u["n_unique"], case
        np.testing.assert_array_equal(uniq.cpu().numpy(), u["unique"], err_msg=case)
        assert np.abs(gates.cpu().numpy() - rgates).max() <= 1e-5, case
        err = o.astype(np.float64) - ref64
        assert np.sqrt((err ** 2).sum()) <= 5e-5 * np.sqrt((ref64 ** 2).sum()), case
        ctx.close()


@pytest.mark.parametrize("block", range(3))
def test_random_valid_chained_and_decoder_blocks_match_the_oracle(block):
    """36 seeded random draws of one teacher-forced block, half of them with the attention stub: shapes, expert counts,
    shared experts, 1 .. 16 tokens, both gate rules, bf16 (both layouts) or FP8 as in the layer test above, 1 .. 3 kv
    heads with 1, 2 or 4 query heads each, head dims 32 .. 128, input scales 0.3 / 1 / 3.  Draws whose routing margin
    on the normalised input is under 1e-4 are skipped (the two sides normalise in different summation orders).
    (The same generator passed 600 draws when this test was written.)"""
    codes = synth.code_table_e4m3()
    bf = lambda a: synth.f32_to_bf16_bits(a.astype(np.float32))
    ran = 0
    for seed in range(12 * block, 12 * block + 12):
        rng = np.random.default_rng(50_000 + seed)
        fp8 = bool(rng.integers(0, 2))
        q = 64 if fp8 else 32
        d, ffn = int(rng.integers(1, 9)) * q, int(rng.integers(1, 13)) * q
        E = int(rng.choice([1, 2, 3, 5, 8, 16, 31, 32, 33, 60, 64, 100, 256]))
        k = int(rng.integers(1, min(E, 16) + 1))
        if rng.random() < 0.5:
            k = min(k, 4)
        ns, T, gm = int(rng.choice([0, 0, 1, 2, 8])), int(rng.integers(1, 17)), int(rng.integers(0, 2))
        tiled = bool(seed & 1) if fp8 else bool(rng.integers(0, 2))
        decoder = bool(rng.integers(0, 2))
        dh, Hkv = int(rng.choice([32, 64, 96, 128])), int(rng.integers(1, 4))
        H = Hkv * int(rng.choice([1, 2, 4]))
        qm = lambda shape: codes[rng.integers(0, len(codes), shape)]
        sc = lambda shape: (rng.uniform(0.5, 1.5, shape) * 2e-3).astype(np.float32)
        W = dict(router_w=bf(rng.normal(0, 0.3, (E, d))))
        if fp8:
            W.update(q1=qm((E, ffn, d)), q3=qm((E, ffn, d)), q2=qm((E, d, ffn)), s1=sc((E, ffn)), s3=sc((E, ffn)), s2=sc((E, d)))
            if ns:
                W.update(sq1=qm((ns, ffn, d)), sq3=qm((ns, ffn, d)), sq2=qm((ns, d, ffn)),
                         ss1=sc((ns, ffn)), ss3=sc((ns, ffn)), ss2=sc((ns, d)))
        else:
            W.update(w1=bf(rng.normal(0, 0.1, (E, ffn, d))), w3=bf(rng.normal(0, 0.1, (E, ffn, d))),
                     w2=bf(rng.normal(0, 0.1, (E, d, ffn))))
            if ns:
                W.update(sw1=bf(rng.normal(0, 0.1, (ns, ffn, d))), sw3=bf(rng.normal(0, 0.1, (ns, ffn, d))),
                         sw2=bf(rng.normal(0, 0.1, (ns, d, ffn))))
        x = (rng.normal(size=(T, d)) * rng.choice([0.3, 1.0, 3.0])).astype(np.float32)
        geo = dict(n_heads=H, n_kv_heads=Hkv, head_dim=dh) if decoder else {}
        ctx = binding.MoeContext(d, ffn, E, k, ns, 16, gate_mode=gm, **geo)
        lw = ctx.weights(_weights_dev(W))
        if tiled or decoder:
            lw = ctx.moe_pack_weights(lw)
        try:
            if decoder:
                A = dict(wqkv=bf(rng.normal(0, 0.08, ((H + 2 * Hkv) * dh, d))), wo=bf(rng.normal(0, 0.08, (d, H * dh))),
                         gamma_attn=bf(1 + 0.1 * rng.normal(size=d)), gamma_moe=bf(1 + 0.1 * rng.normal(size=d)), **geo)
                _decoder_block_check(ctx, lw, _attn_dev(ctx, A), W, A, x, k, ns)
            else:
                gam = bf(1 + 0.1 * rng.normal(size=d))
                _chain_block_check(ctx, lw, W, gam, _dev(gam), x, k, ns)
            ran += 1
        except AssertionError as e:
            if "near-tie" not in str(e):
                raise AssertionError(f"seed={seed} decoder={decoder} fp8={fp8} d={d} ffn={ffn} E={E} k={k} ns={ns} T={T} "
                                     f"gate_mode={gm} tiled={tiled} H={H} Hkv={Hkv} dh={dh}: {e}") from e
        finally:
            ctx.close()
    assert ran >= 10


def test_one_context_many_calls_leftovers_never_matter():
    """One context serves 40 calls in a row with changing T (1 .. 16, so packed and split fragments, inline and separate
    grouping, fused and split-K down projection all alternate), changing layout, input scales from 1e-3 to 30 (gates
    that underflow to 0) and token correlation up to identical tokens; every call is checked against the fp64 oracle.
    Whatever a call leaves in the workspace — fragments, slabs, tables of a larger union — must not reach the next."""
    import torch
    bf = lambda a: synth.f32_to_bf16_bits(a.astype(np.float32))
    for ci, (d, ffn, E, k, ns, gm) in enumerate([(256, 320, 8, 2, 0, 0), (192, 1024, 60, 4, 4, 1)]):
        rng = np.random.default_rng(900 + ci)
        W = dict(router_w=bf(rng.normal(0, 0.3, (E, d))), w1=bf(rng.normal(0, 0.1, (E, ffn, d))),
                 w3=bf(rng.normal(0, 0.1, (E, ffn, d))), w2=bf(rng.normal(0, 0.1, (E, d, ffn))))
        if ns:
            W.update(sw1=bf(rng.normal(0, 0.1, (ns, ffn, d))), sw3=bf(rng.normal(0, 0.1, (ns, ffn, d))),
                     sw2=bf(rng.normal(0, 0.1, (ns, d, ffn))))
        ctx = binding.MoeContext(d, ffn, E, k, ns, 16, gate_mode=gm)
        lw_row = ctx.weights(_weights_dev(W))
        lw_t = ctx.moe_pack_weights(lw_row)
        checked = 0
        for call in range(40):
            T, tiled = int(rng.integers(1, 17)), bool(rng.integers(0, 2))
            scale, rho = float(rng.choice([1e-3, 1.0, 30.0])), float(rng.choice([0.0, 0.9, 1.0]))
            x = ((np.sqrt(rho) * rng.normal(size=(1, d)) + np.sqrt(1 - rho) * rng.normal(size=(T, d))) * scale).astype(np.float32)
            ref64, rids, _ = orc.layer(x, W, k, ns, "f64", gm)
            _, _, logits = orc.route(x, W["router_w"], k, "f64")
            srt = np.sort(logits, axis=1)[:, ::-1][:, :k + 1]
            out = torch.full((T, d), float("nan"), dtype=torch.float32, device="cuda")
            ids = torch.full((T, k), -7, dtype=torch.int32, device="cuda")
            nu = torch.full((1,), -7, dtype=torch.int32, device="cuda")
            ctx.moe_verify_layer(lw_t if tiled else lw_row, _dev(x), out, ids=ids, n_unique=nu)
            torch.cuda.synchronize()
            if np.abs(np.diff(srt, axis=1)).min() <= 1e-9:
                continue                                   # a routing near-tie: either pick is right, not compared
            case = f"config {ci} call {call}: T={T} tiled={tiled} scale={scale} rho={rho}"
            o = out.cpu().numpy()
            assert np.isfinite(o).all(), case
            np.testing.assert_array_equal(ids.cpu().numpy(), rids, err_msg=case)
            assert int(nu.item()) == orc.union(rids, E)["n_unique"], case
            err = o.astype(np.float64) - ref64
            assert np.sqrt((err ** 2).sum()) <= 5e-5 * np.sqrt((ref64 ** 2).sum()), case
            checked += 1
        assert checked >= 35
        ctx.close()


def test_measurement_aids_profile_and_stream_probe():
    """The two measurement aids the benchmark relies on.  Per-kernel profiling: the outputs stay bit-identical with the
    events in the stream, the number of profiled layer-steps is what was run, every stage that has a launch shows
    time, and a read empties the record.  Read-stream probe: every 32-bit word of the buffer reaches the sink exactly
    once (the sink's XOR fold equals the host's), also for sizes that leave waves without work or with a ragged tail."""
    import torch
    cfg = synth.TINY
    W = synth.layer_weights_host(cfg, 12)
    ctx = binding.MoeContext(cfg.d, cfg.ffn, cfg.n_experts, cfg.top_k, 0, 9)
    lw = ctx.moe_pack_weights(ctx.weights(_weights_dev(W)))
    xs = [_dev(synth.hidden_host(cfg, 12, it, T, 0.5)) for it, T in enumerate((1, 4, 9))]
    plain = []
    for x in xs:
        o = torch.zeros((x.shape[0], cfg.d), dtype=torch.float32, device="cuda")
        ctx.moe_verify_layer(lw, x, o)
        plain.append(o)
    torch.cuda.synchronize()
    ctx.moe_ctx_profile(True)
    for rep in range(2):
        for x, want in zip(xs, plain):
            o = torch.zeros_like(want)
            ctx.moe_verify_layer(lw, x, o)
            torch.cuda.synchronize()
            np.testing.assert_array_equal(o.cpu().numpy(), want.cpu().numpy())
    ms, steps = ctx.moe_ctx_profile_read()
    assert steps == 6 and set(ms) == {"route", "gateup", "down", "combine"}
    assert ms["route"] > 0 and ms["gateup"] > 0 and ms["down"] > 0 and ms["combine"] >= 0
    assert sum(ms.values()) < 50.0                                   # six tiny layer-steps: far below 50 ms
    assert ctx.moe_ctx_profile_read()[1] == 0                        # the read forgot the events
    ctx.moe_ctx_profile(False)
    o = torch.zeros_like(plain[0])
    ctx.moe_verify_layer(lw, xs[0], o)
    torch.cuda.synchronize()
    assert ctx.moe_ctx_profile_read()[1] == 0                        # nothing is recorded when switched off
    ctx.close()
    rng = np.random.default_rng(5)
    for n_words in (4, 4 * 64, 4 * 64 * 4096 + 4 * 7, 3_000_000 * 4):
        host = rng.integers(0, 2**32, n_words, dtype=np.uint32)
        src = torch.from_numpy(host.view(np.int32)).cuda()
        sink = torch.zeros(4096, dtype=torch.float32, device="cuda")
        binding.moe_stream_read_probe(src, sink)
        torch.cuda.synchronize()
        fold = np.bitwise_xor.reduce(sink.cpu().numpy().view(np.uint32))
        assert fold == np.bitwise_xor.reduce(host), n_words
    # the gate/up kernel's load twin: every word of the first `slots` matrices of both tensors reaches the sink once
    for slots, tiles, steps in ((1, 1, 1), (2, 5, 7), (3, 4, 13)):
        A = rng.integers(0, 2**16, (3, tiles * 16, steps * 32), dtype=np.uint16)
        B = rng.integers(0, 2**16, (3, tiles * 16, steps * 32), dtype=np.uint16)
        sink = torch.zeros(4096, dtype=torch.float32, device="cuda")
        binding.moe_weight_load_twin(_dev(A), _dev(B), slots, tiles, steps, sink)
        torch.cuda.synchronize()
        fold = np.bitwise_xor.reduce(sink.cpu().numpy().view(np.uint32))
        want = np.bitwise_xor.reduce(A[:slots].reshape(-1).view(np.uint32)) ^ np.bitwise_xor.reduce(B[:slots].reshape(-1).view(np.uint32))
        assert fold == want, (slots, tiles, steps)

