"""GPU test of the entry point that allocates nothing (moe_verify_layer_noalloc): through the C ABI, against the
existing entry point moe_verify_layer on a context of the same shape — same kernels, same launch plan, so the outputs
must agree bit for bit — and against the oracle's bars; several calls in a row on the one fixed workspace, each
smaller or differently shaped than the one before, so every call meets the previous call's leftovers."""
import ctypes

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from oracle import moe_oracle as orc
from paper_2506_20675_amd import binding, synth
from gpu_common import _check_out, _dev, _weights_dev


def _both(shape_args, W, x, tiled, fp8=False):
    """(out, ids, gates, unique, n_unique) from moe_verify_layer_noalloc and from moe_verify_layer on a fresh context."""
    import torch
    d, ffn, E, k, ns, mt = shape_args
    ctx = binding.MoeContext(d, ffn, E, k, ns, mt)
    lw = ctx.weights(_weights_dev(W))
    if tiled:
        lw = ctx.moe_pack_weights(lw)
    T = x.shape[0]
    res = []
    for noalloc in (True, False):
        out = torch.full((T, d), float("nan"), dtype=torch.float32, device="cuda")
        ids = torch.full((T, k), -7, dtype=torch.int32, device="cuda")
        gates = torch.zeros((T, k), dtype=torch.float32, device="cuda")
        uniq = torch.full((E,), -7, dtype=torch.int32, device="cuda")
        nu = torch.full((1,), -7, dtype=torch.int32, device="cuda")
        if noalloc:
            binding.moe_verify_layer_noalloc(ctx.shape, lw, _dev(x), out, ids, gates, uniq, nu)
        else:
            ctx.moe_verify_layer(lw, _dev(x), out, ids, gates, uniq, nu)
        torch.cuda.synchronize()
        res.append([t.cpu().numpy() for t in (out, ids, gates, uniq, nu)])
    ctx.close()
    return res


def test_noalloc_entry_point_matches_the_context_entry_point_call_after_call():
    cfg = synth.TINY
    W = synth.layer_weights_host(cfg, 21)
    rng = np.random.default_rng(2121)
    bf = lambda a: synth.f32_to_bf16_bits(a.astype(np.float32))
    d2, f2, E2, k2, ns2 = 256, 352, 16, 6, 2            # a second geometry: the workspace is laid out anew
    W2 = dict(router_w=bf(rng.normal(0, 0.3, (E2, d2))), w1=bf(rng.normal(0, 0.1, (E2, f2, d2))),
              w3=bf(rng.normal(0, 0.1, (E2, f2, d2))), w2=bf(rng.normal(0, 0.1, (E2, d2, f2))),
              sw1=bf(rng.normal(0, 0.1, (ns2, f2, d2))), sw3=bf(rng.normal(0, 0.1, (ns2, f2, d2))),
              sw2=bf(rng.normal(0, 0.1, (ns2, d2, f2))))
    tiny = (cfg.d, cfg.ffn, cfg.n_experts, cfg.top_k, 0, 16)
    calls = [  # (shape, weights, T, tiled): each input smaller than, or shaped differently from, the one before
        (tiny, W, 16, True), (tiny, W, 9, True), (tiny, W, 3, True), (tiny, W, 1, False),
        ((d2, f2, E2, k2, ns2, 9), W2, 9, True), ((d2, f2, E2, k2, ns2, 9), W2, 2, True), (tiny, W, 5, True),
    ]
    for n, (shape_args, Wh, T, tiled) in enumerate(calls):
        d, ffn, E, k, ns, _ = shape_args
        x = rng.normal(size=(T, d)).astype(np.float32)
        (out, ids, gates, uniq, nu), want = _both(shape_args, Wh, x, tiled)
        case = f"call {n}: shape {shape_args} T={T} tiled={tiled}"
        for got, ref, name in zip((out, ids, gates, uniq, nu), want, ("out", "ids", "gates", "unique", "n_unique")):
            np.testing.assert_array_equal(got, ref, err_msg=f"{case}: {name}")
        ref32, rids, rgates = orc.layer(x, Wh, k, ns, "f32")
        ref64, _, _ = orc.layer(x, Wh, k, ns, "f64")
        np.testing.assert_array_equal(ids, rids, err_msg=case)
        assert int(nu[0]) == orc.union(rids, E)["n_unique"], case
        assert np.abs(gates - rgates).max() <= 1e-5, case
        _check_out(out, ref32, ref64)


def test_noalloc_entry_point_rejects_what_does_not_fit_and_bad_arguments():
    import torch
    L = binding.lib()
    x = torch.zeros((1, 4096), dtype=torch.float32, device="cuda")
    out = torch.zeros((1, 4096), dtype=torch.float32, device="cuda")
    big = binding.MoeShape(4096, 14336, 64, 8, 0, 16, 0, 0, 0, 0)         # 64 live slots of H fragments alone: 58 MB
    dummy = binding.MoeLayerWeights()                                    # never looked at: the size check comes first
    rc = L.moe_verify_layer_noalloc(ctypes.byref(big), ctypes.byref(dummy), x.data_ptr(), 1, out.data_ptr(),
                                    None, None, None, None, None)
    assert rc == -3, rc                                                  # MOE_ERR_WORKSPACE
    assert b"fixed workspace" in L.moe_strerror(rc)
    ok = binding.MoeShape(4096, 14336, 8, 2, 0, 9, 0, 0, 0, 0)           # fits, but the weights are all NULL
    rc = L.moe_verify_layer_noalloc(ctypes.byref(ok), ctypes.byref(dummy), x.data_ptr(), 1, out.data_ptr(),
                                    None, None, None, None, None)
    assert rc == -1, rc
    rc = L.moe_verify_layer_noalloc(ctypes.byref(ok), ctypes.byref(dummy), x.data_ptr(), 10, out.data_ptr(),
                                    None, None, None, None, None)
    assert rc == -1, rc                                                  # T beyond max_tokens
    torch.cuda.synchronize()


def test_noalloc_entry_point_replays_from_a_hip_graph():
    """What the entry point is for: after one eager call (which looks the workspace address up), the call is captured
    in a HIP graph — its workspace preparation is a kernel, not a memset node — and replays, with eager work and
    synchronisation in between, give the eager bits for every input."""
    import torch
    cfg = synth.TINY
    T = 4
    W = synth.layer_weights_host(cfg, 44)
    ctx = binding.MoeContext(cfg.d, cfg.ffn, cfg.n_experts, cfg.top_k, 0, 9)
    lw = ctx.moe_pack_weights(ctx.weights(_weights_dev(W)))
    xs = [_dev(synth.hidden_host(cfg, 44, it, T, 0.5)) for it in range(3)]
    eager = []
    for x in xs:
        o = torch.zeros((T, cfg.d), dtype=torch.float32, device="cuda")
        binding.moe_verify_layer_noalloc(ctx.shape, lw, x, o)
        torch.cuda.synchronize()
        eager.append(o)
    x_static, out = xs[0].clone(), torch.zeros((T, cfg.d), dtype=torch.float32, device="cuda")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        binding.moe_verify_layer_noalloc(ctx.shape, lw, x_static, out)      # warm-up on the capture stream
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            binding.moe_verify_layer_noalloc(ctx.shape, lw, x_static, out)
    torch.cuda.synchronize()
    for rep in range(2):
        for x, want in zip(xs, eager):
            x_static.copy_(x)
            out.fill_(-1.0)
            other = torch.zeros((9, cfg.d), dtype=torch.float32, device="cuda")
            ctx.moe_verify_layer(lw, _dev(synth.hidden_host(cfg, 44, 9, 9, 0.5)), other)   # eager work in between
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(out, want)
    ctx.close()
