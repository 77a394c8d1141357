"""Shared helpers of the GPU parity tests: the HIP path (through the C ABI) against the CPU oracle, element by element.

Bars:
  * expert ids, unique-expert lists/counts, token grouping: bit-exact;
  * gates: |err| <= 1e-5;
  * out: the benchmark's bar  max|err| <= 2e-2 and relative RMS <= 1e-2  against the plain fp32
    oracle, AND the tighter bar this implementation is built to (fp32 accumulation, activations
    carried as bf16 hi+lo pairs): relative RMS <= 5e-5 and max|err| <= 1e-4 * max|ref| against the
    fp64 oracle.  Where it comes from: weights are exact bf16 (or exact E4M3) numbers; an activation
    enters as hi + lo with a residual below 2^-17 |x|; products are exact in fp32 and sums are kept in
    fp32, about sqrt(K) * 2^-24 relative for K terms: an expected relative RMS near 1e-5.
"""
import numpy as np

from oracle import moe_oracle as orc
from paper_2506_20675_amd import binding, synth


def _dev(a):
    import torch
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _weights_dev(W):
    return {k: _dev(v) for k, v in W.items()}


def _tiled(ctx, Wd):
    """Tiled copy of a layer's weights, made once per dict by moe_pack_weights and kept ON the dict (so it lives
    exactly as long as the tensors it was made from and can never be handed to another layer)."""
    if "_tiled" not in Wd:
        Wd["_tiled"] = ctx.moe_pack_weights(ctx.weights(Wd))
    return Wd["_tiled"]


def _run_layer(ctx, Wd, x, tiled=False):
    import torch
    s = ctx.shape
    T = x.shape[0]
    hid = _dev(x)
    out = torch.full((T, s.d), float("nan"), dtype=torch.float32, device="cuda")
    ids = torch.full((T, s.top_k), -7, dtype=torch.int32, device="cuda")
    gates = torch.zeros((T, s.top_k), dtype=torch.float32, device="cuda")
    uniq = torch.full((s.n_experts,), -7, dtype=torch.int32, device="cuda")
    nu = torch.full((1,), -7, dtype=torch.int32, device="cuda")
    lw = _tiled(ctx, Wd) if tiled else ctx.weights(Wd)
    ctx.moe_verify_layer(lw, hid, out, ids, gates, uniq, nu)
    torch.cuda.synchronize()
    return out.cpu().numpy(), ids.cpu().numpy(), gates.cpu().numpy(), uniq.cpu().numpy(), int(nu.item())


def _check_out(out, ref32, ref64):
    assert np.isfinite(out).all()
    err32 = out.astype(np.float64) - ref32
    assert np.abs(err32).max() <= 2e-2
    assert np.sqrt((err32 ** 2).sum() / (ref32.astype(np.float64) ** 2).sum()) <= 1e-2
    err64 = out.astype(np.float64) - ref64
    rel = np.sqrt((err64 ** 2).sum() / (ref64.astype(np.float64) ** 2).sum())
    assert rel <= 5e-5, rel
    assert np.abs(err64).max() <= 1e-4 * np.abs(ref64).max()
    return rel


def _check_layer(cfg_like, W, x, ctx=None, Wd=None, gate_mode=0):
    d, ffn, E, k, ns = cfg_like
    own = ctx is None
    if own:
        ctx = binding.MoeContext(d, ffn, E, k, ns, max_tokens=max(9, x.shape[0]), gate_mode=gate_mode)
        Wd = _weights_dev(W)
    assert ctx.shape.gate_mode == gate_mode
    out, ids, gates, uniq, nu = _run_layer(ctx, Wd, x)
    ref32, rids, rgates = orc.layer(x, W, k, ns, "f32", gate_mode)
    ref64, rids64, _ = orc.layer(x, W, k, ns, "f64", gate_mode)
    # margin between the k-th and (k+1)-th logit: routing is decided in fp64 on both sides, so
    # only margins at the 1e-12 level could legitimately differ
    _, _, logits = orc.route(x, W["router_w"], k, "f64")
    srt = np.sort(logits, axis=1)[:, ::-1]
    if E > k:
        assert (srt[:, k - 1] - srt[:, k]).min() > 1e-9, "seed produces a routing near-tie; pick another"
    np.testing.assert_array_equal(ids, rids)
    np.testing.assert_array_equal(rids, rids64)
    assert np.abs(gates - rgates).max() <= 1e-5
    u = orc.union(rids, E)
    assert nu == u["n_unique"]
    np.testing.assert_array_equal(uniq, u["unique"])
    rel = _check_out(out, ref32, ref64)
    # the tiled weight layout holds the same numbers in another order; its kernels split the sums
    # differently, so it is checked against the oracle in its own right
    out_t, ids_t, gates_t, uniq_t, nu_t = _run_layer(ctx, Wd, x, tiled=True)
    np.testing.assert_array_equal(ids_t, rids)
    np.testing.assert_array_equal(uniq_t, u["unique"])
    assert nu_t == nu and np.abs(gates_t - rgates).max() <= 1e-5
    rel = max(rel, _check_out(out_t, ref32, ref64))
    if own:
        ctx.close()
    return out, rel



def _run_layer_fp8(ctx, Wd, x, tiled=True):
    import torch
    s = ctx.shape
    T = x.shape[0]
    out = torch.full((T, s.d), float("nan"), dtype=torch.float32, device="cuda")
    ids = torch.full((T, s.top_k), -7, dtype=torch.int32, device="cuda")
    gates = torch.zeros((T, s.top_k), dtype=torch.float32, device="cuda")
    uniq = torch.full((s.n_experts,), -7, dtype=torch.int32, device="cuda")
    nu = torch.full((1,), -7, dtype=torch.int32, device="cuda")
    ctx.moe_verify_layer(_tiled(ctx, Wd) if tiled else ctx.weights(Wd), _dev(x), out, ids, gates, uniq, nu)
    torch.cuda.synchronize()
    return out.cpu().numpy(), ids.cpu().numpy(), gates.cpu().numpy(), uniq.cpu().numpy(), int(nu.item())


def _check_layer_fp8(ctx, W, Wd, x, k, ns, row_major=True):
    """The tiled layout (the one that is streamed at speed) and, unless switched off, the plain row-major one the
    oracle reads: other kernels with other summation splits, each held to the oracle in its own right."""
    rel = _check_layer_fp8_one(ctx, W, Wd, x, k, ns, True)
    if row_major:
        rel = max(rel, _check_layer_fp8_one(ctx, W, Wd, x, k, ns, False))
    return rel


def _check_layer_fp8_one(ctx, W, Wd, x, k, ns, tiled):
    gm = ctx.shape.gate_mode
    out, ids, gates, uniq, nu = _run_layer_fp8(ctx, Wd, x, tiled)
    ref32, rids, rgates = orc.layer_fp8(x, W, k, ns, "f32", gm)
    ref64, rids64, _ = orc.layer_fp8(x, W, k, ns, "f64", gm)
    E = W["q1"].shape[0]
    _, _, logits = orc.route(x, W["router_w"], k, "f64")
    srt = np.sort(logits, axis=1)[:, ::-1]
    if E > k:
        assert (srt[:, k - 1] - srt[:, k]).min() > 1e-9, "seed produces a routing near-tie; pick another"
    np.testing.assert_array_equal(ids, rids)
    np.testing.assert_array_equal(rids, rids64)
    assert np.abs(gates - rgates).max() <= 1e-5
    u = orc.union(rids, E)
    assert nu == u["n_unique"]
    np.testing.assert_array_equal(uniq, u["unique"])
    return _check_out(out, ref32, ref64)



def _routing_margin_ok(n, router_w, k, E, need=1e-4):
    """The GPU normalises in another summation order than the oracle, so the two routers see inputs that differ in
    the last bits; their picks agree whenever the k-th/(k+1)-th logit gap is far above that (seeds are screened)."""
    if E <= k:
        return True
    _, _, logits = orc.route(n, router_w, k, "f64")
    srt = np.sort(logits, axis=1)[:, ::-1]
    return (srt[:, k - 1] - srt[:, k]).min() > need and (srt[:, :k - 1] - srt[:, 1:k]).min(initial=1.0) > need


def _chain_block_check(ctx, lw, W, gam, gam_d, x, k, ns, eps=1e-5):
    """One block, teacher-forced: the GPU gets the oracle's input x and must reproduce the oracle's x'."""
    import torch
    T, d = x.shape
    xo = torch.full((T, d), float("nan"), dtype=torch.float32, device="cuda")
    tr = torch.full((1, T, d), float("nan"), dtype=torch.float32, device="cuda")
    nu = torch.full((1,), -3, dtype=torch.int32, device="cuda")
    ctx.moe_chained_stack([lw], [gam_d], _dev(x), xo, eps, tr, nu)
    torch.cuda.synchronize()
    gm = ctx.shape.gate_mode
    r32, n32, ids, _ = orc.chained_block(x, W, gam, k, ns, eps, "f32", gm)
    r64, n64, ids64, _ = orc.chained_block(x, W, gam, k, ns, eps, "f64", gm)
    assert _routing_margin_ok(n64, W["router_w"], k, ctx.shape.n_experts), "seed produces a routing near-tie; pick another"
    np.testing.assert_array_equal(ids, ids64)
    np.testing.assert_array_equal(tr[0].cpu().numpy(), x)                       # the stream entering the block
    assert int(nu.item()) == orc.union(ids64, ctx.shape.n_experts)["n_unique"]
    got = xo.cpu().numpy().astype(np.float64)
    # the update x' - x is what the block computes: held to the same bars as a layer's output
    _check_out((got - x).astype(np.float32), (r32.astype(np.float64) - x).astype(np.float32), r64.astype(np.float64) - x)
    return r64



def _attn_dev(ctx, A):
    return ctx.attn_weights({k: _dev(v) for k, v in A.items() if isinstance(v, np.ndarray)})


def _decoder_block_check(ctx, lw, aw, W, A, x, k, ns, eps=1e-5):
    """One block, teacher-forced on the oracle's input stream."""
    import torch
    T, d = x.shape
    xo = torch.full((T, d), float("nan"), dtype=torch.float32, device="cuda")
    nu = torch.full((1,), -3, dtype=torch.int32, device="cuda")
    ctx.moe_decoder_stack([lw], [aw], _dev(x), xo, eps, None, nu)
    torch.cuda.synchronize()
    gm = ctx.shape.gate_mode
    r32, h32, ids, _ = orc.decoder_block(x, A, W, k, ns, eps, "f32", gm)
    r64, h64, ids64, _ = orc.decoder_block(x, A, W, k, ns, eps, "f64", gm)
    n64 = orc.rmsnorm(h64, A["gamma_moe"], eps, "f64")
    assert _routing_margin_ok(n64, W["router_w"], k, ctx.shape.n_experts), "seed produces a routing near-tie; pick another"
    np.testing.assert_array_equal(ids, ids64)
    assert int(nu.item()) == orc.union(ids64, ctx.shape.n_experts)["n_unique"]
    got = xo.cpu().numpy().astype(np.float64)
    _check_out((got - x).astype(np.float32), (r32.astype(np.float64) - x).astype(np.float32), r64.astype(np.float64) - x)
    return r64

