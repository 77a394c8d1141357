"""Pins for the chained-stack part of the CPU oracle: RMSNorm, residual add, pre-norm MoE block (no GPU)."""
import numpy as np
import pytest

from oracle import moe_oracle as orc
from paper_2506_20675_amd import synth

PRECS = ("f32", "f64")


def _bf16(a):
    return synth.f32_to_bf16_bits(np.asarray(a, np.float32))


@pytest.mark.parametrize("prec", PRECS)
def test_rmsnorm_hand_values_and_invariants(prec):
    ones = _bf16(np.ones(2))
    y = orc.rmsnorm(np.array([[3.0, 4.0]], np.float32), ones, 0.0, prec)
    np.testing.assert_allclose(y[0], [0.6 * 2 ** 0.5, 0.8 * 2 ** 0.5], rtol=2e-7)      # (3,4)/sqrt(12.5) = (0.6, 0.8) * sqrt 2
    rng = np.random.default_rng(51)
    T, d = 5, 48
    x = rng.normal(size=(T, d)).astype(np.float32) * np.array([[0.01], [1], [30], [1e3], [1]], np.float32)
    g1 = _bf16(np.ones(d))
    y = orc.rmsnorm(x, g1, 0.0, prec).astype(np.float64)
    np.testing.assert_allclose((y ** 2).mean(axis=1), 1.0, rtol=1e-6)                 # unit mean square whatever the input scale
    np.testing.assert_array_equal(orc.rmsnorm(x * np.float32(8.0), g1, 0.0, prec), orc.rmsnorm(x, g1, 0.0, prec))   # power of two: exact
    # gamma multiplies element j, and only element j
    gam = _bf16(rng.choice([0.5, 1.0, 2.0, -1.0, 0.25], d))
    yg = orc.rmsnorm(x, gam, 0.0, prec).astype(np.float64)
    np.testing.assert_allclose(yg, y * synth.bf16_bits_to_f32(gam).astype(np.float64), rtol=3e-7, atol=0)
    # rows do not mix; permuting the elements permutes the result (the mean does not care)
    np.testing.assert_array_equal(orc.rmsnorm(x[2:3], gam, 1e-5, prec)[0], orc.rmsnorm(x, gam, 1e-5, prec)[2])
    perm = rng.permutation(d)
    np.testing.assert_allclose(orc.rmsnorm(x[:, perm], g1, 0.0, prec), orc.rmsnorm(x, g1, 0.0, prec)[:, perm], rtol=3e-7)


@pytest.mark.parametrize("prec", PRECS)
def test_rmsnorm_eps_sits_inside_the_root_next_to_the_mean(prec):
    d = 16
    g1 = _bf16(np.ones(d))
    z = orc.rmsnorm(np.zeros((1, d), np.float32), g1, 1e-5, prec)
    assert np.all(z == 0.0)                                                           # no 0/0
    x = np.full((1, d), 2.0, np.float32)                                              # mean square 4
    for eps in (5.0, 12.0, 0.25):
        y = orc.rmsnorm(x, g1, eps, prec)
        np.testing.assert_allclose(y, 2.0 / np.sqrt(4.0 + eps), rtol=3e-7)            # (4+5) -> 2/3, (4+12) -> 1/2
    x2 = np.zeros((1, d), np.float32)
    x2[0, 0] = 4.0                                                                    # sum of squares 16, MEAN 1: tells sum from mean
    np.testing.assert_allclose(orc.rmsnorm(x2, g1, 3.0, prec)[0, 0], 4.0 / 2.0, rtol=3e-7)


@pytest.mark.parametrize("prec", PRECS)
def test_chained_block_wiring(prec):
    """x' - x is the layer applied to the NORMALISED input; the skip path carries x itself; a dead layer leaves x untouched."""
    cfg = synth.TINY
    W = synth.layer_weights_host(cfg, 4)
    gam = synth.norm_gamma_host(cfg, 4)
    T = 3
    x = (synth.hidden_host(cfg, 4, 1, T, 0.5) * np.float32(7.0)).astype(np.float32)   # far from unit scale on purpose
    xo, n, ids, gates = orc.chained_block(x, W, gam, cfg.top_k, 0, 1e-5, prec)
    np.testing.assert_array_equal(n, orc.rmsnorm(x, gam, 1e-5, prec))
    m, ids2, _ = orc.layer(n, W, cfg.top_k, 0, prec)
    np.testing.assert_array_equal(ids, ids2)
    np.testing.assert_allclose(xo.astype(np.float64), x.astype(np.float64) + m.astype(np.float64), rtol=0, atol=2e-6 * np.abs(xo).max())
    # scale invariance of the MoE branch: the block's update depends on the direction of x only (eps is tiny here)
    xo8, _, ids8, _ = orc.chained_block(x * np.float32(8.0), W, gam, cfg.top_k, 0, 0.0, prec)
    xo1, _, ids1, _ = orc.chained_block(x, W, gam, cfg.top_k, 0, 0.0, prec)
    np.testing.assert_array_equal(ids8, ids1)
    np.testing.assert_allclose(xo8 - x * np.float32(8.0), xo1 - x, rtol=0, atol=2e-5 * np.abs(xo1 - x).max() * 8)
    W0 = dict(W)
    W0["w1"] = np.zeros_like(W["w1"])
    xo0, *_ = orc.chained_block(x, W0, gam, cfg.top_k, 0, 1e-5, prec)
    np.testing.assert_array_equal(xo0, x)
    xg0, *_ = orc.chained_block(x, W, np.zeros_like(gam), cfg.top_k, 0, 1e-5, prec)    # gamma = 0 -> the layer sees zeros
    np.testing.assert_array_equal(xg0, x)


def test_chained_stack_is_the_blocks_in_order_and_fp8_variant_runs():
    cfg = synth.TINY
    L, T = 3, 2
    Ws = [synth.layer_weights_host(cfg, 20 + l) for l in range(L)]
    gs = [synth.norm_gamma_host(cfg, 20 + l) for l in range(L)]
    x0 = synth.hidden_host(cfg, 20, 0, T, 0.5)
    xL, trace, ids = orc.chained_stack(x0, Ws, gs, cfg.top_k, 0, 1e-5, "f64")
    x = x0
    for l in range(L):
        np.testing.assert_array_equal(trace[l], x)
        x, *_ = orc.chained_block(x, Ws[l], gs[l], cfg.top_k, 0, 1e-5, "f64")
    np.testing.assert_array_equal(xL, x)
    assert np.abs(xL - x0).max() > 0.1                 # the blocks do something
    # reversing the order of the layers changes the result: the chain is not a sum of independent terms
    xR, *_ = orc.chained_stack(x0, Ws[::-1], gs[::-1], cfg.top_k, 0, 1e-5, "f64")
    assert np.abs(xR - xL).max() > 1e-3
    W8 = synth.layer_weights_fp8_host(cfg, 20)
    x8, n8, i8, _ = orc.chained_block(x0, W8, gs[0], cfg.top_k, 0, 1e-5, "f64")
    m8, j8, _ = orc.layer_fp8(n8, W8, cfg.top_k, 0, "f64")
    np.testing.assert_array_equal(i8, j8)
    np.testing.assert_allclose(x8, x0 + m8, rtol=0, atol=1e-6 * np.abs(x8).max())


# ---------------------------------------------------------------- attention stub of the decoder block
def _attn_case(seed, T=5, d=32, H=4, Hkv=2, dh=8):
    rng = np.random.default_rng(seed)
    wqkv = _bf16(rng.normal(0, 0.3, ((H + 2 * Hkv) * dh, d)))
    wo = _bf16(rng.normal(0, 0.3, (d, H * dh)))
    n = rng.normal(size=(T, d)).astype(np.float32)
    return n, wqkv, wo, (H, Hkv, dh)


def _f64(b):
    return synth.bf16_bits_to_f32(b).astype(np.float64)


@pytest.mark.parametrize("prec", PRECS)
def test_attention_stub_matches_the_tensor_library_attention(prec):
    """Projections by library GEMMs, the core by the tensor library's own causal scaled-dot-product attention with the
    kv heads repeated over their query groups — nothing of the oracle's loops is reused."""
    import torch
    n, wqkv, wo, (H, Hkv, dh) = _attn_case(61)
    T = n.shape[0]
    a = orc.attention_stub(n, wqkv, wo, H, Hkv, dh, prec)
    qkv = torch.from_numpy(n.astype(np.float64) @ _f64(wqkv).T)
    q = qkv[:, :H * dh].reshape(T, H, dh).transpose(0, 1)
    k = qkv[:, H * dh:(H + Hkv) * dh].reshape(T, Hkv, dh).transpose(0, 1).repeat_interleave(H // Hkv, 0)
    v = qkv[:, (H + Hkv) * dh:].reshape(T, Hkv, dh).transpose(0, 1).repeat_interleave(H // Hkv, 0)
    o = torch.nn.functional.scaled_dot_product_attention(q[None], k[None], v[None], is_causal=True)[0]
    ref = o.transpose(0, 1).reshape(T, H * dh).numpy() @ _f64(wo).T
    np.testing.assert_allclose(a, ref, rtol=0, atol=(3e-5 if prec == "f32" else 1e-6) * np.abs(ref).max())


@pytest.mark.parametrize("prec", PRECS)
def test_attention_stub_special_cases(prec):
    n, wqkv, wo, (H, Hkv, dh) = _attn_case(62)
    T, d = n.shape
    a = orc.attention_stub(n, wqkv, wo, H, Hkv, dh, prec)
    # one token attends to itself only: a = Wo . repeat(Wv n); also what row 0 of any longer call gives (causality)
    a1 = orc.attention_stub(n[:1], wqkv, wo, H, Hkv, dh, prec)
    v0 = _f64(wqkv)[(H + Hkv) * dh:] @ n[0].astype(np.float64)
    o0 = np.concatenate([v0[(h // (H // Hkv)) * dh:(h // (H // Hkv) + 1) * dh] for h in range(H)])
    np.testing.assert_allclose(a1[0], _f64(wo) @ o0, rtol=0, atol=(3e-5 if prec == "f32" else 1e-6) * np.abs(a1).max())
    np.testing.assert_array_equal(a[0], a1[0])
    # causal: changing later tokens leaves earlier rows untouched, bit for bit
    n2 = n.copy()
    n2[3:] += 1.0
    a2 = orc.attention_stub(n2, wqkv, wo, H, Hkv, dh, prec)
    np.testing.assert_array_equal(a2[:3], a[:3])
    assert np.abs(a2[3:] - a[3:]).max() > 1e-3
    # zero query weights: all scores equal, so every token gets the running mean of the values up to itself
    wz = wqkv.copy()
    wz[:H * dh] = 0
    az = orc.attention_stub(n, wz, wo, H, Hkv, dh, prec)
    vs = n.astype(np.float64) @ _f64(wqkv)[(H + Hkv) * dh:].T                 # [T, Hkv dh]
    for t in range(T):
        vm = vs[:t + 1].mean(axis=0)
        o = np.concatenate([vm[(h // (H // Hkv)) * dh:(h // (H // Hkv) + 1) * dh] for h in range(H)])
        np.testing.assert_allclose(az[t], _f64(wo) @ o, rtol=0, atol=(3e-5 if prec == "f32" else 1e-6) * np.abs(az).max())


def test_decoder_block_wiring():
    cfg = synth.TINY
    A = synth.attn_weights_host(cfg, 7)
    W = synth.layer_weights_host(cfg, 7)
    assert (A["n_heads"], A["n_kv_heads"], A["head_dim"]) == (4, 1, 128)
    x = synth.hidden_host(cfg, 7, 0, 3, 0.5)
    xo, h, ids, _ = orc.decoder_block(x, A, W, cfg.top_k, 0, 1e-5, "f64")
    a = orc.attention_stub(orc.rmsnorm(x, A["gamma_attn"], 1e-5, "f64"), A["wqkv"], A["wo"], 4, 1, 128, "f64")
    np.testing.assert_allclose(h, x + a, rtol=0, atol=1e-6 * np.abs(h).max())
    xo2, _, ids2, _ = orc.chained_block(h, W, A["gamma_moe"], cfg.top_k, 0, 1e-5, "f64")
    np.testing.assert_array_equal(xo, xo2)
    np.testing.assert_array_equal(ids, ids2)
    assert np.abs(a).max() > 1e-2 and np.abs(xo - h).max() > 1e-2          # both halves contribute
    Az = dict(A)
    Az["wo"] = np.zeros_like(A["wo"])                                       # dead attention half: plain chained block
    xz, hz, *_ = orc.decoder_block(x, Az, W, cfg.top_k, 0, 1e-5, "f64")
    np.testing.assert_array_equal(hz, x)
    np.testing.assert_array_equal(xz, orc.chained_block(x, W, A["gamma_moe"], cfg.top_k, 0, 1e-5, "f64")[0])
