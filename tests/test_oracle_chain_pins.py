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
