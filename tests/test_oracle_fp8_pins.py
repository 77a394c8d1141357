"""Pins for the FP8 (E4M3 codes + per-output-channel scale) part of the CPU oracle (no GPU).

Pinned to things outside the oracle: the format's published corner values (tests/golden), a library
implementation of the same 8-bit type, the already pinned bf16 oracle on weights that are exactly
representable in both formats, library GEMVs, and closed forms on hand-built experts that tell the
per-row scales apart.
"""
import math
import os

import numpy as np
import pytest

from oracle import moe_oracle as orc
from paper_2506_20675_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")
PRECS = ("f32", "f64")


def _library_values():
    """All 256 code values from the tensor library's own float8_e4m3fn type (independent of the oracle)."""
    import torch
    return torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float64).numpy()


FINITE = np.array([c for c in range(256) if c not in (0x7F, 0xFF)], dtype=np.uint8)


def _rand_fp8_expert(rng, d, ffn, pow2_scales):
    q1 = rng.choice(FINITE, (ffn, d))
    q3 = rng.choice(FINITE, (ffn, d))
    q2 = rng.choice(FINITE, (d, ffn))
    if pow2_scales:
        s = lambda n: (2.0 ** rng.integers(-12, -6, n)).astype(np.float32)
    else:
        s = lambda n: rng.uniform(1e-4, 2e-3, n).astype(np.float32)
    return q1, s(ffn), q3, s(ffn), q2, s(d)


def test_e4m3_golden_corner_values():
    rows = []
    with open(os.path.join(GOLD, "fp8_e4m3_values.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                c, v = line.split()
                rows.append((int(c, 16), float(v)))
    assert len(rows) == 12
    vals = orc.fp8_e4m3_values()
    for code, want in rows:
        got = vals[code]
        if math.isnan(want):
            assert math.isnan(got), hex(code)
        else:
            assert got == want and math.copysign(1.0, got) == math.copysign(1.0, want), hex(code)


def test_e4m3_all_codes_match_library_type_and_structure():
    vals = orc.fp8_e4m3_values()
    lib = _library_values()
    assert np.array_equal(np.isnan(vals), np.isnan(lib))
    ok = ~np.isnan(lib)
    assert np.array_equal(vals[ok], lib[ok])
    pos = vals[:0x7F]
    assert np.all(np.diff(pos) > 0)                       # codes are ordered like their values
    assert np.array_equal(vals[0x80:0xFF], -pos)          # sign bit only flips the sign
    assert np.array_equal(pos[16:] / pos[8:-8], np.full(0x7F - 16, 2.0))   # one exponent step doubles a normal value
    assert np.array_equal(pos[1:8], np.arange(1, 8) * 2.0 ** -9)           # subnormals are evenly spaced


@pytest.mark.parametrize("prec", PRECS)
def test_fp8_ffn_equals_bf16_oracle_when_effective_weights_fit_bf16(prec):
    """Power-of-two scales: scale * value(code) is exactly a bf16 number, so the FP8 expert must give the very bits the
    (separately pinned) bf16 expert gives on those weights — any wrong code value, scale index or operand shows."""
    rng = np.random.default_rng(31)
    d, ffn = 24, 40
    q1, s1, q3, s3, q2, s2 = _rand_fp8_expert(rng, d, ffn, pow2_scales=True)
    lib = _library_values()
    w1, w3, w2 = (s1[:, None] * lib[q1]), (s3[:, None] * lib[q3]), (s2[:, None] * lib[q2])
    b1, b3, b2 = (synth.f32_to_bf16_bits(w.astype(np.float32)) for w in (w1, w3, w2))
    for b, w in ((b1, w1), (b3, w3), (b2, w2)):
        assert np.array_equal(synth.bf16_bits_to_f32(b).astype(np.float64), w)     # really exact
    x = rng.normal(size=d).astype(np.float32)
    y8, h8 = orc.expert_ffn_fp8(x, q1, s1, q3, s3, q2, s2, prec)
    y16, h16 = orc.expert_ffn(x, b1, b3, b2, prec)
    np.testing.assert_array_equal(h8, h16)
    np.testing.assert_array_equal(y8, y16)


def test_fp8_ffn_general_scales_is_three_library_gemvs():
    rng = np.random.default_rng(32)
    d, ffn = 40, 72
    q1, s1, q3, s3, q2, s2 = _rand_fp8_expert(rng, d, ffn, pow2_scales=False)
    lib = _library_values()
    x = rng.normal(size=d).astype(np.float32)
    g = (s1.astype(np.float64)[:, None] * lib[q1]) @ x.astype(np.float64)
    u = (s3.astype(np.float64)[:, None] * lib[q3]) @ x.astype(np.float64)
    h = (g / (1.0 + np.exp(-g))) * u
    y = (s2.astype(np.float64)[:, None] * lib[q2]) @ h
    y64, h64 = orc.expert_ffn_fp8(x, q1, s1, q3, s3, q2, s2, "f64")
    np.testing.assert_allclose(h64, h, rtol=1e-12, atol=1e-18)
    np.testing.assert_allclose(y64, y, rtol=1e-11, atol=1e-18)
    y32, _ = orc.expert_ffn_fp8(x, q1, s1, q3, s3, q2, s2, "f32")
    assert np.linalg.norm(y32 - y) / np.linalg.norm(y) < 1e-5


def _fp8_selection_expert(d, rng):
    """ffn = 2d: w1 picks x[r // 2] (code of 1.0), w3 picks 2 x[(r + 1) % d] (code of 2.0), w2 picks h[2c + 1];
    every row has its own scale, so g_r = s1[r] x[r//2], u_r = 2 s3[r] x[(r+1)%d], y_c = s2[c] h[2c+1]."""
    ffn = 2 * d
    q1 = np.zeros((ffn, d), np.uint8)
    q3 = np.zeros((ffn, d), np.uint8)
    q2 = np.zeros((d, ffn), np.uint8)
    for r in range(ffn):
        q1[r, r // 2] = 0x38
        q3[r, (r + 1) % d] = 0x40
    for c in range(d):
        q2[c, 2 * c + 1] = 0x38
    s1 = rng.uniform(0.5, 2.0, ffn).astype(np.float32)
    s3 = rng.uniform(0.5, 2.0, ffn).astype(np.float32)
    s2 = rng.uniform(0.5, 2.0, d).astype(np.float32)
    return q1, s1, q3, s3, q2, s2


def _fp8_selection_closed_form(x, s1, s3, s2):
    d = x.shape[0]
    y = np.empty(d)
    for c in range(d):
        r = 2 * c + 1
        g = float(s1[r]) * float(x[r // 2])
        u = 2.0 * float(s3[r]) * float(x[(r + 1) % d])
        y[c] = float(s2[c]) * (g / (1.0 + math.exp(-g))) * u
    return y


@pytest.mark.parametrize("prec", PRECS)
def test_fp8_row_scales_closed_form(prec):
    """Each of the three scale vectors enters at its own row: a scale taken per column, from the wrong matrix or dropped fails."""
    rng = np.random.default_rng(33)
    d = 12
    q1, s1, q3, s3, q2, s2 = _fp8_selection_expert(d, rng)
    x = rng.normal(size=d).astype(np.float32)
    y, _ = orc.expert_ffn_fp8(x, q1, s1, q3, s3, q2, s2, prec)
    np.testing.assert_allclose(y, _fp8_selection_closed_form(x, s1, s3, s2), rtol=1e-6 if prec == "f32" else 1e-14, atol=1e-12)


@pytest.mark.parametrize("prec", PRECS)
def test_fp8_combine_gate_weighting_experts_and_shared(prec):
    rng = np.random.default_rng(34)
    d, E, T, n_shared = 10, 4, 3, 2
    ex = [_fp8_selection_expert(d, rng) for _ in range(E)]
    sh = [_fp8_selection_expert(d, rng) for _ in range(n_shared)]
    W = dict(q1=np.stack([e[0] for e in ex]), s1=np.stack([e[1] for e in ex]), q3=np.stack([e[2] for e in ex]),
             s3=np.stack([e[3] for e in ex]), q2=np.stack([e[4] for e in ex]), s2=np.stack([e[5] for e in ex]),
             sq1=np.stack([e[0] for e in sh]), ss1=np.stack([e[1] for e in sh]), sq3=np.stack([e[2] for e in sh]),
             ss3=np.stack([e[3] for e in sh]), sq2=np.stack([e[4] for e in sh]), ss2=np.stack([e[5] for e in sh]))
    x = rng.normal(size=(T, d)).astype(np.float32)
    ids = np.array([[3, 0], [1, 2], [2, 3]], np.int32)
    gates = np.array([[0.75, 0.25], [0.5, 0.5], [0.125, 0.875]], np.float32)
    out = orc.combine_fp8(x, W, ids, gates, 0, prec)
    out_s = orc.combine_fp8(x, W, ids, gates, n_shared, prec)
    for t in range(T):
        want = sum(float(gates[t, i]) * _fp8_selection_closed_form(x[t], ex[ids[t, i]][1], ex[ids[t, i]][3], ex[ids[t, i]][5])
                   for i in range(2))
        np.testing.assert_allclose(out[t], want, rtol=2e-6, atol=1e-7)
        want_s = want + sum(_fp8_selection_closed_form(x[t], s[1], s[3], s[5]) for s in sh)
        np.testing.assert_allclose(out_s[t], want_s, rtol=2e-6, atol=1e-7)


@pytest.mark.parametrize("prec", PRECS)
def test_fp8_layer_routes_like_the_bf16_router_and_is_batch_invariant(prec):
    cfg = synth.TINY
    W = synth.layer_weights_fp8_host(cfg, 2)
    T = 4
    x = synth.hidden_host(cfg, 2, 5, T, 0.5)
    out, ids, gates = orc.layer_fp8(x, W, cfg.top_k, 0, prec)
    rids, rgates, _ = orc.route(x, W["router_w"], cfg.top_k, prec)
    np.testing.assert_array_equal(ids, rids)
    np.testing.assert_array_equal(gates, rgates)
    np.testing.assert_array_equal(out, orc.combine_fp8(x, W, ids, gates, 0, prec))
    o1, i1, _ = orc.layer_fp8(x[2:3], W, cfg.top_k, 0, prec)      # verification equals decoding (Section 2.2)
    np.testing.assert_array_equal(o1[0], out[2])
    np.testing.assert_array_equal(i1[0], ids[2])


def test_fp8_layer_f32_close_to_f64_on_tiny_config():
    cfg = synth.TINY
    W = synth.layer_weights_fp8_host(cfg, 0)
    x = synth.hidden_host(cfg, 0, 0, 3, 0.5)
    o32, i32, _ = orc.layer_fp8(x, W, cfg.top_k, 0, "f32")
    o64, i64, _ = orc.layer_fp8(x, W, cfg.top_k, 0, "f64")
    np.testing.assert_array_equal(i32, i64)
    assert np.linalg.norm(o32.astype(np.float64) - o64) / np.linalg.norm(o64) < 1e-5
    assert np.abs(o64).max() > 1e-3      # a live signal, not zeros
