"""Pins for the CPU oracle of the MoE layer (no GPU).

The oracle has no implementation to be compared against, so it is pinned to
things fixed outside it: values printed in the paper (tests/golden), closed forms
on hand-built weights, brute force on tiny inputs, library GEMVs for the special
case top_k = 1, and invariants (batch invariance = the verification-equals-decoding
property of speculative decoding, Section 2.2 of the paper).
"""
import itertools
import math
import os

import numpy as np
import pytest

from oracle import moe_oracle as orc
from paper_2506_20675_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")
PRECS = ("f32", "f64")


def _bf16(a):
    return synth.f32_to_bf16_bits(np.asarray(a, np.float32))


def _rand_layer(seed, d, ffn, E, n_shared=0, sigma=0.05):
    rng = np.random.default_rng(seed)
    W = dict(router_w=_bf16(rng.normal(0, 0.3, (E, d))),
             w1=_bf16(rng.normal(0, sigma, (E, ffn, d))),
             w3=_bf16(rng.normal(0, sigma, (E, ffn, d))),
             w2=_bf16(rng.normal(0, sigma, (E, d, ffn))))
    if n_shared:
        W.update(sw1=_bf16(rng.normal(0, sigma, (n_shared, ffn, d))),
                 sw3=_bf16(rng.normal(0, sigma, (n_shared, ffn, d))),
                 sw2=_bf16(rng.normal(0, sigma, (n_shared, d, ffn))))
    return W, rng


def _golden_rows(name):
    rows = []
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                rows.append([float(v) for v in line.split()])
    return rows


# ---------------------------------------------------------------- routing
@pytest.mark.parametrize("prec", PRECS)
@pytest.mark.parametrize("E,k", [(4, 1), (5, 2), (8, 2), (8, 3), (6, 6)])
def test_route_brute_force(prec, E, k):
    """The chosen set maximises the sum of logits over all C(E,k) subsets; slots are in descending order."""
    rng = np.random.default_rng(100 + E * 10 + k)
    d, T = 24, 7
    x = rng.normal(size=(T, d)).astype(np.float32)
    rw = _bf16(rng.normal(0, 0.5, (E, d)))
    ids, gates, logits = orc.route(x, rw, k, prec)
    ref = x.astype(np.float64) @ synth.bf16_bits_to_f32(rw).astype(np.float64).T   # library GEMM, independent of the C loop
    np.testing.assert_allclose(logits, ref, rtol=0, atol=1e-12)
    for t in range(T):
        best = max(itertools.combinations(range(E), k), key=lambda s: sum(ref[t, e] for e in s))
        assert set(ids[t]) == set(best)
        assert len(set(ids[t])) == k
        sel = ref[t, ids[t]]
        assert np.all(np.diff(sel) <= 0), "slots must be in descending-logit order"


@pytest.mark.parametrize("prec", PRECS)
def test_route_ties_go_to_lower_index_and_uniform_gates(prec):
    d, E, k, T = 16, 8, 3, 2
    x = np.random.default_rng(1).normal(size=(T, d)).astype(np.float32)
    ids, gates, _ = orc.route(x, np.zeros((E, d), np.uint16), k, prec)
    assert (ids == np.arange(k)[None, :]).all()
    np.testing.assert_allclose(gates, 1.0 / k, rtol=1e-7)
    # duplicated rows: experts 2 and 5 identical -> 2 comes first whenever they are adjacent in rank
    rng = np.random.default_rng(2)
    rw = rng.normal(0, 0.5, (E, d)).astype(np.float32)
    rw[5] = rw[2]
    ids, _, _ = orc.route(x, _bf16(rw), E, prec)
    for t in range(T):
        pos = {int(e): i for i, e in enumerate(ids[t])}
        assert pos[5] == pos[2] + 1


@pytest.mark.parametrize("prec", PRECS)
def test_route_topk_equals_E_is_permutation_and_row_permutation_equivariance(prec):
    rng = np.random.default_rng(3)
    d, E, T = 32, 8, 5
    x = rng.normal(size=(T, d)).astype(np.float32)
    rw = _bf16(rng.normal(0, 0.5, (E, d)))
    ids, gates, _ = orc.route(x, rw, E, prec)
    assert (np.sort(ids, axis=1) == np.arange(E)[None, :]).all()
    perm = rng.permutation(E)
    ids2, gates2, _ = orc.route(x, rw[perm], 2, prec)      # new expert j is old expert perm[j]
    ids1, gates1, _ = orc.route(x, rw, 2, prec)
    assert (perm[ids2] == ids1).all()
    np.testing.assert_array_equal(gates1, gates2)


@pytest.mark.parametrize("prec", PRECS)
def test_gates_closed_forms(prec):
    rng = np.random.default_rng(4)
    d, E, T = 48, 8, 9
    x = rng.normal(size=(T, d)).astype(np.float32)
    rw = _bf16(rng.normal(0, 0.4, (E, d)))
    tol = 2e-6 if prec == "f32" else 1e-7      # gates are returned as fp32
    # top-2: logistic of the logit gap
    ids, gates, logits = orc.route(x, rw, 2, prec)
    for t in range(T):
        l0, l1 = logits[t, ids[t, 0]], logits[t, ids[t, 1]]
        assert abs(gates[t, 0] - 1.0 / (1.0 + math.exp(-(l0 - l1)))) < tol
    # top-k: softmax over ALL experts, renormalised over the selected ones
    for k in (1, 3, 8):
        ids, gates, logits = orc.route(x, rw, k, prec)
        full = np.exp(logits - logits.max(axis=1, keepdims=True))
        full /= full.sum(axis=1, keepdims=True)
        sel = np.take_along_axis(full, ids.astype(np.int64), axis=1)
        np.testing.assert_allclose(gates, sel / sel.sum(axis=1, keepdims=True), atol=tol, rtol=0)
        np.testing.assert_allclose(gates.sum(axis=1), 1.0, atol=1e-6)
        assert (gates > 0).all() and (np.diff(gates, axis=1) <= 0).all()


# ---------------------------------------------------------------- union
def test_union_structure_and_paper_example():
    rows = _golden_rows("union_example.txt")
    for n_tok, k, E, max_unique, ratio in rows:
        n_tok, k, E = int(n_tok), int(k), int(E)
        ids = np.arange(n_tok * k, dtype=np.int32).reshape(n_tok, k)      # disjoint choices = the "up to" case
        u = orc.union(ids, E, "f64")
        assert u["n_unique"] == int(max_unique)
        assert u["n_unique"] / k == ratio
    ids = np.array([[5, 2], [2, 7], [7, 5], [0, 2]], np.int32)
    u = orc.union(ids, 8, "f64")
    assert u["n_unique"] == 4 and list(u["unique"][:4]) == [0, 2, 5, 7] and (u["unique"][4:] == -1).all()
    assert list(u["count"]) == [1, 0, 3, 0, 0, 2, 0, 2]
    assert list(u["offset"]) == [0, 1, 1, 4, 4, 4, 6, 6, 8]
    # assignments a = t*top_k + i, grouped by expert, ascending inside each group
    assert list(u["assign"]) == [6, 1, 2, 7, 0, 5, 3, 4]
    with pytest.raises(ValueError):
        orc.union(np.array([[0, 9]], np.int32), 8, "f64")


@pytest.mark.parametrize("prec", PRECS)
def test_union_bounds_and_degenerate_cases(prec):
    cfg = synth.TINY
    W = synth.layer_weights_host(cfg, 0)
    for T in (1, 2, 3, 5, 9):
        for rho in (0.0, 0.5):
            x = synth.hidden_host(cfg, 0, 7, T, rho)
            ids, _, _ = orc.route(x, W["router_w"], cfg.top_k, prec)
            n = orc.union(ids, cfg.n_experts, prec)["n_unique"]
            assert cfg.top_k <= n <= min(cfg.n_experts, T * cfg.top_k)
            if T == 1:
                assert n == cfg.top_k
    # rho = 1: identical tokens -> same experts, union = top_k
    x = synth.hidden_host(cfg, 0, 7, 6, 1.0)
    assert np.abs(x - x[0]).max() == 0
    ids, _, _ = orc.route(x, W["router_w"], cfg.top_k, prec)
    assert orc.union(ids, cfg.n_experts, prec)["n_unique"] == cfg.top_k


def test_union_mean_matches_balls_and_bins():
    """Uniform routing of 8 tokens x top-2 over 8 experts: mean union 'over seven' (closed form 8(1-0.75^8) = 7.199)."""
    (n_tok, k, E, lower, ratio), = _golden_rows("balls_and_bins.txt")
    n_tok, k, E = int(n_tok), int(k), int(E)
    rng = np.random.default_rng(5)
    d, trials = 32, 1500
    tot = 0
    for _ in range(trials):
        rw = _bf16(rng.normal(0, 1.0, (E, d)))       # a fresh random router per draw -> exchangeable experts
        x = rng.normal(size=(n_tok, d)).astype(np.float32)
        ids, _, _ = orc.route(x, rw, k)
        tot += orc.union(ids, E)["n_unique"]
    mean = tot / trials
    closed = E * (1 - (1 - k / E) ** n_tok)
    assert mean > lower
    assert abs(mean - closed) < 0.08
    assert abs(closed / k - ratio) < 0.11            # the paper rounds 3.6 down to "3.5x"


# ---------------------------------------------------------------- expert FFN and combine
def _selection_expert(d, scale=1.0):
    """ffn = 2d expert built from 0/1/2-valued matrices with a closed-form output:
       g_r = x[r // 2], u_r = 2 x[(r + 1) % d], y_c = scale * h[2c + 1]."""
    ffn = 2 * d
    w1 = np.zeros((ffn, d), np.float32)
    w3 = np.zeros((ffn, d), np.float32)
    w2 = np.zeros((d, ffn), np.float32)
    for r in range(ffn):
        w1[r, r // 2] = 1.0
        w3[r, (r + 1) % d] = 2.0
    for c in range(d):
        w2[c, 2 * c + 1] = scale
    return w1, w3, w2


def _selection_closed_form(x, scale=1.0):
    d = x.shape[0]
    y = np.empty(d)
    for c in range(d):
        r = 2 * c + 1
        g = float(x[r // 2])
        u = 2.0 * float(x[(r + 1) % d])
        y[c] = scale * (g / (1.0 + math.exp(-g))) * u
    return y


@pytest.mark.parametrize("prec", PRECS)
def test_expert_ffn_closed_form_selection_matrices(prec):
    """Catches a transposed operand, swapped w1/w3, a wrong activation or a wrong index."""
    d = 12
    x = np.random.default_rng(6).normal(size=d).astype(np.float32)
    w1, w3, w2 = _selection_expert(d, scale=0.5)
    y, h = orc.expert_ffn(x, _bf16(w1), _bf16(w3), _bf16(w2), prec)
    np.testing.assert_allclose(y, _selection_closed_form(x, 0.5), rtol=3e-7 if prec == "f32" else 1e-14, atol=1e-12)
    # silu spot values: silu(0) = 0, silu(1) = 1/(1+e^-1)
    x2 = np.zeros(d, np.float32)
    x2[0] = 1.0
    x2[1] = 0.5
    y2, h2 = orc.expert_ffn(x2, _bf16(w1), _bf16(w3), _bf16(w2), prec)
    assert abs(h2[0] - (1.0 / (1.0 + math.exp(-1.0))) * 2 * 0.5) < 1e-7      # r=0: g=x0=1, u=2*x1
    assert h2[4] == 0.0                                                        # g = x2 = 0 -> silu(0) = 0


@pytest.mark.parametrize("prec", PRECS)
def test_top1_layer_is_three_library_gemvs(prec):
    d, ffn, E, T = 40, 72, 4, 3
    W, rng = _rand_layer(7, d, ffn, E, sigma=0.2)
    x = rng.normal(size=(T, d)).astype(np.float32)
    out, ids, gates = orc.layer(x, W, 1, 0, prec)
    np.testing.assert_allclose(gates, 1.0)
    f = lambda a: synth.bf16_bits_to_f32(a).astype(np.float64)
    for t in range(T):
        e = int(ids[t, 0])
        g = f(W["w1"][e]) @ x[t].astype(np.float64)
        u = f(W["w3"][e]) @ x[t].astype(np.float64)
        y = f(W["w2"][e]) @ ((g / (1.0 + np.exp(-g))) * u)
        np.testing.assert_allclose(out[t], y, rtol=2e-5 if prec == "f32" else 2e-7, atol=1e-6 if prec == "f32" else 1e-9)


@pytest.mark.parametrize("prec", PRECS)
def test_combine_closed_form_gate_weighting_and_shared(prec):
    """Experts that are scaled copies of one closed-form expert: out = base * sum_i gate_i * scale_{e_i} (+ shared scales)."""
    d, E, T = 10, 4, 3
    ffn = 2 * d
    scales = [1.0, 2.0, 0.5, 4.0]
    parts = [_selection_expert(d, s) for s in scales]
    W = dict(w1=_bf16(np.stack([p[0] for p in parts])), w3=_bf16(np.stack([p[1] for p in parts])),
             w2=_bf16(np.stack([p[2] for p in parts])))
    sh = [_selection_expert(d, s) for s in (0.25, 8.0)]
    W.update(sw1=_bf16(np.stack([p[0] for p in sh])), sw3=_bf16(np.stack([p[1] for p in sh])),
             sw2=_bf16(np.stack([p[2] for p in sh])))
    x = np.random.default_rng(8).normal(size=(T, d)).astype(np.float32)
    ids = np.array([[3, 0], [1, 2], [2, 3]], np.int32)
    gates = np.array([[0.75, 0.25], [0.5, 0.5], [0.125, 0.875]], np.float32)
    tol = dict(rtol=1e-6, atol=1e-7)
    out = orc.combine(x, W, ids, gates, 0, prec)
    out_s = orc.combine(x, W, ids, gates, 2, prec)
    for t in range(T):
        base = _selection_closed_form(x[t])
        wsum = sum(float(gates[t, i]) * scales[ids[t, i]] for i in range(2))
        np.testing.assert_allclose(out[t], base * wsum, **tol)
        np.testing.assert_allclose(out_s[t], base * (wsum + 0.25 + 8.0), **tol)   # shared experts: gate 1, always on


@pytest.mark.parametrize("prec", PRECS)
def test_zero_w1_gives_zero_and_dense_masked_agrees(prec):
    d, ffn, E, T, k = 24, 40, 6, 4, 2
    W, rng = _rand_layer(9, d, ffn, E, n_shared=1, sigma=0.2)
    x = rng.normal(size=(T, d)).astype(np.float32)
    out, ids, gates = orc.layer(x, W, k, 1, prec)
    dm = orc.dense_masked(x, W, ids, gates, 1, prec)
    np.testing.assert_allclose(out, dm, rtol=1e-5 if prec == "f32" else 1e-12, atol=1e-6 if prec == "f32" else 1e-13)
    W0 = dict(W)
    W0["w1"] = np.zeros_like(W["w1"])
    W0["sw1"] = np.zeros_like(W["sw1"])
    out0, _, _ = orc.layer(x, W0, k, 1, prec)
    assert np.abs(out0).max() == 0.0


@pytest.mark.parametrize("prec", PRECS)
def test_batch_invariance_and_token_permutation(prec):
    """Verification equals decoding (Section 2.2): row t of the T-token result IS the 1-token result, bit for bit."""
    cfg = synth.TINY
    W = synth.layer_weights_host(cfg, 1)
    T = 5
    x = synth.hidden_host(cfg, 1, 3, T, 0.5)
    out, ids, gates = orc.layer(x, W, cfg.top_k, 0, prec)
    for t in (0, 3):
        o1, i1, g1 = orc.layer(x[t:t + 1], W, cfg.top_k, 0, prec)
        np.testing.assert_array_equal(o1[0], out[t])
        np.testing.assert_array_equal(i1[0], ids[t])
    perm = np.array([4, 2, 0, 1, 3])
    outp, idsp, _ = orc.layer(x[perm], W, cfg.top_k, 0, prec)
    np.testing.assert_array_equal(outp, out[perm])
    np.testing.assert_array_equal(idsp, ids[perm])


def test_f32_oracle_close_to_f64_oracle_on_tiny_config():
    cfg = synth.TINY
    W = synth.layer_weights_host(cfg, 0)
    x = synth.hidden_host(cfg, 0, 0, 9, 0.5)
    o32, i32, g32 = orc.layer(x, W, cfg.top_k, 0, "f32")
    o64, i64, g64 = orc.layer(x, W, cfg.top_k, 0, "f64")
    np.testing.assert_array_equal(i32, i64)          # routing decided in double in both builds
    np.testing.assert_allclose(g32, g64, atol=2e-7)
    rel = np.sqrt(((o32.astype(np.float64) - o64) ** 2).sum() / (o64.astype(np.float64) ** 2).sum())
    assert rel < 1e-5


# ---------------------------------------------------------------- gate variant: softmax over all experts
@pytest.mark.parametrize("prec", PRECS)
def test_softmax_all_gates_against_library_softmax_and_identities(prec):
    """Same picks as the renormalised rule; gates = the library softmax over ALL logits read at the picks; the two rules
    differ by exactly the probability mass of the picks; with top_k = E they coincide; E = 2, top-1 is the logistic."""
    from scipy.special import softmax
    rng = np.random.default_rng(41)
    T, d, E, k = 6, 20, 7, 3
    x = rng.normal(size=(T, d)).astype(np.float32)
    rw = _bf16(rng.normal(0, 0.6, (E, d)))
    ids0, g0, logits = orc.route(x, rw, k, prec)
    ids1, g1, logits1 = orc.route(x, rw, k, prec, gate_mode=orc.GATE_SOFTMAX_ALL)
    np.testing.assert_array_equal(ids0, ids1)
    np.testing.assert_array_equal(logits, logits1)
    p = softmax(logits, axis=1)
    tol = 3e-7 if prec == "f32" else 1e-7          # gates are stored as fp32
    np.testing.assert_allclose(g1, np.take_along_axis(p, ids1, 1), rtol=0, atol=tol)
    assert (g1.sum(axis=1) < 1.0).all()             # mass of the experts that were not picked is missing
    mass = np.take_along_axis(p, ids1, 1).sum(axis=1, keepdims=True)
    np.testing.assert_allclose(g1, g0 * mass, rtol=0, atol=tol)
    _, gE0, _ = orc.route(x, rw, E, prec)
    _, gE1, _ = orc.route(x, rw, E, prec, gate_mode=orc.GATE_SOFTMAX_ALL)
    np.testing.assert_allclose(gE1, gE0, rtol=0, atol=tol)
    rw2 = _bf16(rng.normal(0, 0.6, (2, d)))
    ids2, g2, l2 = orc.route(x, rw2, 1, prec, gate_mode=orc.GATE_SOFTMAX_ALL)
    np.testing.assert_allclose(g2[:, 0], 1.0 / (1.0 + np.exp(-np.abs(l2[:, 0] - l2[:, 1]))), rtol=0, atol=tol)


@pytest.mark.parametrize("prec", PRECS)
def test_softmax_all_layer_scales_each_token_by_its_pick_mass(prec):
    """The layer with the other gate rule = the renormalised layer with every token's routed sum scaled by the mass of
    its picks (shared experts are not gated, so they are left out here)."""
    from scipy.special import softmax
    d, ffn, E, T, k = 24, 40, 6, 4, 2
    W, rng = _rand_layer(43, d, ffn, E, sigma=0.2)
    x = rng.normal(size=(T, d)).astype(np.float32)
    out0, ids0, _ = orc.layer(x, W, k, 0, prec)
    out1, ids1, g1 = orc.layer(x, W, k, 0, prec, gate_mode=orc.GATE_SOFTMAX_ALL)
    np.testing.assert_array_equal(ids0, ids1)
    _, _, logits = orc.route(x, W["router_w"], k, "f64")
    mass = np.take_along_axis(softmax(logits, axis=1), ids1, 1).sum(axis=1, keepdims=True)
    np.testing.assert_allclose(out1, out0 * mass, rtol=2e-5 if prec == "f32" else 1e-6, atol=1e-6)
