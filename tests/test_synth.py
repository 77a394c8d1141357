"""Host-side checks of the seeded input generator (no GPU)."""
import numpy as np

from paper_2506_20675_amd import synth


def test_streams_are_deterministic_and_sliceable():
    key = synth.stream_key(2, 7, synth.T_W1)
    a = synth.normal_bf16(key, 0.02, 10_000)
    b = synth.normal_bf16(key, 0.02, 10_000)
    assert (a == b).all()
    for start, count in ((0, 17), (4, 100), (6, 33), (9999, 1), (1023, 4097)):
        assert (synth.normal_bf16(key, 0.02, count, start) == a[start:start + count]).all()
    other = synth.normal_bf16(synth.stream_key(2, 7, synth.T_W3), 0.02, 10_000)
    assert (a != other).mean() > 0.9


def test_threaded_c_twin_equals_numpy_definition():
    key = synth.stream_key(3, 1, synth.T_W3)
    for count, start in ((1 << 17, 0), ((1 << 17) + 3, 8), (100_001, 6), (70_000, 1)):
        a = synth.normal_bf16(key, 0.02, count, start)
        b = synth.normal_bf16(key, 0.02, count, start, force_numpy=True)
        assert a.shape == b.shape and (a == b).all()


def test_weight_distribution():
    w = synth.bf16_bits_to_f32(synth.normal_bf16(synth.stream_key(1, 0, synth.T_W2), 0.02, 400_000)).astype(np.float64)
    assert abs(w.mean()) < 2e-4
    assert abs(w.std() - 0.02) < 3e-4
    assert abs((np.abs(w) < 0.02).mean() - 0.6827) < 0.01
    assert abs((np.abs(w) < 0.04).mean() - 0.9545) < 0.005
    r = synth.bf16_bits_to_f32(synth.normal_bf16(synth.stream_key(1, 0, synth.T_ROUTER), 0.05, 100_000))
    assert abs(r.std() - 0.05) < 1e-3


def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 2 ** -7, 1.0 + 3 * 2 ** -8, -2.5, 0.0], np.float32)
    bits = synth.f32_to_bf16_bits(x)
    back = synth.bf16_bits_to_f32(bits)
    assert list(back) == [1.0, 1.0, 1.0 + 2 ** -7, 1.0 + 2 ** -6, -2.5, 0.0]   # ties go to the even mantissa


def test_hidden_prefix_property_and_correlation():
    cfg = synth.TINY
    x9 = synth.hidden_host(cfg, 3, 11, 9, 0.5)
    x4 = synth.hidden_host(cfg, 3, 11, 4, 0.5)
    assert (x9[:4] == x4).all()
    assert x9.dtype == np.float32 and x9.shape == (9, cfg.d)
    big = synth.MIXTRAL
    for rho in (0.0, 0.5, 0.9):
        x = synth.hidden_host(big, 0, 0, 6, rho).astype(np.float64)
        assert abs(x.std() - 1.0) < 0.03
        c = np.corrcoef(x)
        off = c[~np.eye(6, dtype=bool)]
        assert abs(off.mean() - rho) < 0.04
    assert (synth.hidden_host(cfg, 0, 0, 3, 0.5) != synth.hidden_host(cfg, 1, 0, 3, 0.5)).any()
    assert (synth.hidden_host(cfg, 0, 0, 3, 0.5) != synth.hidden_host(cfg, 0, 1, 3, 0.5)).any()


def test_layer_weight_shapes():
    W = synth.layer_weights_host(synth.TINY, 0)
    assert W["router_w"].shape == (8, 512) and W["w1"].shape == (8, 1024, 512) and W["w2"].shape == (8, 512, 1024)
    assert all(v.dtype == np.uint16 for v in W.values())
    assert synth.MIXTRAL.expert_bytes == 352_321_536
    assert {c.name for c in synth.CONFIGS.values()} == {"tiny", "mixtral-8x7b-shaped", "olmoe-like", "deepseek-v2-lite-like",
                                                        "phi-3.5-moe-like", "qwen1.5-moe-like"}
    assert len({c.config_id for c in synth.CONFIGS.values()}) == len(synth.CONFIGS)
    assert all(c.d % 64 == 0 and c.ffn % 64 == 0 for c in synth.CONFIGS.values())      # FP8 needs 64-wide steps


def test_regimes_and_causal_acceptance():
    r = synth.regime_sequence(600)
    assert set(np.unique(r)) <= set(synth.ACCEPT_RATES)
    blocks = r.reshape(-1, synth.REGIME_PERIOD)
    assert (blocks == blocks[:, :1]).all()
    assert (np.diff(blocks[:, 0]) != 0).all()            # every switch goes to a different rate
    u = synth.acceptance_uniforms(2000)
    assert u.shape == (2000, synth.K_MAX) and (u > 0).all() and (u < 1).all()
    for p in (0.1, 0.4, 0.8):
        for K in (0, 1, 4, 8):
            tok = np.array([synth.tokens_emitted(u[i], p, K) for i in range(2000)])
            assert tok.min() >= 1 and tok.max() <= K + 1
            expect = (1 - p ** (K + 1)) / (1 - p)            # mean of 1 + leading successes
            assert abs(tok.mean() - expect) < 0.12
    # nested in K: a longer draft never emits fewer tokens on the same iteration
    assert all(synth.tokens_emitted(u[i], 0.8, 8) >= synth.tokens_emitted(u[i], 0.8, 3) for i in range(200))


def test_fp8_code_streams_and_scales():
    """E4M3 code streams: finite codes only, numpy definition == threaded C twin, any slice regenerates, and the
    effective weights scale * value(code) have the bf16 recipe's spread."""
    tab = synth.code_table_e4m3()
    grid = synth.e4m3_grid()
    assert tab.dtype == np.uint8 and tab.shape == (65536,)
    assert not np.isin(tab, (0x7F, 0xFF, 0x80)).any()                  # no NaN code, no negative zero
    assert grid[tab[0]] == -448.0 and grid[tab[-1]] == 448.0
    assert np.all(np.diff(grid[tab]) >= 0)                             # monotone in the quantile index
    key = synth.stream_key(9, 9, 9)
    a = synth.codes_e4m3(key, 70_001, 5, force_numpy=True)
    assert np.array_equal(a[100:200], synth.codes_e4m3(key, 100, 105, force_numpy=True))
    import os
    if os.path.exists(synth.synth_lib_path()):
        assert np.array_equal(a, synth.codes_e4m3(key, 70_001, 5))
    W = synth.layer_weights_fp8_host(synth.TINY, 0)
    assert W["q1"].shape == (8, 1024, 512) and W["s1"].shape == (8, 1024) and W["q2"].shape == (8, 512, 1024)
    assert W["s2"].shape == (8, 512) and W["s1"].dtype == np.float32 and W["q3"].dtype == np.uint8
    assert np.array_equal(W["router_w"], synth.layer_weights_host(synth.TINY, 0)["router_w"])
    w = W["s1"].astype(np.float64)[:, :, None] * grid[W["q1"]]
    assert abs(w.std() - synth.SIGMA_EXPERT) < 0.002 and abs(w.mean()) < 1e-4
    base = synth.SIGMA_EXPERT * 4.32 / 448.0
    assert W["s1"].min() >= 0.75 * base * 0.999 and W["s1"].max() <= 1.25 * base * 1.001
    assert synth.MIXTRAL.expert_bytes_fp8 == 176_160_768
