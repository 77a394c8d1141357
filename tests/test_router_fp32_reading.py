"""The router's integer decision under the other possible reading of "fp32 router logits".

The oracle (and the HIP router) accumulate the logits in fp64, where an fp32 activation times a bf16 weight is exact,
so that the top-k decision does not depend on the order of summation.  A plain fp32 accumulator — one running sum,
j ascending, product and sum each rounded to fp32, no fused multiply-add — is the other reading.  This file recomputes
the logits that way in numpy (outside oracle/) and checks that the picks, their order and hence the expert unions are
IDENTICAL on every seeded input that a reported result rests on: the benchmark's timed steps, its latency-vs-K
sample and its oracle sample on the Mixtral-shaped layer, the same for the two fine-grained shapes, and the seeded
layer-steps of the GPU parity tests.  So the choice of reading changes no reported number."""
import numpy as np
import pytest

from oracle import moe_oracle as orc
from paper_2506_20675_amd import synth


def _bf16_to_f32(bits):
    return (bits.astype(np.uint32) << 16).view(np.float32)


def _logits_fp32_sequential(x, rw_bits):
    """logit[t, e] with ONE fp32 accumulator per (t, e), j ascending; numpy float32 ops round after every operation."""
    w = _bf16_to_f32(rw_bits)
    acc = np.zeros((x.shape[0], w.shape[0]), dtype=np.float32)
    for j in range(x.shape[1]):
        acc = acc + x[:, j, None] * w[None, :, j]
    return acc


def _topk_lower_index_wins(logits, k):
    return np.argsort(-logits, axis=1, kind="stable")[:, :k].astype(np.int32)


def _router(cfg, layer):
    return synth.normal_bf16(synth.weight_key(cfg, layer, synth.T_ROUTER), synth.SIGMA_ROUTER,
                             cfg.n_experts * cfg.d).reshape(cfg.n_experts, cfg.d)


def _check(cfg, draws):
    """draws: (layer, iteration, T, rho).  All tokens of one layer go through the sequential sum together."""
    by_layer = {}
    for layer, it, T, rho in draws:
        by_layer.setdefault(layer, []).append(synth.hidden_host(cfg, layer, it, T, rho))
    n_tok, min_gap = 0, np.inf
    for layer, xs in by_layer.items():
        rw = _router(cfg, layer)
        x = np.concatenate(xs)
        l32 = _logits_fp32_sequential(x, rw)
        ids64, _, l64 = orc.route(x, rw, cfg.top_k, "f64")
        np.testing.assert_array_equal(_topk_lower_index_wins(l32, cfg.top_k), ids64,
                                      err_msg=f"{cfg.name} layer {layer}: fp32 and fp64 accumulation pick different experts")
        assert np.abs(l32 - l64).max() < 1e-4                 # the two sums differ by rounding only
        srt = np.sort(l64, axis=1)[:, ::-1][:, :cfg.top_k + 1]
        min_gap = min(min_gap, np.abs(np.diff(srt, axis=1)).min())
        n_tok += x.shape[0]
    return n_tok, min_gap


def _bench_draws(L, rho=0.5, steps=180, warmup=18):
    timed = [(i % L, i, i % 9 + 1, rho) for i in range(warmup + steps)]                       # bench.py's step(i)
    by_k = [(j % L, 50_000 + 100 * k + j, k + 1, rho) for k in range(9) for j in range(20)]   # its latency-vs-K sample
    cpu = [(0, 10_000 + n, T, rho) for n, T in enumerate(tuple(range(1, 10)) + (9,))]         # its oracle sample
    return timed + by_k + cpu


def test_mixtral_bench_inputs_route_the_same_under_fp32_accumulation():
    n, gap = _check(synth.MIXTRAL, _bench_draws(8) + _bench_draws(8, steps=20, warmup=5))
    assert n > 2000 and gap > 1e-4           # far above the ~1e-5 the two sums can differ by


@pytest.mark.parametrize("cfg", [synth.OLMOE, synth.DEEPSEEK], ids=lambda c: c.name)
def test_fine_grained_bench_inputs_route_the_same_under_fp32_accumulation(cfg):
    n, _ = _check(cfg, _bench_draws(16))
    assert n > 1000


def test_gpu_parity_inputs_route_the_same_under_fp32_accumulation():
    T_rho = ((1, 0.5), (2, 0.0), (5, 0.9), (9, 0.0), (9, 0.5), (9, 0.9))
    for cfg in (synth.TINY, synth.OLMOE, synth.DEEPSEEK, synth.MIXTRAL):                       # router parity
        _check(cfg, [(0, 100 + it, T, rho) for it, (T, rho) in enumerate(T_rho)])
    _check(synth.MIXTRAL, [(0, 300, 1, 0.5), (0, 301, 9, 0.0), (0, 302, 4, 0.5), (0, 303, 8, 0.9), (0, 500, 1, 0.5), (0, 501, 5, 0.0)])   # full size, bf16 and FP8
    for cfg in (synth.OLMOE, synth.DEEPSEEK):
        _check(cfg, [(1, 200, 1, 0.5), (1, 201, 4, 0.0), (1, 202, 9, 0.9), (1, 400, 1, 0.5), (1, 401, 9, 0.9)])
    for cfg in (synth.PHI35, synth.QWEN15):
        _check(cfg, [(1, 600, 1, 0.5), (1, 601, 8, 0.0), (1, 602, 9, 0.9)])
    tiny = [(0, T, T, 0.5) for T in (1, 2, 3, 5, 9)] + [(0, 60 + T, T, 0.5) for T in (1, 5, 9, 16)]
    tiny += [(0, 40 + T, T, 0.5) for T in (1, 3, 9)] + [(2, 5, 9, 0.5), (0, 0, 3, 0.5)]
    tiny += [(10 + l, 0, 4, 0.5) for l in range(3)] + [(6, 0, 1, 0.5)] + [(12, it, T, 0.5) for it, T in enumerate((1, 4, 9))]
    _check(synth.TINY, tiny)
    _check(synth.MIXTRAL, [(l, 700, 9, 0.5) for l in range(32)])                                # the 32-layer stack test
