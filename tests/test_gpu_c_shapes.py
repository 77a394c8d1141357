"""GPU parity, part 3: the gate rule 'softmax over all experts' and the remaining Table 1 shapes.
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from oracle import moe_oracle as orc
from paper_2506_20675_amd import binding, synth
from gpu_common import (_check_layer, _check_out, _dev, _run_layer, _tiled, _weights_dev)


from gpu_common import _check_layer_fp8


@pytest.mark.parametrize("E,k,T,d", [(8, 2, 9, 512), (60, 4, 5, 2048), (256, 16, 3, 96), (3, 3, 2, 64), (16, 1, 16, 1056)])
def test_route_parity_softmax_all_gates(E, k, T, d):
    import torch
    rng = np.random.default_rng(E * 1000 + k * 10 + T)
    x = rng.normal(size=(T, d)).astype(np.float32)
    rw = synth.f32_to_bf16_bits(rng.normal(0, 0.1, (E, d)).astype(np.float32))
    ctx = binding.MoeContext(d, 64, E, k, 0, 16, gate_mode=binding.MOE_GATE_SOFTMAX_ALL)
    ids = torch.full((T, k), -1, dtype=torch.int32, device="cuda")
    gates = torch.zeros((T, k), dtype=torch.float32, device="cuda")
    ctx.moe_route(_dev(x), _dev(rw), ids, gates)
    torch.cuda.synchronize()
    rids, rgates, logits = orc.route(x, rw, k, "f32", orc.GATE_SOFTMAX_ALL)
    srt = np.sort(logits, axis=1)[:, ::-1]
    if E > k:
        assert (srt[:, k - 1] - srt[:, k]).min() > 1e-9
    np.testing.assert_array_equal(ids.cpu().numpy(), rids)
    assert np.abs(gates.cpu().numpy() - rgates).max() <= 1e-5
    if E > k:
        assert (gates.cpu().numpy().sum(axis=1) < 1.0).all()
    ctx.close()


@pytest.mark.parametrize("cfg,weights", [(synth.PHI35, "bf16"), (synth.QWEN15, "bf16"), (synth.QWEN15, "fp8")],
                         ids=lambda v: v if isinstance(v, str) else v.name)
def test_layer_parity_remaining_table1_shapes(cfg, weights):
    """Phi-3.5-like (16 experts, top-2) and Qwen1.5-like (60 routed top-4 + 4 shared, gates = softmax over all experts)."""
    ctx = binding.MoeContext(cfg.d, cfg.ffn, cfg.n_experts, cfg.top_k, cfg.n_shared, 9, gate_mode=cfg.gate_mode)
    W = synth.layer_weights_fp8_host(cfg, 1) if weights == "fp8" else synth.layer_weights_host(cfg, 1)
    Wd = _weights_dev(W)
    for it, (T, rho) in enumerate(((1, 0.5), (8, 0.0), (9, 0.9))):
        x = synth.hidden_host(cfg, 1, 600 + it, T, rho)
        if weights == "fp8":
            _check_layer_fp8(ctx, W, Wd, x, cfg.top_k, cfg.n_shared)
        else:
            _check_layer((cfg.d, cfg.ffn, cfg.n_experts, cfg.top_k, cfg.n_shared), W, x, ctx, Wd, gate_mode=cfg.gate_mode)
    ctx.close()


