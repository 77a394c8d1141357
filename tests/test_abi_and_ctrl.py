"""CPU-side checks of the C-ABI library: it loads, exports every declared symbol, refuses to work
without a GPU, and its host-side controller replays exactly like the policy oracle."""
import math
import os
import re

import numpy as np
import pytest

from oracle import cascade_oracle as co
from paper_2506_20675_amd import binding, synth
from test_cascade_pins import bins_cost

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "cascade_moe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b((?:moe|cascade)_[a-z0-9_]+)\s*\(", text)
    return sorted(set(names))


def test_library_loads_and_exports_every_declared_symbol():
    L = binding.lib()
    declared = _declared_functions()
    assert len(declared) >= 15
    for name in declared:
        assert hasattr(L, name), f"{name} declared in the header but not exported"
    assert sorted(binding.EXPORTS) == declared
    assert L.moe_abi_version() == 2
    assert binding._strerror(0) == "ok" and "shape" in binding._strerror(-2)


def test_no_cpu_fallback_without_gpu():
    import torch
    if torch.cuda.is_available():
        pytest.skip("GPU present")
    with pytest.raises(binding.MoeError) as e:
        binding.MoeContext(512, 1024, 8, 2)
    assert e.value.status == -4       # MOE_ERR_HIP: the product path refuses to run without a device


def test_shape_validation_is_host_side():
    L = binding.lib()
    import ctypes
    h = ctypes.c_void_p()
    for bad, code in (((500, 1024, 8, 2, 0, 9), -2), ((512, 1000, 8, 2, 0, 9), -2), ((512, 1024, 8, 9, 0, 9), -1),
                      ((512, 1024, 300, 2, 0, 9), -2), ((512, 1024, 8, 2, 0, 17), -2), ((512, 1024, 8, 0, 0, 9), -1),
                      ((512, 1024, 8, 2, 9, 9), -2), ((512, 1024, 8, 2, 0, 9, 2), -1)):
        s = binding.MoeShape(*bad)
        assert L.moe_ctx_create(ctypes.byref(s), ctypes.byref(h)) == code
        assert not h.value
    assert L.moe_ctx_create(None, ctypes.byref(h)) == -1


def test_utility_matches_paper_examples_and_oracle():
    assert binding.cascade_utility(1.5, 2.0, 1.0) == 0.75
    assert binding.cascade_utility(1.0, 5.0, 5.0) == 1.0
    assert math.isnan(binding.cascade_utility(1.0, 0.0, 1.0))
    assert math.isnan(binding.cascade_utility(1.0, 1.0, -2.0))
    rng = np.random.default_rng(0)
    for _ in range(200):
        a, b, c = rng.uniform(0.1, 9, 3)
        assert binding.cascade_utility(a, b, c) == co.utility(a, b, c)     # bit-identical doubles


def test_default_params_are_the_papers():
    p = binding.cascade_default_params()
    assert (p.t_trial, p.max_trials, p.s_set, p.k_start, p.base_iters, p.base_refresh) == (4, 4, 16, 3, 4, 100)
    assert p.k_max == 8 and p.converge_frac == 0.10 and p.backoff == 1 and p.hillclimb == 1
    q = co.Params()
    for f in ("t_trial", "max_trials", "s_set", "k_max", "k_start", "base_iters", "base_refresh", "s_max",
              "converge_frac", "backoff", "hillclimb"):
        assert getattr(p, f) == getattr(q, f)


def _replay(seed, n_iter=2500):
    rng = np.random.default_rng(seed)
    kw = dict(t_trial=int(rng.integers(1, 6)), max_trials=int(rng.integers(1, 6)), s_set=int(rng.integers(1, 24)),
              k_max=int(rng.integers(1, 9)), base_iters=int(rng.integers(1, 6)), base_refresh=int(rng.integers(5, 150)),
              s_max=int(rng.choice([0, 64])), backoff=int(rng.integers(0, 3)), hillclimb=int(rng.integers(0, 2)))
    if seed == 0:
        kw = {}
    kw["k_start"] = int(rng.integers(1, kw.get("k_max", 8) + 1)) if seed else 3
    ref = co.Controller(co.Params(**kw))
    dut = binding.CascadeController(**kw)
    regimes = synth.regime_sequence(n_iter, seed)
    u = synth.acceptance_uniforms(n_iter, seed)
    noise = rng.uniform(0.85, 1.15, n_iter)
    for i in range(n_iter):
        k = ref.next_k()
        assert dut.next_k() == k, f"iteration {i}: C controller chose {dut.next_k()}, oracle {k}"
        tok = synth.tokens_emitted(u[i], regimes[i], k)
        t = 3.7e-3 * bins_cost(k) * noise[i]
        ref.observe(k, tok, t)
        dut.observe(k, tok, t)
        st = dut.state()
        assert st.phase == ref.phase and st.s_cur == ref.s_cur and st.iters == ref.iters
        assert st.t_base == ref.t_base or (math.isnan(st.t_base) and math.isnan(ref.t_base))
    assert dut.state().trial_iters == ref.spec_trial_iters


@pytest.mark.parametrize("seed", range(8))
def test_c_controller_replays_like_the_oracle(seed):
    _replay(seed)


def test_c_controller_rejects_bad_observations():
    c = binding.CascadeController()
    for args in ((1, 1, 1.0), (0, 2, 1.0), (0, 0, 1.0), (0, 1, 0.0), (0, 1, float("nan")), (0, 1, float("inf"))):
        with pytest.raises(binding.MoeError):
            c.observe(*args)
    assert c.state().iters == 0
    with pytest.raises(ValueError):
        binding.CascadeController(k_start=9)
    with pytest.raises(ValueError):
        binding.CascadeController(t_trial=0)


def test_header_is_plain_c11_and_structs_match_the_binding(tmp_path):
    """The boundary is a C ABI: the header must compile as C11 on its own, and the ctypes mirrors of its structs must
    have the sizes the C compiler gives them."""
    import ctypes
    import os
    import subprocess
    inc = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include")
    src = tmp_path / "sizes.c"
    src.write_text('#include <stdio.h>\n#include "cascade_moe.h"\n'
                   'int main(void) { printf("%zu %zu %zu %zu %zu\\n", sizeof(moe_shape), sizeof(moe_layer_weights), '
                   'sizeof(moe_attn_weights), sizeof(cascade_params), sizeof(moe_plan_info)); return 0; }\n')
    exe = tmp_path / "sizes"
    subprocess.run(["gcc", "-std=c11", "-pedantic", "-Wall", "-Werror", "-I", inc, str(src), "-o", str(exe)], check=True)
    sizes = [int(v) for v in subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()]
    assert sizes == [ctypes.sizeof(binding.MoeShape), ctypes.sizeof(binding.MoeLayerWeights),
                     ctypes.sizeof(binding.MoeAttnWeights), ctypes.sizeof(binding.CascadeParams),
                     ctypes.sizeof(binding.MoePlanInfo)]


def test_launch_plan_is_host_arithmetic_with_sane_invariants():
    """moe_plan_query needs no device.  For every benchmark shape, weight type and T: the split-K factor is a power of
    two that leaves every wave at least 4 k-steps, the workspace rule (slabs per slot <= 16) holds, tile counts are
    from the instantiated set, the fused down + combine launch is chosen exactly for tiled weights with few tokens in
    flight (T <= 5 with bf16 — 6 where d gives at least 256 row tiles —, T <= 4 with FP8 weights; unions of at most 32
    slots), and the launch count follows from
    the choices."""
    from paper_2506_20675_amd import synth
    seen_fused = seen_split = False
    for cfg in (synth.TINY, synth.MIXTRAL, synth.OLMOE, synth.DEEPSEEK, synth.PHI35, synth.QWEN15):
        for dtype in (binding.MOE_WEIGHT_BF16, binding.MOE_WEIGHT_FP8_E4M3):
            for layout in (binding.MOE_LAYOUT_TILED, binding.MOE_LAYOUT_ROW_MAJOR):
                prev_slots = 0.0
                for T in range(1, 17):
                    p = binding.moe_plan_query(cfg.d, cfg.ffn, cfg.n_experts, cfg.top_k, cfg.n_shared, 16, T, layout, dtype)
                    assert p["routed_slots"] == min(cfg.n_experts, T * cfg.top_k)
                    assert cfg.top_k + cfg.n_shared <= p["expected_slots"] + 1e-9 <= p["routed_slots"] + cfg.n_shared + 1e-9
                    assert p["expected_slots"] > prev_slots            # more tokens in flight, larger union (Section 2.4)
                    prev_slots = p["expected_slots"]
                    assert p["wide_router"] == (cfg.n_experts >= 32) and p["packed_fragments"] == (T <= 8)
                    assert p["gu_tiles"] in (1, 2, 4) and p["dn_tiles"] in (1, 2, 4)
                    ks, nsteps = p["dn_split_k"], cfg.ffn // (64 if dtype else 32)
                    assert 1 <= ks <= 16 and ks & (ks - 1) == 0
                    assert ks == 1 or nsteps // (4 * ks) >= 4
                    want_fused = (layout == binding.MOE_LAYOUT_TILED and p["expected_slots"] <= 32
                                  and T <= (4 if dtype else (6 if cfg.d // 16 >= 256 else 5)))
                    assert (p["dn_fused_chunks"] > 0) == want_fused
                    if p["dn_fused_chunks"] > 0:
                        seen_fused = True
                        assert nsteps // p["dn_fused_chunks"] >= 8 or p["dn_fused_chunks"] == 1   # >= 8 k-steps per item
                    else:
                        seen_split = True
                    router = 2 if (p["wide_router"] or T > 1) else 1
                    assert p["launches"] == router + 1 + (1 if p["dn_fused_chunks"] > 0 else 2)
    assert seen_fused and seen_split
    # the Mixtral-shaped layer without speculation: three launches (router, gate/up, fused down + combine); with
    # eight drafts: five (router, grouping, gate/up, split-K down with four slabs per slot, slab sum)
    p = binding.moe_plan_query(4096, 14336, 8, 2, 0, 9, 1)
    assert (p["launches"], p["dn_fused_chunks"]) == (3, 8)
    p = binding.moe_plan_query(4096, 14336, 8, 2, 0, 9, 9)
    assert (p["launches"], p["dn_split_k"], p["dn_tiles"], p["dn_fused_chunks"]) == (5, 4, 4, 0)
    for bad in (dict(T=0), dict(T=10), dict(layout=7), dict(dtype=5)):
        with pytest.raises(binding.MoeError):
            binding.moe_plan_query(4096, 14336, 8, 2, 0, 9, **{"T": 1, **bad})
    with pytest.raises(binding.MoeError):
        binding.moe_plan_query(4096, 14336 + 32, 8, 2, 0, 9, 1, dtype=binding.MOE_WEIGHT_FP8_E4M3)  # FP8 needs ffn % 64
