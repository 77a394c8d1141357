"""Seeded synthetic inputs for the MoE verification path (test/bench infrastructure).

This module holds NO arithmetic of the method itself (no routing, no FFN, no
utility).  It only produces the workload: bf16 weight tensors, fp32 hidden
states with a tunable token-to-token correlation, and the draft-acceptance
trace that stands in for a drafter + rejection sampler.  Both the CPU oracle's
tests and the HIP path's tests/bench draw their inputs from here so that the two
sides see bit-identical data while sharing none of the method's code.

Everything is a pure function of (BASE_SEED, integer fields...) through a
counter-based generator (the splitmix64 output function applied to
key + (counter+1)*GOLDEN), so any tensor, or any slice of one, can be
regenerated anywhere.  bf16 weights use integer-only steps after a one-off
table build (hash -> 16-bit index -> table of bf16 normal quantiles), which is
what lets the device fill kernel in csrc/synth_fill.hip reproduce the host
values bit for bit without trusting device transcendentals.

Shapes follow the paper's Table 1 (hidden size, expert count, top-k, shared
experts); value distributions follow the benchmark recipe: expert weights
~N(0, 0.02^2), router weights ~N(0, 0.05^2), hidden x_t = sqrt(rho) z_shared +
sqrt(1-rho) z_t with z ~ N(0,1), where rho stands in for the expert affinity of
consecutive tokens discussed in Section 2.4 of the paper.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from functools import lru_cache

import numpy as np

BASE_SEED = 20675
_MASK = (1 << 64) - 1
GOLDEN = 0x9E3779B97F4A7C15
_M1 = 0xBF58476D1CE4E5B9
_M2 = 0x94D049BB133111EB

# tensor ids (one random stream per tensor)
T_ROUTER, T_W1, T_W3, T_W2, T_SW1, T_SW3, T_SW2 = 1, 2, 3, 4, 5, 6, 7
T_Z_SHARED, T_Z_TOKEN, T_ACCEPT, T_REGIME = 8, 9, 10, 11
# FP8 variants of the expert tensors: code streams and per-row scale streams
T_Q = {"q1": 12, "q3": 13, "q2": 14, "sq1": 15, "sq3": 16, "sq2": 17}
T_S = {"s1": 18, "s3": 19, "s2": 20, "ss1": 21, "ss3": 22, "ss2": 23}
T_GAMMA = 24   # RMSNorm weight of the block in front of a layer (chained stack)
T_WQKV, T_WO, T_GAMMA_ATTN = 25, 26, 27   # attention stub of the decoder block

SIGMA_EXPERT = 0.02
SIGMA_ROUTER = 0.05


@dataclass(frozen=True)
class MoEConfig:
    """Geometry of one synthetic MoE layer."""
    name: str
    config_id: int
    d: int
    ffn: int
    n_experts: int
    top_k: int
    n_shared: int = 0
    gate_mode: int = 0   # 0: softmax over the picked logits; 1: softmax over all experts, picks not renormalised

    @property
    def expert_bytes(self) -> int:
        return 3 * self.d * self.ffn * 2

    @property
    def expert_bytes_fp8(self) -> int:
        return 3 * self.d * self.ffn


# The four single-layer workloads; the 32-layer stack reuses MIXTRAL with layer = 0..31.
TINY = MoEConfig("tiny", 1, 512, 1024, 8, 2, 0)
MIXTRAL = MoEConfig("mixtral-8x7b-shaped", 2, 4096, 14336, 8, 2, 0)
OLMOE = MoEConfig("olmoe-like", 3, 2048, 1024, 64, 8, 0)
DEEPSEEK = MoEConfig("deepseek-v2-lite-like", 4, 2048, 1408, 64, 6, 2)
# The two remaining rows of the paper's Table 1 (expert count, top-k, shared experts, hidden size from the table;
# the expert intermediate sizes are not in the paper and are taken from the public model cards: 6400 and 1408).
PHI35 = MoEConfig("phi-3.5-moe-like", 6, 4096, 6400, 16, 2, 0)
QWEN15 = MoEConfig("qwen1.5-moe-like", 7, 2048, 1408, 60, 4, 4, gate_mode=1)
CONFIGS = {c.name: c for c in (TINY, MIXTRAL, OLMOE, DEEPSEEK, PHI35, QWEN15)}


# ----------------------------------------------------------------------------
# counter-based generator
# ----------------------------------------------------------------------------
def _mix_int(z: int) -> int:
    z &= _MASK
    z = ((z ^ (z >> 30)) * _M1) & _MASK
    z = ((z ^ (z >> 27)) * _M2) & _MASK
    return z ^ (z >> 31)


def stream_key(*fields: int, base: int = BASE_SEED) -> int:
    """Fold integer fields (config id, layer, tensor id, iteration, ...) into a 64-bit stream key."""
    k = _mix_int(base + GOLDEN)
    for f in fields:
        k = _mix_int((k ^ _mix_int((int(f) + GOLDEN) & _MASK)) + GOLDEN)
    return k


def _mix_arr(z: np.ndarray) -> np.ndarray:
    z = z.copy()
    z ^= z >> np.uint64(30)
    z *= np.uint64(_M1)
    z ^= z >> np.uint64(27)
    z *= np.uint64(_M2)
    z ^= z >> np.uint64(31)
    return z


def hash_blocks(key: int, first_block: int, n_blocks: int) -> np.ndarray:
    """64-bit hashes for counters first_block .. first_block+n_blocks-1 of stream `key`."""
    with np.errstate(over="ignore"):
        ctr = np.arange(first_block + 1, first_block + n_blocks + 1, dtype=np.uint64)
        ctr *= np.uint64(GOLDEN)
        ctr += np.uint64(key)
        return _mix_arr(ctr)


def uniforms(key: int, n: int, first: int = 0) -> np.ndarray:
    """fp64 uniforms in the open interval (0, 1)."""
    h = hash_blocks(key, first, n)
    return ((h >> np.uint64(11)).astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


def std_normal(key: int, n: int) -> np.ndarray:
    """fp64 N(0,1) draws (host only): Box-Muller on two counter-based uniforms per value."""
    u = uniforms(key, 2 * n)
    return np.sqrt(-2.0 * np.log(u[0::2])) * np.cos(2.0 * np.pi * u[1::2])


# ----------------------------------------------------------------------------
# bf16 helpers (storage format only)
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


@lru_cache(maxsize=8)
def normal_table_bf16(sigma: float) -> np.ndarray:
    """65536 equiprobable N(0, sigma^2) quantile mid-points, rounded to bf16 bits.

    Indexing this table with 16 hash bits gives a 65536-level discretised normal
    (tails end at +-4.32 sigma) — indistinguishable from a true normal once the
    value has only bf16's 8 significant bits, and exactly reproducible on device.
    """
    from scipy.special import ndtri
    z = ndtri((np.arange(65536, dtype=np.float64) + 0.5) / 65536.0)
    return f32_to_bf16_bits((sigma * z).astype(np.float32))


def normal_bf16(key: int, sigma: float, count: int, start: int = 0, force_numpy: bool = False) -> np.ndarray:
    """`count` bf16 values (uint16 bits) of stream `key`, elements start .. start+count-1.

    Element i uses 16-bit field (i % 4) of the hash of counter i // 4.  Large requests go through
    the threaded C twin of this loop when the generator library is built (same integers; a test
    checks the two against each other); the numpy code below is the definition.
    """
    table = normal_table_bf16(sigma)
    if not force_numpy and count >= (1 << 16) and os.path.exists(synth_lib_path()):
        lib = _load_synth_lib()
        lo = start % 4
        buf = np.empty(count + lo, dtype=np.uint16)
        rc = lib.synth_fill_bf16_host(buf.ctypes.data_as(ctypes.c_void_p), ctypes.c_uint64(key),
                                      ctypes.c_uint64(start - lo), ctypes.c_uint64(count + lo),
                                      table.ctypes.data_as(ctypes.c_void_p), min(16, os.cpu_count() or 1))
        if rc != 0:
            raise RuntimeError("synth_fill_bf16_host failed")
        return buf[lo:]
    b0 = start // 4
    b1 = (start + count + 3) // 4
    out = np.empty((b1 - b0) * 4, dtype=np.uint16)
    step = 1 << 24  # blocks per chunk: bounds temporaries to ~128 MiB
    for s in range(b0, b1, step):
        n = min(step, b1 - s)
        h = hash_blocks(key, s, n)
        idx = h.view(np.uint16).reshape(n, 4)  # little-endian: field j = bits 16j..16j+15
        out[(s - b0) * 4:(s - b0 + n) * 4] = table[idx.reshape(-1)]
    lo = start - b0 * 4
    return out[lo:lo + count]


# ----------------------------------------------------------------------------
# layer tensors
# ----------------------------------------------------------------------------
def weight_spec(cfg: MoEConfig):
    """(name, tensor id, shape, sigma) of every weight tensor of a layer."""
    spec = [
        ("router_w", T_ROUTER, (cfg.n_experts, cfg.d), SIGMA_ROUTER),
        ("w1", T_W1, (cfg.n_experts, cfg.ffn, cfg.d), SIGMA_EXPERT),
        ("w3", T_W3, (cfg.n_experts, cfg.ffn, cfg.d), SIGMA_EXPERT),
        ("w2", T_W2, (cfg.n_experts, cfg.d, cfg.ffn), SIGMA_EXPERT),
    ]
    if cfg.n_shared:
        spec += [
            ("sw1", T_SW1, (cfg.n_shared, cfg.ffn, cfg.d), SIGMA_EXPERT),
            ("sw3", T_SW3, (cfg.n_shared, cfg.ffn, cfg.d), SIGMA_EXPERT),
            ("sw2", T_SW2, (cfg.n_shared, cfg.d, cfg.ffn), SIGMA_EXPERT),
        ]
    return spec


def weight_key(cfg: MoEConfig, layer: int, tensor_id: int) -> int:
    return stream_key(cfg.config_id, layer, tensor_id)


def layer_weights_host(cfg: MoEConfig, layer: int = 0) -> dict:
    """All weight tensors of one layer as uint16 (bf16 bit patterns) numpy arrays, row-major."""
    out = {}
    for name, tid, shape, sigma in weight_spec(cfg):
        n = int(np.prod(shape))
        out[name] = normal_bf16(weight_key(cfg, layer, tid), sigma, n).reshape(shape)
    return out


# ----------------------------------------------------------------------------
# FP8 (E4M3) expert weights: 8-bit codes + one fp32 scale per output channel (storage format only)
# ----------------------------------------------------------------------------
E4M3_MAX = 448.0


@lru_cache(maxsize=1)
def e4m3_grid() -> np.ndarray:
    """Value of each of the 256 E4M3 codes (sign, 4 exponent bits biased by 7, 3 mantissa bits, no
    infinities, S.1111.111 = NaN).  Used only to pick codes for synthetic weights."""
    c = np.arange(256)
    ex, man = (c >> 3) & 15, c & 7
    mag = np.where(ex == 0, man / 8.0 * 2.0 ** -6, (1.0 + man / 8.0) * 2.0 ** (ex - 7.0))
    mag = np.where((ex == 15) & (man == 7), np.nan, mag)
    return np.where(c >= 128, -mag, mag)


@lru_cache(maxsize=1)
def code_table_e4m3() -> np.ndarray:
    """65536 E4M3 codes: the equiprobable N(0,1) quantile mid-points, stretched so that the outermost one
    (4.32 sigma) lands on the largest finite value 448, each replaced by the nearest finite code."""
    from scipy.special import ndtri
    z = ndtri((np.arange(65536, dtype=np.float64) + 0.5) / 65536.0)
    target = z * (E4M3_MAX / z[-1])
    grid = e4m3_grid()
    finite = np.flatnonzero(~np.isnan(grid) & ~((grid == 0) & (np.arange(256) >= 128)))  # drop NaNs and -0
    order = finite[np.argsort(grid[finite], kind="stable")]
    vals = grid[order]
    hi = np.clip(np.searchsorted(vals, target), 1, len(vals) - 1)
    lo = hi - 1
    pick = np.where(np.abs(target - vals[lo]) <= np.abs(vals[hi] - target), lo, hi)
    return order[pick].astype(np.uint8)


def codes_e4m3(key: int, count: int, start: int = 0, force_numpy: bool = False) -> np.ndarray:
    """`count` E4M3 codes (uint8) of stream `key`, elements start .. start+count-1: element i is
    code_table_e4m3()[16-bit field (i % 4) of the hash of counter i // 4] — the same walk as normal_bf16."""
    table = code_table_e4m3()
    if not force_numpy and count >= (1 << 16) and os.path.exists(synth_lib_path()):
        lib = _load_synth_lib()
        lo = start % 4
        buf = np.empty(count + lo, dtype=np.uint8)
        rc = lib.synth_fill_u8_host(buf.ctypes.data_as(ctypes.c_void_p), ctypes.c_uint64(key),
                                    ctypes.c_uint64(start - lo), ctypes.c_uint64(count + lo),
                                    table.ctypes.data_as(ctypes.c_void_p), min(16, os.cpu_count() or 1))
        if rc != 0:
            raise RuntimeError("synth_fill_u8_host failed")
        return buf[lo:]
    b0 = start // 4
    b1 = (start + count + 3) // 4
    out = np.empty((b1 - b0) * 4, dtype=np.uint8)
    step = 1 << 24
    for s in range(b0, b1, step):
        n = min(step, b1 - s)
        h = hash_blocks(key, s, n)
        idx = h.view(np.uint16).reshape(n, 4)
        out[(s - b0) * 4:(s - b0 + n) * 4] = table[idx.reshape(-1)]
    lo = start - b0 * 4
    return out[lo:lo + count]


def channel_scales(key: int, rows: int, sigma: float = SIGMA_EXPERT) -> np.ndarray:
    """One fp32 scale per output channel: the value that maps code magnitude 448 to 4.32 sigma, times a
    per-row factor uniform in [0.75, 1.25) (rows of a real checkpoint do not share one scale)."""
    u = uniforms(key, rows)
    base = sigma * 4.32 / E4M3_MAX
    return (base * (0.75 + 0.5 * u)).astype(np.float32)


def fp8_weight_spec(cfg: MoEConfig):
    """(code tensor, scale tensor, code shape) of every FP8 expert tensor of a layer."""
    spec = [("q1", "s1", (cfg.n_experts, cfg.ffn, cfg.d)), ("q3", "s3", (cfg.n_experts, cfg.ffn, cfg.d)),
            ("q2", "s2", (cfg.n_experts, cfg.d, cfg.ffn))]
    if cfg.n_shared:
        spec += [("sq1", "ss1", (cfg.n_shared, cfg.ffn, cfg.d)), ("sq3", "ss3", (cfg.n_shared, cfg.ffn, cfg.d)),
                 ("sq2", "ss2", (cfg.n_shared, cfg.d, cfg.ffn))]
    return spec


def layer_weights_fp8_host(cfg: MoEConfig, layer: int = 0) -> dict:
    """FP8 layer: router_w as in layer_weights_host (bf16 bits); q* uint8 codes, row-major; s* fp32 [.., rows]."""
    out = {"router_w": normal_bf16(weight_key(cfg, layer, T_ROUTER), SIGMA_ROUTER,
                                   cfg.n_experts * cfg.d).reshape(cfg.n_experts, cfg.d)}
    for qn, sn, shape in fp8_weight_spec(cfg):
        out[qn] = codes_e4m3(weight_key(cfg, layer, T_Q[qn]), int(np.prod(shape))).reshape(shape)
        out[sn] = channel_scales(weight_key(cfg, layer, T_S[sn]), shape[0] * shape[1]).reshape(shape[:2])
    return out


def norm_gamma_host(cfg: MoEConfig, layer: int) -> np.ndarray:
    """RMSNorm weight gamma[d] of the block in front of `layer`, bf16 bits: 1 + 0.1 z (trained norms sit near 1)."""
    z = bf16_bits_to_f32(normal_bf16(weight_key(cfg, layer, T_GAMMA), 0.1, cfg.d, force_numpy=True))
    return f32_to_bf16_bits(np.float32(1.0) + z)


def attn_geometry(cfg: MoEConfig):
    """(query heads, kv heads, head dim) of the attention stub: head dim 128, hidden/128 query heads, a quarter as
    many kv heads (the grouped-query shape of the Mixtral family: 32 / 8 / 128 at hidden 4096)."""
    dh = 128 if cfg.d % 128 == 0 else 64
    H = cfg.d // dh
    return H, max(1, H // 4), dh


def attn_weights_host(cfg: MoEConfig, layer: int) -> dict:
    """Attention stub weights of block `layer`: wqkv [(H + 2 Hkv) dh, d], wo [d, H dh] ~ N(0, 0.02^2) bf16 bits, the
    two norm weights, and the geometry."""
    H, Hkv, dh = attn_geometry(cfg)
    nq, nout = H * dh, (H + 2 * Hkv) * dh
    g = bf16_bits_to_f32(normal_bf16(weight_key(cfg, layer, T_GAMMA_ATTN), 0.1, cfg.d, force_numpy=True))
    return {"wqkv": normal_bf16(weight_key(cfg, layer, T_WQKV), SIGMA_EXPERT, nout * cfg.d).reshape(nout, cfg.d),
            "wo": normal_bf16(weight_key(cfg, layer, T_WO), SIGMA_EXPERT, cfg.d * nq).reshape(cfg.d, nq),
            "gamma_attn": f32_to_bf16_bits(np.float32(1.0) + g), "gamma_moe": norm_gamma_host(cfg, layer),
            "n_heads": H, "n_kv_heads": Hkv, "head_dim": dh}


def hidden_host(cfg: MoEConfig, layer: int, iteration: int, T: int, rho: float) -> np.ndarray:
    """hidden[T, d] fp32.  Row t does not depend on T (nested K sweeps see nested inputs)."""
    d = cfg.d
    zs = std_normal(stream_key(cfg.config_id, layer, T_Z_SHARED, iteration), d)
    x = np.empty((T, d), dtype=np.float32)
    a, b = np.sqrt(rho), np.sqrt(1.0 - rho)
    for t in range(T):
        zt = std_normal(stream_key(cfg.config_id, layer, T_Z_TOKEN, iteration, t), d)
        x[t] = (a * zs + b * zt).astype(np.float32)
    return x


# ----------------------------------------------------------------------------
# draft acceptance trace (stand-in for drafter + rejection sampler)
# ----------------------------------------------------------------------------
ACCEPT_RATES = (0.1, 0.4, 0.8)
REGIME_PERIOD = 50
K_MAX = 8


def regime_sequence(n_iter: int, seed_field: int = 0, rates=ACCEPT_RATES, period: int = REGIME_PERIOD) -> np.ndarray:
    """Per-iteration mean acceptance rate: held for `period` iterations, then switches
    uniformly to one of the other rates."""
    n_reg = (n_iter + period - 1) // period
    u = uniforms(stream_key(5, seed_field, T_REGIME), n_reg)
    idx = np.empty(n_reg, dtype=np.int64)
    idx[0] = min(int(u[0] * len(rates)), len(rates) - 1)
    for r in range(1, n_reg):
        step = 1 + min(int(u[r] * (len(rates) - 1)), len(rates) - 2)
        idx[r] = (idx[r - 1] + step) % len(rates)
    return np.repeat(np.asarray(rates, dtype=np.float64)[idx], period)[:n_iter]


def acceptance_uniforms(n_iter: int, seed_field: int = 0, k_max: int = K_MAX) -> np.ndarray:
    """u[n_iter, k_max]: draft j of iteration i is individually correct iff u[i, j] < p_i."""
    return uniforms(stream_key(5, seed_field, T_ACCEPT), n_iter * k_max).reshape(n_iter, k_max)


def tokens_emitted(u_row: np.ndarray, p: float, K: int) -> int:
    """1 + number of leading correct drafts among the first K (causal acceptance, Section 2.2 / 5.4)."""
    a = 0
    while a < K and u_row[a] < p:
        a += 1
    return 1 + a


# ----------------------------------------------------------------------------
# device fill (bit-identical to normal_bf16) — separate tiny library, not the product .so
# ----------------------------------------------------------------------------
_SYNTH_LIB = None


def synth_lib_path() -> str:
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), "libmoe_synth.so")


def _load_synth_lib():
    global _SYNTH_LIB
    if _SYNTH_LIB is None:
        path = synth_lib_path()
        if not os.path.exists(path):
            raise RuntimeError(f"{path} not built; run `python -c 'import __graft_entry__ as g; g.build()'`")
        import torch  # noqa: F401  (one HIP runtime per process: let torch load its copy first)
        lib = ctypes.CDLL(path)
        lib.synth_fill_bf16.restype = ctypes.c_int
        lib.synth_fill_bf16.argtypes = [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint64, ctypes.c_uint64,
                                        ctypes.c_void_p, ctypes.c_void_p]
        lib.synth_fill_bf16_host.restype = ctypes.c_int
        lib.synth_fill_bf16_host.argtypes = [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint64, ctypes.c_uint64,
                                             ctypes.c_void_p, ctypes.c_int]
        lib.synth_fill_u8.restype = ctypes.c_int
        lib.synth_fill_u8.argtypes = lib.synth_fill_bf16.argtypes
        lib.synth_fill_u8_host.restype = ctypes.c_int
        lib.synth_fill_u8_host.argtypes = lib.synth_fill_bf16_host.argtypes
        _SYNTH_LIB = lib
    return _SYNTH_LIB


_DEV_TABLES = {}


def fill_normal_bf16_device(dst, key: int, sigma: float, start: int = 0, stream_ptr: int = 0) -> None:
    """Fill a contiguous torch int16/uint16/bfloat16 CUDA tensor with elements start.. of stream `key`."""
    import torch
    assert dst.is_cuda and dst.is_contiguous() and dst.element_size() == 2
    lib = _load_synth_lib()
    tkey = (float(sigma), dst.device.index)
    if tkey not in _DEV_TABLES:
        tab = torch.from_numpy(normal_table_bf16(sigma).view(np.int16).copy()).to(dst.device)
        _DEV_TABLES[tkey] = tab
    tab = _DEV_TABLES[tkey]
    if stream_ptr == 0:
        stream_ptr = torch.cuda.current_stream(dst.device).cuda_stream
    rc = lib.synth_fill_bf16(ctypes.c_void_p(dst.data_ptr()), ctypes.c_uint64(key), ctypes.c_uint64(start),
                             ctypes.c_uint64(dst.numel()), ctypes.c_void_p(tab.data_ptr()),
                             ctypes.c_void_p(stream_ptr))
    if rc != 0:
        raise RuntimeError(f"synth_fill_bf16 failed with HIP error {rc}")


def layer_weights_device(cfg: MoEConfig, layer: int, device="cuda:0") -> dict:
    """Same tensors as layer_weights_host, generated directly in HBM (int16 storage of bf16 bits)."""
    import torch
    out = {}
    for name, tid, shape, sigma in weight_spec(cfg):
        t = torch.empty(shape, dtype=torch.int16, device=device)
        fill_normal_bf16_device(t, weight_key(cfg, layer, tid), sigma)
        out[name] = t
    return out


def fill_codes_e4m3_device(dst, key: int, start: int = 0, stream_ptr: int = 0) -> None:
    """Fill a contiguous torch uint8 CUDA tensor with elements start.. of code stream `key`."""
    import torch
    assert dst.is_cuda and dst.is_contiguous() and dst.element_size() == 1
    lib = _load_synth_lib()
    tkey = ("e4m3", dst.device.index)
    if tkey not in _DEV_TABLES:
        _DEV_TABLES[tkey] = torch.from_numpy(code_table_e4m3().copy()).to(dst.device)
    tab = _DEV_TABLES[tkey]
    if stream_ptr == 0:
        stream_ptr = torch.cuda.current_stream(dst.device).cuda_stream
    rc = lib.synth_fill_u8(ctypes.c_void_p(dst.data_ptr()), ctypes.c_uint64(key), ctypes.c_uint64(start),
                           ctypes.c_uint64(dst.numel()), ctypes.c_void_p(tab.data_ptr()), ctypes.c_void_p(stream_ptr))
    if rc != 0:
        raise RuntimeError(f"synth_fill_u8 failed with HIP error {rc}")


def layer_weights_fp8_device(cfg: MoEConfig, layer: int, device="cuda:0") -> dict:
    """Same tensors as layer_weights_fp8_host: codes generated directly in HBM, scales and router uploaded."""
    import torch
    rw = torch.empty((cfg.n_experts, cfg.d), dtype=torch.int16, device=device)
    fill_normal_bf16_device(rw, weight_key(cfg, layer, T_ROUTER), SIGMA_ROUTER)
    out = {"router_w": rw}
    for qn, sn, shape in fp8_weight_spec(cfg):
        t = torch.empty(shape, dtype=torch.uint8, device=device)
        fill_codes_e4m3_device(t, weight_key(cfg, layer, T_Q[qn]))
        out[qn] = t
        sc = channel_scales(weight_key(cfg, layer, T_S[sn]), shape[0] * shape[1]).reshape(shape[:2])
        out[sn] = torch.from_numpy(sc).to(device)
    return out
