"""ctypes front end of oracle/moe_oracle.c — TEST INFRASTRUCTURE, not a product path.

Only tests/, the smoke check and the bench's cpu_baseline leg may import this.
It marshals numpy arrays into the plain C oracle and nothing else; the HIP
library is never imported here.

Two builds of the same C source exist: precision="f32" (the plain fp32 oracle the
parity bar is stated against) and precision="f64" (accuracy reference).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "moe_oracle.c")
_LIBS = {}

_u16p = ctypes.POINTER(ctypes.c_uint16)
_f32p = ctypes.POINTER(ctypes.c_float)
_i32p = ctypes.POINTER(ctypes.c_int32)
_f64p = ctypes.POINTER(ctypes.c_double)
_u8p = ctypes.POINTER(ctypes.c_uint8)


def lib_path(precision: str) -> str:
    return os.path.join(_HERE, f"liboracle_{precision}.so")


def build(force: bool = True) -> None:
    """Compile both precisions with gcc (no fast-math, no contraction: sums stay in source order)."""
    for prec, real in (("f32", "float"), ("f64", "double")):
        out = lib_path(prec)
        if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(_SRC):
            continue
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off", "-fno-fast-math",
               f"-DREAL={real}", _SRC, "-o", out, "-lm"]
        subprocess.run(cmd, check=True)


def _load(path: str, precision: str):
    """dlopen one build of the oracle and declare its signatures."""
    L = ctypes.CDLL(path)
    L.oracle_real_bytes.restype = ctypes.c_int
    L.oracle_route.restype = ctypes.c_int
    L.oracle_route.argtypes = [_f32p, _u16p] + [ctypes.c_int] * 4 + [_i32p, _f32p, _f64p]
    L.oracle_route_softmax_all.restype = ctypes.c_int
    L.oracle_route_softmax_all.argtypes = L.oracle_route.argtypes
    L.oracle_union.restype = ctypes.c_int
    L.oracle_union.argtypes = [_i32p] + [ctypes.c_int] * 3 + [_i32p] * 5
    L.oracle_expert_ffn.restype = None
    L.oracle_expert_ffn.argtypes = [_f32p, _u16p, _u16p, _u16p, ctypes.c_int, ctypes.c_int,
                                    ctypes.c_void_p, ctypes.c_void_p]
    comb = [_f32p] + [ctypes.c_int] * 6 + [_u16p] * 6 + [_i32p, _f32p, _f32p]
    L.oracle_combine.restype = ctypes.c_int
    L.oracle_combine.argtypes = comb
    L.oracle_dense_masked.restype = ctypes.c_int
    L.oracle_dense_masked.argtypes = comb
    L.oracle_layer.restype = ctypes.c_int
    L.oracle_layer.argtypes = [_f32p] + [ctypes.c_int] * 6 + [_u16p] * 7 + [_i32p, _f32p, _f32p]
    L.oracle_rmsnorm.restype = None
    L.oracle_rmsnorm.argtypes = [_f32p, _u16p, ctypes.c_int, ctypes.c_int, ctypes.c_double, _f32p]
    L.oracle_residual_add.restype = None
    L.oracle_residual_add.argtypes = [_f32p, _f32p, ctypes.c_size_t, _f32p]
    L.oracle_attention_stub.restype = ctypes.c_int
    L.oracle_attention_stub.argtypes = [_f32p, _u16p, _u16p] + [ctypes.c_int] * 5 + [_f32p]
    L.oracle_fp8_e4m3_value.restype = ctypes.c_double
    L.oracle_fp8_e4m3_value.argtypes = [ctypes.c_uint8]
    L.oracle_expert_ffn_fp8.restype = None
    L.oracle_expert_ffn_fp8.argtypes = [_f32p, _u8p, _f32p, _u8p, _f32p, _u8p, _f32p, ctypes.c_int, ctypes.c_int,
                                        ctypes.c_void_p, ctypes.c_void_p]
    fp8w = [_u8p] * 3 + [_f32p] * 3 + [_u8p] * 3 + [_f32p] * 3
    L.oracle_combine_fp8.restype = ctypes.c_int
    L.oracle_combine_fp8.argtypes = [_f32p] + [ctypes.c_int] * 6 + fp8w + [_i32p, _f32p, _f32p]
    L.oracle_layer_fp8.restype = ctypes.c_int
    L.oracle_layer_fp8.argtypes = [_f32p] + [ctypes.c_int] * 6 + [_u16p] + fp8w + [_i32p, _f32p, _f32p]
    assert L.oracle_real_bytes() == (4 if precision == "f32" else 8)
    return L


def _lib(precision: str):
    if precision not in ("f32", "f64"):
        raise ValueError(precision)
    if precision not in _LIBS:
        build(force=False)
        _LIBS[precision] = _load(lib_path(precision), precision)
    return _LIBS[precision]


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(_f32p)


def _u16(a):
    if a is None:
        return None, None
    a = np.ascontiguousarray(a)
    if a.dtype != np.uint16:
        a = a.view(np.uint16)
    return a, a.ctypes.data_as(_u16p)


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(_i32p)


GATE_RENORM_TOPK, GATE_SOFTMAX_ALL = 0, 1


def route(hidden, router_w, top_k, precision="f32", gate_mode=GATE_RENORM_TOPK):
    """-> ids[T,top_k] int32, gates[T,top_k] fp32, logits[T,E] fp64.
    gate_mode 0: gates = softmax over the selected logits; 1: softmax over all E logits, picks not renormalised."""
    hidden, hp = _f32(hidden)
    router_w, rp = _u16(router_w)
    T, d = hidden.shape
    E = router_w.shape[0]
    assert router_w.shape == (E, d)
    ids = np.empty((T, top_k), np.int32)
    gates = np.empty((T, top_k), np.float32)
    logits = np.empty((T, E), np.float64)
    if gate_mode not in (GATE_RENORM_TOPK, GATE_SOFTMAX_ALL):
        raise ValueError(gate_mode)
    fn = _lib(precision).oracle_route if gate_mode == GATE_RENORM_TOPK else _lib(precision).oracle_route_softmax_all
    rc = fn(hp, rp, T, d, E, top_k, ids.ctypes.data_as(_i32p), gates.ctypes.data_as(_f32p),
            logits.ctypes.data_as(_f64p))
    if rc:
        raise ValueError("oracle_route: bad sizes")
    return ids, gates, logits


def union(ids, n_experts, precision="f32"):
    """-> dict(unique[E] (-1 padded), n_unique, count[E], offset[E+1], assign[T*top_k])."""
    ids, ip = _i32(ids)
    T, top_k = ids.shape
    E = n_experts
    unique = np.empty(E, np.int32)
    n = np.zeros(1, np.int32)
    count = np.empty(E, np.int32)
    offset = np.empty(E + 1, np.int32)
    assign = np.full(T * top_k, -1, np.int32)
    rc = _lib(precision).oracle_union(ip, T, top_k, E, *(a.ctypes.data_as(_i32p) for a in (unique, n, count, offset, assign)))
    if rc:
        raise ValueError("oracle_union: expert id out of range")
    return dict(unique=unique, n_unique=int(n[0]), count=count, offset=offset, assign=assign)


def expert_ffn(x, w1, w3, w2, precision="f32"):
    """One SwiGLU expert on one token: x[d], w1/w3[ffn,d], w2[d,ffn] (bf16 bits) -> y[d] (fp64 array of REAL values)."""
    x, xp = _f32(x)
    w1, p1 = _u16(w1)
    w3, p3 = _u16(w3)
    w2, p2 = _u16(w2)
    ffn, d = w1.shape
    assert w3.shape == (ffn, d) and w2.shape == (d, ffn) and x.shape == (d,)
    dt = np.float32 if precision == "f32" else np.float64
    h = np.empty(ffn, dt)
    y = np.empty(d, dt)
    _lib(precision).oracle_expert_ffn(xp, p1, p3, p2, d, ffn, h.ctypes.data, y.ctypes.data)
    return y.astype(np.float64), h.astype(np.float64)


def _combine_like(fn_name, hidden, W, ids, gates, top_k, n_shared, precision):
    hidden, hp = _f32(hidden)
    T, d = hidden.shape
    w1, p1 = _u16(W["w1"])
    w3, p3 = _u16(W["w3"])
    w2, p2 = _u16(W["w2"])
    E, ffn, _ = w1.shape
    assert w1.shape == (E, ffn, d) and w3.shape == (E, ffn, d) and w2.shape == (E, d, ffn)
    sw1, q1 = _u16(W.get("sw1") if n_shared else None)
    sw3, q3 = _u16(W.get("sw3") if n_shared else None)
    sw2, q2 = _u16(W.get("sw2") if n_shared else None)
    if n_shared:
        assert sw1.shape == (n_shared, ffn, d) and sw2.shape == (n_shared, d, ffn)
    ids, ip = _i32(ids)
    gates, gp = _f32(gates)
    assert ids.shape == (T, top_k) and gates.shape == (T, top_k)
    out = np.empty((T, d), np.float32)
    fn = getattr(_lib(precision), fn_name)
    rc = fn(hp, T, d, ffn, E, top_k, n_shared, p1, p3, p2, q1, q3, q2, ip, gp, out.ctypes.data_as(_f32p))
    if rc:
        raise ValueError(f"{fn_name}: expert id out of range")
    return out


def combine(hidden, W, ids, gates, n_shared=0, precision="f32"):
    """out[T,d] for a GIVEN routing (ids, gates)."""
    return _combine_like("oracle_combine", hidden, W, ids, gates, np.asarray(ids).shape[1], n_shared, precision)


def dense_masked(hidden, W, ids, gates, n_shared=0, precision="f32"):
    return _combine_like("oracle_dense_masked", hidden, W, ids, gates, np.asarray(ids).shape[1], n_shared, precision)


def layer(hidden, W, top_k, n_shared=0, precision="f32", gate_mode=GATE_RENORM_TOPK):
    """Route + combine.  W: dict with router_w, w1, w3, w2 (and sw1, sw3, sw2).  -> out, ids, gates."""
    if gate_mode != GATE_RENORM_TOPK:      # the other gate rule: its own routing call, then the same combine
        ids, gates, _ = route(hidden, W["router_w"], top_k, precision, gate_mode)
        return combine(hidden, W, ids, gates, n_shared, precision), ids, gates
    hidden, hp = _f32(hidden)
    T, d = hidden.shape
    rw, pr = _u16(W["router_w"])
    w1, p1 = _u16(W["w1"])
    w3, p3 = _u16(W["w3"])
    w2, p2 = _u16(W["w2"])
    E, ffn, _ = w1.shape
    assert rw.shape == (E, d) and w1.shape == (E, ffn, d) and w3.shape == (E, ffn, d) and w2.shape == (E, d, ffn)
    sw1, q1 = _u16(W.get("sw1") if n_shared else None)
    sw3, q3 = _u16(W.get("sw3") if n_shared else None)
    sw2, q2 = _u16(W.get("sw2") if n_shared else None)
    if n_shared:
        assert sw1.shape == (n_shared, ffn, d) and sw3.shape == (n_shared, ffn, d) and sw2.shape == (n_shared, d, ffn)
    ids = np.empty((T, top_k), np.int32)
    gates = np.empty((T, top_k), np.float32)
    out = np.empty((T, d), np.float32)
    rc = _lib(precision).oracle_layer(hp, T, d, ffn, E, top_k, n_shared, pr, p1, p3, p2, q1, q3, q2,
                                      ids.ctypes.data_as(_i32p), gates.ctypes.data_as(_f32p),
                                      out.ctypes.data_as(_f32p))
    if rc:
        raise ValueError("oracle_layer: bad sizes")
    return out, ids, gates


# ---------------------------------------------------------------------------------------------
# FP8 (E4M3 codes + one fp32 scale per output channel) expert weights
# ---------------------------------------------------------------------------------------------
def _u8(a):
    if a is None:
        return None, None
    a = np.ascontiguousarray(a)
    if a.dtype != np.uint8:
        a = a.view(np.uint8)
    return a, a.ctypes.data_as(_u8p)


def _f32n(a):
    if a is None:
        return None, None
    return _f32(a)


def fp8_e4m3_values(codes=None, precision="f64"):
    """Value of each E4M3 code (default: all 256) as fp64; the two NaN codes give NaN."""
    L = _lib(precision)
    codes = np.arange(256, dtype=np.uint8) if codes is None else np.asarray(codes, dtype=np.uint8)
    return np.array([L.oracle_fp8_e4m3_value(int(c)) for c in codes.reshape(-1)], dtype=np.float64).reshape(codes.shape)


def expert_ffn_fp8(x, q1, s1, q3, s3, q2, s2, precision="f32"):
    """One FP8 SwiGLU expert on one token: q1/q3 [ffn,d] codes, s1/s3 [ffn]; q2 [d,ffn], s2 [d] -> y[d], h[ffn]."""
    x, xp = _f32(x)
    q1, p1 = _u8(q1)
    q3, p3 = _u8(q3)
    q2, p2 = _u8(q2)
    s1, c1 = _f32(s1)
    s3, c3 = _f32(s3)
    s2, c2 = _f32(s2)
    ffn, d = q1.shape
    assert q3.shape == (ffn, d) and q2.shape == (d, ffn) and x.shape == (d,)
    assert s1.shape == (ffn,) and s3.shape == (ffn,) and s2.shape == (d,)
    dt = np.float32 if precision == "f32" else np.float64
    h = np.empty(ffn, dt)
    y = np.empty(d, dt)
    _lib(precision).oracle_expert_ffn_fp8(xp, p1, c1, p3, c3, p2, c2, d, ffn, h.ctypes.data, y.ctypes.data)
    return y.astype(np.float64), h.astype(np.float64)


def _fp8_weight_args(W, E, ffn, d, n_shared):
    """Marshal q1,q3,q2,s1,s3,s2 (+ sq*, ss* for shared experts) of a weight dict; returns (keepalive, pointers)."""
    keep, ptrs = [], []
    for name, shape in (("q1", (E, ffn, d)), ("q3", (E, ffn, d)), ("q2", (E, d, ffn))):
        a, p = _u8(W[name])
        assert a.shape == shape, (name, a.shape, shape)
        keep.append(a), ptrs.append(p)
    for name, shape in (("s1", (E, ffn)), ("s3", (E, ffn)), ("s2", (E, d))):
        a, p = _f32(W[name])
        assert a.shape == shape, (name, a.shape, shape)
        keep.append(a), ptrs.append(p)
    for name, shape in (("sq1", (n_shared, ffn, d)), ("sq3", (n_shared, ffn, d)), ("sq2", (n_shared, d, ffn))):
        a, p = _u8(W.get(name) if n_shared else None)
        if n_shared:
            assert a.shape == shape, (name, a.shape, shape)
        keep.append(a), ptrs.append(p)
    for name, shape in (("ss1", (n_shared, ffn)), ("ss3", (n_shared, ffn)), ("ss2", (n_shared, d))):
        a, p = _f32n(W.get(name) if n_shared else None)
        if n_shared:
            assert a.shape == shape, (name, a.shape, shape)
        keep.append(a), ptrs.append(p)
    return keep, ptrs


def combine_fp8(hidden, W, ids, gates, n_shared=0, precision="f32"):
    """out[T,d] for a GIVEN routing, FP8 experts.  W: q1,q3,q2 (uint8 codes), s1,s3,s2 (fp32 row scales), shared: sq*, ss*."""
    hidden, hp = _f32(hidden)
    T, d = hidden.shape
    E, ffn, _ = np.asarray(W["q1"]).shape
    keep, ptrs = _fp8_weight_args(W, E, ffn, d, n_shared)
    ids, ip = _i32(ids)
    gates, gp = _f32(gates)
    top_k = ids.shape[1]
    assert ids.shape == (T, top_k) and gates.shape == (T, top_k)
    out = np.empty((T, d), np.float32)
    rc = _lib(precision).oracle_combine_fp8(hp, T, d, ffn, E, top_k, n_shared, *ptrs, ip, gp, out.ctypes.data_as(_f32p))
    if rc:
        raise ValueError("oracle_combine_fp8: expert id out of range")
    return out


def layer_fp8(hidden, W, top_k, n_shared=0, precision="f32", gate_mode=GATE_RENORM_TOPK):
    """Route (bf16 router_w) + FP8 combine.  -> out, ids, gates."""
    if gate_mode != GATE_RENORM_TOPK:
        ids, gates, _ = route(hidden, W["router_w"], top_k, precision, gate_mode)
        return combine_fp8(hidden, W, ids, gates, n_shared, precision), ids, gates
    hidden, hp = _f32(hidden)
    T, d = hidden.shape
    rw, pr = _u16(W["router_w"])
    E, ffn, _ = np.asarray(W["q1"]).shape
    assert rw.shape == (E, d)
    keep, ptrs = _fp8_weight_args(W, E, ffn, d, n_shared)
    ids = np.empty((T, top_k), np.int32)
    gates = np.empty((T, top_k), np.float32)
    out = np.empty((T, d), np.float32)
    rc = _lib(precision).oracle_layer_fp8(hp, T, d, ffn, E, top_k, n_shared, pr, *ptrs, ids.ctypes.data_as(_i32p),
                                          gates.ctypes.data_as(_f32p), out.ctypes.data_as(_f32p))
    if rc:
        raise ValueError("oracle_layer_fp8: bad sizes")
    return out, ids, gates


# ---------------------------------------------------------------------------------------------
# Chained stack: pre-norm residual blocks  x' = x + Layer(RMSNorm(x) * gamma)
# ---------------------------------------------------------------------------------------------
def rmsnorm(x, gamma, eps=1e-5, precision="f32"):
    """x[T,d] fp32, gamma[d] bf16 bits -> RMSNorm(x) * gamma, fp32 [T,d]."""
    x, xp = _f32(x)
    gamma, gp = _u16(gamma)
    T, d = x.shape
    assert gamma.shape == (d,)
    y = np.empty((T, d), np.float32)
    _lib(precision).oracle_rmsnorm(xp, gp, T, d, float(eps), y.ctypes.data_as(_f32p))
    return y


def residual_add(x, delta, precision="f32"):
    x, xp = _f32(x)
    delta, dp = _f32(delta)
    assert x.shape == delta.shape
    out = np.empty_like(x)
    _lib(precision).oracle_residual_add(xp, dp, x.size, out.ctypes.data_as(_f32p))
    return out


def chained_block(x, W, gamma, top_k, n_shared=0, eps=1e-5, precision="f32", gate_mode=GATE_RENORM_TOPK):
    """One pre-norm residual MoE block.  W: bf16 layer dict, or FP8 layer dict (has "q1").
    -> x_out[T,d], normed[T,d] (what the layer saw), ids, gates."""
    n = rmsnorm(x, gamma, eps, precision)
    fn = layer_fp8 if "q1" in W else layer
    m, ids, gates = fn(n, W, top_k, n_shared, precision, gate_mode)
    return residual_add(x, m, precision), n, ids, gates


def chained_stack(x0, layers, gammas, top_k, n_shared=0, eps=1e-5, precision="f32", gate_mode=GATE_RENORM_TOPK):
    """Blocks applied one after another.  -> x_L, list of the residual stream entering each block, list of ids."""
    x = np.ascontiguousarray(x0, dtype=np.float32)
    trace, all_ids = [], []
    for W, g in zip(layers, gammas):
        trace.append(x)
        x, _, ids, _ = chained_block(x, W, g, top_k, n_shared, eps, precision, gate_mode)
        all_ids.append(ids)
    return x, trace, all_ids


# ---------------------------------------------------------------------------------------------
# Decoder block with the attention stub:  h = x + Attn(RMSNorm(x) g_a) ;  x' = h + Layer(RMSNorm(h) g_m)
# ---------------------------------------------------------------------------------------------
def attention_stub(n, wqkv, wo, n_heads, n_kv_heads, head_dim, precision="f32"):
    """Causal grouped-query self-attention among the T rows of n[T,d] (no cache, no rotation) -> a[T,d] fp32.
    wqkv: [(H + 2 Hkv) dh, d] bf16 bits (q heads, k heads, v heads); wo: [d, H dh] bf16 bits."""
    n, np_ = _f32(n)
    wqkv, pq = _u16(wqkv)
    wo, po = _u16(wo)
    T, d = n.shape
    assert wqkv.shape == ((n_heads + 2 * n_kv_heads) * head_dim, d) and wo.shape == (d, n_heads * head_dim)
    a = np.empty((T, d), np.float32)
    rc = _lib(precision).oracle_attention_stub(np_, pq, po, T, d, n_heads, n_kv_heads, head_dim, a.ctypes.data_as(_f32p))
    if rc:
        raise ValueError("oracle_attention_stub: bad sizes")
    return a


def decoder_block(x, A, W, top_k, n_shared=0, eps=1e-5, precision="f32", gate_mode=GATE_RENORM_TOPK):
    """A: dict(wqkv, wo, gamma_attn, gamma_moe, n_heads, n_kv_heads, head_dim); W: the MoE layer (bf16 or FP8 dict).
    -> x_out, h (the stream after the attention half), ids, gates."""
    n = rmsnorm(x, A["gamma_attn"], eps, precision)
    h = residual_add(x, attention_stub(n, A["wqkv"], A["wo"], A["n_heads"], A["n_kv_heads"], A["head_dim"], precision),
                     precision)
    x_out, _, ids, gates = chained_block(h, W, A["gamma_moe"], top_k, n_shared, eps, precision, gate_mode)
    return x_out, h, ids, gates


def decoder_stack(x0, attn, layers, top_k, n_shared=0, eps=1e-5, precision="f32", gate_mode=GATE_RENORM_TOPK):
    """-> x_L, list of the stream entering each block, list of ids."""
    x = np.ascontiguousarray(x0, dtype=np.float32)
    trace, all_ids = [], []
    for A, W in zip(attn, layers):
        trace.append(x)
        x, _, ids, _ = decoder_block(x, A, W, top_k, n_shared, eps, precision, gate_mode)
        all_ids.append(ids)
    return x, trace, all_ids
