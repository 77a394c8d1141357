"""Thin ctypes binding of libcascade_moe.so (declared in include/cascade_moe.h).

Argument marshalling only: every step of the MoE verification path runs in the HIP
kernels of the library, and the policy (utility, test-and-set loop) in its C code.
torch is used for device memory and streams.  There is no fallback: if the library
is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, byref, c_double, c_float, c_int32, c_int64, c_uint16, c_void_p

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcascade_moe.so")

MOE_OK = 0
STATUS_NAMES = {0: "MOE_OK", -1: "MOE_ERR_INVALID_ARG", -2: "MOE_ERR_UNSUPPORTED_SHAPE", -3: "MOE_ERR_WORKSPACE",
                -4: "MOE_ERR_HIP", -5: "MOE_ERR_UNIMPLEMENTED"}

EXPORTS = ("moe_strerror", "moe_abi_version", "moe_ctx_create", "moe_ctx_destroy", "moe_ctx_workspace_bytes", "moe_ctx_tune",
           "moe_route", "moe_group", "moe_verify_layer", "moe_verify_layer_noalloc", "moe_verify_stack", "moe_chained_stack", "moe_decoder_stack", "moe_pack_matrix",
           "moe_stream_read_probe", "moe_weight_load_twin", "moe_plan_query",
           "moe_ctx_profile", "moe_ctx_profile_read", "moe_pack_weights",
           "cascade_utility", "cascade_default_params", "cascade_ctrl_create", "cascade_ctrl_destroy",
           "cascade_next_k", "cascade_observe", "cascade_get_state")


class MoeError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: {STATUS_NAMES.get(status, status)} ({_strerror(status)})")


class MoeShape(ctypes.Structure):
    _fields_ = [(n, c_int32) for n in ("d", "ffn", "n_experts", "top_k", "n_shared", "max_tokens", "gate_mode",
                                       "n_heads", "n_kv_heads", "head_dim")]


class MoeLayerWeights(ctypes.Structure):
    _fields_ = ([(n, c_void_p) for n in ("router_w", "w1", "w3", "w2", "sw1", "sw3", "sw2")]
                + [("layout", c_int32), ("dtype", c_int32)]
                + [(n, c_void_p) for n in ("w1_scale", "w3_scale", "w2_scale", "sw1_scale", "sw3_scale", "sw2_scale")])


class MoeAttnWeights(ctypes.Structure):
    _fields_ = [(n, c_void_p) for n in ("wqkv", "wo", "gamma_attn", "gamma_moe")]


class MoePlanInfo(ctypes.Structure):
    _fields_ = ([(n, c_int32) for n in ("routed_slots", "wide_router", "packed_fragments", "gu_tiles", "dn_tiles",
                                        "dn_split_k", "dn_fused_chunks", "launches")]
                + [("expected_slots", ctypes.c_double)])


MOE_LAYOUT_ROW_MAJOR, MOE_LAYOUT_TILED = 0, 1
MOE_WEIGHT_BF16, MOE_WEIGHT_FP8_E4M3 = 0, 1
MOE_GATE_RENORM_TOPK, MOE_GATE_SOFTMAX_ALL = 0, 1


class CascadeParams(ctypes.Structure):
    _fields_ = [("t_trial", c_int32), ("max_trials", c_int32), ("s_set", c_int32), ("k_max", c_int32),
                ("k_start", c_int32), ("base_iters", c_int32), ("base_refresh", c_int32), ("s_max", c_int32),
                ("converge_frac", c_double), ("backoff", c_int32), ("hillclimb", c_int32)]


class CascadeState(ctypes.Structure):
    _fields_ = [("phase", c_int32), ("cur_k", c_int32), ("s_cur", c_int32), ("trials_done", c_int32),
                ("iters", c_int64), ("trial_iters", c_int64), ("t_base", c_double), ("last_utility", c_double)]


_LIB = None


def lib():
    """dlopen the library once and declare every signature."""
    global _LIB
    if _LIB is not None:
        return _LIB
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is not built. Run: python -c 'import __graft_entry__ as g; g.build()'")
    # torch owns the device memory handed to the library, so both must sit on ONE HIP runtime: import
    # torch first, so that the library's libamdhip64 dependency resolves to the copy torch has loaded
    import torch  # noqa: F401
    L = ctypes.CDLL(LIB_PATH)
    L.moe_strerror.restype = ctypes.c_char_p
    L.moe_strerror.argtypes = [ctypes.c_int]
    L.moe_abi_version.restype = ctypes.c_int
    L.moe_ctx_create.restype = ctypes.c_int
    L.moe_ctx_create.argtypes = [POINTER(MoeShape), POINTER(c_void_p)]
    L.moe_ctx_destroy.restype = ctypes.c_int
    L.moe_ctx_destroy.argtypes = [c_void_p]
    L.moe_ctx_workspace_bytes.restype = c_int64
    L.moe_ctx_workspace_bytes.argtypes = [c_void_p]
    L.moe_ctx_tune.restype = ctypes.c_int
    L.moe_ctx_tune.argtypes = [c_void_p, c_int32, c_int32, c_int32, c_int32]
    L.moe_route.restype = ctypes.c_int
    L.moe_route.argtypes = [c_void_p, c_void_p, c_void_p, c_int32, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]
    L.moe_group.restype = ctypes.c_int
    L.moe_group.argtypes = [c_void_p, c_void_p, c_int32] + [c_void_p] * 6
    L.moe_verify_layer.restype = ctypes.c_int
    L.moe_verify_layer.argtypes = [c_void_p, POINTER(MoeLayerWeights), c_void_p, c_int32, c_void_p,
                                   c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]
    L.moe_verify_layer_noalloc.restype = ctypes.c_int
    L.moe_verify_layer_noalloc.argtypes = [POINTER(MoeShape), POINTER(MoeLayerWeights), c_void_p, c_int32, c_void_p,
                                           c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]
    L.moe_chained_stack.restype = ctypes.c_int
    L.moe_chained_stack.argtypes = [c_void_p, POINTER(MoeLayerWeights), POINTER(c_void_p), c_int32, c_void_p, c_int32,
                                    ctypes.c_float, c_void_p, c_void_p, c_void_p, c_void_p]
    L.moe_decoder_stack.restype = ctypes.c_int
    L.moe_decoder_stack.argtypes = [c_void_p, POINTER(MoeLayerWeights), POINTER(MoeAttnWeights), c_int32, c_void_p,
                                    c_int32, ctypes.c_float, c_void_p, c_void_p, c_void_p, c_void_p]
    L.moe_pack_matrix.restype = ctypes.c_int
    L.moe_pack_matrix.argtypes = [c_void_p, c_void_p, c_void_p, c_int64, c_int32, c_int32, c_void_p]
    L.moe_verify_stack.restype = ctypes.c_int
    L.moe_verify_stack.argtypes = [c_void_p, POINTER(MoeLayerWeights), c_int32, c_void_p, c_int32, c_void_p,
                                   c_void_p, c_void_p]
    L.moe_pack_weights.restype = ctypes.c_int
    L.moe_pack_weights.argtypes = [c_void_p, POINTER(MoeLayerWeights), POINTER(MoeLayerWeights), c_void_p]
    L.moe_ctx_profile.restype = ctypes.c_int
    L.moe_ctx_profile.argtypes = [c_void_p, c_int32]
    L.moe_ctx_profile_read.restype = ctypes.c_int
    L.moe_ctx_profile_read.argtypes = [c_void_p, POINTER(c_double), POINTER(c_int64)]
    L.moe_plan_query.restype = ctypes.c_int
    L.moe_plan_query.argtypes = [ctypes.POINTER(MoeShape), c_int32, c_int32, c_int32, ctypes.POINTER(MoePlanInfo)]
    L.moe_stream_read_probe.restype = ctypes.c_int
    L.moe_stream_read_probe.argtypes = [c_void_p, c_int64, c_void_p, c_void_p]
    L.moe_weight_load_twin.restype = ctypes.c_int
    L.moe_weight_load_twin.argtypes = [c_void_p, c_void_p, c_int32, c_int32, c_int32, c_int64, c_void_p, c_void_p]
    L.cascade_utility.restype = c_double
    L.cascade_utility.argtypes = [c_double, c_double, c_double]
    L.cascade_default_params.restype = None
    L.cascade_default_params.argtypes = [POINTER(CascadeParams)]
    L.cascade_ctrl_create.restype = c_void_p
    L.cascade_ctrl_create.argtypes = [POINTER(CascadeParams)]
    L.cascade_ctrl_destroy.restype = None
    L.cascade_ctrl_destroy.argtypes = [c_void_p]
    L.cascade_next_k.restype = c_int32
    L.cascade_next_k.argtypes = [c_void_p]
    L.cascade_observe.restype = ctypes.c_int
    L.cascade_observe.argtypes = [c_void_p, c_int32, c_int32, c_double]
    L.cascade_get_state.restype = None
    L.cascade_get_state.argtypes = [c_void_p, POINTER(CascadeState)]
    _LIB = L
    return L


def _strerror(status: int) -> str:
    try:
        return lib().moe_strerror(status).decode()
    except Exception:
        return "?"


def _check(status: int, what: str):
    if status != MOE_OK:
        raise MoeError(status, what)


def _ptr(t):
    return None if t is None else c_void_p(t.data_ptr())


def _stream_ptr(stream):
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return c_void_p(stream.cuda_stream)


def _want(t, dtype, shape, name):
    import torch
    if t is None:
        return
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.is_contiguous() and t.dtype == dtype
            and tuple(t.shape) == tuple(shape)):
        raise ValueError(f"{name}: expected contiguous CUDA tensor {dtype} {tuple(shape)}, got "
                         f"{getattr(t, 'dtype', None)} {tuple(getattr(t, 'shape', ()))}")


def _want_bf16(t, shape, name):
    import torch
    if t is None:
        return
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.is_contiguous() and t.element_size() == 2
            and t.dtype in (torch.int16, torch.uint16, torch.bfloat16) and tuple(t.shape) == tuple(shape)):
        raise ValueError(f"{name}: expected contiguous CUDA 16-bit tensor {tuple(shape)}")


class LayerWeights:
    """Device pointers of one layer's weights (tensors stay owned by the caller).
    dtype = MOE_WEIGHT_BF16: 16-bit expert tensors; MOE_WEIGHT_FP8_E4M3: uint8 codes + fp32 per-row `scales`
    (w1_scale [E,ffn], w3_scale [E,ffn], w2_scale [E,d], then the three of the shared experts)."""

    def __init__(self, shape: "MoeShape", router_w, w1, w3, w2, sw1=None, sw3=None, sw2=None, layout=0,
                 dtype=MOE_WEIGHT_BF16, scales=None):
        import torch
        E, d, f, ns = shape.n_experts, shape.d, shape.ffn, shape.n_shared
        _want_bf16(router_w, (E, d), "router_w")
        if dtype == MOE_WEIGHT_BF16:
            want = _want_bf16
        else:
            want = lambda t, shp, name: _want(t, torch.uint8, shp, name)
        want(w1, (E, f, d), "w1")
        want(w3, (E, f, d), "w3")
        want(w2, (E, d, f), "w2")
        if ns:
            want(sw1, (ns, f, d), "sw1")
            want(sw3, (ns, f, d), "sw3")
            want(sw2, (ns, d, f), "sw2")
            if sw1 is None or sw3 is None or sw2 is None:
                raise ValueError("shared expert weights required")
        self.tensors = (router_w, w1, w3, w2, sw1, sw3, sw2)
        self.scales = tuple(scales) if scales is not None else (None,) * 6
        if dtype == MOE_WEIGHT_FP8_E4M3:
            shapes = ((E, f), (E, f), (E, d), (ns, f), (ns, f), (ns, d))
            for t, shp, name in zip(self.scales, shapes, ("w1_scale", "w3_scale", "w2_scale", "sw1_scale", "sw3_scale",
                                                          "sw2_scale")):
                if t is None and (ns or not name.startswith("s")):
                    raise ValueError(f"{name} required for FP8 weights")
                _want(t, torch.float32, shp, name)
        self.dtype = dtype
        self.geometry = (d, f, E, ns)        # the tensors were checked against these sizes
        self.c = MoeLayerWeights(*[None if t is None else t.data_ptr() for t in self.tensors], layout, dtype,
                                 *[None if t is None else t.data_ptr() for t in self.scales])


class MoeContext:
    """Owns a moe_ctx (device workspace for one layer geometry on the current device)."""

    def __init__(self, d, ffn, n_experts, top_k, n_shared=0, max_tokens=9, gate_mode=MOE_GATE_RENORM_TOPK,
                 n_heads=0, n_kv_heads=0, head_dim=0):
        self.shape = MoeShape(d, ffn, n_experts, top_k, n_shared, max_tokens, gate_mode, n_heads, n_kv_heads, head_dim)
        self._h = c_void_p()
        _check(lib().moe_ctx_create(byref(self.shape), byref(self._h)), "moe_ctx_create")

    def close(self):
        if self._h:
            lib().moe_ctx_destroy(self._h)
            self._h = c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _same_geometry(self, *layers) -> None:
        """The library sees raw pointers: weights validated for another geometry would be read out of bounds."""
        s = self.shape
        mine = (s.d, s.ffn, s.n_experts, s.n_shared)
        for lw in layers:
            if lw.geometry != mine:
                raise ValueError(f"layer weights were built for (d, ffn, E, n_shared) = {lw.geometry}, "
                                 f"this context is {mine}")

    @property
    def workspace_bytes(self) -> int:
        return int(lib().moe_ctx_workspace_bytes(self._h))

    def weights(self, W: dict) -> LayerWeights:
        """bf16 layer from a dict with router_w, w1, w3, w2 (sw1, sw3, sw2); FP8 layer from a dict with router_w,
        q1, q3, q2 (uint8 codes), s1, s3, s2 (fp32 per-row scales) and sq*/ss* for shared experts."""
        if "q1" in W:
            return LayerWeights(self.shape, W["router_w"], W["q1"], W["q3"], W["q2"], W.get("sq1"), W.get("sq3"),
                                W.get("sq2"), dtype=MOE_WEIGHT_FP8_E4M3,
                                scales=(W["s1"], W["s3"], W["s2"], W.get("ss1"), W.get("ss3"), W.get("ss2")))
        return LayerWeights(self.shape, W["router_w"], W["w1"], W["w3"], W["w2"], W.get("sw1"), W.get("sw3"),
                            W.get("sw2"))

    def moe_ctx_tune(self, gu_tiles=0, dn_tiles=0, dn_split_k=0, fused_down=-1) -> None:
        _check(lib().moe_ctx_tune(self._h, gu_tiles, dn_tiles, dn_split_k, fused_down), "moe_ctx_tune")

    KERNELS = ("route", "gateup", "down", "combine")

    def moe_ctx_profile(self, enable: bool) -> None:
        _check(lib().moe_ctx_profile(self._h, 1 if enable else 0), "moe_ctx_profile")

    def moe_ctx_profile_read(self):
        """-> ({kernel: summed ms}, number of layer-steps) since profiling was enabled / last read."""
        ms = (c_double * 4)()
        n = c_int64()
        _check(lib().moe_ctx_profile_read(self._h, ms, byref(n)), "moe_ctx_profile_read")
        return dict(zip(self.KERNELS, [float(v) for v in ms])), int(n.value)

    def moe_pack_weights(self, src: LayerWeights, stream=None, in_place_of=None) -> LayerWeights:
        """Re-layout src (row-major) into freshly allocated tiled buffers; returns the tiled LayerWeights."""
        import torch
        self._same_geometry(src)
        bufs = [None if t is None else torch.empty_like(t) for t in src.tensors]
        bufs[0] = src.tensors[0]            # router is shared, it stays row-major
        dst = LayerWeights(self.shape, *bufs, layout=0, dtype=src.dtype, scales=src.scales)
        _check(lib().moe_pack_weights(self._h, byref(src.c), byref(dst.c), _stream_ptr(stream)), "moe_pack_weights")
        return dst

    # ---- device calls (same names as the C ABI) -------------------------------------------
    def moe_route(self, hidden, router_w, ids=None, gates=None, unique_experts=None, n_unique=None, stream=None):
        import torch
        s = self.shape
        T = hidden.shape[0]
        _want(hidden, torch.float32, (T, s.d), "hidden")
        _want_bf16(router_w, (s.n_experts, s.d), "router_w")
        _want(ids, torch.int32, (T, s.top_k), "ids")
        _want(gates, torch.float32, (T, s.top_k), "gates")
        _want(unique_experts, torch.int32, (s.n_experts,), "unique_experts")
        _want(n_unique, torch.int32, (1,), "n_unique")
        _check(lib().moe_route(self._h, _ptr(hidden), _ptr(router_w), T, _ptr(ids), _ptr(gates), _ptr(unique_experts),
                               _ptr(n_unique), _stream_ptr(stream)), "moe_route")

    def moe_group(self, ids, unique_experts=None, n_unique=None, expert_count=None, expert_offset=None, assign=None,
                  stream=None):
        import torch
        s = self.shape
        T = ids.shape[0]
        _want(ids, torch.int32, (T, s.top_k), "ids")
        _want(unique_experts, torch.int32, (s.n_experts,), "unique_experts")
        _want(n_unique, torch.int32, (1,), "n_unique")
        _want(expert_count, torch.int32, (s.n_experts,), "expert_count")
        _want(expert_offset, torch.int32, (s.n_experts + 1,), "expert_offset")
        _want(assign, torch.int32, (T * s.top_k,), "assign")
        _check(lib().moe_group(self._h, _ptr(ids), T, _ptr(unique_experts), _ptr(n_unique), _ptr(expert_count),
                               _ptr(expert_offset), _ptr(assign), _stream_ptr(stream)), "moe_group")

    def moe_verify_layer(self, weights: LayerWeights, hidden, out, ids=None, gates=None, unique_experts=None,
                         n_unique=None, stream=None):
        import torch
        s = self.shape
        T = hidden.shape[0]
        _want(hidden, torch.float32, (T, s.d), "hidden")
        _want(out, torch.float32, (T, s.d), "out")
        _want(ids, torch.int32, (T, s.top_k), "ids")
        _want(gates, torch.float32, (T, s.top_k), "gates")
        _want(unique_experts, torch.int32, (s.n_experts,), "unique_experts")
        _want(n_unique, torch.int32, (1,), "n_unique")
        self._same_geometry(weights)
        _check(lib().moe_verify_layer(self._h, byref(weights.c), _ptr(hidden), T, _ptr(out), _ptr(ids), _ptr(gates),
                                      _ptr(unique_experts), _ptr(n_unique), _stream_ptr(stream)), "moe_verify_layer")

    def moe_verify_stack(self, layers, hidden, out, n_unique_per_layer=None, stream=None):
        import torch
        s = self.shape
        L, T = hidden.shape[0], hidden.shape[1]
        if L != len(layers):
            raise ValueError("hidden.shape[0] must equal the number of layers")
        _want(hidden, torch.float32, (L, T, s.d), "hidden")
        _want(out, torch.float32, (L, T, s.d), "out")
        _want(n_unique_per_layer, torch.int32, (L,), "n_unique_per_layer")
        self._same_geometry(*layers)
        arr = (MoeLayerWeights * L)(*[lw.c for lw in layers])
        _check(lib().moe_verify_stack(self._h, arr, L, _ptr(hidden), T, _ptr(out), _ptr(n_unique_per_layer),
                                      _stream_ptr(stream)), "moe_verify_stack")


    def moe_chained_stack(self, layers, gammas, x_in, x_out, eps=1e-5, trace=None, n_unique_per_layer=None,
                          stream=None):
        """L pre-norm residual MoE blocks, each feeding the next.  gammas: L CUDA tensors [d] (16-bit)."""
        import torch
        s = self.shape
        L, T = len(layers), x_in.shape[0]
        if len(gammas) != L:
            raise ValueError("one norm weight per layer")
        _want(x_in, torch.float32, (T, s.d), "x_in")
        _want(x_out, torch.float32, (T, s.d), "x_out")
        _want(trace, torch.float32, (L, T, s.d), "trace")
        _want(n_unique_per_layer, torch.int32, (L,), "n_unique_per_layer")
        for g in gammas:
            _want_bf16(g, (s.d,), "gamma")
        self._same_geometry(*layers)
        arr = (MoeLayerWeights * L)(*[lw.c for lw in layers])
        garr = (c_void_p * L)(*[g.data_ptr() for g in gammas])
        _check(lib().moe_chained_stack(self._h, arr, garr, L, _ptr(x_in), T, ctypes.c_float(eps), _ptr(x_out),
                                       _ptr(trace), _ptr(n_unique_per_layer), _stream_ptr(stream)), "moe_chained_stack")


    def moe_pack_matrix(self, src, stream=None):
        """Tiled copy of one row-major 2-D weight matrix (16-bit tensor: bf16; uint8 tensor: FP8 codes)."""
        import torch
        if not (isinstance(src, torch.Tensor) and src.is_cuda and src.is_contiguous() and src.dim() == 2):
            raise ValueError("src: contiguous 2-D CUDA tensor expected")
        dtype = MOE_WEIGHT_FP8_E4M3 if src.element_size() == 1 else MOE_WEIGHT_BF16
        dst = torch.empty_like(src)
        _check(lib().moe_pack_matrix(self._h, _ptr(src), _ptr(dst), src.shape[0], src.shape[1], dtype,
                                     _stream_ptr(stream)), "moe_pack_matrix")
        return dst

    def attn_weights(self, A: dict, stream=None) -> "AttnWeights":
        """Attention stub weights from a dict with row-major wqkv, wo (packed here) and gamma_attn, gamma_moe."""
        s = self.shape
        nq, nqkv = s.n_heads * s.head_dim, (s.n_heads + 2 * s.n_kv_heads) * s.head_dim
        _want_bf16(A["wqkv"], (nqkv, s.d), "wqkv")
        _want_bf16(A["wo"], (s.d, nq), "wo")
        _want_bf16(A["gamma_attn"], (s.d,), "gamma_attn")
        _want_bf16(A["gamma_moe"], (s.d,), "gamma_moe")
        return AttnWeights(self.moe_pack_matrix(A["wqkv"], stream), self.moe_pack_matrix(A["wo"], stream),
                           A["gamma_attn"], A["gamma_moe"])

    def moe_decoder_stack(self, layers, attn, x_in, x_out, eps=1e-5, trace=None, n_unique_per_layer=None, stream=None):
        """L decoder blocks (attention stub + MoE), each feeding the next.  attn: L AttnWeights."""
        import torch
        s = self.shape
        L, T = len(layers), x_in.shape[0]
        if len(attn) != L:
            raise ValueError("one set of attention weights per layer")
        _want(x_in, torch.float32, (T, s.d), "x_in")
        _want(x_out, torch.float32, (T, s.d), "x_out")
        _want(trace, torch.float32, (L, T, s.d), "trace")
        _want(n_unique_per_layer, torch.int32, (L,), "n_unique_per_layer")
        self._same_geometry(*layers)
        arr = (MoeLayerWeights * L)(*[lw.c for lw in layers])
        aarr = (MoeAttnWeights * L)(*[a.c for a in attn])
        _check(lib().moe_decoder_stack(self._h, arr, aarr, L, _ptr(x_in), T, ctypes.c_float(eps), _ptr(x_out),
                                       _ptr(trace), _ptr(n_unique_per_layer), _stream_ptr(stream)), "moe_decoder_stack")


class AttnWeights:
    """Device pointers of one block's attention stub (tiled wqkv, wo; norm weights); keeps the tensors alive."""

    def __init__(self, wqkv_tiled, wo_tiled, gamma_attn, gamma_moe):
        self.tensors = (wqkv_tiled, wo_tiled, gamma_attn, gamma_moe)
        self.c = MoeAttnWeights(*[t.data_ptr() for t in self.tensors])


def moe_plan_query(d, ffn, n_experts, top_k, n_shared=0, max_tokens=9, T=1, layout=MOE_LAYOUT_TILED,
                   dtype=MOE_WEIGHT_BF16, gate_mode=0, n_heads=0, n_kv_heads=0, head_dim=0) -> dict:
    """Launch plan of one layer-step (host arithmetic only; needs no GPU)."""
    shape = MoeShape(d, ffn, n_experts, top_k, n_shared, max_tokens, gate_mode, n_heads, n_kv_heads, head_dim)
    info = MoePlanInfo()
    _check(lib().moe_plan_query(ctypes.byref(shape), T, layout, dtype, ctypes.byref(info)), "moe_plan_query")
    return {n: getattr(info, n) for n, _ in MoePlanInfo._fields_}


def moe_verify_layer_noalloc(shape: MoeShape, weights: LayerWeights, hidden, out, ids=None, gates=None,
                             unique_experts=None, n_unique=None, stream=None):
    """moe_verify_layer on the library's fixed workspace: no context, no allocation inside the call."""
    import torch
    s = shape
    T = hidden.shape[0]
    _want(hidden, torch.float32, (T, s.d), "hidden")
    _want(out, torch.float32, (T, s.d), "out")
    _want(ids, torch.int32, (T, s.top_k), "ids")
    _want(gates, torch.float32, (T, s.top_k), "gates")
    _want(unique_experts, torch.int32, (s.n_experts,), "unique_experts")
    _want(n_unique, torch.int32, (1,), "n_unique")
    if weights.geometry != (s.d, s.ffn, s.n_experts, s.n_shared):
        raise ValueError(f"layer weights were built for (d, ffn, E, n_shared) = {weights.geometry}")
    _check(lib().moe_verify_layer_noalloc(byref(s), byref(weights.c), _ptr(hidden), T, _ptr(out), _ptr(ids), _ptr(gates),
                                          _ptr(unique_experts), _ptr(n_unique), _stream_ptr(stream)),
           "moe_verify_layer_noalloc")


def moe_stream_read_probe(src, sink, stream=None):
    nbytes = src.numel() * src.element_size()
    _check(lib().moe_stream_read_probe(_ptr(src), nbytes - nbytes % 16, _ptr(sink), _stream_ptr(stream)),
           "moe_stream_read_probe")


def moe_weight_load_twin(a, b, slots, tiles, steps, sink, stream=None):
    """The tiled bf16 gate/up kernel's weight loads alone, over the first `slots` matrices of a and b ([n, rows, K])."""
    slot_stride = a.stride(0) * a.element_size()
    _check(lib().moe_weight_load_twin(_ptr(a), _ptr(b), slots, tiles, steps, slot_stride, _ptr(sink), _stream_ptr(stream)),
           "moe_weight_load_twin")


# ---- host side ---------------------------------------------------------------------------------
def cascade_utility(tokens_per_iter: float, t_verify: float, t_base: float) -> float:
    return float(lib().cascade_utility(tokens_per_iter, t_verify, t_base))


def cascade_default_params() -> CascadeParams:
    p = CascadeParams()
    lib().cascade_default_params(byref(p))
    return p


class CascadeController:
    """Per-request controller: K = next_k(); run the iteration; observe(K, tokens, time)."""

    def __init__(self, params: CascadeParams | None = None, **overrides):
        p = params or cascade_default_params()
        for k, v in overrides.items():
            if not hasattr(p, k):
                raise AttributeError(k)
            setattr(p, k, v)
        self.params = p
        self._h = lib().cascade_ctrl_create(byref(p))
        if not self._h:
            raise ValueError("cascade_ctrl_create: bad parameters")

    def close(self):
        if self._h:
            lib().cascade_ctrl_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def next_k(self) -> int:
        return int(lib().cascade_next_k(self._h))

    def observe(self, k_used: int, tokens_emitted: int, t_iter: float) -> None:
        _check(lib().cascade_observe(self._h, k_used, tokens_emitted, t_iter), "cascade_observe")

    def state(self) -> CascadeState:
        st = CascadeState()
        lib().cascade_get_state(self._h, byref(st))
        return st
