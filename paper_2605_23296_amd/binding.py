"""ctypes binding over libcompact.so: argument marshalling only.

The functions keep the names of the C ABI (include/compact.h).  `Layer` is a
thin convenience holder that owns torch-allocated device buffers (KV slabs,
workspace) and passes their addresses down; every step of the computation
runs in the library's kernels.  There is no fallback: if the library has not
been built, `lib()` raises.
"""
import ctypes as C
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libcompact.so")

COMPACT_FP32, COMPACT_BF16 = 0, 1
K_NONE, K_GEMM, K_ATTN_PREFILL, K_ATTN_DECODE, K_GEMM_SKINNY = 0, 1, 2, 3, 4
ERR_NAMES = {0: "OK", 1: "EINVAL", 2: "ESHAPE", 3: "ECAPACITY", 4: "EWORKSPACE", 5: "EUNSUPPORTED", 6: "EHIP"}

EXPORTS = [
    "compact_create", "compact_destroy", "compact_last_error", "compact_workspace_bytes",
    "compact_prefill", "compact_decode_step", "compact_layer_forward",
    "compact_profile_select", "compact_profile_read",
    "compact_rmsnorm", "compact_rope_kvwrite", "compact_gemm", "compact_attn_prefill",
    "compact_attn_decode", "compact_attn_decode_noalloc", "compact_moe_route", "compact_moe_ffn",
    "compact_prefix_workspace_bytes", "compact_prefix_decode_step", "compact_attn_decode_prefix",
    "compact_stack_workspace_bytes", "compact_stack_forward", "compact_prefill_extend", "compact_mxfp4_dequant",
    "compact_mixed_workspace_bytes", "compact_mixed_forward",
    "compact_prefix_stack_workspace_bytes", "compact_prefix_stack_forward",
]


class LayerCfg(C.Structure):
    _fields_ = [("d_model", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("ffn_dim", C.c_int32), ("n_experts", C.c_int32),
                ("top_k", C.c_int32), ("rms_eps", C.c_float), ("rope_theta", C.c_float),
                ("dtype", C.c_int32)]


class Weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("g_attn", "w_qkv", "w_o", "g_ffn", "w_gate_up", "w_down",
                                          "w_router", "w_exp_gate_up", "w_exp_down",
                                          "w_exp_gate_up_q", "w_exp_gate_up_s", "w_exp_down_q", "w_exp_down_s")]


class KV(C.Structure):
    _fields_ = [("d_k", C.c_void_p), ("d_v", C.c_void_p),
                ("h_slab_offset", C.POINTER(C.c_int64)), ("h_capacity", C.POINTER(C.c_int32)),
                ("h_len", C.POINTER(C.c_int32)), ("h_pos_offset", C.POINTER(C.c_int32))]


class RouteOut(C.Structure):
    _fields_ = [("d_expert_idx", C.c_void_p), ("d_gate", C.c_void_p)]


class CompactError(RuntimeError):
    def __init__(self, code, detail):
        super().__init__("libcompact: %s (%d): %s" % (ERR_NAMES.get(code, "?"), code, detail))
        self.code = code
        self.detail = detail


_lib = None


def lib():
    """Loads libcompact.so; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("libcompact.so is not built: run `python -m paper_2605_23296_amd.build` "
                           "(there is no fallback path)")
    L = C.CDLL(LIB_PATH)
    vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
    P = C.POINTER
    L.compact_create.argtypes = [P(LayerCfg), P(vp)]
    L.compact_destroy.argtypes = [vp]
    L.compact_destroy.restype = None
    L.compact_last_error.argtypes = [vp]
    L.compact_last_error.restype = C.c_char_p
    L.compact_workspace_bytes.argtypes = [vp, i64, i32, i32, P(sz)]
    L.compact_prefill.argtypes = [vp, P(Weights), i32, P(i32), vp, P(KV), vp, P(RouteOut), vp, sz, vp]
    L.compact_decode_step.argtypes = [vp, P(Weights), i32, vp, P(KV), vp, P(RouteOut), vp, sz, vp]
    L.compact_prefill_extend.argtypes = [vp, P(Weights), i32, P(i32), vp, P(KV), vp, P(RouteOut), vp, sz, vp]
    L.compact_layer_forward.argtypes = [vp, P(Weights), i32, P(i32), vp, i32, vp, P(KV), vp, vp, vp, vp, sz, vp]
    L.compact_profile_select.argtypes = [vp, i32]
    L.compact_profile_read.argtypes = [vp, P(i64), P(C.c_double)]
    L.compact_rmsnorm.argtypes = [vp, vp, vp, vp, i64, vp]
    L.compact_rope_kvwrite.argtypes = [vp, i32, P(i32), vp, P(KV), vp]
    L.compact_gemm.argtypes = [vp, vp, vp, vp, vp, i64, i32, i32, i32, vp, sz, vp]
    L.compact_attn_prefill.argtypes = [vp, i32, P(i32), vp, P(KV), vp, vp]
    L.compact_attn_decode.argtypes = [vp, i32, vp, P(KV), vp, vp, sz, vp]
    L.compact_moe_route.argtypes = [vp, vp, vp, i64, vp, vp, vp, vp, sz, vp]
    L.compact_moe_ffn.argtypes = [vp, P(Weights), vp, vp, vp, vp, i64, vp, vp, sz, vp]
    L.compact_prefix_workspace_bytes.argtypes = [vp, i32, i32, i32, P(sz)]
    L.compact_prefix_decode_step.argtypes = [vp, P(Weights), i32, vp, P(KV), P(i32), P(KV), vp, P(RouteOut), vp, sz, vp]
    L.compact_attn_decode_prefix.argtypes = [vp, i32, vp, P(KV), P(i32), P(KV), vp, vp, sz, vp]
    L.compact_mixed_workspace_bytes.argtypes = [vp, i32, i32, i32, P(sz)]
    L.compact_mixed_forward.argtypes = [vp, P(Weights), i32, P(i32), vp, i32, vp, P(KV), i32, vp, vp, vp, sz, vp]
    L.compact_prefix_stack_workspace_bytes.argtypes = [vp, i64, i32, i32, P(sz)]
    L.compact_prefix_stack_forward.argtypes = [vp, i32, P(Weights), i32, P(i32), i64, vp, i32, vp, P(KV), P(KV), vp, vp, sz, vp]
    L.compact_mxfp4_dequant.argtypes = [vp, vp, vp, i64, i32, vp, vp]
    L.compact_stack_workspace_bytes.argtypes = [vp, i64, i32, i32, P(sz)]
    L.compact_stack_forward.argtypes = [vp, i32, P(Weights), i32, P(i32), vp, i32, vp, P(KV), vp, vp, vp, sz, vp]
    for name in EXPORTS:
        fn = getattr(L, name)
        if name not in ("compact_destroy", "compact_last_error"):
            fn.restype = C.c_int
    _lib = L
    return L


def _ptr(t):
    if t is None:
        return None
    assert t.is_contiguous()
    return C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _i32arr(vals):
    return (C.c_int32 * len(vals))(*[int(v) for v in vals])


def make_cfg(layer):
    """layer: workloads.LayerConfig (or any object with the same fields)."""
    return LayerCfg(layer.d_model, layer.n_q_heads, layer.n_kv_heads, layer.head_dim, layer.ffn_dim,
                    layer.n_experts, layer.top_k, layer.rms_eps, layer.rope_theta,
                    COMPACT_BF16 if layer.dtype == "bf16" else COMPACT_FP32)


class KVCache:
    """Torch-allocated K/V slabs for N blocks plus the host arrays of compact_kv."""

    def __init__(self, layer, capacities, device, dtype, pos_offset=None):
        self.N = len(capacities)
        caps = [(int(c) + 7) // 8 * 8 for c in capacities]
        per_tok = layer.n_kv_heads * layer.head_dim
        offs, total = [], 0
        for c in caps:
            offs.append(total)
            total += c * per_tok
        self.k = torch.empty(max(total, 8), dtype=dtype, device=device)
        self.v = torch.empty(max(total, 8), dtype=dtype, device=device)
        self.h_slab_offset = (C.c_int64 * self.N)(*offs)
        self.h_capacity = _i32arr(caps)
        self.h_len = _i32arr([0] * self.N)
        self.h_pos_offset = None if pos_offset is None else _i32arr(pos_offset)
        self.layer = layer
        self.caps, self.offs = caps, offs
        self.c = KV(self.k.data_ptr(), self.v.data_ptr(), self.h_slab_offset, self.h_capacity, self.h_len,
                    self.h_pos_offset if self.h_pos_offset is not None else C.cast(None, C.POINTER(C.c_int32)))

    def lens(self):
        return [int(v) for v in self.h_len]

    def block_k(self, b):
        """K rows of block b as [len, Hkv, hd]."""
        L, Hkv, hd = self.h_len[b], self.layer.n_kv_heads, self.layer.head_dim
        slab = self.k[self.offs[b]:self.offs[b] + self.caps[b] * Hkv * hd].view(Hkv, self.caps[b], hd)
        return slab[:, :L, :].permute(1, 0, 2)

    def block_v(self, b):
        """V rows of block b as [len, Hkv, hd] (the slab stores them transposed)."""
        L, Hkv, hd = self.h_len[b], self.layer.n_kv_heads, self.layer.head_dim
        slab = self.v[self.offs[b]:self.offs[b] + self.caps[b] * Hkv * hd].view(Hkv, hd, self.caps[b])
        return slab[:, :, :L].permute(2, 0, 1)


class Layer:
    """One layer context plus its weight pointers."""

    def __init__(self, layer, weights):
        self.L = lib()
        self.layer = layer
        self.cfg = make_cfg(layer)
        self.ctx = C.c_void_p()
        rc = self.L.compact_create(C.byref(self.cfg), C.byref(self.ctx))
        if rc != 0:
            raise CompactError(rc, self.L.compact_last_error(None).decode())
        self.weights = weights          # keeps the tensors alive
        self.w = Weights()
        for name, _ in Weights._fields_:
            t = weights.get(name) if weights is not None else None
            setattr(self.w, name, t.data_ptr() if t is not None else None)
        self.ws = None
        self.torch_dtype = torch.bfloat16 if layer.dtype == "bf16" else torch.float32

    def close(self):
        if self.ctx:
            self.L.compact_destroy(self.ctx)
            self.ctx = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def check(self, rc):
        if rc != 0:
            raise CompactError(rc, self.L.compact_last_error(self.ctx).decode())

    # -- workspace ------------------------------------------------------------
    def workspace_bytes(self, max_tokens, max_blocks, max_kv_len):
        n = C.c_size_t()
        self.check(self.L.compact_workspace_bytes(self.ctx, max_tokens, max_blocks, max_kv_len, C.byref(n)))
        return n.value

    def ensure_workspace(self, max_tokens, max_blocks, max_kv_len, device):
        need = self.workspace_bytes(max_tokens, max_blocks, max_kv_len)
        if self.ws is None or self.ws.numel() < need:
            self.ws = torch.empty(need, dtype=torch.uint8, device=device)
        return self.ws

    def _ws(self):
        return (C.c_void_p(self.ws.data_ptr()), self.ws.numel()) if self.ws is not None else (None, 0)

    # -- layer calls ------------------------------------------------------------
    def compact_prefill(self, cu_seqlens, x, kv, y, route=None):
        wsp, wsn = self._ws()
        r = None if route is None else C.byref(RouteOut(route[0].data_ptr(), route[1].data_ptr()))
        self.check(self.L.compact_prefill(self.ctx, C.byref(self.w), len(cu_seqlens) - 1, _i32arr(cu_seqlens),
                                          _ptr(x), C.byref(kv.c), _ptr(y), r, wsp, wsn, _stream()))

    def compact_prefill_extend(self, cu_seqlens, x, kv, y, route=None):
        wsp, wsn = self._ws()
        r = None if route is None else C.byref(RouteOut(route[0].data_ptr(), route[1].data_ptr()))
        self.check(self.L.compact_prefill_extend(self.ctx, C.byref(self.w), len(cu_seqlens) - 1, _i32arr(cu_seqlens),
                                                 _ptr(x), C.byref(kv.c), _ptr(y), r, wsp, wsn, _stream()))

    def compact_decode_step(self, x, kv, y, route=None):
        wsp, wsn = self._ws()
        r = None if route is None else C.byref(RouteOut(route[0].data_ptr(), route[1].data_ptr()))
        self.check(self.L.compact_decode_step(self.ctx, C.byref(self.w), kv.N, _ptr(x), C.byref(kv.c), _ptr(y),
                                              r, wsp, wsn, _stream()))

    def compact_layer_forward(self, cu_seqlens, x_prefill, x_decode, kv, y_prefill, y_last, y_decode):
        wsp, wsn = self._ws()
        S = 0 if x_decode is None else x_decode.shape[0]
        self.check(self.L.compact_layer_forward(
            self.ctx, C.byref(self.w), len(cu_seqlens) - 1, _i32arr(cu_seqlens), _ptr(x_prefill), S,
            _ptr(x_decode), C.byref(kv.c), _ptr(y_prefill), _ptr(y_last), _ptr(y_decode), wsp, wsn, _stream()))

    # -- mixed batches (chunked prefill interleaved with decode) --------------------
    def mixed_workspace_bytes(self, max_batched_tokens, max_blocks, max_kv_len):
        n = C.c_size_t()
        self.check(self.L.compact_mixed_workspace_bytes(self.ctx, max_batched_tokens, max_blocks, max_kv_len, C.byref(n)))
        return n.value

    def compact_mixed_forward(self, cu_seqlens, x_prefill, x_decode, kv, max_batched_tokens, y_last, y_decode):
        wsp, wsn = self._ws()
        S = 0 if x_decode is None else x_decode.shape[0]
        self.check(self.L.compact_mixed_forward(
            self.ctx, C.byref(self.w), len(cu_seqlens) - 1, _i32arr(cu_seqlens), _ptr(x_prefill), S, _ptr(x_decode),
            C.byref(kv.c), max_batched_tokens, _ptr(y_last), _ptr(y_decode), wsp, wsn, _stream()))

    # -- a depth of layers --------------------------------------------------------
    def stack_workspace_bytes(self, max_tokens, max_blocks, max_kv_len):
        n = C.c_size_t()
        self.check(self.L.compact_stack_workspace_bytes(self.ctx, max_tokens, max_blocks, max_kv_len, C.byref(n)))
        return n.value

    def compact_stack_forward(self, layer_weights, cu_seqlens, x_prefill, x_decode, kvs, y_last, y_decode):
        """layer_weights: one dict of device tensors per layer; kvs: one KVCache per layer (same geometry)."""
        wsp, wsn = self._ws()
        nl = len(layer_weights)
        warr = (Weights * nl)()
        for l, wd in enumerate(layer_weights):
            for name, _ in Weights._fields_:
                t = wd.get(name)
                setattr(warr[l], name, t.data_ptr() if t is not None else None)
        karr = (KV * nl)()
        for l, kv in enumerate(kvs):
            for name, _ in KV._fields_:
                setattr(karr[l], name, getattr(kv.c, name))
        S = 0 if x_decode is None else x_decode.shape[0]
        self.check(self.L.compact_stack_forward(
            self.ctx, nl, warr, len(cu_seqlens) - 1, _i32arr(cu_seqlens), _ptr(x_prefill), S, _ptr(x_decode), karr,
            _ptr(y_last), _ptr(y_decode), wsp, wsn, _stream()))

    def prefix_stack_workspace_bytes(self, history_tokens, n_workers, max_tail_len):
        n = C.c_size_t()
        self.check(self.L.compact_prefix_stack_workspace_bytes(self.ctx, history_tokens, n_workers, max_tail_len, C.byref(n)))
        return n.value

    def compact_prefix_stack_forward(self, layer_weights, prefix_len, x_history, x_decode, shared, tails, y_decode):
        """layer_weights: one dict per layer; shared, tails: one KVCache per layer."""
        wsp, wsn = self._ws()
        nl = len(layer_weights)
        warr = (Weights * nl)()
        for l, wd in enumerate(layer_weights):
            for name, _ in Weights._fields_:
                t = wd.get(name)
                setattr(warr[l], name, t.data_ptr() if t is not None else None)
        sarr, tarr = (KV * nl)(), (KV * nl)()
        for l in range(nl):
            for name, _ in KV._fields_:
                setattr(sarr[l], name, getattr(shared[l].c, name))
                setattr(tarr[l], name, getattr(tails[l].c, name))
        S = 0 if x_decode is None else x_decode.shape[0]
        self.check(self.L.compact_prefix_stack_forward(
            self.ctx, nl, warr, tails[0].N, _i32arr(prefix_len), x_history.shape[0], _ptr(x_history), S, _ptr(x_decode),
            sarr, tarr, _ptr(y_decode), wsp, wsn, _stream()))

    # -- prefix-aware layout ------------------------------------------------------
    def prefix_workspace_bytes(self, n_workers, max_prefix_len, max_tail_len):
        n = C.c_size_t()
        self.check(self.L.compact_prefix_workspace_bytes(self.ctx, n_workers, max_prefix_len, max_tail_len, C.byref(n)))
        return n.value

    def compact_prefix_decode_step(self, x, shared, prefix_len, tails, y, route=None):
        wsp, wsn = self._ws()
        r = None if route is None else C.byref(RouteOut(route[0].data_ptr(), route[1].data_ptr()))
        self.check(self.L.compact_prefix_decode_step(self.ctx, C.byref(self.w), tails.N, _ptr(x), C.byref(shared.c),
                                                     _i32arr(prefix_len), C.byref(tails.c), _ptr(y), r, wsp, wsn, _stream()))

    def compact_attn_decode_prefix(self, q, shared, prefix_len, tails, o):
        wsp, wsn = self._ws()
        self.check(self.L.compact_attn_decode_prefix(self.ctx, tails.N, _ptr(q), C.byref(shared.c), _i32arr(prefix_len),
                                                     C.byref(tails.c), _ptr(o), wsp, wsn, _stream()))

    # -- profiling --------------------------------------------------------------
    def compact_profile_select(self, klass):
        self.check(self.L.compact_profile_select(self.ctx, klass))

    def compact_profile_read(self):
        n, ms = C.c_int64(), C.c_double()
        self.check(self.L.compact_profile_read(self.ctx, C.byref(n), C.byref(ms)))
        return n.value, ms.value

    # -- per-kernel entry points --------------------------------------------------
    def compact_mxfp4_dequant(self, codes, scales, out):
        """codes uint8 [..., K/2], scales uint8 [..., K/32] -> out bf16 [..., K]."""
        K = codes.shape[-1] * 2
        self.check(self.L.compact_mxfp4_dequant(self.ctx, _ptr(codes), _ptr(scales), codes.numel() // (K // 2), K, _ptr(out),
                                                _stream()))

    def compact_rmsnorm(self, x, g, y):
        self.check(self.L.compact_rmsnorm(self.ctx, _ptr(x), _ptr(g), _ptr(y), x.shape[0], _stream()))

    def compact_rope_kvwrite(self, cu_seqlens, qkv, kv):
        self.check(self.L.compact_rope_kvwrite(self.ctx, len(cu_seqlens) - 1, _i32arr(cu_seqlens), _ptr(qkv),
                                               C.byref(kv.c), _stream()))

    def compact_gemm(self, a, b, r, c, epilogue=0):
        wsp, wsn = self._ws()
        M, K = a.shape
        N = c.shape[1]
        self.check(self.L.compact_gemm(self.ctx, _ptr(a), _ptr(b), _ptr(r), _ptr(c), M, N, K, epilogue, wsp, wsn,
                                       _stream()))

    def compact_attn_prefill(self, cu_seqlens, qkv, kv, o):
        self.check(self.L.compact_attn_prefill(self.ctx, len(cu_seqlens) - 1, _i32arr(cu_seqlens), _ptr(qkv),
                                               C.byref(kv.c), _ptr(o), _stream()))

    def compact_attn_decode(self, q, kv, o):
        wsp, wsn = self._ws()
        self.check(self.L.compact_attn_decode(self.ctx, kv.N, _ptr(q), C.byref(kv.c), _ptr(o), wsp, wsn, _stream()))

    def compact_attn_decode_noalloc(self, q, kv, o):
        self.check(self.L.compact_attn_decode_noalloc(self.ctx, kv.N, _ptr(q), C.byref(kv.c), _ptr(o), _stream()))

    def compact_moe_route(self, m, w_router, idx, gate, logits=None):
        wsp, wsn = self._ws()
        self.check(self.L.compact_moe_route(self.ctx, _ptr(m), _ptr(w_router), m.shape[0], _ptr(idx), _ptr(gate),
                                            _ptr(logits), wsp, wsn, _stream()))

    def compact_moe_ffn(self, m, h, idx, gate, y):
        wsp, wsn = self._ws()
        self.check(self.L.compact_moe_ffn(self.ctx, C.byref(self.w), _ptr(m), _ptr(h), _ptr(idx), _ptr(gate),
                                          m.shape[0], _ptr(y), wsp, wsn, _stream()))
