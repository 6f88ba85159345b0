"""Host-side checks of the C ABI: the library loads, exports every symbol the
header declares, and rejects bad arguments before touching the device."""
import ctypes as C
import os
import re

import pytest

from paper_2605_23296_amd import binding as B
from paper_2605_23296_amd.workloads import WORKLOADS, LayerConfig

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_symbols():
    text = open(os.path.join(ROOT, "include", "compact.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(compact_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = B.lib()
    syms = header_symbols()
    assert len(syms) >= 16
    for s in syms:
        assert hasattr(L, s), s
    assert sorted(B.EXPORTS) == syms


def test_create_validates_cfg():
    L = B.lib()
    good = WORKLOADS["tiny_fp32"].layer
    ctx = C.c_void_p()
    assert L.compact_create(C.byref(B.make_cfg(good)), C.byref(ctx)) == 0
    L.compact_destroy(ctx)
    bad = [
        (dict(head_dim=48), 2), (dict(n_kv_heads=3), 2), (dict(d_model=100), 2),
        (dict(n_experts=4, top_k=0), 2), (dict(n_experts=4, top_k=5), 2), (dict(d_model=0), 1),
        (dict(dtype="fp32", rope_theta=-1.0), 1),
        (dict(dtype="bf16", n_experts=12, top_k=2), 2),     # bf16 storage: experts in multiples of 8
    ]
    for kw, code in bad:
        d = good.as_dict()
        d.update(kw)
        cfg = B.make_cfg(LayerConfig(**d))
        assert L.compact_create(C.byref(cfg), C.byref(ctx)) == code, kw
        assert L.compact_last_error(None) != b""
    cfg = B.make_cfg(good)
    cfg.dtype = 7
    assert L.compact_create(C.byref(cfg), C.byref(ctx)) == 5
    assert L.compact_create(None, C.byref(ctx)) == 1


def test_workspace_bytes_grows_with_the_problem():
    lay = B.Layer(WORKLOADS["dense_8x4096"].layer, None)
    a = lay.workspace_bytes(1024, 4, 2048)
    b = lay.workspace_bytes(32768, 8, 4352)
    assert 0 < a < b
    # n, qkv, o, h, act for 32768 tokens in bf16
    assert b > 32768 * 2 * (4096 * 3 + 6144 + 14336)
    with pytest.raises(B.CompactError) as e:
        lay.workspace_bytes(-1, 4, 16)
    assert e.value.code == 1


def test_workspace_holds_a_model_width_row_where_the_projection_rows_are_narrower():
    """A layer whose stacked q/k/v rows are narrower than d_model: the attention scratch must
    still hold [T, d_model] (a forward pass without a prefill output buffer puts the feed-forward
    result there), so the workspace grows with d_model like that of a layer with wide rows."""
    T = 4096
    narrow = LayerConfig(d_model=1024, n_q_heads=4, n_kv_heads=4, head_dim=64, ffn_dim=1024, dtype="bf16")   # 768 columns
    wide = LayerConfig(d_model=1024, n_q_heads=8, n_kv_heads=4, head_dim=64, ffn_dim=1024, dtype="bf16")     # 1024 columns
    a = B.Layer(narrow, None).workspace_bytes(T, 4, 64) - B.Layer(narrow, None).workspace_bytes(0, 4, 64)
    b = B.Layer(wide, None).workspace_bytes(T, 4, 64) - B.Layer(wide, None).workspace_bytes(0, 4, 64)
    # per token: n (d) + scratch (max(cols, d)) + o (Dq) + h (fp32 d) + act (F): only o differs
    assert b - a == T * 2 * (8 - 4) * 64
    assert a >= T * (2 * 1024 + 2 * 1024 + 2 * 256 + 4 * 1024 + 2 * 1024)


def _fake_layer(name="tiny_fp32"):
    layer = WORKLOADS[name].layer

    class T:  # stand-in for a device tensor: validation never dereferences it
        def __init__(self, addr):
            self.addr = addr

        def data_ptr(self):
            return self.addr

    names = ["g_attn", "w_qkv", "w_o", "g_ffn", "w_gate_up", "w_down"]
    return B.Layer(layer, {n: T(0x1000 * (i + 1)) for i, n in enumerate(names)})


def _kv(caps, lens, offs=None):
    n = len(caps)
    offs = offs or [i * 1 << 20 for i in range(n)]
    keep = dict(off=(C.c_int64 * n)(*offs), cap=(C.c_int32 * n)(*caps), len=(C.c_int32 * n)(*lens))
    kv = B.KV(0x10000, 0x20000, keep["off"], keep["cap"], keep["len"], C.cast(None, C.POINTER(C.c_int32)))
    return kv, keep


def test_layer_calls_reject_bad_arguments_without_a_device():
    lay = _fake_layer()
    L, ctx, w = lay.L, lay.ctx, C.byref(lay.w)
    x = C.c_void_p(0x30000)
    ws = C.c_void_p(0x40000)
    kv, keep = _kv([128, 128], [0, 0])
    cu = (C.c_int32 * 3)(0, 100, 200)

    def prefill(cu=cu, x=x, kv=kv, y=x, ws=ws, n=2, w=w):
        return L.compact_prefill(ctx, w, n, cu, x, C.byref(kv) if kv is not None else None, y, None, ws, 1 << 30, None)

    assert prefill(n=0) == 1
    assert prefill(cu=None) == 1
    assert prefill(cu=(C.c_int32 * 3)(0, 100, 100)) == 1          # empty block
    assert b"empty" in L.compact_last_error(ctx)
    assert prefill(cu=(C.c_int32 * 3)(0, 100, 50)) == 1           # not increasing
    assert prefill(cu=(C.c_int32 * 3)(1, 100, 200)) == 1          # does not start at 0
    assert prefill(x=None) == 1
    assert prefill(y=None) == 1
    assert prefill(kv=None) == 1
    assert prefill(ws=None) == 4
    assert prefill(w=None) == 1
    assert prefill(cu=(C.c_int32 * 3)(0, 129, 200)) == 3          # block longer than its slab
    kv2, k2 = _kv([128, 100], [0, 0])
    assert prefill(kv=kv2) == 1                                   # capacity not a multiple of 8
    kv3, k3 = _kv([128, 128], [0, 0], offs=[0, 12])
    assert prefill(kv=kv3) == 1                                   # slab offset not a multiple of 8

    # decode: len + 1 must fit the slab
    kv4, k4 = _kv([128, 128], [128, 5])
    assert L.compact_decode_step(ctx, w, 2, x, C.byref(kv4), x, None, ws, 1 << 30, None) == 3
    assert k4["len"][0] == 128 and k4["len"][1] == 5              # untouched on failure
    kv5, k5 = _kv([128, 128], [5, 5])
    assert L.compact_decode_step(ctx, w, 2, None, C.byref(kv5), x, None, ws, 1 << 30, None) == 1
    assert L.compact_decode_step(ctx, w, 2, x, C.byref(kv5), x, None, None, 0, None) == 4

    # forward: prefill rows + decode steps must fit
    assert L.compact_layer_forward(ctx, w, 2, cu, x, 29, x, C.byref(kv), x, None, x, ws, 1 << 30, None) == 3
    assert L.compact_layer_forward(ctx, w, 2, cu, x, -1, x, C.byref(kv), x, None, x, ws, 1 << 30, None) == 1
    assert L.compact_layer_forward(ctx, w, 2, cu, x, 4, None, C.byref(kv), x, None, x, ws, 1 << 30, None) == 1


def test_kernel_hooks_reject_bad_arguments_without_a_device():
    lay = _fake_layer()
    L, ctx = lay.L, lay.ctx
    p = C.c_void_p(0x1000)
    assert L.compact_rmsnorm(ctx, None, p, p, 4, None) == 1
    assert L.compact_gemm(ctx, p, p, None, None, 4, 8, 8, 0, None, 0, None) == 1
    assert L.compact_gemm(ctx, p, p, None, p, 4, 8, 8, 3, None, 0, None) == 1
    assert L.compact_moe_route(ctx, p, p, 4, p, p, p, None, 0, None) == 1     # dense layer: no experts
    kv, keep = _kv([128], [0])
    assert L.compact_attn_decode(ctx, 1, p, C.byref(kv), p, None, 0, None) == 3   # empty cache
    blay = _fake_layer("dense_8x4096")
    assert blay.L.compact_gemm(blay.ctx, p, p, None, p, 128, 64, 100, 0, None, 0, None) == 2


def test_no_alloc_decode_attention_checks_its_limits_without_a_device():
    lay = _fake_layer("dense_8x4096")
    L = B.lib()
    q, o = C.c_void_p(0x3000), C.c_void_p(0x4000)
    kv, keep = _kv([16] * 65, [8] * 65)
    assert L.compact_attn_decode_noalloc(lay.ctx, 65, q, C.byref(kv), o, None) == 3        # more than 64 blocks
    assert b"64 blocks" in L.compact_last_error(lay.ctx)
    kv, keep = _kv([8208] * 64, [8200] * 64)
    assert L.compact_attn_decode_noalloc(lay.ctx, 64, q, C.byref(kv), o, None) == 3        # records beyond 32 MiB
    assert b"32 MiB" in L.compact_last_error(lay.ctx)
    kv, keep = _kv([16], [17])
    assert L.compact_attn_decode_noalloc(lay.ctx, 1, q, C.byref(kv), o, None) == 3         # h_len beyond the slab
    kv, keep = _kv([16], [8])
    assert L.compact_attn_decode_noalloc(lay.ctx, 1, None, C.byref(kv), o, None) == 1
    assert L.compact_attn_decode_noalloc(lay.ctx, 0, q, C.byref(kv), o, None) == 1
    assert L.compact_attn_decode_noalloc(_fake_layer("tiny_fp32").ctx, 1, q, C.byref(kv), o, None) == 5   # fp32 storage


def test_prefix_aware_calls_reject_bad_arguments_without_a_device():
    lay = _fake_layer("dense_8x4096")
    L, ctx, w = lay.L, lay.ctx, C.byref(lay.w)
    x = C.c_void_p(0x30000)
    ws = C.c_void_p(0x40000)
    shared, ks = _kv([1024], [1000])
    tails, kt = _kv([64, 64, 64], [0, 3, 64])

    def step(prefix, tails=tails, shared=shared, n=3, ws=ws, x=x):
        pl = (C.c_int32 * len(prefix))(*prefix) if prefix is not None else None
        return L.compact_prefix_decode_step(ctx, w, n, x, C.byref(shared) if shared is not None else None, pl,
                                            C.byref(tails) if tails is not None else None, x, None, ws, 1 << 30, None)

    assert step([100, 200, 300]) == 3                     # worker 2's tail is full
    assert b"tail" in L.compact_last_error(ctx)
    tails2, kt2 = _kv([64, 64, 64], [0, 3, 5])
    assert step([100, 50, 300], tails=tails2) == 1        # prefixes must not decrease
    assert step([100, 200, 1001], tails=tails2) == 1      # prefix beyond the shared rows
    assert step(None, tails=tails2) == 1
    assert step([100, 200, 300], tails=tails2, shared=None) == 1
    assert step([100, 200, 300], tails=None) == 1
    assert step([100, 200, 300], tails=tails2, ws=None) == 4
    assert step([100, 200, 300], tails=tails2, x=None) == 1
    assert step([100, 200, 300], tails=tails2, n=0) == 1
    assert kt2["len"][1] == 3                             # untouched on failure
    n = C.c_size_t()
    assert L.compact_prefix_workspace_bytes(ctx, 8, 32768, 256, C.byref(n)) == 0 and n.value > 0
    small = n.value
    assert L.compact_prefix_workspace_bytes(ctx, 8, 65536, 256, C.byref(n)) == 0 and n.value > small
    assert L.compact_prefix_workspace_bytes(ctx, 0, 32768, 256, C.byref(n)) == 1
    # fp32 storage has no prefix-aware path
    flay = _fake_layer()
    s32, _k1 = _kv([128], [100])
    t32, _k2 = _kv([16, 16], [0, 0])
    pl = (C.c_int32 * 2)(50, 100)
    assert flay.L.compact_prefix_decode_step(flay.ctx, C.byref(flay.w), 2, x, C.byref(s32), pl, C.byref(t32), x, None, ws,
                                             1 << 30, None) == 5


def test_stack_call_rejects_bad_arguments_without_a_device():
    lay = _fake_layer()
    L, ctx = lay.L, lay.ctx
    x = C.c_void_p(0x30000)
    ws = C.c_void_p(0x40000)
    cu = (C.c_int32 * 3)(0, 100, 200)
    warr = (B.Weights * 2)()
    for l in range(2):
        for name, _ in B.Weights._fields_:
            setattr(warr[l], name, getattr(lay.w, name))

    def kvarr(caps_per_layer, offs_per_layer=None):
        arr, keep = (B.KV * len(caps_per_layer))(), []
        for l, caps in enumerate(caps_per_layer):
            kv, k = _kv(caps, [0] * len(caps), None if offs_per_layer is None else offs_per_layer[l])
            keep.append(k)
            for name, _ in B.KV._fields_:
                setattr(arr[l], name, getattr(kv, name))
        return arr, keep

    def stack(nl=2, w=warr, kv=None, steps=4, xd=x, yd=x, ws=ws, wsn=1 << 30):
        return L.compact_stack_forward(ctx, nl, w, 2, cu, x, steps, xd, kv, None, yd, ws, wsn, None)

    good, keep = kvarr([[128, 128], [128, 128]])
    assert stack(nl=0, kv=good) == 1
    assert stack(w=None, kv=good) == 1
    assert stack(kv=None) == 1
    assert stack(kv=good, steps=-1) == 1
    assert stack(kv=good, xd=None) == 1
    assert stack(kv=good, ws=None) == 4
    assert stack(kv=good, steps=29) == 3                       # 100 + 29 rows do not fit 128
    other_caps, k2 = kvarr([[128, 128], [128, 136]])
    assert stack(kv=other_caps) == 1                           # layer 1's slabs differ from layer 0's
    assert b"geometry" in L.compact_last_error(ctx)
    other_offs, k3 = kvarr([[128, 128], [128, 128]], [[0, 1 << 20], [0, 1 << 21]])
    assert stack(kv=other_offs) == 1
    assert keep[1]["len"][0] == 0                              # untouched on failure
    n, m = C.c_size_t(), C.c_size_t()
    assert L.compact_stack_workspace_bytes(ctx, 512, 4, 160, C.byref(n)) == 0
    assert L.compact_workspace_bytes(ctx, 512, 4, 160, C.byref(m)) == 0
    assert n.value >= m.value + 2 * 512 * 256 * 4 + 2 * 4 * 256 * 4
    assert L.compact_stack_workspace_bytes(ctx, 512, 0, 160, C.byref(n)) == 1


def test_prefill_extend_rejects_bad_arguments_without_a_device():
    lay = _fake_layer()
    L, ctx, w = lay.L, lay.ctx, C.byref(lay.w)
    x = C.c_void_p(0x30000)
    ws = C.c_void_p(0x40000)
    cu = (C.c_int32 * 3)(0, 100, 200)
    kv, keep = _kv([128, 128], [28, 29])
    call = lambda kv=kv, y=x, ws=ws: L.compact_prefill_extend(ctx, w, 2, cu, x, C.byref(kv), y, None, ws, 1 << 30, None)
    assert call() == 3                                    # block 1: 29 cached + 100 new rows > 128
    assert b"chunk" in L.compact_last_error(ctx)
    assert keep["len"][0] == 28 and keep["len"][1] == 29  # untouched on failure
    kv2, keep2 = _kv([128, 128], [-1, 0])
    assert call(kv=kv2) == 1
    kv3, _ = _kv([128, 128], [28, 28])
    assert call(kv=kv3, y=None) == 1
    assert call(kv=kv3, ws=None) == 4


def test_mixed_forward_rejects_bad_arguments_without_a_device():
    lay = _fake_layer()
    L, ctx, w = lay.L, lay.ctx, C.byref(lay.w)
    x = C.c_void_p(0x30000)
    ws = C.c_void_p(0x40000)
    cu = (C.c_int32 * 3)(0, 100, 200)
    kv, keep = _kv([128, 128], [0, 0])
    call = lambda budget=64, steps=4, xd=x, ws=ws, kv=kv: L.compact_mixed_forward(
        ctx, w, 2, cu, x, steps, xd, C.byref(kv) if kv is not None else None, budget, None, x, ws, 1 << 30, None)
    assert call(budget=2) == 1                         # every decoding block needs a row of its own, plus a chunk row
    assert b"max_batched_tokens" in L.compact_last_error(ctx)
    assert call(steps=-1) == 1
    assert call(xd=None) == 1
    assert call(ws=None) == 4
    assert call(kv=None) == 1
    assert call(steps=29) == 3                         # 100 + 29 rows do not fit 128
    n, m = C.c_size_t(), C.c_size_t()
    assert L.compact_mixed_workspace_bytes(ctx, 64, 2, 160, C.byref(n)) == 0
    assert L.compact_workspace_bytes(ctx, 200, 2, 160, C.byref(m)) == 0
    assert 0 < n.value < m.value                       # sized by the budget, not by the 200 prefill tokens


def test_prefix_stack_call_rejects_bad_arguments_without_a_device():
    lay = _fake_layer("dense_8x4096")
    L, ctx = lay.L, lay.ctx
    x = C.c_void_p(0x30000)
    ws = C.c_void_p(0x40000)
    warr = (B.Weights * 2)()
    for l in range(2):
        for name, _ in B.Weights._fields_:
            setattr(warr[l], name, getattr(lay.w, name))

    def kvarr(caps, lens, n=2, caps1=None):
        arr, keep = (B.KV * n)(), []
        for l in range(n):
            kv, k = _kv(caps if (l == 0 or caps1 is None) else caps1, list(lens))
            keep.append(k)
            for name, _ in B.KV._fields_:
                setattr(arr[l], name, getattr(kv, name))
        return arr, keep

    shared, ks = kvarr([1024], [0])
    tails, kt = kvarr([64, 64, 64], [0, 0, 0])

    def call(prefix=(100, 200, 1000), T=1000, steps=4, nl=2, shared=shared, tails=tails, ws=ws, xd=x):
        pl = (C.c_int32 * len(prefix))(*prefix)
        return L.compact_prefix_stack_forward(ctx, nl, warr, 3, pl, T, x, steps, xd, shared, tails, x, ws, 1 << 40, None)

    assert call(nl=0) == 1
    assert call(T=0) == 1
    assert call(T=1025) == 3                                  # the history does not fit the shared cache
    assert call(prefix=(100, 50, 1000)) == 1                  # prefixes must not decrease
    assert call(prefix=(100, 200, 1001)) == 1                 # prefix beyond the history
    assert call(steps=65) == 3                                # tails too small
    assert call(steps=-1) == 1
    assert call(xd=None) == 1
    assert call(ws=None) == 4
    other, ko = kvarr([64, 64, 64], [0, 0, 0], caps1=[64, 64, 72])
    assert call(tails=other) == 1
    assert b"geometry" in L.compact_last_error(ctx)
    assert ks[0]["len"][0] == 0 and ks[1]["len"][0] == 0      # untouched on failure
    n = C.c_size_t()
    assert L.compact_prefix_stack_workspace_bytes(ctx, 1000, 3, 8, C.byref(n)) == 0 and n.value > 0
    flay = _fake_layer()                                      # fp32 storage has no prefix-aware path
    w32 = (B.Weights * 1)()
    for name, _ in B.Weights._fields_:
        setattr(w32[0], name, getattr(flay.w, name))
    s32, _a = kvarr([128], [0], n=1)
    t32, _b = kvarr([16, 16, 16], [0, 0, 0], n=1)
    pl = (C.c_int32 * 3)(10, 20, 100)
    assert flay.L.compact_prefix_stack_forward(flay.ctx, 1, w32, 3, pl, 100, x, 2, x, s32, t32, x, ws, 1 << 40, None) == 5
