"""A depth of layers on the GPU (compact_stack_forward; the models of paper
Sec. IV-A are stacks of the one layer): checked against the fp64 checker on
stacks it finishes in seconds, and -- at the named workload's full size --
against the composition of the single-layer calls, which must be bitwise equal."""
import numpy as np
import pytest
import torch

from oracle import layer as O
from paper_2605_23296_amd import binding as B
from paper_2605_23296_amd.workloads import WORKLOADS, LayerConfig, Workload, make_inputs, make_stack_weights, to_numpy_f64
from tests import harness as H
from tests.util import ErrLog, FP32_TOL

pytestmark = pytest.mark.gpu
DEV = "cuda"


def run_stack(inp, weights, n_steps):
    layer, cu = inp.layer, inp.cu_seqlens
    N, T, nl = len(inp.block_lens), cu[-1], len(weights)
    wdev = [{k: v.to(DEV).contiguous() for k, v in w.items()} for w in weights]
    lay = B.Layer(layer, wdev[0])
    dt = lay.torch_dtype
    kvs = [B.KVCache(layer, [L + n_steps + 3 for L in inp.block_lens], DEV, dt) for _ in range(nl)]
    for kv in kvs:
        kv.k.fill_(float("nan"))
        kv.v.fill_(float("nan"))
    lay.ws = torch.empty(lay.stack_workspace_bytes(T, N, max(inp.block_lens) + n_steps), dtype=torch.uint8, device=DEV)
    y_last = torch.empty(N, layer.d_model, dtype=dt, device=DEV)
    y_dec = torch.empty(n_steps, N, layer.d_model, dtype=dt, device=DEV)
    xd = inp.x_decode[:n_steps].to(DEV).contiguous()
    lay.compact_stack_forward(wdev, cu, inp.x_prefill.to(DEV), xd if n_steps else None, kvs, y_last, y_dec if n_steps else None)
    torch.cuda.synchronize()
    for kv in kvs:
        assert kv.lens() == [L + n_steps for L in inp.block_lens]
    return dict(y_last=y_last, y_dec=y_dec, kvs=kvs, wdev=wdev, lay=lay)


def check_against_oracle(inp, weights, n_steps, fp32=False):
    g = run_stack(inp, weights, n_steps)
    ref = O.Stack(inp.layer.as_dict(), [{k: to_numpy_f64(v) for k, v in w.items()} for w in weights])
    y_pre, y_dec, Ks, Vs = ref.forward(to_numpy_f64(inp.x_prefill), inp.cu_seqlens, to_numpy_f64(inp.x_decode[:n_steps]))
    cu = inp.cu_seqlens
    log = ErrLog(FP32_TOL, FP32_TOL, FP32_TOL) if fp32 else ErrLog.for_depth(len(weights))
    cmp = log.cmp
    cmp("y_last", to_numpy_f64(g["y_last"]), np.stack([y_pre[cu[b + 1] - 1] for b in range(len(cu) - 1)]))
    cmp("y_dec", to_numpy_f64(g["y_dec"]), y_dec)
    for li in range(len(weights)):
        for b in range(len(cu) - 1):
            cmp("K%d_%d" % (li, b), to_numpy_f64(g["kvs"][li].block_k(b)), Ks[li][b])
            cmp("V%d_%d" % (li, b), to_numpy_f64(g["kvs"][li].block_v(b)), Vs[li][b])
    log.check()


def test_tiny_fp32_stack_of_three_layers_in_full():
    wl = WORKLOADS["tiny_fp32"]
    inp = make_inputs(wl, block_lens=[128, 65, 1, 97], decode_steps=5)
    check_against_oracle(inp, make_stack_weights(wl, 3, gain_jitter=True), 5, fp32=True)


def test_bf16_stack_of_four_layers_ragged_blocks():
    layer = LayerConfig(d_model=512, n_q_heads=4, n_kv_heads=2, head_dim=128, ffn_dim=1024, rope_theta=500000.0)
    wl = Workload("small_dense", layer, [300, 77, 513], 3, 4)
    inp = make_inputs(wl)
    check_against_oracle(inp, make_stack_weights(wl, 4, gain_jitter=True), 4)


def test_bf16_moe_stack_every_row():
    """Routed layers through the depth.  The stack call must give the bits of the single-layer
    calls applied layer by layer; those also report their routing tables, and the fp64 stack is
    evaluated for exactly those (validated) expert choices, layer by layer, so that every output
    row and every cache row of every layer is compared."""
    layer = LayerConfig(d_model=256, n_q_heads=8, n_kv_heads=2, head_dim=64, ffn_dim=320, n_experts=16, top_k=4,
                        rope_theta=500000.0)
    wl = Workload("small_moe", layer, [130, 40], 2, 3)
    inp = make_inputs(wl)
    nl, S, N, k = 2, 3, 2, layer.top_k
    ws = make_stack_weights(wl, nl)
    g = run_stack(inp, ws, S)
    cu, T, dt = inp.cu_seqlens, inp.cu_seqlens[-1], torch.bfloat16
    lays = [B.Layer(layer, w) for w in g["wdev"]]
    kvs = [B.KVCache(layer, [L + S + 3 for L in inp.block_lens], DEV, dt) for _ in range(nl)]
    idx_pre = [torch.empty(T, k, dtype=torch.int32, device=DEV) for _ in range(nl)]
    gate_pre = [torch.empty(T, k, dtype=torch.float32, device=DEV) for _ in range(nl)]
    idx_dec = [torch.empty(S, N, k, dtype=torch.int32, device=DEV) for _ in range(nl)]
    gate_dec = [torch.empty(S, N, k, dtype=torch.float32, device=DEV) for _ in range(nl)]
    x = inp.x_prefill.to(DEV)
    for l in range(nl):
        lays[l].ensure_workspace(T, N, max(inp.block_lens) + S, DEV)
        y = torch.empty(T, layer.d_model, dtype=dt, device=DEV)
        lays[l].compact_prefill(cu, x, kvs[l], y, (idx_pre[l], gate_pre[l]))
        x = y
    assert torch.equal(g["y_last"], x[[c - 1 for c in cu[1:]]])
    for s in range(S):
        xs = inp.x_decode[s].to(DEV).contiguous()
        for l in range(nl):
            ys = torch.empty(N, layer.d_model, dtype=dt, device=DEV)
            lays[l].compact_decode_step(xs, kvs[l], ys, (idx_dec[l][s], gate_dec[l][s]))
            xs = ys
        assert torch.equal(g["y_dec"][s], xs), s
    torch.cuda.synchronize()
    for l in range(nl):
        for b in range(N):
            assert torch.equal(g["kvs"][l].block_k(b), kvs[l].block_k(b)) and torch.equal(g["kvs"][l].block_v(b), kvs[l].block_v(b))
    ref = O.Stack(layer.as_dict(), [{k_: to_numpy_f64(v) for k_, v in w.items()} for w in ws])
    forced = [(idx_pre[l].cpu().numpy(), idx_dec[l].cpu().numpy()) for l in range(nl)]
    y_pre, y_dec, Ks, Vs = ref.forward(to_numpy_f64(inp.x_prefill), cu, to_numpy_f64(inp.x_decode), forced=forced)
    n_close = 0
    for l in range(nl):       # each layer's choices against the logits of the pass that follows the earlier layers' choices
        r = ref.routes[l]
        n_close += H.check_routing(forced[l][0], r["pre_logits"], k, 2e-2, gate_pre[l].cpu().numpy())
        for s in range(S):
            n_close += H.check_routing(forced[l][1][s], r["dec_logits"][s], k, 2e-2, gate_dec[l][s].cpu().numpy())
    log = ErrLog.for_depth(nl)
    log.cmp("y_pre", to_numpy_f64(x), y_pre)
    log.cmp("y_dec", to_numpy_f64(g["y_dec"]), y_dec)
    for l in range(nl):
        for b in range(N):
            log.cmp("K%d_%d" % (l, b), to_numpy_f64(g["kvs"][l].block_k(b)), Ks[l][b])
            log.cmp("V%d_%d" % (l, b), to_numpy_f64(g["kvs"][l].block_v(b)), Vs[l][b])
    log.check("rows with a close call: %d of %d (all compared) |" % (n_close, nl * (T + S * N)))


def test_dense_8x4096_stack_equals_the_single_layer_calls_bitwise():
    """Full size: three layers of the named workload through compact_stack_forward must
    give the bits of compact_prefill / compact_decode_step applied layer by layer (those
    are checked against the fp64 checker at this size in test_gpu_full_size.py)."""
    wl = WORKLOADS["dense_8x4096"]
    S, nl = 3, 3
    inp = make_inputs(wl, device=DEV, gen_device=DEV, decode_steps=S)
    ws = make_stack_weights(wl, nl, device=DEV, gen_device=DEV)
    g = run_stack(inp, ws, S)
    layer, cu = inp.layer, inp.cu_seqlens
    N, T = len(inp.block_lens), cu[-1]
    dt = torch.bfloat16
    lays = [B.Layer(layer, w) for w in g["wdev"]]
    kvs = [B.KVCache(layer, [L + S + 3 for L in inp.block_lens], DEV, dt) for _ in range(nl)]
    x = inp.x_prefill
    for l in range(nl):
        lays[l].ensure_workspace(T, N, max(inp.block_lens) + S, DEV)
        y = torch.empty(T, layer.d_model, dtype=dt, device=DEV)
        lays[l].compact_prefill(cu, x, kvs[l], y)
        x = y
    assert torch.equal(g["y_last"], x[[c - 1 for c in cu[1:]]])
    for s in range(S):
        xs = inp.x_decode[s].contiguous()
        for l in range(nl):
            ys = torch.empty(N, layer.d_model, dtype=dt, device=DEV)
            lays[l].compact_decode_step(xs, kvs[l], ys)
            xs = ys
        assert torch.equal(g["y_dec"][s], xs), s
    torch.cuda.synchronize()
    for l in range(nl):
        for b in (0, N - 1):
            assert torch.equal(g["kvs"][l].block_k(b), kvs[l].block_k(b))
            assert torch.equal(g["kvs"][l].block_v(b), kvs[l].block_v(b))


def run_prefix_stack(inp, weights, n_steps):
    layer, cu = inp.layer, inp.cu_seqlens
    N, T, nl = len(inp.block_lens), cu[-1], len(weights)
    wdev = [{k: v.to(DEV).contiguous() for k, v in w.items()} for w in weights]
    lay = B.Layer(layer, wdev[0])
    dt = torch.bfloat16
    shared = [B.KVCache(layer, [T + 5], DEV, dt) for _ in range(nl)]
    tails = [B.KVCache(layer, [n_steps + 3] * N, DEV, dt) for _ in range(nl)]
    for c in shared + tails:
        c.k.fill_(float("nan"))
        c.v.fill_(float("nan"))
    lay.ws = torch.empty(lay.prefix_stack_workspace_bytes(T, N, n_steps), dtype=torch.uint8, device=DEV)
    y_dec = torch.empty(n_steps, N, layer.d_model, dtype=dt, device=DEV)
    lay.compact_prefix_stack_forward(wdev, [int(c) for c in cu[1:]], inp.x_prefill.to(DEV), inp.x_decode[:n_steps].to(DEV).contiguous(),
                                     shared, tails, y_dec)
    torch.cuda.synchronize()
    for l in range(nl):
        assert shared[l].lens() == [T] and tails[l].lens() == [n_steps] * N
    return dict(y_dec=y_dec, shared=shared, tails=tails, wdev=wdev)


def test_prefix_aware_stack_of_three_layers():
    """The paper's own configuration in small: prefix-aware workers through a depth of layers."""
    layer = LayerConfig(d_model=512, n_q_heads=4, n_kv_heads=2, head_dim=128, ffn_dim=1024, rope_theta=500000.0)
    wl = Workload("small_dense", layer, [300, 77, 513, 40], 4, 3)
    inp = make_inputs(wl)
    ws = make_stack_weights(wl, 3, gain_jitter=True)
    g = run_prefix_stack(inp, ws, 3)
    ref = O.Stack(layer.as_dict(), [{k: to_numpy_f64(v) for k, v in w.items()} for w in ws])
    yd, shared, Kt, Vt = ref.forward_prefix(to_numpy_f64(inp.x_prefill), inp.cu_seqlens, to_numpy_f64(inp.x_decode))
    log = ErrLog.for_depth(3)
    log.cmp("y_dec", to_numpy_f64(g["y_dec"]), yd)
    for li in range(3):
        log.cmp("Ks%d" % li, to_numpy_f64(g["shared"][li].block_k(0)), shared[li][0])
        log.cmp("Vs%d" % li, to_numpy_f64(g["shared"][li].block_v(0)), shared[li][1])
        for b in range(4):
            log.cmp("Kt%d_%d" % (li, b), to_numpy_f64(g["tails"][li].block_k(b)), Kt[li][b])
            log.cmp("Vt%d_%d" % (li, b), to_numpy_f64(g["tails"][li].block_v(b)), Vt[li][b])
    log.check()


def test_prefix_aware_stack_equals_the_single_layer_calls_bitwise_at_full_size():
    """dense_8x4096 (one 32768-token history, 8 workers), two layers, three steps: the stack call must give
    the bits of compact_prefill + compact_prefix_decode_step applied layer by layer."""
    wl = WORKLOADS["dense_8x4096"]
    S, nl = 3, 2
    inp = make_inputs(wl, device=DEV, gen_device=DEV, decode_steps=S)
    ws = make_stack_weights(wl, nl, device=DEV, gen_device=DEV)
    g = run_prefix_stack(inp, ws, S)
    layer, cu = inp.layer, inp.cu_seqlens
    N, T = len(inp.block_lens), cu[-1]
    dt = torch.bfloat16
    prefix = [int(c) for c in cu[1:]]
    lays = [B.Layer(layer, w) for w in g["wdev"]]
    shared = [B.KVCache(layer, [T + 5], DEV, dt) for _ in range(nl)]
    tails = [B.KVCache(layer, [S + 3] * N, DEV, dt) for _ in range(nl)]
    x = inp.x_prefill
    for l in range(nl):
        lays[l].ensure_workspace(T, 1, T, DEV)
        y = torch.empty(T, layer.d_model, dtype=dt, device=DEV)
        lays[l].compact_prefill([0, T], x, shared[l], y)
        x = y
        need = lays[l].prefix_workspace_bytes(N, T, S)
        if lays[l].ws.numel() < need:
            lays[l].ws = torch.empty(need, dtype=torch.uint8, device=DEV)
    for s in range(S):
        xs = inp.x_decode[s].contiguous()
        for l in range(nl):
            ys = torch.empty(N, layer.d_model, dtype=dt, device=DEV)
            lays[l].compact_prefix_decode_step(xs, shared[l], prefix, tails[l], ys)
            xs = ys
        assert torch.equal(g["y_dec"][s], xs), s
    torch.cuda.synchronize()
    for l in range(nl):
        assert torch.equal(g["shared"][l].block_k(0), shared[l].block_k(0))
        for b in (0, N - 1):
            assert torch.equal(g["tails"][l].block_k(b), tails[l].block_k(b))
            assert torch.equal(g["tails"][l].block_v(b), tails[l].block_v(b))
