"""A prefill cut into chunks on the GPU (compact_prefill_extend; paper Sec. IV-B
chunked prefill, and a worker's own block behind a cached prefix): checked against
the fp64 checker's prefill in one piece through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import layer as O
from paper_2605_23296_amd import binding as B
from paper_2605_23296_amd.workloads import WORKLOADS, LayerConfig, Workload, make_inputs, to_numpy_f64
from tests import harness as H
from tests.util import ErrLog, FP32_TOL

pytestmark = pytest.mark.gpu
DEV = "cuda"


def run_chunked(inp, cuts_per_block, n_steps=0, pos_offset=None):
    """Block b's tokens arrive in chunks of cuts_per_block[b] rows; call c holds the
    c-th chunk of every block that still has one.  Then n_steps decode steps."""
    layer, cu = inp.layer, inp.cu_seqlens
    N, T = len(inp.block_lens), cu[-1]
    lay = B.Layer(layer, {k: v.to(DEV).contiguous() for k, v in inp.weights.items()})
    dt = lay.torch_dtype
    kv = B.KVCache(layer, [L + n_steps + 5 for L in inp.block_lens], DEV, dt, pos_offset)
    kv.k.fill_(float("nan"))
    kv.v.fill_(float("nan"))
    lay.ensure_workspace(T, N, max(inp.block_lens) + n_steps, DEV)
    x = inp.x_prefill.to(DEV)
    y = torch.full((T, layer.d_model), float("nan"), dtype=dt, device=DEV)
    moe = layer.n_experts > 0
    idx_all = torch.full((T, max(layer.top_k, 1)), -1, dtype=torch.int32, device=DEV)
    gate_all = torch.zeros((T, max(layer.top_k, 1)), dtype=torch.float32, device=DEV)
    starts = [[0] + list(np.cumsum(c)) for c in cuts_per_block]
    n_calls = max(len(c) for c in cuts_per_block)
    for c in range(n_calls):
        blocks = [b for b in range(N) if c < len(cuts_per_block[b])]
        rows = [torch.arange(cu[b] + starts[b][c], cu[b] + starts[b][c + 1]) for b in blocks]
        cu_c = [0] + list(np.cumsum([len(r) for r in rows]))
        idx = torch.cat(rows).to(DEV)
        sub = B.KVCache.__new__(B.KVCache)          # a view of the chosen blocks' slabs
        sub.N, sub.layer = len(blocks), layer
        sub.k, sub.v = kv.k, kv.v
        sub.caps, sub.offs = [kv.caps[b] for b in blocks], [kv.offs[b] for b in blocks]
        import ctypes as C
        sub.h_slab_offset = (C.c_int64 * len(blocks))(*sub.offs)
        sub.h_capacity = (C.c_int32 * len(blocks))(*sub.caps)
        sub.h_len = (C.c_int32 * len(blocks))(*[kv.h_len[b] for b in blocks])
        sub.h_pos_offset = None if pos_offset is None else (C.c_int32 * len(blocks))(*[pos_offset[b] for b in blocks])
        sub.c = B.KV(kv.k.data_ptr(), kv.v.data_ptr(), sub.h_slab_offset, sub.h_capacity, sub.h_len,
                     sub.h_pos_offset if sub.h_pos_offset is not None else C.cast(None, C.POINTER(C.c_int32)))
        yc = torch.empty(len(idx), layer.d_model, dtype=dt, device=DEV)
        route = None
        if moe:
            route = (torch.empty(len(idx), layer.top_k, dtype=torch.int32, device=DEV),
                     torch.empty(len(idx), layer.top_k, dtype=torch.float32, device=DEV))
        lay.compact_prefill_extend([int(v) for v in cu_c], x[idx].contiguous(), sub, yc, route)
        y[idx] = yc
        if moe:
            idx_all[idx], gate_all[idx] = route
        for i, b in enumerate(blocks):
            kv.h_len[b] = sub.h_len[i]
    assert kv.lens() == list(inp.block_lens)
    y_dec = torch.empty(n_steps, N, layer.d_model, dtype=dt, device=DEV)
    xd = inp.x_decode[:n_steps].to(DEV).contiguous()
    for s in range(n_steps):
        lay.compact_decode_step(xd[s], kv, y_dec[s])
    torch.cuda.synchronize()
    return dict(y=y, y_dec=y_dec, kv=kv, idx=idx_all, gate=gate_all)


def check(inp, cuts, n_steps, fp32=False, pos_offset=None):
    g = run_chunked(inp, cuts, n_steps, pos_offset)
    ref = O.Layer(inp.layer.as_dict(), {k: to_numpy_f64(v) for k, v in inp.weights.items()})
    pre, y_dec, Ks, Vs, _ = ref.forward(to_numpy_f64(inp.x_prefill), inp.cu_seqlens, to_numpy_f64(inp.x_decode[:n_steps]), pos_offset)
    log = ErrLog(FP32_TOL, FP32_TOL, FP32_TOL) if fp32 else ErrLog()
    cmp = log.cmp
    cmp("y", to_numpy_f64(g["y"]), np.concatenate([p["y"] for p in pre]))
    if n_steps:
        cmp("y_dec", to_numpy_f64(g["y_dec"]), y_dec)
    for b in range(len(inp.block_lens)):
        cmp("K%d" % b, to_numpy_f64(g["kv"].block_k(b)), Ks[b])
        cmp("V%d" % b, to_numpy_f64(g["kv"].block_v(b)), Vs[b])
    log.check()


def test_tiny_fp32_chunked_prefill_in_full():
    inp = make_inputs(WORKLOADS["tiny_fp32"], block_lens=[128, 65, 1, 97], decode_steps=3, gain_jitter=True)
    check(inp, [[50, 13, 65], [64, 1], [1], [8, 80, 9]], 3, fp32=True, pos_offset=[0, 7, 3, 100])


def test_bf16_chunked_prefill_every_tile_edge():
    """Chunk boundaries on and off the 64-token KV tiles, the 128-row query tiles and the
    8-row alignment of the transposed V slab; a one-row chunk; head_dim 128."""
    layer = LayerConfig(d_model=512, n_q_heads=4, n_kv_heads=2, head_dim=128, ffn_dim=1024, rope_theta=500000.0)
    wl = Workload("small_dense", layer, [700, 130, 257], 3, 2)
    inp = make_inputs(wl, gain_jitter=True)
    check(inp, [[128, 64, 3, 1, 300, 204], [130], [5, 123, 129]], 2)


def test_bf16_chunked_prefill_head_dim_64_routed_layer_every_row():
    layer = LayerConfig(d_model=256, n_q_heads=8, n_kv_heads=2, head_dim=64, ffn_dim=320, n_experts=16, top_k=4,
                        rope_theta=500000.0)
    wl = Workload("small_moe", layer, [200, 75], 2, 0)
    inp = make_inputs(wl)
    g = run_chunked(inp, [[64, 100, 36], [70, 5]])
    ref = O.Layer(layer.as_dict(), {k: to_numpy_f64(v) for k, v in inp.weights.items()})
    pre = ref.prefill(to_numpy_f64(inp.x_prefill), inp.cu_seqlens)
    log, n_close = ErrLog(), 0
    gi, gg = g["idx"].cpu().numpy(), g["gate"].cpu().numpy()
    y = to_numpy_f64(g["y"])
    for b in range(2):
        sl = slice(inp.cu_seqlens[b], inp.cu_seqlens[b + 1])
        log.cmp("K%d" % b, to_numpy_f64(g["kv"].block_k(b)), pre[b]["K"])
        log.cmp("V%d" % b, to_numpy_f64(g["kv"].block_v(b)), pre[b]["V"])
        n_close += H.check_routing(gi[sl], pre[b]["logits"], layer.top_k, 2e-2, gg[sl])
        log.cmp("y%d" % b, y[sl], ref.ffn(pre[b]["h"], forced_idx=gi[sl])[0])       # every row
    log.check("rows with a close call: %d of %d (all compared) |" % (n_close, inp.cu_seqlens[-1]))


def test_dense_8x4096_in_chunks_of_1024_matches_the_one_piece_prefill():
    """Full size: the named workload prefilled in four chunks of 1024 rows per block.  K/V rows
    are bitwise those of the one-piece compact_prefill (projections are row-wise); the outputs
    agree within the bf16 tolerance (the softmax runs over the same rows, tiled differently)."""
    wl = WORKLOADS["dense_8x4096"]
    inp = make_inputs(wl, device=DEV, gen_device=DEV, decode_steps=0)
    g = run_chunked(inp, [[1024] * 4] * 8)
    layer, cu = inp.layer, inp.cu_seqlens
    lay = B.Layer(layer, inp.weights)
    kv = B.KVCache(layer, [L + 5 for L in inp.block_lens], DEV, torch.bfloat16)
    lay.ensure_workspace(cu[-1], 8, 4096, DEV)
    y = torch.empty(cu[-1], layer.d_model, dtype=torch.bfloat16, device=DEV)
    lay.compact_prefill(cu, inp.x_prefill, kv, y)
    torch.cuda.synchronize()
    for b in (0, 7):
        assert torch.equal(g["kv"].block_k(b), kv.block_k(b))
        assert torch.equal(g["kv"].block_v(b), kv.block_v(b))
    d = (g["y"].float() - y.float()).norm(dim=1) / y.float().norm(dim=1)
    assert d.max().item() < 2e-2, d.max().item()
