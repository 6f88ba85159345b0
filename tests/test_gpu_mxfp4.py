"""Block-scaled 4-bit expert weights on the GPU (paper Sec. IV-B "mxfp4 weights";
OCP Microscaling Formats v1.0): the expansion to bf16 is checked bit for bit against
the checker's field-by-field definition, routed decode steps that stream the 4-bit
arrays against the fp64 layer whose expert weights are that definition's values."""
import numpy as np
import pytest
import torch

from oracle import layer as O
from oracle import mxfp4 as Q
from paper_2605_23296_amd import binding as B
from paper_2605_23296_amd.workloads import (WORKLOADS, LayerConfig, Workload, make_inputs, make_mxfp4_experts,
                                            to_numpy_f64)
from tests import harness as H
from tests.util import ErrLog

pytestmark = pytest.mark.gpu
DEV = "cuda"


def test_expansion_is_bit_exact_for_every_code_and_a_range_of_scales():
    lay = B.Layer(WORKLOADS["moe_16x8192"].layer, None)
    g = torch.Generator().manual_seed(5)
    rows, K = 37, 320
    codes = torch.randint(0, 256, (rows, K // 2), generator=g, dtype=torch.uint8)
    codes[0, :128] = torch.arange(256, dtype=torch.int32)[:128].to(torch.uint8)        # every byte value once ...
    codes[1, :128] = (torch.arange(256, dtype=torch.int32)[128:]).to(torch.uint8)      # ... over two rows
    scales = torch.randint(100, 140, (rows, K // 32), generator=g, dtype=torch.uint8)
    scales[2] = torch.tensor([8, 60, 119, 120, 126, 127, 128, 130, 200, 246], dtype=torch.uint8)
    out = torch.empty(rows, K, dtype=torch.bfloat16, device=DEV)
    lay.compact_mxfp4_dequant(codes.to(DEV), scales.to(DEV), out)
    torch.cuda.synchronize()
    ref = Q.dequantize(codes.numpy(), scales.numpy())
    got = to_numpy_f64(out)
    assert np.array_equal(got, ref)
    assert np.array_equal(np.signbit(got), np.signbit(ref))      # -0.0 stays -0.0


def build(layer, block_lens, steps, seed=0, scale_spread=0):
    wl = Workload("q4", layer, block_lens, len(block_lens), steps, seed=seed)
    inp = make_inputs(wl)
    gen = torch.Generator().manual_seed(seed + 77)
    q4 = make_mxfp4_experts(layer, gen, scale_spread=scale_spread)
    return inp, q4


def oracle_weights(inp, q4):
    w = {k: to_numpy_f64(v) for k, v in inp.weights.items() if not k.startswith("w_exp_")}
    w["w_exp_gate_up"] = Q.dequantize(q4["w_exp_gate_up_q"].numpy(), q4["w_exp_gate_up_s"].numpy())
    w["w_exp_down"] = Q.dequantize(q4["w_exp_down_q"].numpy(), q4["w_exp_down_s"].numpy())
    return w


def device_weights(lay0, inp, q4):
    """The library's inputs: the 4-bit arrays plus the bf16 copy its own expansion writes."""
    w = {k: v.to(DEV).contiguous() for k, v in inp.weights.items() if not k.startswith("w_exp_")}
    for k, v in q4.items():
        w[k] = v.to(DEV).contiguous()
    for name in ("w_exp_gate_up", "w_exp_down"):
        c, s = w[name + "_q"], w[name + "_s"]
        out = torch.empty(c.shape[:-1] + (c.shape[-1] * 2,), dtype=torch.bfloat16, device=DEV)
        lay0.compact_mxfp4_dequant(c, s, out)
        w[name] = out
    return w


@pytest.mark.parametrize("d,F,spread,lens", [(256, 320, 0, None), (1216, 1088, 0, None), (1216, 1088, 30, None),
                                             (256, 320, 0, [7] * 48), (256, 320, 0, [5] * 70)])
def test_routed_decode_steps_streaming_4bit_experts(d, F, spread, lens):
    """d = 256: one k-slice of two MFMA groups; d = 1216 / F = 1088: a full 1024-wide slice plus a
    slice of 6 (2) blocks, i.e. a partial group of four.  Empty experts, experts with several rows.
    spread = 30: scale bytes from 56 to 181 (2^-71 .. 2^54) through the streaming kernels, every
    expert's contribution still O(1) (workloads.make_mxfp4_experts)."""
    layer = LayerConfig(d_model=d, n_q_heads=8, n_kv_heads=2, head_dim=64, ffn_dim=F, n_experts=16, top_k=4,
                        rope_theta=500000.0)
    lens = lens or [70, 33, 129, 5, 64]     # 48 blocks: experts with more than 16 rows, streamed tile by tile
    inp, q4 = build(layer, lens, 3, scale_spread=spread)
    if spread:
        sc = torch.cat([q4["w_exp_gate_up_s"].flatten(), q4["w_exp_down_s"].flatten()])
        assert int(sc.min()) <= 60 and int(sc.max()) >= 180
    lay0 = B.Layer(layer, None)
    w = device_weights(lay0, inp, q4)
    lay = B.Layer(layer, w)
    N, S, cu = len(lens), 3, inp.cu_seqlens
    dt = torch.bfloat16
    kv = B.KVCache(layer, [L + S for L in inp.block_lens], DEV, dt)
    lay.ensure_workspace(cu[-1], N, max(inp.block_lens) + S, DEV)
    y_pre = torch.empty(cu[-1], d, dtype=dt, device=DEV)
    lay.compact_prefill(cu, inp.x_prefill.to(DEV), kv, y_pre)
    xd = inp.x_decode.to(DEV).contiguous()
    y_dec = torch.empty(S, N, d, dtype=dt, device=DEV)
    idx = torch.empty(S, N, 4, dtype=torch.int32, device=DEV)
    gate = torch.empty(S, N, 4, dtype=torch.float32, device=DEV)
    for s in range(S):
        lay.compact_decode_step(xd[s], kv, y_dec[s], (idx[s], gate[s]))
    torch.cuda.synchronize()

    ref = O.Layer(layer.as_dict(), oracle_weights(inp, q4))
    pre, yd, Ks, Vs, routes = ref.forward(to_numpy_f64(inp.x_prefill), cu, to_numpy_f64(inp.x_decode))
    log, n_close = ErrLog(), 0
    for s in range(S):
        logits = np.stack([routes[s][b][2] for b in range(N)])
        h = np.stack([routes[s][b][3] for b in range(N)])
        gi = idx[s].cpu().numpy()
        n_close += H.check_routing(gi, logits, 4, 8e-3, gate[s].cpu().numpy())
        log.cmp("y_dec%d" % s, to_numpy_f64(y_dec[s]), ref.ffn(h, forced_idx=gi)[0])     # every row
    log.check("rows with a close call: %d of %d (all compared) |" % (n_close, S * N))


def test_4bit_and_16bit_paths_agree_on_the_same_values():
    """The 4-bit streaming kernels and the 16-bit ones read the same numbers (the bf16 copy is
    the exact expansion), so a decode step must agree far inside the bf16 tolerance."""
    layer = LayerConfig(d_model=1216, n_q_heads=8, n_kv_heads=2, head_dim=64, ffn_dim=1088, n_experts=16, top_k=4,
                        rope_theta=500000.0)
    inp, q4 = build(layer, [40, 17, 9], 2, seed=3)
    lay0 = B.Layer(layer, None)
    w = device_weights(lay0, inp, q4)
    w16 = {k: v for k, v in w.items() if not k.endswith(("_q", "_s"))}
    outs = []
    for ww in (w, w16):
        lay = B.Layer(layer, ww)
        kv = B.KVCache(layer, [L + 2 for L in inp.block_lens], DEV, torch.bfloat16)
        lay.ensure_workspace(inp.cu_seqlens[-1], 3, 64, DEV)
        y_pre = torch.empty(inp.cu_seqlens[-1], 1216, dtype=torch.bfloat16, device=DEV)
        lay.compact_prefill(inp.cu_seqlens, inp.x_prefill.to(DEV), kv, y_pre)
        y = torch.empty(2, 3, 1216, dtype=torch.bfloat16, device=DEV)
        idx = torch.empty(2, 3, 4, dtype=torch.int32, device=DEV)
        gate = torch.empty(2, 3, 4, dtype=torch.float32, device=DEV)
        for s in range(2):
            lay.compact_decode_step(inp.x_decode[s].to(DEV).contiguous(), kv, y[s], (idx[s], gate[s]))
        torch.cuda.synchronize()
        outs.append((y.float().cpu(), idx.cpu()))
    assert torch.equal(outs[0][1], outs[1][1])                 # routing does not depend on the expert format
    d = (outs[0][0] - outs[1][0]).norm(dim=-1) / outs[1][0].norm(dim=-1)
    assert d.max().item() < 4e-3, d.max().item()               # only the split of K differs (1024- vs 512-wide slices)


def test_more_than_16_blocks_stream_the_4bit_arrays_tile_by_tile():
    """With 20 .. 64 blocks an expert can receive more than 16 rows: the routing plan cuts its rows into tiles of 16
    and the expert is streamed once per tile, from the 4-bit arrays when they are given.  40 blocks on 16 experts
    (10 rows per expert on average, up to two tiles): against the 16-bit path on the expanded values."""
    layer = LayerConfig(d_model=256, n_q_heads=8, n_kv_heads=2, head_dim=64, ffn_dim=320, n_experts=16, top_k=4,
                        rope_theta=500000.0)
    inp, q4 = build(layer, [9] * 40, 2, seed=5)
    lay0 = B.Layer(layer, None)
    w = device_weights(lay0, inp, q4)
    w16 = {k: v for k, v in w.items() if not k.endswith(("_q", "_s"))}
    outs = []
    for ww in (w, w16):
        lay = B.Layer(layer, ww)
        kv = B.KVCache(layer, [L + 2 for L in inp.block_lens], DEV, torch.bfloat16)
        lay.ensure_workspace(inp.cu_seqlens[-1], 40, 16, DEV)
        y_last = torch.empty(40, 256, dtype=torch.bfloat16, device=DEV)
        y = torch.empty(2, 40, 256, dtype=torch.bfloat16, device=DEV)
        lay.compact_layer_forward(inp.cu_seqlens, inp.x_prefill.to(DEV), inp.x_decode.to(DEV).contiguous(), kv, None, y_last, y)
        torch.cuda.synchronize()
        outs.append((y.float().cpu(), y_last.clone()))
    assert torch.equal(outs[0][1], outs[1][1])                 # the prefill reads the 16-bit copy either way
    d = (outs[0][0] - outs[1][0]).norm(dim=-1) / outs[1][0].norm(dim=-1)
    assert d.max().item() < 4e-3, d.max().item()               # only the split of K differs (1024- vs 512-wide slices)
