"""fp32 storage mode against the fp64 checker: the tiny layer in full, at 1e-5."""
import numpy as np
import pytest
import torch

from paper_2605_23296_amd import binding as B
from paper_2605_23296_amd.workloads import WORKLOADS, make_inputs, to_numpy_f64
from tests import harness as H
from tests.util import rel_err

pytestmark = pytest.mark.gpu
TOL = 1e-5     # fp32 mode: max |g - r| / max(|r|, rms(r)) per output tensor


def check_forward(inp, pos_offset=None, tol=TOL):
    g = H.gpu_forward(inp, pos_offset=pos_offset)
    r = H.oracle_forward(inp, pos_offset=pos_offset)
    y_pre = np.concatenate([p["y"] for p in r["pre"]])
    errs = dict(y_prefill=rel_err(g["y_prefill"], y_pre), y_decode=rel_err(g["y_decode"], r["y_decode"]))
    last = np.stack([p["y"][-1] for p in r["pre"]])
    errs["y_last"] = rel_err(g["y_last"], last)
    for b in range(len(inp.block_lens)):
        assert g["lens"][b] == inp.block_lens[b] + inp.x_decode.shape[0]
        errs["K%d" % b] = rel_err(g["K"][b], r["K"][b])
        errs["V%d" % b] = rel_err(g["V"][b], r["V"][b])
    print({k: "%.2e" % v for k, v in errs.items()})
    assert max(errs.values()) < tol, errs
    return g, r


def test_tiny_fp32_layer_in_full():
    check_forward(make_inputs(WORKLOADS["tiny_fp32"]))


def test_ragged_blocks_with_gain_and_position_offsets():
    # lengths straddling every tile edge of the row kernels: 1, 63..65, 127..129, a long ragged tail
    lens = [1, 63, 64, 65, 127, 128, 129, 257, 2]
    inp = make_inputs(WORKLOADS["tiny_fp32"], block_lens=lens, decode_steps=3, gain_jitter=True)
    check_forward(inp, pos_offset=[0, 5, 1000, 0, 7, 0, 4000, 1, 0])


def test_head_dim_128_fp32():
    wl = WORKLOADS["tiny_fp32"]
    import copy
    wl = copy.deepcopy(wl)
    wl.layer.head_dim, wl.layer.n_q_heads, wl.layer.n_kv_heads, wl.layer.rope_theta = 128, 4, 1, 500000.0
    check_forward(make_inputs(wl, block_lens=[70, 33], decode_steps=2))


def test_step_by_step_api_matches_forward_call():
    inp = make_inputs(WORKLOADS["tiny_fp32"], block_lens=[40, 9, 77], decode_steps=4)
    ref = H.gpu_forward(inp)
    lay = H.gpu_layer(inp)
    layer = inp.layer
    N, S, T = 3, 4, inp.cu_seqlens[-1]
    kv = B.KVCache(layer, [L + S for L in inp.block_lens], "cuda", torch.float32)
    lay.ensure_workspace(T, N, max(inp.block_lens) + S, "cuda")
    x = inp.x_prefill.cuda()
    y = torch.empty_like(x)
    lay.compact_prefill(inp.cu_seqlens, x, kv, y)
    assert kv.lens() == inp.block_lens
    ys = []
    for s in range(S):
        ys.append(torch.empty(N, layer.d_model, device="cuda"))
        lay.compact_decode_step(inp.x_decode[s].cuda().contiguous(), kv, ys[-1])
    torch.cuda.synchronize()
    assert kv.lens() == [L + S for L in inp.block_lens]
    assert np.array_equal(to_numpy_f64(y), ref["y_prefill"])
    assert np.array_equal(to_numpy_f64(torch.stack(ys)), ref["y_decode"])
    for b in range(N):
        assert np.array_equal(to_numpy_f64(kv.block_k(b)), ref["K"][b])
        assert np.array_equal(to_numpy_f64(kv.block_v(b)), ref["V"][b])


def test_batched_equals_one_block_at_a_time_bitwise():
    """Sec. IV: per-block results are independent of the rest of the batch."""
    import copy
    inp = make_inputs(WORKLOADS["tiny_fp32"], block_lens=[40, 9, 77, 128], decode_steps=3)
    full = H.gpu_forward(inp)
    for b, L in enumerate(inp.block_lens):
        one = copy.copy(inp)
        one.block_lens, one.cu_seqlens = [L], [0, L]
        one.x_prefill = inp.x_prefill[inp.cu_seqlens[b]:inp.cu_seqlens[b + 1]].contiguous()
        one.x_decode = inp.x_decode[:, b:b + 1].contiguous()
        g = H.gpu_forward(one)
        assert np.array_equal(g["y_prefill"], full["y_prefill"][inp.cu_seqlens[b]:inp.cu_seqlens[b + 1]])
        assert np.array_equal(g["y_decode"][:, 0], full["y_decode"][:, b])
        assert np.array_equal(g["K"][0], full["K"][b]) and np.array_equal(g["V"][0], full["V"][b])


def test_forty_thousand_tiny_blocks_grow_the_metadata_buffer():
    """40 000 blocks of one to three tokens: the block table alone (32 bytes a block) outgrows the context's first
    metadata buffer, which is replaced on the way; a small batch before and after must give the same bits, and
    sampled blocks of the big batch match the checker (prefill rows, caches and one decode step)."""
    wl = WORKLOADS["tiny_fp32"]
    small = make_inputs(wl, block_lens=[5, 1, 9], decode_steps=1)
    n = 40000
    lens = [1 + (b * 7) % 3 for b in range(n)]
    big = make_inputs(wl, block_lens=lens, decode_steps=1)
    lay = H.gpu_layer(big)                      # same weights for all three calls (same seed, same layer)
    before = H.gpu_forward(small, lay=lay)
    g = H.gpu_forward(big, lay=lay)
    after = H.gpu_forward(small, lay=lay)
    for k in ("y_prefill", "y_decode", "y_last"):
        assert np.array_equal(before[k], after[k]), k
    ref = H.oracle_layer(big)
    cu = big.cu_seqlens
    xp, xd = to_numpy_f64(big.x_prefill), to_numpy_f64(big.x_decode)
    worst = 0.0
    for b in [0, 1, 2, 4095, 4096, 20000, 32767, 32768, n - 2, n - 1]:
        r = ref.prefill_block(xp[cu[b]:cu[b + 1]])
        worst = max(worst, rel_err(g["y_prefill"][cu[b]:cu[b + 1]], r["y"]))
        d = ref.decode_block(xd[0, b], r["K"], r["V"])
        worst = max(worst, rel_err(g["y_decode"][0, b], d["y"]), rel_err(g["K"][b], d["K"]), rel_err(g["V"][b], d["V"]))
        assert g["lens"][b] == lens[b] + 1
    assert worst < TOL, worst


@pytest.mark.parametrize("kw", [
    dict(n_q_heads=6, n_kv_heads=2, head_dim=64), dict(n_q_heads=3, n_kv_heads=1, head_dim=128),
    dict(n_q_heads=16, n_kv_heads=1, head_dim=64), dict(n_q_heads=4, n_kv_heads=4, head_dim=128),
    dict(n_experts=6, top_k=2), dict(n_experts=12, top_k=3), dict(n_experts=8, top_k=1),
    dict(n_experts=256, top_k=8, ffn_dim=64), dict(d_model=64, n_q_heads=1, n_kv_heads=1, head_dim=64, ffn_dim=64),
    dict(d_model=2112, n_q_heads=6, n_kv_heads=2, head_dim=128, ffn_dim=1344),
], ids=lambda kw: "-".join("%s%s" % (k[:4], v) for k, v in kw.items()))
def test_unusual_layer_shapes_fp32(kw):
    """Layer shapes no named workload has, in fp32 storage at 1e-5 (routed layers: the routing is then decided in
    fp32 against fp64, and a row whose logits nearly tie is checked with the choice the GPU made)."""
    from paper_2605_23296_amd.workloads import LayerConfig, Workload
    base = dict(d_model=512, n_q_heads=8, n_kv_heads=2, head_dim=64, ffn_dim=256, rope_theta=500000.0, dtype="fp32")
    base.update(kw)
    layer = LayerConfig(**base)
    inp = make_inputs(Workload("odd_shape", layer, [70, 3, 129], 3, 3), gain_jitter=True)
    if layer.n_experts == 0:
        check_forward(inp)
        return
    from tests.test_gpu_layer_bf16 import check_moe
    check_moe(inp, margin_rel=1e-4, fp32=True)
