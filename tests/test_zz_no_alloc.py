"""The allocation-free decode attention (compact_attn_decode_noalloc: partial records and
work list in a fixed device array inside the library) against compact_attn_decode (the same
kernels with a caller workspace and host-built lists): bit-identical outputs, on calls in a
row that share the array, the later ones smaller than the first."""
import numpy as np
import pytest
import torch

from oracle import layer as O
from paper_2605_23296_amd import binding as B
from paper_2605_23296_amd.workloads import WORKLOADS, to_numpy_f64
from tests.util import rel_err

pytestmark = pytest.mark.gpu
DEV = "cuda"


def rnd(shape, seed):
    g = torch.Generator(device="cpu").manual_seed(seed)
    return torch.randn(shape, generator=g, dtype=torch.float32).to(torch.bfloat16).to(DEV)


def make_case(layer, lens, seed):
    Hq, Hkv, hd = layer.n_q_heads, layer.n_kv_heads, layer.head_dim
    kv = B.KVCache(layer, [L + (b % 3) * 8 for b, L in enumerate(lens)], DEV, torch.bfloat16)
    kv.k.fill_(float("nan"))
    kv.v.fill_(float("nan"))
    Ks, Vs = [], []
    for b, L in enumerate(lens):
        k, v = rnd((L, Hkv, hd), seed + 10 * b), rnd((L, Hkv, hd), seed + 10 * b + 1)
        kv.h_len[b] = L
        kv.block_k(b).copy_(k)
        kv.block_v(b).copy_(v)
        Ks.append(k)
        Vs.append(v)
    return kv, Ks, Vs, rnd((len(lens), Hq * hd), seed + 5)


def run_both(lay, layer, lens, seed, check_oracle_blocks=()):
    kv, Ks, Vs, q = make_case(layer, lens, seed)
    N = len(lens)
    want = torch.full_like(q, float("nan"))
    lay.ws = torch.empty(lay.workspace_bytes(0, N, max(lens)), dtype=torch.uint8, device=DEV)
    lay.compact_attn_decode(q, kv, want)
    got = torch.full_like(q, float("nan"))
    lay.ws = None                                         # the entry point under test takes no workspace
    lay.compact_attn_decode_noalloc(q, kv, got)
    torch.cuda.synchronize()
    assert not torch.isnan(want.float()).any()
    assert torch.equal(got, want), (lens, (got.float() - want.float()).abs().max().item())
    Hq, hd = layer.n_q_heads, layer.head_dim
    for b in check_oracle_blocks:
        ref = O.gqa_attention(to_numpy_f64(q[b]).reshape(1, Hq, hd), to_numpy_f64(Ks[b]), to_numpy_f64(Vs[b]),
                              visible=np.array([lens[b]])).reshape(-1)
        assert rel_err(to_numpy_f64(got[b]), ref) < 3e-2


def test_no_alloc_decode_attention_equals_the_workspace_entry_point_on_calls_in_a_row():
    layer = WORKLOADS["dense_8x4096"].layer
    lay = B.Layer(layer, None)
    # chunk edges, a long cache, 14 blocks; then smaller calls that leave most of the array's old contents in place
    run_both(lay, layer, [1, 2, 31, 32, 33, 64, 65, 255, 256, 257, 511, 513, 4097, 8448], 21, check_oracle_blocks=(0, 9, 13))
    run_both(lay, layer, [300, 40], 22, check_oracle_blocks=(0, 1))
    run_both(lay, layer, [7], 23, check_oracle_blocks=(0,))
    run_both(lay, layer, [2048 + 3 * b for b in range(64)], 24, check_oracle_blocks=(63,))   # the 64-block limit


def test_no_alloc_decode_attention_head_dim_64_group_of_8():
    layer = WORKLOADS["moe_16x8192"].layer
    lay = B.Layer(layer, None)
    run_both(lay, layer, [5, 256, 300, 2049], 25, check_oracle_blocks=(1, 3))
    run_both(lay, layer, [3, 257], 26, check_oracle_blocks=(1,))


def test_no_alloc_decode_attention_rejects_sizes_beyond_its_scratch():
    layer = WORKLOADS["dense_8x4096"].layer
    lay = B.Layer(layer, None)
    kv, _, _, q = make_case(layer, [8] * 65, 27)
    o = torch.empty_like(q)
    with pytest.raises(B.CompactError) as e:
        lay.compact_attn_decode_noalloc(q, kv, o)
    assert e.value.code == 3 and "64 blocks" in e.value.detail
    # 64 blocks x 32 heads x 9 chunks x 130 floats fit; 64 blocks x 33 chunks x 32 x 130 x 4 = 35 MB do not
    kv2 = B.KVCache(layer, [8208] * 64, DEV, torch.bfloat16)
    for b in range(64):
        kv2.h_len[b] = 8200
    q2 = rnd((64, layer.n_q_heads * layer.head_dim), 28)
    with pytest.raises(B.CompactError) as e:
        lay.compact_attn_decode_noalloc(q2, kv2, torch.empty_like(q2))
    assert e.value.code == 3 and "32 MiB" in e.value.detail
