"""Per-kernel parity: each HIP kernel (through its C-ABI entry point) against
the fp64 checker's function for the same step, on seeded inputs whose sizes
span several tiles and a ragged tail."""
import copy

import numpy as np
import pytest
import torch

from oracle import layer as O
from paper_2605_23296_amd import binding as B
from paper_2605_23296_amd.workloads import WORKLOADS, LayerConfig, to_numpy_f64
from tests.util import rel_err, rms_err

pytestmark = pytest.mark.gpu

TOL = {"bf16": 2e-2, "fp32": 1e-5}
DENSE = WORKLOADS["dense_8x4096"].layer
MOE = WORKLOADS["moe_16x8192"].layer


def rnd(shape, dtype, seed, std=1.0, device="cuda"):
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    return (torch.randn(shape, generator=g, dtype=torch.float32) * std).to(dtype).to(device)


def tdtype(layer):
    return torch.bfloat16 if layer.dtype == "bf16" else torch.float32


def fp32_variant(layer):
    l2 = copy.deepcopy(layer)
    l2.dtype = "fp32"
    return l2


# ---------------------------------------------------------------- RMSNorm
@pytest.mark.parametrize("layer", [DENSE, MOE, fp32_variant(MOE)], ids=["d4096", "d2880", "d2880_fp32"])
def test_rmsnorm(layer):
    dt = tdtype(layer)
    lay = B.Layer(layer, None)
    x = rnd((37, layer.d_model), dt, 1, std=3.0)
    g = (1 + rnd((layer.d_model,), torch.float32, 2, std=0.1)).to(dt)
    y = torch.empty_like(x)
    lay.compact_rmsnorm(x, g, y)
    torch.cuda.synchronize()
    ref = O.rmsnorm(to_numpy_f64(x), to_numpy_f64(g), layer.rms_eps)
    assert rel_err(to_numpy_f64(y), ref) < (5e-3 if layer.dtype == "bf16" else 1e-6)


# ---------------------------------------------------------------- GEMM
GEMM_SHAPES = [
    # M, N, K, epilogue, residual
    (300, 512, 256, 0, False),      # M tail inside a 256-row tile
    (513, 2880, 192, 0, True),      # N not a multiple of the 256-column tile, residual
    (1024, 6144, 4096, 0, False),   # QKV shape, several tiles
    (257, 1408, 512, 1, False),     # SwiGLU epilogue with a column tail
    (1, 4096, 4096, 0, True),       # weight-streaming path, one row
    (8, 6144, 4096, 0, False),      # weight-streaming path, decode batch of 8
    (64, 4096, 14336, 0, True),     # weight-streaming path, 64 rows, long K
    (33, 2880, 2880, 0, False),     # weight-streaming path, K with a short last slice
    (65, 512, 128, 0, False),       # just above the weight-streaming limit
    # several tiles per CU, tails in both directions
    (4196, 4360, 256, 0, True),     # 17 x 18 tiles of 8 k-tiles, row tail of 100, column tail of 8, residual
    (4196, 4360, 1088, 0, False),   # 34 k-tiles
    (4352, 4096, 320, 0, False),    # 10 k-tiles
    (4352, 4096, 192, 0, False),    # 6 k-tiles
    (4196, 2184, 512, 1, False),    # SwiGLU epilogue: 17 x 18 tiles of 128 output columns, column tail of 8
    (8192, 8192, 4096, 0, True),    # 1024 tiles: four per workgroup
]


@pytest.mark.parametrize("M,N,K,epi,res", GEMM_SHAPES)
def test_gemm_bf16(M, N, K, epi, res):
    lay = B.Layer(DENSE, None)
    lay.ws = torch.empty(64 << 20, dtype=torch.uint8, device="cuda")
    a = rnd((M, K), torch.bfloat16, 3)
    b = rnd(((2 if epi else 1) * N, K), torch.bfloat16, 4, std=0.05)
    r = rnd((M, N), torch.bfloat16, 5) if res else None
    c = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    lay.compact_gemm(a, b, r, c, epi)
    torch.cuda.synchronize()
    A, Bm = to_numpy_f64(a), to_numpy_f64(b)
    if epi:
        ref = O.silu(O.linear(A, Bm[:N])) * O.linear(A, Bm[N:])
    else:
        ref = O.linear(A, Bm) + (to_numpy_f64(r) if res else 0.0)
    assert rel_err(to_numpy_f64(c), ref) < 1e-2


@pytest.mark.parametrize("M,N,K,epi,res", [(100, 192, 80, 0, True), (70, 96, 64, 1, False), (3, 256, 1024, 0, False)])
def test_gemm_fp32(M, N, K, epi, res):
    lay = B.Layer(fp32_variant(DENSE), None)
    a = rnd((M, K), torch.float32, 3)
    b = rnd(((2 if epi else 1) * N, K), torch.float32, 4, std=0.05)
    r = rnd((M, N), torch.float32, 5) if res else None
    c = torch.empty((M, N), dtype=torch.float32, device="cuda")
    lay.compact_gemm(a, b, r, c, epi)
    torch.cuda.synchronize()
    A, Bm = to_numpy_f64(a), to_numpy_f64(b)
    ref = O.silu(O.linear(A, Bm[:N])) * O.linear(A, Bm[N:]) if epi else O.linear(A, Bm) + (to_numpy_f64(r) if res else 0.0)
    assert rel_err(to_numpy_f64(c), ref) < 1e-5


# ---------------------------------------------------------------- rotary + KV write, prefill attention
def attention_case(layer, lens, seed, pos_offset=None, edit=None):
    """qkv rows -> (GPU: rope_kvwrite + attn_prefill) vs (checker: rope + gqa_attention)."""
    dt = tdtype(layer)
    lay = B.Layer(layer, None)
    cu = [0]
    for L in lens:
        cu.append(cu[-1] + L)
    Dq, Dkv, hd = layer.Dq, layer.Dkv, layer.head_dim
    qkv = rnd((cu[-1], Dq + 2 * Dkv), dt, seed)
    if edit is not None:
        qkv = edit(qkv, cu)
    qkv_in = to_numpy_f64(qkv)
    kv = B.KVCache(layer, [L + 3 for L in lens], "cuda", dt, pos_offset)
    # poison the slabs: rows past a block's length must never reach a result
    kv.k.fill_(float("nan"))
    kv.v.fill_(float("nan"))
    lay.compact_rope_kvwrite(cu, qkv, kv)
    o = torch.empty((cu[-1], Dq), dtype=dt, device="cuda")
    lay.compact_attn_prefill(cu, qkv, kv, o)
    torch.cuda.synchronize()
    assert kv.lens() == list(lens)
    # bf16: q, k, the probabilities and o are each rounded to 8 mantissa bits, and the
    # inputs here are unit-variance (scores of unit variance): the worst of ~10^6
    # outputs sits near 5 sigma of that rounding noise, so the max-error bound is
    # loose and the rms bound carries the check (a structural mistake gives O(1)).
    tol = 5e-2 if layer.dtype == "bf16" else 1e-5
    rms_tol = 6e-3 if layer.dtype == "bf16" else 1e-6
    worst = 0.0
    for b, L in enumerate(lens):
        rows = qkv_in[cu[b]:cu[b + 1]]
        pos = (0 if pos_offset is None else pos_offset[b]) + np.arange(L)
        q = O.rope(rows[:, :Dq].reshape(L, layer.n_q_heads, hd), pos, layer.rope_theta)
        k = O.rope(rows[:, Dq:Dq + Dkv].reshape(L, layer.n_kv_heads, hd), pos, layer.rope_theta)
        v = rows[:, Dq + Dkv:].reshape(L, layer.n_kv_heads, hd)
        assert rel_err(to_numpy_f64(kv.block_k(b)), k) < (1e-2 if layer.dtype == "bf16" else 1e-5)
        assert np.array_equal(to_numpy_f64(kv.block_v(b)), v)
        ref = O.gqa_attention(q, k, v, visible=np.arange(L) + 1).reshape(L, Dq)
        e = rel_err(to_numpy_f64(o[cu[b]:cu[b + 1]]), ref)
        assert rms_err(to_numpy_f64(o[cu[b]:cu[b + 1]]), ref) < rms_tol
        worst = max(worst, e)
    assert worst < tol, worst
    return lay, kv, qkv


def test_prefill_attention_bf16_hd128_ragged():
    # 1 token; one short of / exactly / one past the 64-token KV tile and the 128-row query tile; longer ragged
    attention_case(DENSE, [1, 63, 64, 65, 127, 128, 129, 300, 641], seed=11, pos_offset=[0, 3, 0, 100, 0, 7, 0, 4000, 9])


@pytest.mark.parametrize("pattern", ["growing", "sink"])
@pytest.mark.parametrize("layer_name", ["dense", "moe"])
def test_prefill_attention_when_the_scaling_reference_has_to_move(layer_name, pattern):
    """Scores that keep growing along a block (every new tile of 64 keys outgrows the running reference by 2^8, so
    the reference moves and the accumulators are rescaled tile after tile) and an attention sink (token 0 outweighs
    everything after it by 2^60: the reference is set once and never moves).  The structure sits in the rotary pair
    with the lowest frequency, which positions up to a few thousand leave practically unrotated."""
    layer = copy.deepcopy(DENSE if layer_name == "dense" else MOE)
    if layer_name == "moe":
        layer.n_q_heads, layer.n_kv_heads = 16, 2
    hd, Hq, Hkv = layer.head_dim, layer.n_q_heads, layer.n_kv_heads
    Dq, Dkv = Hq * hd, Hkv * hd
    per_key = 8.0 / 64.0 / (16.0 * 1.4426950408889634 / np.sqrt(hd))   # k value that adds 2^8 per 64 keys at q = 16

    def edit(qkv, cu):
        q = qkv[:, :Dq].view(-1, Hq, hd)
        k = qkv[:, Dq:Dq + Dkv].view(-1, Hkv, hd)
        q[:, :, hd // 2 - 1] = 16.0
        q[:, :, hd - 1] = 0.0
        k[:, :, hd - 1] = 0.0
        for b in range(len(cu) - 1):
            j = torch.arange(cu[b + 1] - cu[b], device=qkv.device, dtype=torch.float32)
            if pattern == "growing":
                val = j * per_key
            else:
                val = torch.zeros_like(j)
                val[0] = 60.0 * 64.0 / 8.0 * per_key
            k[cu[b]:cu[b + 1], :, hd // 2 - 1] = val.to(qkv.dtype)[:, None]
        return qkv

    attention_case(layer, [1, 64, 65, 300, 777], seed=17, edit=edit)


def test_prefill_attention_bf16_hd64_group_of_8():
    small = copy.deepcopy(MOE)
    small.n_q_heads, small.n_kv_heads = 16, 2
    attention_case(small, [200, 1, 77, 513], seed=12)


def test_prefill_attention_bf16_odd_gqa_group_takes_the_one_head_per_workgroup_kernel():
    # the two-heads-per-workgroup kernel needs an even GQA group; 3 query heads per KV head and plain
    # multi-head attention (group of 1) run the four-wavefront kernel at head_dim 128
    g3 = copy.deepcopy(DENSE)
    g3.n_q_heads, g3.n_kv_heads = 6, 2
    attention_case(g3, [1, 64, 129, 300, 385], seed=14, pos_offset=[0, 5, 0, 900, 3])
    mha = copy.deepcopy(DENSE)
    mha.n_q_heads, mha.n_kv_heads = 3, 3
    attention_case(mha, [65, 200], seed=15)


def test_prefill_attention_bf16_two_heads_per_workgroup_long_block():
    # long enough for the four-stage K/V ring to wrap several times (34 tiles), ragged last tile
    two = copy.deepcopy(DENSE)
    two.n_q_heads, two.n_kv_heads = 4, 2
    attention_case(two, [2150, 130], seed=16)


def test_prefill_attention_fp32():
    l2 = fp32_variant(DENSE)
    l2.n_q_heads, l2.n_kv_heads = 8, 2
    attention_case(l2, [70, 5, 129], seed=13)


# ---------------------------------------------------------------- decode attention
def decode_case(layer, lens, seed, grow=None):
    dt = tdtype(layer)
    lay = B.Layer(layer, None)
    N, Hq, Hkv, hd = len(lens), layer.n_q_heads, layer.n_kv_heads, layer.head_dim
    kv = B.KVCache(layer, [L + (b % 3) * 8 for b, L in enumerate(lens)], "cuda", dt)
    kv.k.fill_(float("nan"))
    kv.v.fill_(float("nan"))
    Ks, Vs = [], []
    for b, L in enumerate(lens):
        k = rnd((L, Hkv, hd), dt, seed + 10 * b)
        v = rnd((L, Hkv, hd), dt, seed + 10 * b + 1)
        if grow is not None:   # scores that grow (or fall) along the cache: k[j][0] = grow * j against q[0] = 16
            k[:, :, 0] = (torch.arange(L, device=k.device, dtype=torch.float32) * grow).to(dt)[:, None]
        cap = kv.caps[b]
        kslab = kv.k[kv.offs[b]:kv.offs[b] + cap * Hkv * hd].view(Hkv, cap, hd)
        vslab = kv.v[kv.offs[b]:kv.offs[b] + cap * Hkv * hd].view(Hkv, hd, cap)
        kslab[:, :L, :] = k.permute(1, 0, 2)
        vslab[:, :, :L] = v.permute(1, 2, 0)
        kv.h_len[b] = L
        Ks.append(to_numpy_f64(k))
        Vs.append(to_numpy_f64(v))
    q = rnd((N, Hq * hd), dt, seed + 5)
    if grow is not None:
        q.view(N, Hq, hd)[:, :, 0] = 16.0
    o = torch.empty_like(q)
    lay.ws = torch.empty(lay.workspace_bytes(0, N, max(lens)), dtype=torch.uint8, device="cuda")
    lay.compact_attn_decode(q, kv, o)
    torch.cuda.synchronize()
    qn = to_numpy_f64(q).reshape(N, Hq, hd)
    worst = 0.0
    for b, L in enumerate(lens):
        ref = O.gqa_attention(qn[b:b + 1], Ks[b], Vs[b], visible=np.array([L])).reshape(-1)
        worst = max(worst, rel_err(to_numpy_f64(o[b]), ref))
        assert rms_err(to_numpy_f64(o[b]), ref) < (6e-3 if layer.dtype == "bf16" else 1e-6)
    assert worst < (3e-2 if layer.dtype == "bf16" else 1e-5), worst


def test_decode_attention_bf16_hd128_chunk_edges():
    # lengths around the 32-token window, the 64-token wavefront share and the 256-token chunk
    decode_case(DENSE, [1, 2, 31, 32, 33, 64, 65, 255, 256, 257, 511, 513, 4097, 8448], seed=21)


def test_decode_attention_bf16_hd64_group_of_8():
    decode_case(MOE, [5, 256, 300, 2049], seed=22)


@pytest.mark.parametrize("layer_name", ["dense", "moe"])
def test_decode_attention_many_ragged_blocks_repeats_bit_for_bit(layer_name):
    """48 ragged blocks (shares of the persistent workgroups cross block and KV-head boundaries, records are
    buffered and flushed several times per workgroup): twenty launches give identical bits, and the first matches
    the checker on sampled blocks."""
    layer = DENSE if layer_name == "dense" else MOE
    dt = torch.bfloat16
    lay = B.Layer(layer, None)
    rng = np.random.default_rng(77)
    lens = [int(v) for v in rng.integers(1, 3000, size=48)]
    N, Hq, Hkv, hd = len(lens), layer.n_q_heads, layer.n_kv_heads, layer.head_dim
    kv = B.KVCache(layer, [L + 5 for L in lens], "cuda", dt)
    gen = torch.Generator(device="cuda").manual_seed(5)
    kv.k.copy_(torch.randn(kv.k.shape, generator=gen, device="cuda", dtype=torch.float32).to(dt))
    kv.v.copy_(torch.randn(kv.v.shape, generator=gen, device="cuda", dtype=torch.float32).to(dt))
    for b, L in enumerate(lens):
        kv.h_len[b] = L
    q = rnd((N, Hq * hd), dt, 9)
    lay.ws = torch.empty(lay.workspace_bytes(0, N, max(lens)), dtype=torch.uint8, device="cuda")
    outs = []
    for _ in range(20):
        o = torch.empty_like(q)
        lay.compact_attn_decode(q, kv, o)
        outs.append(o)
    torch.cuda.synchronize()
    first = outs[0].view(torch.int16)
    for o in outs[1:]:
        assert torch.equal(first, o.view(torch.int16))
    qn = to_numpy_f64(q).reshape(N, Hq, hd)
    for b in (0, 7, 23, 47, int(np.argmax(lens)), int(np.argmin(lens))):
        ref = O.gqa_attention(qn[b:b + 1], to_numpy_f64(kv.block_k(b)), to_numpy_f64(kv.block_v(b)),
                              visible=np.array([lens[b]])).reshape(-1)
        assert rms_err(to_numpy_f64(outs[0][b]), ref) < 6e-3 and rel_err(to_numpy_f64(outs[0][b]), ref) < 3e-2


@pytest.mark.parametrize("sign", [1.0, -1.0])
def test_decode_attention_scores_that_grow_or_fall_along_the_cache(sign):
    """2^8 more (or less) per 64 cached rows: the running maximum moves at every step of the walk through an item,
    and the chunks' records differ by hundreds of binary orders when they are merged."""
    for layer in (DENSE, MOE):
        per_key = 8.0 / 64.0 / (16.0 * 1.4426950408889634 / np.sqrt(layer.head_dim))
        decode_case(layer, [1, 100, 129, 256, 257, 700, 2049], seed=41, grow=sign * per_key)


def test_decode_attention_fp32():
    l2 = fp32_variant(DENSE)
    l2.n_q_heads, l2.n_kv_heads = 8, 2
    decode_case(l2, [1, 7, 130], seed=23)


def test_decode_attention_identical_keys_returns_mean_of_values():
    """The closed form the checker is pinned with, straight on the GPU kernel."""
    layer = DENSE
    lay = B.Layer(layer, None)
    L, Hq, Hkv, hd = 300, layer.n_q_heads, layer.n_kv_heads, layer.head_dim
    kv = B.KVCache(layer, [L], "cuda", torch.bfloat16)
    cap = kv.caps[0]
    krow = rnd((Hkv, 1, hd), torch.bfloat16, 31)
    kv.k.view(Hkv, cap, hd)[:, :L, :] = krow
    v = rnd((Hkv, hd, L), torch.bfloat16, 32)
    kv.v.view(Hkv, hd, cap)[:, :, :L] = v
    kv.h_len[0] = L
    q = rnd((1, Hq * hd), torch.bfloat16, 33)
    o = torch.empty_like(q)
    lay.ws = torch.empty(lay.workspace_bytes(0, 1, L), dtype=torch.uint8, device="cuda")
    lay.compact_attn_decode(q, kv, o)
    torch.cuda.synchronize()
    mean = to_numpy_f64(v).mean(-1)                      # [Hkv, hd]
    want = np.repeat(mean, Hq // Hkv, axis=0).reshape(-1)
    assert rel_err(to_numpy_f64(o[0]), want) < 1e-2


# ---------------------------------------------------------------- router
@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
def test_router_topk_indices_bit_exact(dtype):
    """Same rounded router input on both sides; indices must be identical for
    every row whose checker margins exceed 1e-4 * max|logit| (fp32-vs-fp64
    accumulation can only flip closer calls), and valid everywhere."""
    layer = copy.deepcopy(MOE)
    layer.dtype = dtype
    dt = tdtype(layer)
    lay = B.Layer(layer, None)
    rows, E, k = 3000, layer.n_experts, layer.top_k
    m = rnd((rows, layer.d_model), dt, 41)
    wr = rnd((E, layer.d_model), dt, 42, std=0.02)
    # planted exact ties: experts 7 and 90 share a weight row, as do 3 and 4
    wr[90] = wr[7]
    wr[4] = wr[3]
    idx = torch.empty((rows, k), dtype=torch.int32, device="cuda")
    gate = torch.empty((rows, k), dtype=torch.float32, device="cuda")
    logits = torch.empty((rows, E), dtype=torch.float32, device="cuda")
    lay.compact_moe_route(m, wr, idx, gate, logits)
    torch.cuda.synchronize()
    ref_logits = O.router_logits(to_numpy_f64(m), to_numpy_f64(wr))
    ref_idx, ref_gate = O.topk_route(ref_logits, k)
    assert rel_err(to_numpy_f64(logits), ref_logits) < 1e-5
    gi = idx.cpu().numpy()
    srt = -np.sort(-ref_logits, axis=-1)
    gaps = srt[:, :k] - srt[:, 1:k + 1]                   # gaps inside the top-k and to the runner-up
    # exact ties (planted duplicates) are decided by index, not by margin
    margin_ok = np.all((gaps > 1e-4 * np.abs(ref_logits).max()) | (gaps == 0.0), axis=-1)
    assert margin_ok.mean() > 0.95
    assert np.array_equal(gi[margin_ok], ref_idx[margin_ok])
    tied = [r for r in range(rows) if 7 in ref_idx[r] and 90 in ref_idx[r]]
    assert len(tied) > 0                                  # the planted tie is exercised
    for r in np.nonzero(~margin_ok)[0]:                   # near ties: any of the tied candidates is valid
        assert len(set(gi[r])) == k
        assert np.all(ref_logits[r, gi[r]] >= srt[r, k - 1] - 1e-4 * np.abs(ref_logits).max())
    np.testing.assert_allclose(gate.cpu().numpy()[margin_ok], ref_gate[margin_ok], atol=2e-5)
    np.testing.assert_allclose(gate.cpu().numpy().sum(-1), 1.0, atol=1e-5)


def test_router_full_size_ordered_indices():
    """The routed workload's whole routing table: 131072 rows x d 2880 through the router's
    entry point, router weights drawn as the workload's, the same bf16 rows on both sides.
    Ordered top-4 indices must equal the checker's on every row whose margins (inside the
    top 4 and to the runner-up) exceed 1e-4 * max|logit|; the remaining rows must hold a
    valid choice, and every gate row is the softmax over its four logits."""
    wl = WORKLOADS["moe_16x8192"]
    layer = wl.layer
    rows, E, k, d = sum(wl.block_lens), layer.n_experts, layer.top_k, layer.d_model
    assert rows == 131072 and E == 128 and k == 4 and d == 2880
    wr = rnd((E, d), torch.bfloat16, 43, std=0.02)            # drawn as the workload's router, N(0, 0.02)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(97)
    m = torch.randn((rows, d), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)  # unit-rms rows
    lay = B.Layer(layer, None)
    idx = torch.empty((rows, k), dtype=torch.int32, device="cuda")
    gate = torch.empty((rows, k), dtype=torch.float32, device="cuda")
    logits = torch.empty((rows, E), dtype=torch.float32, device="cuda")
    lay.compact_moe_route(m, wr, idx, gate, logits)
    torch.cuda.synchronize()
    gi, gg, gl = idx.cpu().numpy(), gate.cpu().numpy().astype(np.float64), logits.cpu().numpy().astype(np.float64)
    wr64 = to_numpy_f64(wr)
    n_exact = n_close = 0
    worst_logit = 0.0
    CH = 8192
    for r0 in range(0, rows, CH):
        ref_logits = O.router_logits(to_numpy_f64(m[r0:r0 + CH]), wr64)
        ref_idx, ref_gate = O.topk_route(ref_logits, k)
        scale = np.abs(ref_logits).max()
        worst_logit = max(worst_logit, float(np.abs(gl[r0:r0 + CH] - ref_logits).max() / scale))
        srt = -np.sort(-ref_logits, axis=-1)
        gaps = srt[:, :k] - srt[:, 1:k + 1]
        clear = np.all(gaps > 1e-4 * scale, axis=-1)
        g = gi[r0:r0 + CH]
        assert np.array_equal(g[clear], ref_idx[clear]), "ordered expert indices differ on rows with clear margins"
        np.testing.assert_allclose(gg[r0:r0 + CH][clear], ref_gate[clear], atol=2e-5)
        n_exact += int(clear.sum())
        for r in np.nonzero(~clear)[0]:
            assert len(set(g[r].tolist())) == k
            assert np.all(ref_logits[r, g[r]] >= srt[r, k - 1] - 1e-4 * scale)
            n_close += 1
    print("router at full size: %d rows ordered-exact, %d rows with a margin under 1e-4 (valid choice), worst logit error %.2e"
          % (n_exact, n_close, worst_logit))
    # four gaps per row, each under 1e-4 * max|logit| ~ 5e-4 with probability ~ 3e-3
    assert n_exact + n_close == rows and n_close < rows // 40
    assert worst_logit < 1e-5
    np.testing.assert_allclose(gg.sum(-1), 1.0, atol=1e-5)


# ---------------------------------------------------------------- expert feed-forward
@pytest.mark.parametrize("dtype,rows", [("fp32", 150), ("bf16", 700), ("bf16", 5)])
def test_moe_ffn_with_given_routing(dtype, rows):
    layer = LayerConfig(d_model=256, n_q_heads=4, n_kv_heads=2, head_dim=64, ffn_dim=320,
                        n_experts=8, top_k=3, dtype=dtype)
    dt = tdtype(layer)
    E, k, d, F = 8, 3, 256, 320
    w = dict(w_router=rnd((E, d), dt, 50, 0.05), w_exp_gate_up=rnd((E, 2 * F, d), dt, 51, 0.05),
             w_exp_down=rnd((E, d, F), dt, 52, 0.05), g_attn=rnd((d,), dt, 53), w_qkv=rnd((8, d), dt, 54),
             w_o=rnd((d, 8), dt, 55), g_ffn=rnd((d,), dt, 56))
    lay = B.Layer(layer, w)
    m = rnd((rows, d), dt, 57)
    h = rnd((rows, d), dt, 58)
    # routing: expert 5 gets no row at all, expert 2 gets every row
    g = torch.Generator().manual_seed(59)
    others = [0, 1, 3, 4, 6, 7]
    idx_np = np.zeros((rows, k), dtype=np.int32)
    for r in range(rows):
        pick = torch.randperm(len(others), generator=g)[:2].tolist()
        idx_np[r] = [others[pick[0]], 2, others[pick[1]]]
    gate_np = np.random.default_rng(60).dirichlet(np.ones(k), size=rows).astype(np.float32)
    idx = torch.from_numpy(idx_np).cuda()
    gate = torch.from_numpy(gate_np).cuda()
    y = torch.empty_like(m)
    lay.ws = torch.empty(64 << 20, dtype=torch.uint8, device="cuda")
    lay.compact_moe_ffn(m, h, idx, gate, y)
    torch.cuda.synchronize()
    ref = to_numpy_f64(h) + O.moe_ffn(to_numpy_f64(m), idx_np, gate_np.astype(np.float64),
                                      to_numpy_f64(w["w_exp_gate_up"]), to_numpy_f64(w["w_exp_down"]))
    assert rel_err(to_numpy_f64(y), ref) < TOL[dtype]
