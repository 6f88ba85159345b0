"""Step-by-step decoding keeps its uploaded plan between calls.  Whatever the library
reuses, a sequence of compact_decode_step / compact_prefix_decode_step calls must give
the bits of the same steps taken through a context that has never seen an earlier call
(a fresh context per step), also when other calls come in between, a cache is edited by
the caller, or the blocks cross a chunk boundary of the decode attention."""
import pytest
import torch

from paper_2605_23296_amd import binding as B
from paper_2605_23296_amd.workloads import WORKLOADS, make_inputs

pytestmark = pytest.mark.gpu
DEV = "cuda"
DT = torch.bfloat16


def same_bits(a, b):
    """Bitwise equality of two bf16 tensors (whole slabs include rows nobody has written, which may
    hold NaN patterns that compare unequal to themselves as numbers)."""
    return torch.equal(a.view(torch.int16), b.view(torch.int16))


def weights_on_device(inp):
    return {k: v.to(DEV).contiguous() for k, v in inp.weights.items()}


def prefilled(inp, w, caps):
    lay = B.Layer(inp.layer, w)
    T, N = inp.cu_seqlens[-1], len(inp.block_lens)
    kv = B.KVCache(inp.layer, caps, DEV, DT)
    lay.ensure_workspace(T, N, max(caps), DEV)
    y = torch.empty(T, inp.layer.d_model, dtype=DT, device=DEV)
    lay.compact_prefill(inp.cu_seqlens, inp.x_prefill.to(DEV), kv, y)
    return lay, kv


def clone_kv(inp, kv, caps):
    c = B.KVCache(inp.layer, caps, DEV, DT)
    c.k.copy_(kv.k)
    c.v.copy_(kv.v)
    for b in range(kv.N):
        c.h_len[b] = kv.h_len[b]
    return c


def step_fresh(inp, w, ws, x, kv, y):
    """One decode step through a context of its own."""
    lay = B.Layer(inp.layer, w)
    lay.ws = ws
    lay.compact_decode_step(x, kv, y)
    torch.cuda.synchronize()


def test_steps_across_chunk_boundaries_match_fresh_contexts_bitwise():
    lens = [250, 255, 511, 40]
    S = 8
    inp = make_inputs(WORKLOADS["dense_8x4096"], block_lens=lens, decode_steps=S)
    w = weights_on_device(inp)
    caps = [L + S for L in lens]
    lay, kv_a = prefilled(inp, w, caps)
    kv_b = clone_kv(inp, kv_a, caps)
    xd = inp.x_decode.to(DEV).contiguous()
    ya = torch.empty(S, len(lens), inp.layer.d_model, dtype=DT, device=DEV)
    yb = torch.empty_like(ya)
    for s in range(S):
        lay.compact_decode_step(xd[s], kv_a, ya[s])
        step_fresh(inp, w, lay.ws, xd[s], kv_b, yb[s])
    torch.cuda.synchronize()
    assert kv_a.lens() == kv_b.lens() == [L + S for L in lens]
    assert torch.equal(ya, yb)
    assert same_bits(kv_a.k, kv_b.k) and same_bits(kv_a.v, kv_b.v)


def test_other_calls_and_edited_lengths_between_steps():
    """Between steps: a prefill of another cache through the same context, a second cache
    of the same geometry stepped alternately, and a block the caller rolls back by two rows."""
    lens = [130, 300, 77]
    S = 6
    inp = make_inputs(WORKLOADS["dense_8x4096"], block_lens=lens, decode_steps=S)
    w = weights_on_device(inp)
    caps = [L + S + 8 for L in lens]
    lay, kv_a = prefilled(inp, w, caps)
    kv_ref = clone_kv(inp, kv_a, caps)
    kv_alt = clone_kv(inp, kv_a, caps)       # same lengths and capacities, other slabs
    kv_alt_ref = clone_kv(inp, kv_a, caps)
    other = B.KVCache(inp.layer, caps, DEV, DT)
    xd = inp.x_decode.to(DEV).contiguous()
    N, d = len(lens), inp.layer.d_model
    y = torch.empty(S, 2, N, d, dtype=DT, device=DEV)
    yr = torch.empty_like(y)
    y_pre = torch.empty(inp.cu_seqlens[-1], d, dtype=DT, device=DEV)
    for s in range(S):
        if s == 2:
            lay.compact_prefill(inp.cu_seqlens, inp.x_prefill.to(DEV), other, y_pre)
        if s == 4:
            for c in (kv_a, kv_ref):
                c.h_len[1] -= 2
        lay.compact_decode_step(xd[s], kv_a, y[s, 0])
        step_fresh(inp, w, lay.ws, xd[s], kv_ref, yr[s, 0])
        if s % 2 == 1:
            lay.compact_decode_step(xd[s], kv_alt, y[s, 1])
            step_fresh(inp, w, lay.ws, xd[s], kv_alt_ref, yr[s, 1])
        else:
            y[s, 1].zero_()
            yr[s, 1].zero_()
    torch.cuda.synchronize()
    assert kv_a.lens() == kv_ref.lens() == [lens[0] + S, lens[1] + S - 2, lens[2] + S]
    assert kv_alt.lens() == kv_alt_ref.lens() == [L + S // 2 for L in lens]
    assert torch.equal(y, yr)
    for a, r in ((kv_a, kv_ref), (kv_alt, kv_alt_ref)):
        assert same_bits(a.k, r.k) and same_bits(a.v, r.v)


def test_steps_up_to_the_last_row_of_the_slabs():
    """The kept plan never reaches past a slab: stepping until every block is full works,
    the next step is refused."""
    lens = [20, 9]
    inp = make_inputs(WORKLOADS["dense_8x4096"], block_lens=lens, decode_steps=5)
    w = weights_on_device(inp)
    caps = [24, 16]                       # room for 4 and 7 more rows
    lay, kv = prefilled(inp, w, caps)
    kv_ref = clone_kv(inp, kv, caps)
    xd = inp.x_decode.to(DEV).contiguous()
    y = torch.empty(5, 2, inp.layer.d_model, dtype=DT, device=DEV)
    yr = torch.empty_like(y)
    for s in range(4):
        lay.compact_decode_step(xd[s], kv, y[s])
        step_fresh(inp, w, lay.ws, xd[s], kv_ref, yr[s])
    assert torch.equal(y[:4], yr[:4]) and same_bits(kv.k, kv_ref.k)
    with pytest.raises(B.CompactError) as e:
        lay.compact_decode_step(xd[4], kv, y[4])
    assert e.value.code == 3      # COMPACT_ECAPACITY
    assert kv.lens() == [24, 13]


def test_prefix_aware_steps_across_a_tail_chunk_boundary():
    wl = WORKLOADS["dense_8x4096"]
    layer = wl.layer
    lens = [100, 157, 43]
    S = 5
    inp = make_inputs(wl, block_lens=lens, decode_steps=S)
    w = weights_on_device(inp)
    T, N = inp.cu_seqlens[-1], len(lens)
    lay = B.Layer(layer, w)
    shared = B.KVCache(layer, [T], DEV, DT)
    lay.ensure_workspace(T, 1, T, DEV)
    y_pre = torch.empty(T, layer.d_model, dtype=DT, device=DEV)
    lay.compact_prefill([0, T], inp.x_prefill.to(DEV), shared, y_pre)
    need = lay.prefix_workspace_bytes(N, T, 254 + S)
    if lay.ws.numel() < need:
        lay.ws = torch.empty(need, dtype=torch.uint8, device=DEV)
    prefix = [int(c) for c in inp.cu_seqlens[1:]]
    g = torch.Generator(device="cpu").manual_seed(7)
    start = [254, 3, 255]                    # tails that already hold rows; two of them cross row 256
    caps = [t + S + 1 for t in start]

    def tails():
        t = B.KVCache(layer, caps, DEV, DT)
        return t

    ta = tails()
    ta.k.copy_((torch.randn(ta.k.shape, generator=g) * 0.5).to(DT))
    ta.v.copy_((torch.randn(ta.v.shape, generator=g) * 0.5).to(DT))
    for b in range(N):
        ta.h_len[b] = start[b]
    tb = tails()
    tb.k.copy_(ta.k)
    tb.v.copy_(ta.v)
    for b in range(N):
        tb.h_len[b] = start[b]
    xd = inp.x_decode.to(DEV).contiguous()
    ya = torch.empty(S, N, layer.d_model, dtype=DT, device=DEV)
    yb = torch.empty_like(ya)
    for s in range(S):
        lay.compact_prefix_decode_step(xd[s], shared, prefix, ta, ya[s])
        fresh = B.Layer(layer, w)
        fresh.ws = lay.ws
        fresh.compact_prefix_decode_step(xd[s], shared, prefix, tb, yb[s])
        torch.cuda.synchronize()
    assert ta.lens() == tb.lens() == [t + S for t in start]
    assert torch.equal(ya, yb)
    assert same_bits(ta.k, tb.k) and same_bits(ta.v, tb.v)
