"""Mixed batches on the GPU (compact_mixed_forward: prefill chunks of some blocks in one
batch with decode tokens of others, paper Sec. IV-B chunked prefill): the schedule must
not change what is computed, so the outputs are checked against the fp64 checker's plain
prefill-then-decode pass, through the C ABI, for several token budgets."""
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


def run_mixed(inp, budget, pos_offset=None, weights=None):
    layer, cu = inp.layer, inp.cu_seqlens
    N, S = len(inp.block_lens), inp.x_decode.shape[0]
    lay = B.Layer(layer, weights or {k: v.to(DEV).contiguous() for k, v in inp.weights.items()})
    dt = lay.torch_dtype
    kv = B.KVCache(layer, [L + S + 3 for L in inp.block_lens], DEV, dt, pos_offset)
    kv.k.fill_(float("nan"))
    kv.v.fill_(float("nan"))
    lay.ws = torch.empty(lay.mixed_workspace_bytes(budget, N, max(inp.block_lens) + S), dtype=torch.uint8, device=DEV)
    y_last = torch.full((N, layer.d_model), float("nan"), dtype=dt, device=DEV)
    y_dec = torch.full((S, N, layer.d_model), float("nan"), dtype=dt, device=DEV)
    lay.compact_mixed_forward(cu, inp.x_prefill.to(DEV), inp.x_decode.to(DEV).contiguous() if S else None, kv, budget,
                              y_last, y_dec if S else None)
    torch.cuda.synchronize()
    assert kv.lens() == [L + S for L in inp.block_lens]
    return dict(y_last=y_last, y_dec=y_dec, kv=kv)


def check(inp, budget, fp32, ref_out, pos_offset=None):
    g = run_mixed(inp, budget, pos_offset)
    pre, y_dec, Ks, Vs = ref_out[:4]
    log = ErrLog(FP32_TOL, FP32_TOL, FP32_TOL) if fp32 else ErrLog()
    cmp = log.cmp
    cmp("y_last", to_numpy_f64(g["y_last"]), np.stack([p["y"][-1] for p in pre]))
    if y_dec.shape[0]:
        cmp("y_dec", to_numpy_f64(g["y_dec"]), y_dec)
    for b in range(len(inp.block_lens)):
        cmp("K%d" % b, to_numpy_f64(g["kv"].block_k(b)), Ks[b])
        cmp("V%d" % b, to_numpy_f64(g["kv"].block_v(b)), Vs[b])
    log.check("budget %d |" % budget)


def oracle_pass(inp, pos_offset=None):
    ref = O.Layer(inp.layer.as_dict(), {k: to_numpy_f64(v) for k, v in inp.weights.items()})
    pre, y_dec, Ks, Vs, routes = ref.forward(to_numpy_f64(inp.x_prefill), inp.cu_seqlens, to_numpy_f64(inp.x_decode), pos_offset)
    return pre, y_dec, Ks, Vs, routes, ref


def test_tiny_fp32_mixed_schedules_in_full():
    inp = make_inputs(WORKLOADS["tiny_fp32"], block_lens=[128, 65, 1, 97], decode_steps=5, gain_jitter=True)
    po = [0, 7, 3, 100]
    ref = oracle_pass(inp, po)
    for budget in (5, 64, 100, 1000):       # 5: chunks of 1-5 rows; 1000: everything in one step
        check(inp, budget, True, ref, po)


def test_bf16_mixed_schedules_ragged_blocks():
    """Budgets on and off the tile sizes; early blocks decode while late ones still prefill
    (budget 256: block 0 alone needs three steps), and finish their steps before the others."""
    layer = LayerConfig(d_model=512, n_q_heads=4, n_kv_heads=2, head_dim=128, ffn_dim=1024, rope_theta=500000.0)
    wl = Workload("small_dense", layer, [700, 130, 257, 40], 4, 6)
    inp = make_inputs(wl, gain_jitter=True)
    ref = oracle_pass(inp)
    for budget in (256, 203, 4096):
        check(inp, budget, False, ref)


def test_bf16_mixed_schedule_with_more_than_64_blocks():
    """70 short blocks: the steps after the last prefill chunk are decode steps of 70 rows (two groups of 35 through
    the projection kernels), and a budget of 100 rows mixes up to 70 decode rows with chunk rows before that."""
    layer = LayerConfig(d_model=512, n_q_heads=4, n_kv_heads=2, head_dim=128, ffn_dim=1024, rope_theta=500000.0)
    lens = [(7 * b) % 31 + 1 for b in range(70)]
    inp = make_inputs(Workload("many_blocks", layer, lens, 70, 3), gain_jitter=True)
    ref = oracle_pass(inp)
    for budget in (100, 4096):
        check(inp, budget, False, ref)


def test_bf16_mixed_routed_layer_every_row():
    """The mixed call does not report its routing tables, so the checker lists, per row, every
    expert set that is a valid top-k choice when logits closer than the rounding margin may
    swap (one set on most rows, two or three at a near-tie), evaluates the layer for each, and
    the GPU's row must match one of them within the tolerances.  Every row is compared."""
    layer = LayerConfig(d_model=256, n_q_heads=8, n_kv_heads=2, head_dim=64, ffn_dim=320, n_experts=16, top_k=4,
                        rope_theta=500000.0)
    wl = Workload("small_moe", layer, [200, 75, 30], 3, 4)
    inp = make_inputs(wl)
    g = run_mixed(inp, 96)
    pre, y_dec, Ks, Vs, routes, ref = oracle_pass(inp)
    k, N, S = layer.top_k, 3, 4
    log = ErrLog()
    for b in range(N):
        log.cmp("K%d" % b, to_numpy_f64(g["kv"].block_k(b)), Ks[b])
        log.cmp("V%d" % b, to_numpy_f64(g["kv"].block_v(b)), Vs[b])
    scale = max(np.abs(p["logits"]).max() for p in pre)
    n_multi = 0

    def best_candidate(got, h, logits):
        """got [d]; the candidate evaluation closest to it."""
        cands = H.routing_candidates(logits, k, 2e-2 * scale)
        assert 1 <= len(cands) <= 20
        ys = [ref.ffn(h[None], forced_idx=np.array([c]))[0][0] for c in cands]
        return min(ys, key=lambda y: np.linalg.norm(y - got)), len(cands) > 1

    got_last = to_numpy_f64(g["y_last"])
    want = []
    for b in range(N):
        y, multi = best_candidate(got_last[b], pre[b]["h"][-1], pre[b]["logits"][-1])
        want.append(y)
        n_multi += multi
    log.cmp("y_last", got_last, np.stack(want))
    got_dec = to_numpy_f64(g["y_dec"])
    for s in range(S):
        want = []
        for b in range(N):
            y, multi = best_candidate(got_dec[s, b], routes[s][b][3], routes[s][b][2])
            want.append(y)
            n_multi += multi
        log.cmp("y_dec%d" % s, got_dec[s], np.stack(want))
    log.check("rows with more than one valid expert set: %d of %d (all compared) |" % (n_multi, N + S * N))


def test_dense_ragged32_mixed_matches_the_plain_pass_at_full_size():
    """The named ragged workload (32 blocks of 512..8192 tokens) with 8 decode steps under an 8192-token
    budget against compact_layer_forward (which test_gpu_full_size.py checks against the fp64 checker at
    this size): prefill K/V rows bitwise (projections are row-wise), everything else within the bf16 tolerance."""
    wl = WORKLOADS["dense_ragged32"]
    S = 8
    inp = make_inputs(wl, device=DEV, gen_device=DEV, decode_steps=S)
    g = run_mixed(inp, 8192, weights=inp.weights)
    layer, cu, lens = inp.layer, inp.cu_seqlens, inp.block_lens
    N, T = len(lens), cu[-1]
    lay = B.Layer(layer, inp.weights)
    dt = torch.bfloat16
    kv = B.KVCache(layer, [L + S + 3 for L in lens], DEV, dt)
    lay.ensure_workspace(T, N, max(lens) + S, DEV)
    y_last = torch.empty(N, layer.d_model, dtype=dt, device=DEV)
    y_dec = torch.empty(S, N, layer.d_model, dtype=dt, device=DEV)
    lay.compact_layer_forward(cu, inp.x_prefill, inp.x_decode.contiguous(), kv, None, y_last, y_dec)
    torch.cuda.synchronize()

    def vec_err(a, b):
        a, b = a.float(), b.float()
        return ((a - b).norm(dim=-1) / b.norm(dim=-1)).max().item()

    assert vec_err(g["y_last"], y_last) < 2e-2
    assert vec_err(g["y_dec"], y_dec) < 2e-2
    for b in (0, int(np.argmin(lens)), int(np.argmax(lens)), N - 1):
        L = lens[b]
        assert torch.equal(g["kv"].block_k(b)[:L], kv.block_k(b)[:L])
        assert torch.equal(g["kv"].block_v(b)[:L], kv.block_v(b)[:L])
        assert vec_err(g["kv"].block_k(b)[L:].reshape(S, -1), kv.block_k(b)[L:].reshape(S, -1)) < 2e-2
        assert vec_err(g["kv"].block_v(b)[L:].reshape(S, -1), kv.block_v(b)[L:].reshape(S, -1)) < 2e-2


def test_mixed_degenerate_schedules_fp32():
    """The smallest budget the call accepts (one chunk row per step once every block decodes), blocks of
    one token, no decode steps at all, and a single block."""
    wl = WORKLOADS["tiny_fp32"]
    inp = make_inputs(wl, block_lens=[5, 1, 9], decode_steps=3, gain_jitter=True)
    check(inp, 4, True, oracle_pass(inp))
    inp0 = make_inputs(wl, block_lens=[5, 1, 9], decode_steps=0)
    check(inp0, 4, True, oracle_pass(inp0))
    one = make_inputs(wl, block_lens=[33], decode_steps=2)
    check(one, 16, True, oracle_pass(one))


def test_mixed_random_schedules_fp32():
    """Random block lengths, step counts and budgets (seeded): the schedule never changes the result."""
    wl = WORKLOADS["tiny_fp32"]
    rng = np.random.default_rng(2024)
    for _ in range(6):
        n = int(rng.integers(1, 7))
        lens = [int(v) for v in rng.integers(1, 150, size=n)]
        steps = int(rng.integers(0, 7))
        budget = int(rng.integers(n + 1, 200))
        inp = make_inputs(wl, block_lens=lens, decode_steps=steps, gain_jitter=True)
        print("lens", lens, "steps", steps, end=" ")
        check(inp, budget, True, oracle_pass(inp))
