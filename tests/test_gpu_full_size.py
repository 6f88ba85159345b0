"""The named workloads at their full sizes, in the launch configuration the
benchmark times (one compact_layer_forward call over all blocks; the routed
layer through compact_prefill + compact_decode_step so that its routing tables
can be read back), checked against the fp64 checker on sampled outputs.

Blocks are independent (paper Sec. IV), so the checker recomputes a few whole
blocks of the batch -- first, last, and for ragged batches the shortest and the
longest -- from the same seeded inputs: every cached K and V row of those
blocks, the layer output at query rows that straddle every kernel tile edge
plus random ones, and the decode outputs at the first, second, middle and last
step.  Tolerances are those of tests/test_gpu_layer_bf16.py.  The router at
full size (131072 rows, ordered indices against the checker on the same input) is
checked through its own entry point in tests/test_gpu_kernels.py; here every row of
the prefill's routing table must hold four distinct experts and gates that sum to one."""
import numpy as np
import pytest
import torch

from oracle import layer as O
from paper_2605_23296_amd import binding as B
from paper_2605_23296_amd.workloads import WORKLOADS, make_inputs, make_mxfp4_experts, to_numpy_f64
from tests import harness as H
from tests.util import ErrLog

pytestmark = pytest.mark.gpu
# Routed layer: the GPU routes from its bf16 activations, the checker from fp64 ones.
# The bf16 rounding of the 2880 normalised inputs moves a logit by about 0.4 % of the
# logits' spread (sigma ~ 1), i.e. ~1e-3 of max|logit| ~ 4; experts whose logits are
# closer than 8e-3 * max|logit| (about eight such sigmas) may legitimately swap
# (tests/harness.py, check_routing).  Every row's output is compared, the checker's
# feed-forward being evaluated for the experts the GPU chose.
MOE_MARGIN = 8e-3


class LazyF64:
    """Widens slices of a large device tensor to float64 numpy on demand (the
    expert weights of the routed layer would take 25 GB as float64)."""

    def __init__(self, t):
        self.t = t
        self.shape = tuple(t.shape)

    def __getitem__(self, key):
        return to_numpy_f64(self.t[key])


class LazyQ4:
    """Expert weights given as block-scaled 4-bit arrays: expert e is expanded to float64 on
    demand by the checker's own definition of the format (oracle/mxfp4.py), from the codes."""

    def __init__(self, codes, scales):
        self.codes, self.scales = codes, scales
        self.shape = tuple(codes.shape[:-1]) + (codes.shape[-1] * 2,)

        self._last = (None, None)

    def __getitem__(self, key):
        from oracle import mxfp4 as Q
        key = key if isinstance(key, tuple) else (key,)
        e = int(key[0])
        if self._last[0] != e:
            self._last = (e, Q.dequantize(self.codes[e].cpu().numpy(), self.scales[e].cpu().numpy()))
        return self._last[1][key[1:]] if len(key) > 1 else self._last[1]


def sample_rows(L, rng, n=10):
    edges = [0, 1, 31, 32, 63, 64, 65, 127, 128, 129, 255, 256, 257, 2047, 2048, L - 129, L - 128, L - 65, L - 64, L - 2, L - 1]
    return sorted(set([r for r in edges if 0 <= r < L] + [int(v) for v in rng.integers(0, L, size=n)]))


def run_gpu(inp, with_routes):
    layer = inp.layer
    dev = "cuda"
    lay = B.Layer(layer, inp.weights)
    dt = lay.torch_dtype
    lens, S, N, T = inp.block_lens, inp.x_decode.shape[0], len(inp.block_lens), inp.cu_seqlens[-1]
    kv = B.KVCache(layer, [L + S for L in lens], dev, dt)
    kv.k.fill_(float("nan"))
    kv.v.fill_(float("nan"))
    lay.ensure_workspace(T, N, max(lens) + S, dev)
    y_pre = torch.empty(T, layer.d_model, dtype=dt, device=dev)
    y_last = torch.empty(N, layer.d_model, dtype=dt, device=dev)
    y_dec = torch.empty(S, N, layer.d_model, dtype=dt, device=dev)
    out = dict(y_pre=y_pre, y_last=y_last, y_dec=y_dec, kv=kv, lay=lay)
    xd = inp.x_decode.contiguous()
    if not with_routes:
        lay.compact_layer_forward(inp.cu_seqlens, inp.x_prefill, xd, kv, y_pre, y_last, y_dec)
    else:
        k = layer.top_k
        out["idx_pre"] = torch.empty(T, k, dtype=torch.int32, device=dev)
        out["gate_pre"] = torch.empty(T, k, dtype=torch.float32, device=dev)
        out["idx_dec"] = torch.empty(S, N, k, dtype=torch.int32, device=dev)
        out["gate_dec"] = torch.empty(S, N, k, dtype=torch.float32, device=dev)
        lay.compact_prefill(inp.cu_seqlens, inp.x_prefill, kv, y_pre, (out["idx_pre"], out["gate_pre"]))
        for s in range(S):
            lay.compact_decode_step(xd[s], kv, y_dec[s], (out["idx_dec"][s], out["gate_dec"][s]))
    torch.cuda.synchronize()
    assert kv.lens() == [L + S for L in lens]
    return out


def check_workload(name, blocks=None, n_rows=10, mxfp4=False):
    wl = WORKLOADS[name]
    inp = make_inputs(wl, device="cuda", gen_device="cuda")
    q4 = None
    if mxfp4:
        # the experts are 4-bit arrays; the library expands them into its 16-bit copy (read by the prefill),
        # the checker expands the same arrays by its own definition
        gen = torch.Generator(device="cuda")
        gen.manual_seed(wl.seed + 77)
        q4 = make_mxfp4_experts(inp.layer, gen, "cuda")
        lay0 = B.Layer(inp.layer, None)
        for nm in ("w_exp_gate_up", "w_exp_down"):
            lay0.compact_mxfp4_dequant(q4[nm + "_q"], q4[nm + "_s"], inp.weights[nm])
        inp.weights.update(q4)
        torch.cuda.synchronize()
    layer, lens, cu = inp.layer, inp.block_lens, inp.cu_seqlens
    N, S = len(lens), inp.x_decode.shape[0]
    moe = layer.n_experts > 0
    g = run_gpu(inp, with_routes=moe)
    if blocks is None:
        blocks = sorted(set([0, N - 1, int(np.argmin(lens)), int(np.argmax(lens))]))
    steps = sorted(set([0, 1, S // 2, S - 1]))
    rng = np.random.default_rng(11)

    w = {}
    for k_, v in inp.weights.items():
        if k_.endswith(("_q", "_s")):
            continue
        if k_.startswith("w_exp_"):
            w[k_] = LazyQ4(q4[k_ + "_q"], q4[k_ + "_s"]) if mxfp4 else LazyF64(v)
        else:
            w[k_] = to_numpy_f64(v)
    ref = O.Layer(layer.as_dict(), w)
    log, n_close, n_routed = ErrLog(), 0, 0
    cmp = log.cmp

    for b in blocks:
        L = lens[b]
        rows = sample_rows(L, rng, n_rows)
        x = to_numpy_f64(inp.x_prefill[cu[b]:cu[b + 1]])
        xd = to_numpy_f64(inp.x_decode[:, b:b + 1])
        pre, yd, Ks, Vs, routes = ref.forward_sampled(x, [0, L], xd, [rows], steps)
        cmp("K%d" % b, to_numpy_f64(g["kv"].block_k(b)), Ks[0])
        cmp("V%d" % b, to_numpy_f64(g["kv"].block_v(b)), Vs[0])
        y_rows = to_numpy_f64(g["y_pre"][cu[b]:cu[b + 1]][rows])
        if not moe:
            cmp("y_pre%d" % b, y_rows, pre[0]["y"])
            assert np.array_equal(to_numpy_f64(g["y_last"][b]), to_numpy_f64(g["y_pre"][cu[b + 1] - 1]))
            for s in steps:
                cmp("y_dec%d_%d" % (s, b), to_numpy_f64(g["y_dec"][s, b]), yd[s][0])
        else:
            k = layer.top_k
            idx_rows = g["idx_pre"][cu[b]:cu[b + 1]][rows].cpu().numpy()
            gate_rows = g["gate_pre"][cu[b]:cu[b + 1]][rows].cpu().numpy()
            n_close += H.check_routing(idx_rows, pre[0]["logits"], k, MOE_MARGIN, gate_rows)
            n_routed += len(rows)
            cmp("y_pre%d" % b, y_rows, ref.ffn(pre[0]["h"], forced_idx=idx_rows)[0])
            for s in steps:
                _, _, logits_s, h_s = routes[s]
                idx_s = g["idx_dec"][s, b:b + 1].cpu().numpy()
                n_close += H.check_routing(idx_s, logits_s, k, MOE_MARGIN, g["gate_dec"][s, b:b + 1].cpu().numpy())
                n_routed += 1
                cmp("y_dec%d_%d" % (s, b), to_numpy_f64(g["y_dec"][s, b:b + 1]), ref.ffn(h_s, forced_idx=idx_s)[0])
    log.check("%s blocks %s lens %s | routed rows with a close call: %d of %d (all compared) |"
              % (name, blocks, [lens[b] for b in blocks], n_close, n_routed))
    if moe:
        idx_all = g["idx_pre"]
        srt = idx_all.sort(dim=1).values
        assert bool(((idx_all >= 0) & (idx_all < layer.n_experts)).all()) and bool((srt[:, 1:] != srt[:, :-1]).all())
        assert bool(((g["gate_pre"].sum(dim=1) - 1).abs() < 1e-5).all())
    # nothing outside the blocks' own rows was written: the slab tails stay poisoned
    kvc = g["kv"]
    for b in blocks:
        Hkv, hd, cap, Lb = layer.n_kv_heads, layer.head_dim, kvc.caps[b], lens[b] + S
        if cap > Lb:
            slab = kvc.k[kvc.offs[b]:kvc.offs[b] + cap * Hkv * hd].view(Hkv, cap, hd)
            assert torch.isnan(slab[:, Lb:, :].float()).all()


def test_dense_8x4096_full_size():
    check_workload("dense_8x4096")


def test_dense_64x2048_full_size():
    check_workload("dense_64x2048")


def test_dense_ragged32_full_size():
    check_workload("dense_ragged32")


def test_moe_16x8192_full_size():
    check_workload("moe_16x8192", blocks=[0, 15], n_rows=6)


def test_moe_16x8192_full_size_with_4bit_experts():
    """The routed workload with block-scaled 4-bit experts (bench.py --mxfp4): decode steps stream the
    4-bit arrays, the prefill reads their expansion; the checker's experts come from the same arrays."""
    check_workload("moe_16x8192", blocks=[0, 15], n_rows=6, mxfp4=True)
