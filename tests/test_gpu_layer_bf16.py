"""bf16 storage mode against the fp64 checker, whole layer, reduced sizes.

Tolerance.  The layer's outputs are hidden-state vectors (one per token) and
cached K/V head vectors; the bound is on each vector's relative error,
max_t ||g_t - r_t||_2 / ||r_t||_2 <= 2e-2.  An element-wise bound at the same
2e-2 cannot hold for a bf16 pipeline at these sizes whatever the kernels do:
the storage roundings that any bf16 layer has (normalised activations, the
SwiGLU intermediate, attention probabilities and output, the final result; unit
roundoff 2^-8) add up to an rms relative error of about 0.4 % of the output
scale, and the largest of 10^5..10^8 such errors sits at 4.5..6 sigma, i.e.
2..2.5 %.  So the element-wise error (floored at the tensor's rms) is bounded at
5e-2 -- far outside rounding noise, well inside any indexing or masking
mistake, which shows up as O(1) -- and the vector bound carries the 2e-2."""
import copy

import numpy as np
import pytest
import torch

from paper_2605_23296_amd.workloads import WORKLOADS, Workload, LayerConfig, make_inputs
from tests import harness as H
from tests.util import rel_err, vec_rel_err

pytestmark = pytest.mark.gpu
TOL = 2e-2          # per-vector relative error
ELEM_TOL = 5e-2     # element-wise, floored at rms(r)


def sample_rows(L, rng, n=12):
    edges = [0, 1, 31, 32, 63, 64, 65, 127, 128, 129, 255, 256, L - 2, L - 1]
    rows = sorted(set([r for r in edges if 0 <= r < L] + list(rng.integers(0, L, size=n))))
    return rows


def check_dense(inp, steps=None, pos_offset=None, sampled=True):
    rng = np.random.default_rng(5)
    S = inp.x_decode.shape[0]
    g = H.gpu_forward(inp, pos_offset=pos_offset)
    lay = H.oracle_layer(inp)
    rows = [sample_rows(L, rng) if sampled else list(range(L)) for L in inp.block_lens]
    steps = list(range(S)) if steps is None else steps
    from paper_2605_23296_amd.workloads import to_numpy_f64
    pre, yd, Ks, Vs, _ = lay.forward_sampled(to_numpy_f64(inp.x_prefill), inp.cu_seqlens, to_numpy_f64(inp.x_decode),
                                             rows, steps, pos_offset)
    errs, elem = {}, {}

    def cmp(name, got, ref):
        errs[name] = vec_rel_err(got, ref)
        elem[name] = rel_err(got, ref)

    for b, L in enumerate(inp.block_lens):
        cmp("y_pre%d" % b, g["y_prefill"][inp.cu_seqlens[b]:inp.cu_seqlens[b + 1]][rows[b]], pre[b]["y"])
        cmp("K%d" % b, g["K"][b], Ks[b])
        cmp("V%d" % b, g["V"][b], Vs[b])
        assert g["lens"][b] == L + S
    for s in steps:
        cmp("y_dec%d" % s, g["y_decode"][s], yd[s])
    worst, worst_e = max(errs, key=errs.get), max(elem, key=elem.get)
    print("worst vector error", worst, "%.3e" % errs[worst], "| worst element error", worst_e, "%.3e" % elem[worst_e])
    assert errs[worst] < TOL, {k: "%.2e" % v for k, v in errs.items()}
    assert elem[worst_e] < ELEM_TOL, {k: "%.2e" % v for k, v in elem.items()}
    return g


def test_tiny_layer_in_bf16_in_full():
    wl = copy.deepcopy(WORKLOADS["tiny_fp32"])
    wl.layer.dtype = "bf16"
    check_dense(make_inputs(wl), sampled=False)


def test_dense_8b_layer_ragged_blocks():
    inp = make_inputs(WORKLOADS["dense_8x4096"], block_lens=[300, 1, 513, 64, 129], decode_steps=3, gain_jitter=True)
    check_dense(inp, pos_offset=[0, 17, 0, 4000, 3])


def test_dense_batched_equals_one_block_at_a_time_bitwise():
    """Sec. IV: a block's result does not depend on the blocks it is batched with."""
    inp = make_inputs(WORKLOADS["dense_8x4096"], block_lens=[300, 70, 513], decode_steps=2)
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


def test_run_to_run_determinism():
    inp = make_inputs(WORKLOADS["dense_8x4096"], block_lens=[257, 300], decode_steps=2)
    a = H.gpu_forward(inp)
    b = H.gpu_forward(inp)
    assert np.array_equal(a["y_prefill"], b["y_prefill"]) and np.array_equal(a["y_decode"], b["y_decode"])


def check_moe(inp, margin_rel, tol):
    from paper_2605_23296_amd.workloads import to_numpy_f64
    g = H.gpu_forward_steps(inp)
    r = H.oracle_forward(inp)
    k = inp.layer.top_k
    S = inp.x_decode.shape[0]
    n_unsafe = 0
    errs = {}
    err_fn = rel_err if inp.layer.dtype == "fp32" else vec_rel_err
    for b, L in enumerate(inp.block_lens):
        sl = slice(inp.cu_seqlens[b], inp.cu_seqlens[b + 1])
        ok, nu = H.routed_rows_match(g["idx_prefill"][sl], r["pre"][b]["idx"], r["pre"][b]["logits"], k, margin_rel)
        n_unsafe += nu
        errs["y_pre%d" % b] = err_fn(g["y_prefill"][sl][ok], r["pre"][b]["y"][ok])
        errs["K%d" % b] = err_fn(g["K"][b], r["K"][b])
        errs["V%d" % b] = err_fn(g["V"][b], r["V"][b])
    for s in range(S):
        idx_ref = np.stack([r["routes"][s][b][0] for b in range(len(inp.block_lens))])
        logits_ref = np.stack([r["routes"][s][b][2] for b in range(len(inp.block_lens))])
        ok, nu = H.routed_rows_match(g["idx_decode"][s], idx_ref, logits_ref, k, margin_rel)
        n_unsafe += nu
        if ok.any():
            errs["y_dec%d" % s] = err_fn(g["y_decode"][s][ok], r["y_decode"][s][ok])
    worst = max(errs, key=errs.get)
    print("worst", worst, "%.3e" % errs[worst], "rows with a close call:", n_unsafe)
    assert errs[worst] < tol, {k_: "%.2e" % v for k_, v in errs.items()}
    total = inp.cu_seqlens[-1] + S * len(inp.block_lens)
    assert n_unsafe < 0.5 * total


SMALL_MOE = LayerConfig(d_model=256, n_q_heads=8, n_kv_heads=2, head_dim=64, ffn_dim=320, n_experts=16, top_k=4,
                        rope_theta=500000.0)


def test_small_moe_layer_fp32():
    layer = copy.deepcopy(SMALL_MOE)
    layer.dtype = "fp32"
    wl = Workload("small_moe", layer, [130, 40, 1, 77], 4, 3)
    check_moe(make_inputs(wl), margin_rel=1e-5, tol=1e-5)


def test_small_moe_layer_bf16():
    wl = Workload("small_moe", copy.deepcopy(SMALL_MOE), [300, 40, 1, 513], 4, 3)
    check_moe(make_inputs(wl), margin_rel=2e-2, tol=TOL)


def test_moe_120b_shape_reduced():
    layer = copy.deepcopy(WORKLOADS["moe_16x8192"].layer)
    layer.n_experts = 16            # same expert shape, fewer experts: bounds the checker's time
    wl = Workload("moe_reduced", layer, [200, 65], 2, 2)
    check_moe(make_inputs(wl), margin_rel=2e-2, tol=TOL)
