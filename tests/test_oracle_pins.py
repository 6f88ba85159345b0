"""Pins for the fp64 checker: invariants, closed forms, a hand-worked case and
library special cases.  Each is chosen so that a plausible mistake in
oracle/layer.py (dropped term, wrong sign or index, transposed operand, wrong
mask edge) fails at least one of them.  CPU only."""
import math
import os

import numpy as np
import pytest
import torch

from oracle import layer as O
from tests.util import read_golden

HERE = os.path.dirname(os.path.abspath(__file__))


def small_cfg(**kw):
    cfg = dict(d_model=32, n_q_heads=4, n_kv_heads=2, head_dim=8, ffn_dim=48,
               n_experts=0, top_k=0, rms_eps=1e-5, rope_theta=10000.0)
    cfg.update(kw)
    return cfg


def small_weights(cfg, rng, std=0.2):
    d, F = cfg["d_model"], cfg["ffn_dim"]
    Dq = cfg["n_q_heads"] * cfg["head_dim"]
    Dkv = cfg["n_kv_heads"] * cfg["head_dim"]
    w = dict(g_attn=1 + 0.1 * rng.standard_normal(d), g_ffn=1 + 0.1 * rng.standard_normal(d),
             w_qkv=std * rng.standard_normal((Dq + 2 * Dkv, d)),
             w_o=std * rng.standard_normal((d, Dq)))
    if cfg["n_experts"] == 0:
        w["w_gate_up"] = std * rng.standard_normal((2 * F, d))
        w["w_down"] = std * rng.standard_normal((d, F))
    else:
        E = cfg["n_experts"]
        w["w_router"] = std * rng.standard_normal((E, d))
        w["w_exp_gate_up"] = std * rng.standard_normal((E, 2 * F, d))
        w["w_exp_down"] = std * rng.standard_normal((E, d, F))
    return w


# ---------------------------------------------------------------- softmax / attention core
def test_softmax_rows_sum_to_one_and_nonnegative(rng):
    q = rng.standard_normal((9, 16)) * 3
    k = rng.standard_normal((9, 16)) * 3
    p = O.attention_probs(q, k, visible=np.arange(9) + 1)
    assert np.all(p >= 0)
    np.testing.assert_allclose(p.sum(-1), 1.0, atol=1e-14)
    # masked entries are exactly zero: strictly upper triangle
    assert np.all(np.triu(p, 1) == 0)
    # the diagonal is visible (inclusive causal mask)
    assert np.all(np.diag(p) > 0)


def test_identical_keys_give_running_mean_of_values(rng):
    L, hd = 7, 8
    q = rng.standard_normal((L, hd))
    k = np.tile(rng.standard_normal((1, hd)), (L, 1))
    v = rng.standard_normal((L, hd))
    o = O.attention_head(q, k, v, visible=np.arange(L) + 1)
    want = np.cumsum(v, axis=0) / (np.arange(L) + 1)[:, None]
    np.testing.assert_allclose(o, want, atol=1e-14)


def test_zero_query_gives_running_mean_through_whole_layer_attention(rng):
    # q = 0 so the rotary embedding cannot break the tie between keys
    L, hd = 5, 8
    q = np.zeros((L, 2, hd))
    k = rng.standard_normal((L, 1, hd))
    v = rng.standard_normal((L, 1, hd))
    o = O.gqa_attention(q, k, v, visible=np.arange(L) + 1)
    want = np.cumsum(v[:, 0], axis=0) / (np.arange(L) + 1)[:, None]
    np.testing.assert_allclose(o[:, 0], want, atol=1e-14)
    np.testing.assert_allclose(o[:, 1], want, atol=1e-14)


def test_two_token_case_worked_by_hand():
    g = read_golden(os.path.join(HERE, "golden", "two_token_attention.txt"))
    q = np.stack([g["q0"], g["q1"]])
    k = np.stack([g["k0"], g["k1"]])
    v = np.stack([g["v0"], g["v1"]])
    p = O.attention_probs(q, k, visible=[1, 2])
    np.testing.assert_allclose(p[0], [1.0, 0.0], atol=1e-15)
    np.testing.assert_allclose(p[1], g["p1"], atol=1e-15)
    o = O.attention_head(q, k, v, visible=[1, 2])
    np.testing.assert_allclose(o[0], g["o0"], atol=1e-14)
    np.testing.assert_allclose(o[1], g["o1"], atol=1e-14)
    # and with the rotary embedding applied at positions 0, 1 first
    qr = O.rope(q[:, None, :], np.array([0, 1]), 10000.0)[:, 0]
    kr = O.rope(k[:, None, :], np.array([0, 1]), 10000.0)[:, 0]
    o = O.attention_head(qr, kr, v, visible=[1, 2])
    np.testing.assert_allclose(o[1], g["o1"], atol=1e-14)


def test_scale_is_one_over_sqrt_head_dim():
    # a single query against two keys; closed form of the weight ratio
    hd = 16
    q = np.ones((1, hd))
    k = np.stack([np.zeros(hd), np.full(hd, 0.5)])
    p = O.attention_probs(q, k, visible=[2])
    # score difference = hd*0.5/sqrt(hd) = 0.5*sqrt(hd) = 2
    np.testing.assert_allclose(p[0, 1] / p[0, 0], math.exp(2.0), rtol=1e-13)


def test_attention_core_equals_library_sdpa(rng):
    L, Hq, Hkv, hd = 11, 4, 2, 8
    q = rng.standard_normal((L, Hq, hd))
    k = rng.standard_normal((L, Hkv, hd))
    v = rng.standard_normal((L, Hkv, hd))
    o = O.gqa_attention(q, k, v, visible=np.arange(L) + 1)
    tq, tk, tv = (torch.from_numpy(a).permute(1, 0, 2)[None] for a in (q, k, v))
    ref = torch.nn.functional.scaled_dot_product_attention(
        tq, tk, tv, is_causal=True, enable_gqa=True)[0].permute(1, 0, 2).numpy()
    np.testing.assert_allclose(o, ref, atol=1e-12)


# ---------------------------------------------------------------- rotary embedding
def test_rope_identity_at_position_zero_and_norm_preserving(rng):
    x = rng.standard_normal((6, 3, 16))
    np.testing.assert_array_equal(O.rope(x, np.zeros(6, dtype=int), 5e5), x)
    r = O.rope(x, np.arange(6) * 37, 5e5)
    np.testing.assert_allclose(np.linalg.norm(r, axis=-1), np.linalg.norm(x, axis=-1), rtol=1e-13)


def test_rope_inner_product_depends_only_on_relative_position(rng):
    q = rng.standard_normal((1, 1, 16))
    k = rng.standard_normal((1, 1, 16))

    def dot(m, n):
        return float(np.sum(O.rope(q, np.array([m]), 1e4) * O.rope(k, np.array([n]), 1e4)))

    assert abs(dot(5, 2) - dot(103, 100)) < 1e-12
    assert abs(dot(5, 2) - dot(2, 5)) > 1e-3        # sign of the rotation matters


def test_rope_equals_complex_multiplication(rng):
    # pair (x_i, x_{i+hd/2}) read as the complex number x_i + 1j x_{i+hd/2},
    # multiplied by exp(1j * pos * theta^(-2i/hd))
    T, H, hd, theta = 5, 2, 8, 500000.0
    x = rng.standard_normal((T, H, hd))
    pos = np.array([0, 1, 7, 100, 4095])
    z = x[..., :hd // 2] + 1j * x[..., hd // 2:]
    ang = pos[:, None] * theta ** (-np.arange(hd // 2) / (hd // 2))
    z = z * np.exp(1j * ang)[:, None, :]
    want = np.concatenate([z.real, z.imag], axis=-1)
    np.testing.assert_allclose(O.rope(x, pos, theta), want, atol=1e-12)


def test_rope_first_pair_rotates_by_position_radians():
    # frequency of pair 0 is theta^0 = 1: position 1 rotates (1, 0) to (cos 1, sin 1)
    x = np.zeros((1, 1, 4))
    x[0, 0, 0] = 1.0
    r = O.rope(x, np.array([1]), 10000.0)
    np.testing.assert_allclose(r[0, 0], [math.cos(1.0), 0.0, math.sin(1.0), 0.0], atol=1e-15)
    # pair 1 of hd=4 has frequency theta^(-1/2)
    x = np.zeros((1, 1, 4))
    x[0, 0, 1] = 1.0
    r = O.rope(x, np.array([3]), 10000.0)
    np.testing.assert_allclose(r[0, 0], [0.0, math.cos(0.03), 0.0, math.sin(0.03)], atol=1e-15)


# ---------------------------------------------------------------- RMSNorm
def test_rmsnorm_unit_rms_scale_invariance_and_library(rng):
    x = rng.standard_normal((4, 64)) * 5
    n = O.rmsnorm(x, np.ones(64), 0.0)
    np.testing.assert_allclose(np.sqrt(np.mean(n * n, -1)), 1.0, rtol=1e-13)
    np.testing.assert_allclose(O.rmsnorm(3.7 * x, np.ones(64), 0.0), n, rtol=1e-13)
    g = 1 + 0.1 * rng.standard_normal(64)
    ref = torch.nn.functional.rms_norm(torch.from_numpy(x), (64,), torch.from_numpy(g), 1e-5).numpy()
    np.testing.assert_allclose(O.rmsnorm(x, g, 1e-5), ref, rtol=1e-13)
    # eps sits inside the square root, added to the mean square
    one = O.rmsnorm(np.array([[2.0, 2.0]]), np.ones(2), 5.0)
    np.testing.assert_allclose(one, [[2 / 3.0, 2 / 3.0]], rtol=1e-15)


# ---------------------------------------------------------------- SwiGLU
def test_silu_and_swiglu_special_cases(rng):
    assert O.silu(np.array(0.0)) == 0.0
    np.testing.assert_allclose(O.silu(np.array(40.0)), 40.0, rtol=1e-15)
    np.testing.assert_allclose(O.silu(np.array(1.0)), 1 / (1 + math.exp(-1.0)), rtol=1e-15)
    m = rng.standard_normal((3, 8))
    wu = rng.standard_normal((12, 8))
    wd = rng.standard_normal((8, 12))
    assert np.all(O.swiglu_ffn(m, np.zeros((12, 8)), wu, wd) == 0)
    wg = rng.standard_normal((12, 8))
    ref = torch.nn.functional.linear(
        torch.nn.functional.silu(torch.from_numpy(m @ wg.T)) * torch.from_numpy(m @ wu.T),
        torch.from_numpy(wd)).numpy()
    np.testing.assert_allclose(O.swiglu_ffn(m, wg, wu, wd), ref, rtol=1e-12, atol=1e-12)
    # gate and up are not interchangeable: silu is applied to the gate only
    assert np.max(np.abs(O.swiglu_ffn(m, wu, wg, wd) - ref)) > 1e-3


# ---------------------------------------------------------------- router / MoE
def test_topk_route_is_brute_force_argsort_with_ties_to_lower_index(rng):
    logits = rng.standard_normal((50, 16))
    logits[3, 5] = logits[3, 9] = 10.0         # exact tie at the top
    logits[4, :] = 0.0                         # all equal
    idx, gate = O.topk_route(logits, 4)
    for r in range(50):
        brute = sorted(range(16), key=lambda e: (-logits[r, e], e))[:4]
        assert list(idx[r]) == brute
    assert list(idx[3][:2]) == [5, 9]
    assert list(idx[4]) == [0, 1, 2, 3]
    np.testing.assert_allclose(gate.sum(-1), 1.0, atol=1e-14)
    # gate = softmax over the selected logits only
    r = 7
    e = np.exp(logits[r, idx[r]])
    np.testing.assert_allclose(gate[r], e / e.sum(), rtol=1e-13)
    # equivalently: softmax over all experts, renormalised over the top-k
    full = np.exp(logits[r]) / np.exp(logits[r]).sum()
    np.testing.assert_allclose(gate[r], full[idx[r]] / full[idx[r]].sum(), rtol=1e-12)


def test_moe_with_identical_experts_equals_dense(rng):
    cfg = small_cfg(n_experts=6, top_k=3)
    w = small_weights(cfg, rng)
    w["w_exp_gate_up"][:] = w["w_exp_gate_up"][0]
    w["w_exp_down"][:] = w["w_exp_down"][0]
    dense_cfg = small_cfg()
    wd = {k: v for k, v in w.items() if not k.startswith("w_exp") and k != "w_router"}
    wd["w_gate_up"] = w["w_exp_gate_up"][0]
    wd["w_down"] = w["w_exp_down"][0]
    x = rng.standard_normal((9, cfg["d_model"]))
    y_moe = O.Layer(cfg, w).prefill_block(x)["y"]
    y_dense = O.Layer(dense_cfg, wd).prefill_block(x)["y"]
    np.testing.assert_allclose(y_moe, y_dense, atol=1e-12)


def test_moe_one_hot_router_and_expert_permutation(rng):
    cfg = small_cfg(n_experts=5, top_k=2)
    w = small_weights(cfg, rng)
    m = rng.standard_normal((4, cfg["d_model"]))
    idx, gate = O.topk_route(O.router_logits(m, w["w_router"]), 2)
    out = O.moe_ffn(m, idx, gate, w["w_exp_gate_up"], w["w_exp_down"])
    F = cfg["ffn_dim"]
    # definition, token by token
    for r in range(4):
        want = sum(gate[r, s] * O.swiglu_ffn(m[r:r + 1], w["w_exp_gate_up"][e, :F],
                                             w["w_exp_gate_up"][e, F:], w["w_exp_down"][e])[0]
                   for s, e in enumerate(idx[r]))
        np.testing.assert_allclose(out[r], want, atol=1e-12)
    # rows over experts account for k rows per token
    assert sum(int(np.sum(idx == e)) for e in range(5)) == 2 * 4
    # permuting the experts permutes the indices only
    perm = np.array([3, 0, 4, 1, 2])          # new expert j is old expert perm[j]
    idx2, gate2 = O.topk_route(O.router_logits(m, w["w_router"][perm]), 2)
    np.testing.assert_array_equal(perm[idx2], idx)
    out2 = O.moe_ffn(m, idx2, gate2, w["w_exp_gate_up"][perm], w["w_exp_down"][perm])
    np.testing.assert_allclose(out2, out, atol=1e-12)
    # a router row that dominates picks its expert first
    wr = np.zeros_like(w["w_router"])
    wr[2] = 50 * m[0] / np.dot(m[0], m[0])
    idx3, gate3 = O.topk_route(O.router_logits(m[:1], wr), 2)
    assert idx3[0, 0] == 2 and gate3[0, 0] > 0.999


def test_forced_expert_choice_follows_the_routed_layer_definition(rng):
    """The forced-choice evaluation the parity tests use at router near-ties: row r goes to
    the given experts, gated by the softmax over its own logits at those experts."""
    cfg = small_cfg(n_experts=6, top_k=3)
    w = small_weights(cfg, rng)
    lay = O.Layer(cfg, w)
    F = cfg["ffn_dim"]
    h = rng.standard_normal((7, cfg["d_model"]))
    y, idx, gate, logits = lay.ffn(h)
    # its own choice forced on it changes nothing, bit for bit
    y1, idx1, gate1, _ = lay.ffn(h, forced_idx=idx)
    assert np.array_equal(y1, y) and np.array_equal(idx1, idx) and np.array_equal(gate1, gate)
    # the order inside a choice only permutes the gates
    y2, _, gate2, _ = lay.ffn(h, forced_idx=idx[:, ::-1])
    np.testing.assert_allclose(y2, y, atol=1e-13)
    np.testing.assert_allclose(gate2, gate[:, ::-1], atol=1e-15)
    # another choice, against the definition written out token by token
    other = np.stack([rng.permutation(6)[:3] for _ in range(7)])
    y3, idx3, gate3, _ = lay.ffn(h, forced_idx=other)
    m = O.rmsnorm(h, w["g_ffn"], cfg["rms_eps"])
    for r in range(7):
        e = np.exp(logits[r, other[r]])
        g = e / e.sum()
        np.testing.assert_allclose(gate3[r], g, rtol=1e-13)
        want = h[r] + sum(g[s] * O.swiglu_ffn(m[r:r + 1], w["w_exp_gate_up"][ex, :F], w["w_exp_gate_up"][ex, F:],
                                               w["w_exp_down"][ex])[0] for s, ex in enumerate(other[r]))
        np.testing.assert_allclose(y3[r], want, atol=1e-12)
    assert not np.allclose(y3, y)
    # identical experts: any choice gives the dense layer
    w2 = dict(w)
    w2["w_exp_gate_up"] = np.repeat(w["w_exp_gate_up"][:1], 6, axis=0)
    w2["w_exp_down"] = np.repeat(w["w_exp_down"][:1], 6, axis=0)
    lay2 = O.Layer(cfg, w2)
    np.testing.assert_allclose(lay2.ffn(h, forced_idx=other)[0], lay2.ffn(h)[0], atol=1e-12)


def test_forced_choice_threads_through_blocks_steps_and_the_stack(rng):
    cfg = small_cfg(n_experts=5, top_k=2)
    ws = [small_weights(cfg, rng) for _ in range(2)]
    x = rng.standard_normal((11, cfg["d_model"]))
    xd = rng.standard_normal((3, 2, cfg["d_model"]))
    cu = [0, 7, 11]
    lay = O.Layer(cfg, ws[0])
    pre, yd, Ks, Vs, routes = lay.forward(x, cu, xd)
    # forcing the pass's own choices reproduces it; the reported h is the FFN half's input
    pre2 = lay.prefill(x, cu, forced_idx=[p["idx"] for p in pre])
    for a, b in zip(pre, pre2):
        assert np.array_equal(a["y"], b["y"])
        assert np.array_equal(lay.ffn(a["h"])[0], a["y"])
    Kc, Vc = [p["K"] for p in pre], [p["V"] for p in pre]
    for s in range(3):
        st = lay.decode_step(xd[s], Kc, Vc, forced_idx=np.stack([routes[s][b][0] for b in range(2)]))
        for b in range(2):
            assert np.array_equal(st[b]["y"], yd[s, b])
            assert np.array_equal(lay.ffn(routes[s][b][3][None])[0][0], yd[s, b])
            Kc[b], Vc[b] = st[b]["K"], st[b]["V"]
    # a different choice in one decode row moves that row only
    alt = np.stack([routes[0][b][0] for b in range(2)]).copy()
    alt[1] = [(alt[1, 0] + 1) % 5, (alt[1, 0] + 2) % 5]
    st = lay.decode_step(xd[0], [p["K"] for p in pre], [p["V"] for p in pre], forced_idx=alt)
    assert np.array_equal(st[0]["y"], yd[0, 0]) and not np.allclose(st[1]["y"], yd[0, 1])
    # the stack: forcing every layer's own choices reproduces the pass
    stack = O.Stack(cfg, ws)
    y_pre, y_dec, _, _ = stack.forward(x, cu, xd)
    forced = [(r["pre_idx"], np.stack(r["dec_idx"])) for r in stack.routes]
    y_pre2, y_dec2, _, _ = stack.forward(x, cu, xd, forced=forced)
    assert np.array_equal(y_pre, y_pre2) and np.array_equal(y_dec, y_dec2)
    # a changed choice in layer 0 reaches the last layer's output of that row
    forced[0][0][3] = [(forced[0][0][3, 0] + 1) % 5, (forced[0][0][3, 0] + 2) % 5]
    y_pre3, _, _, _ = stack.forward(x, cu, xd, forced=forced)
    assert np.array_equal(y_pre3[:3], y_pre[:3]) and not np.allclose(y_pre3[3], y_pre[3])


# ---------------------------------------------------------------- whole layer
@pytest.mark.parametrize("moe", [False, True])
def test_batched_equals_one_block_at_a_time(rng, moe):
    """The method's central equivalence (Sec. IV: per-block results are produced
    independently and concatenated in block order)."""
    cfg = small_cfg(n_experts=4, top_k=2) if moe else small_cfg()
    lay = O.Layer(cfg, small_weights(cfg, rng))
    lens = [5, 1, 9, 3]
    cu = np.concatenate([[0], np.cumsum(lens)])
    x = rng.standard_normal((cu[-1], cfg["d_model"]))
    xd = rng.standard_normal((3, len(lens), cfg["d_model"]))
    pre, yd, Ks, Vs, _ = lay.forward(x, cu, xd)
    for b, L in enumerate(lens):
        pre1, yd1, K1, V1, _ = lay.forward(x[cu[b]:cu[b + 1]], [0, L], xd[:, b:b + 1])
        assert np.array_equal(pre[b]["y"], pre1[0]["y"])
        assert np.array_equal(yd[:, b], yd1[:, 0])
        assert np.array_equal(Ks[b], K1[0]) and np.array_equal(Vs[b], V1[0])
        assert Ks[b].shape[0] == L + 3
    # and a block's result changes if its own tokens change (the test is not vacuous)
    x2 = x.copy()
    x2[cu[2]] += 1.0
    pre2 = lay.prefill(x2, cu)
    assert not np.array_equal(pre2[2]["y"], pre[2]["y"])
    for b in (0, 1, 3):
        assert np.array_equal(pre2[b]["y"], pre[b]["y"])


def test_prefill_then_decode_equals_longer_prefill(rng):
    cfg = small_cfg()
    lay = O.Layer(cfg, small_weights(cfg, rng))
    L = 6
    x = rng.standard_normal((L + 2, cfg["d_model"]))
    full = lay.prefill_block(x, pos0=3)
    part = lay.prefill_block(x[:L], pos0=3)
    s1 = lay.decode_block(x[L], part["K"], part["V"], pos0=3)
    s2 = lay.decode_block(x[L + 1], s1["K"], s1["V"], pos0=3)
    np.testing.assert_allclose(s1["y"], full["y"][L], atol=1e-12)
    np.testing.assert_allclose(s2["y"], full["y"][L + 1], atol=1e-12)
    np.testing.assert_allclose(s2["K"], full["K"], atol=1e-13)
    np.testing.assert_allclose(s2["V"], full["V"], atol=1e-13)


def test_causality(rng):
    cfg = small_cfg()
    lay = O.Layer(cfg, small_weights(cfg, rng))
    x = rng.standard_normal((8, cfg["d_model"]))
    y = lay.prefill_block(x)["y"]
    x2 = x.copy()
    x2[5] += 1.0
    y2 = lay.prefill_block(x2)["y"]
    assert np.array_equal(y2[:5], y[:5])
    assert np.all(np.max(np.abs(y2[5:] - y[5:]), axis=-1) > 1e-6)


def test_row_subset_equals_full(rng):
    cfg = small_cfg()
    lay = O.Layer(cfg, small_weights(cfg, rng))
    x = rng.standard_normal((10, cfg["d_model"]))
    full = lay.prefill_block(x)
    sub = lay.prefill_block(x, rows=[0, 4, 9])
    np.testing.assert_allclose(sub["y"], full["y"][[0, 4, 9]], atol=1e-13)
    assert np.array_equal(sub["K"], full["K"])


def test_gqa_equals_mha_with_duplicated_kv_weights(rng):
    cfg = small_cfg()                                   # 4 q heads on 2 kv heads
    w = small_weights(cfg, rng)
    hd, Dq, Dkv = cfg["head_dim"], 32, 16
    mha = small_cfg(n_kv_heads=4)
    w2 = dict(w)
    wq, wk, wv = w["w_qkv"][:Dq], w["w_qkv"][Dq:Dq + Dkv], w["w_qkv"][Dq + Dkv:]
    dup = lambda m: np.repeat(m.reshape(2, hd, -1), 2, axis=0).reshape(4 * hd, -1)
    w2["w_qkv"] = np.concatenate([wq, dup(wk), dup(wv)])
    x = rng.standard_normal((7, cfg["d_model"]))
    np.testing.assert_allclose(O.Layer(cfg, w).prefill_block(x)["y"],
                               O.Layer(mha, w2).prefill_block(x)["y"], atol=1e-12)


@pytest.mark.parametrize("theta", [10000.0, 500000.0])
def test_whole_layer_against_library_routines(rng, theta):
    """Independent composition of the same layer from torch fp64 CPU routines
    (rms_norm, linear, scaled_dot_product_attention with grouped KV, silu); the
    rotary step is restated with complex numbers.  Pins the residual structure,
    the order of the two norms, the QKV row split and the head grouping."""
    cfg = small_cfg(rope_theta=theta)
    w = small_weights(cfg, rng)
    L, d, Hq, Hkv, hd, F = 9, 32, 4, 2, 8, 48
    x = rng.standard_normal((L, d))
    got = O.Layer(cfg, w).prefill_block(x, pos0=2)["y"]

    tw = {k: torch.from_numpy(np.asarray(v)) for k, v in w.items()}
    tx = torch.from_numpy(x)
    TF = torch.nn.functional
    n = TF.rms_norm(tx, (d,), tw["g_attn"], 1e-5)
    qkv = TF.linear(n, tw["w_qkv"])
    q, k, v = qkv.split([Hq * hd, Hkv * hd, Hkv * hd], dim=-1)

    def rot(t, H):
        t = t.reshape(L, H, hd)
        z = torch.complex(t[..., :hd // 2], t[..., hd // 2:])
        ang = (torch.arange(L, dtype=torch.float64) + 2)[:, None] * \
            theta ** (-torch.arange(hd // 2, dtype=torch.float64) / (hd // 2))
        z = z * torch.polar(torch.ones_like(ang), ang)[:, None, :]
        return torch.cat([z.real, z.imag], -1)

    q, k, v = rot(q, Hq), rot(k, Hkv), v.reshape(L, Hkv, hd)
    o = TF.scaled_dot_product_attention(q.permute(1, 0, 2)[None], k.permute(1, 0, 2)[None],
                                        v.permute(1, 0, 2)[None], is_causal=True, enable_gqa=True)
    o = o[0].permute(1, 0, 2).reshape(L, Hq * hd)
    h = tx + TF.linear(o, tw["w_o"])
    m = TF.rms_norm(h, (d,), tw["g_ffn"], 1e-5)
    gu = TF.linear(m, tw["w_gate_up"])
    y = h + TF.linear(TF.silu(gu[:, :F]) * gu[:, F:], tw["w_down"])
    np.testing.assert_allclose(got, y.numpy(), atol=1e-11)


@pytest.mark.parametrize("moe", [False, True])
def test_sampled_forward_equals_full_forward(rng, moe):
    cfg = small_cfg(n_experts=4, top_k=2) if moe else small_cfg()
    lay = O.Layer(cfg, small_weights(cfg, rng))
    lens = [6, 2, 9]
    cu = np.concatenate([[0], np.cumsum(lens)])
    x = rng.standard_normal((cu[-1], cfg["d_model"]))
    xd = rng.standard_normal((5, 3, cfg["d_model"]))
    pos = [0, 11, 3]
    pre, yd, Ks, Vs, routes = lay.forward(x, cu, xd, pos_offset=pos)
    rows = [[0, 5], [1], [3, 8]]
    spre, syd, sK, sV, sroutes = lay.forward_sampled(x, cu, xd, rows, steps=[0, 3, 4], pos_offset=pos)
    for b in range(3):
        np.testing.assert_allclose(spre[b]["y"], pre[b]["y"][rows[b]], atol=1e-12)
        np.testing.assert_allclose(sK[b], Ks[b], atol=1e-13)
        np.testing.assert_allclose(sV[b], Vs[b], atol=1e-13)
    for s in (0, 3, 4):
        np.testing.assert_allclose(syd[s], yd[s], atol=1e-12)
        if moe:
            for b in range(3):
                assert np.array_equal(sroutes[s][0][b], routes[s][b][0])


def test_linear_is_x_times_w_transposed(rng):
    x = rng.standard_normal((3, 5))
    w = rng.standard_normal((4, 5))
    want = np.array([[sum(x[i, k] * w[j, k] for k in range(5)) for j in range(4)] for i in range(3)])
    np.testing.assert_allclose(O.linear(x, w), want, atol=1e-14)


# ---------------------------------------------------------------------------
# prefix-aware layout (paper Sec. IV, Dispatch: worker k's prompt is blocks 1..k)
# ---------------------------------------------------------------------------
def _small_layer(rng, moe=False):
    cfg = dict(d_model=64, n_q_heads=4, n_kv_heads=2, head_dim=16, ffn_dim=96, n_experts=8 if moe else 0,
               top_k=2 if moe else 0, rms_eps=1e-5, rope_theta=10000.0)
    d, Dq, Dkv, F = 64, 64, 32, 96
    w = dict(g_attn=1 + 0.1 * rng.standard_normal(d), g_ffn=1 + 0.1 * rng.standard_normal(d),
             w_qkv=0.2 * rng.standard_normal((Dq + 2 * Dkv, d)), w_o=0.2 * rng.standard_normal((d, Dq)))
    if moe:
        w.update(w_router=rng.standard_normal((8, d)), w_exp_gate_up=0.2 * rng.standard_normal((8, 2 * F, d)),
                 w_exp_down=0.2 * rng.standard_normal((8, d, F)))
    else:
        w.update(w_gate_up=0.2 * rng.standard_normal((2 * F, d)), w_down=0.2 * rng.standard_normal((d, F)))
    return O.Layer(cfg, w)


@pytest.mark.parametrize("moe", [False, True])
def test_prefix_aware_worker_equals_a_lone_run_on_its_truncated_history(rng, moe):
    """Worker k of the prefix-aware layout sees blocks 1..k and nothing else: its
    decode outputs must equal those of an ordinary single-block run whose block is
    the history cut after block k (a different code path: one private cache)."""
    lay = _small_layer(rng, moe)
    lens = [5, 9, 3, 7]
    cu = np.concatenate([[0], np.cumsum(lens)])
    x = rng.standard_normal((cu[-1], 64))
    xd = rng.standard_normal((4, len(lens), 64))
    pre, yd, Kt, Vt = lay.forward_prefix(x, cu, xd)
    for b in range(len(lens)):
        T_b = int(cu[b + 1])
        pre1, yd1, Ks1, Vs1, _ = lay.forward(x[:T_b], [0, T_b], xd[:, b:b + 1])
        np.testing.assert_allclose(yd[:, b], yd1[:, 0], rtol=1e-10, atol=1e-12)
        np.testing.assert_allclose(Kt[b], Ks1[0][T_b:], rtol=1e-10, atol=1e-12)
        np.testing.assert_allclose(Vt[b], Vs1[0][T_b:], rtol=1e-10, atol=1e-12)
        # the shared cache rows of the worker's prefix are those of the lone run too
        np.testing.assert_allclose(pre["K"][:T_b], pre1[0]["K"], rtol=1e-10, atol=1e-12)


def test_prefix_aware_worker_ignores_the_history_after_its_block(rng):
    lay = _small_layer(rng)
    lens = [6, 4, 8]
    cu = np.concatenate([[0], np.cumsum(lens)])
    x = rng.standard_normal((cu[-1], 64))
    xd = rng.standard_normal((3, 3, 64))
    _, yd, _, _ = lay.forward_prefix(x, cu, xd)
    x2 = x.copy()
    x2[cu[2]:] += 3.0                      # perturb block 3 only
    _, yd2, _, _ = lay.forward_prefix(x2, cu, xd)
    np.testing.assert_array_equal(yd[:, :2], yd2[:, :2])
    assert np.abs(yd[:, 2] - yd2[:, 2]).max() > 1e-3


def test_prefix_aware_identical_keys_give_the_mean_over_prefix_and_tail(rng):
    """Zero query weights: every score is 0, so the attention output is the plain mean
    of the values over the worker's prefix rows and its tail rows (the new token
    included) -- checks which rows a worker sees."""
    lay = _small_layer(rng)
    lay.w["w_qkv"][:lay.Dq] = 0.0
    lens = [4, 6]
    cu = np.concatenate([[0], np.cumsum(lens)])
    x = rng.standard_normal((cu[-1], 64))
    xd = rng.standard_normal((2, 2, 64))
    pre, yd, Kt, Vt = lay.forward_prefix(x, cu, xd)
    for b in range(2):
        V = np.concatenate([pre["V"][:cu[b + 1]], Vt[b]], axis=0)          # [rows, Hkv, hd]
        mean_v = V.mean(axis=0)                                             # after both steps
        o = np.repeat(mean_v, lay.Hq // lay.Hkv, axis=0).reshape(-1)
        h = xd[1, b] + o @ lay.w["w_o"].T
        y, _, _, _ = lay.ffn(h[None])
        np.testing.assert_allclose(yd[1, b], y[0], rtol=1e-10, atol=1e-12)


# ---------------------------------------------------------------------------
# a depth of layers (the full stack the workers run, paper Sec. IV-A models)
# ---------------------------------------------------------------------------
def _torch_layer(tx, tw, theta, Hq, Hkv, hd, F, d):
    """One dense layer over ONE block from torch fp64 library routines (independent of the oracle's code)."""
    TF = torch.nn.functional
    L = tx.shape[0]
    n = TF.rms_norm(tx, (d,), tw["g_attn"], 1e-5)
    q, k, v = TF.linear(n, tw["w_qkv"]).split([Hq * hd, Hkv * hd, Hkv * hd], dim=-1)

    def rot(t, H):
        t = t.reshape(L, H, hd)
        z = torch.complex(t[..., :hd // 2], t[..., hd // 2:])
        ang = torch.arange(L, dtype=torch.float64)[:, None] * theta ** (-torch.arange(hd // 2, dtype=torch.float64) / (hd // 2))
        z = z * torch.polar(torch.ones_like(ang), ang)[:, None, :]
        return torch.cat([z.real, z.imag], -1)

    q, k, v = rot(q, Hq), rot(k, Hkv), v.reshape(L, Hkv, hd)
    o = TF.scaled_dot_product_attention(q.permute(1, 0, 2)[None], k.permute(1, 0, 2)[None], v.permute(1, 0, 2)[None],
                                        is_causal=True, enable_gqa=True)[0].permute(1, 0, 2).reshape(L, Hq * hd)
    h = tx + TF.linear(o, tw["w_o"])
    gu = TF.linear(TF.rms_norm(h, (d,), tw["g_ffn"], 1e-5), tw["w_gate_up"])
    return h + TF.linear(TF.silu(gu[:, :F]) * gu[:, F:], tw["w_down"]), k, v


def test_stack_prefill_equals_library_layers_applied_in_turn(rng):
    """Three different layers: the stack's last-layer output and the K rows cached by
    the LAST layer equal torch fp64 layers applied one after the other to each block
    (a wrong hand-over between layers, or one layer's cache filed under another, fails)."""
    cfg = small_cfg()
    ws = [small_weights(cfg, rng) for _ in range(3)]
    lens = [7, 4]
    cu = [0, 7, 11]
    x = rng.standard_normal((11, 32))
    y_pre, _, Ks, Vs = O.Stack(cfg, ws).forward(x, cu, None)
    for b in range(2):
        t = torch.from_numpy(x[cu[b]:cu[b + 1]])
        for li, w in enumerate(ws):
            tw = {k: torch.from_numpy(np.asarray(v)) for k, v in w.items()}
            t, k, v = _torch_layer(t, tw, cfg["rope_theta"], 4, 2, 8, 48, 32)
            np.testing.assert_allclose(Ks[li][b], k.numpy(), atol=1e-10)
            np.testing.assert_allclose(Vs[li][b], v.numpy(), atol=1e-10)
        np.testing.assert_allclose(y_pre[cu[b]:cu[b + 1]], t.numpy(), atol=1e-10)


def test_stack_of_one_layer_is_the_layer(rng):
    cfg = small_cfg()
    w = small_weights(cfg, rng)
    cu = [0, 5, 8]
    x = rng.standard_normal((8, 32))
    xd = rng.standard_normal((3, 2, 32))
    pre, yd, Ks, Vs, _ = O.Layer(cfg, w).forward(x, cu, xd)
    y_pre, yd2, Ks2, Vs2 = O.Stack(cfg, [w]).forward(x, cu, xd)
    np.testing.assert_array_equal(np.concatenate([p["y"] for p in pre]), y_pre)
    np.testing.assert_array_equal(yd, yd2)
    np.testing.assert_array_equal(Ks[1], Ks2[0][1])


def test_stack_skips_an_identity_layer(rng):
    """A layer whose output and down projections are zero adds nothing to the residual
    stream: inserting it anywhere leaves every other layer's outputs and caches alone,
    in prefill and in decode."""
    cfg = small_cfg()
    wa, wb = small_weights(cfg, rng), small_weights(cfg, rng)
    wi = small_weights(cfg, rng)
    wi["w_o"] = np.zeros_like(wi["w_o"])
    wi["w_down"] = np.zeros_like(wi["w_down"])
    cu = [0, 6, 9]
    x = rng.standard_normal((9, 32))
    xd = rng.standard_normal((2, 2, 32))
    y2, yd2, K2, V2 = O.Stack(cfg, [wa, wb]).forward(x, cu, xd)
    y3, yd3, K3, V3 = O.Stack(cfg, [wa, wi, wb]).forward(x, cu, xd)
    np.testing.assert_allclose(y3, y2, atol=1e-12)
    np.testing.assert_allclose(yd3, yd2, atol=1e-12)
    for b in range(2):
        np.testing.assert_allclose(K3[2][b], K2[1][b], atol=1e-12)
        np.testing.assert_allclose(V3[0][b], V2[0][b], atol=1e-12)
        assert K3[1][b].shape[0] == K2[1][b].shape[0]   # the identity layer caches every row too


def test_stack_decode_equals_a_longer_prefill(rng):
    """Feeding a block's next token as a decode step through the whole depth gives the
    last row of a prefill over the block with that token appended (every layer's cache
    must take the row its own predecessor produced)."""
    cfg = small_cfg()
    ws = [small_weights(cfg, rng) for _ in range(3)]
    x = rng.standard_normal((8, 32))
    st = O.Stack(cfg, ws)
    y_full, _, K_full, _ = st.forward(x, [0, 8], None)
    _, yd, K_inc, _ = st.forward(x[:6], [0, 6], x[6:8].reshape(2, 1, 32))
    np.testing.assert_allclose(yd[:, 0], y_full[6:8], atol=1e-11)
    for li in range(3):
        np.testing.assert_allclose(K_inc[li][0], K_full[li][0], atol=1e-11)


def test_stack_batched_equals_one_block_at_a_time(rng):
    cfg = small_cfg()
    ws = [small_weights(cfg, rng) for _ in range(2)]
    cu = [0, 4, 9, 12]
    x = rng.standard_normal((12, 32))
    xd = rng.standard_normal((2, 3, 32))
    st = O.Stack(cfg, ws)
    y, yd, _, _ = st.forward(x, cu, xd)
    for b in range(3):
        y1, yd1, _, _ = st.forward(x[cu[b]:cu[b + 1]], [0, cu[b + 1] - cu[b]], xd[:, b:b + 1])
        np.testing.assert_array_equal(y[cu[b]:cu[b + 1]], y1)
        np.testing.assert_array_equal(yd[:, b], yd1[:, 0])


# ---------------------------------------------------------------------------
# a prefill cut into chunks (paper Sec. IV-B: chunked prefill on the server)
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("moe", [False, True])
@pytest.mark.parametrize("cuts", [[4], [1, 5], [3, 3, 4], [10]])
def test_chunked_prefill_equals_the_prefill_in_one_piece(rng, moe, cuts):
    """Cutting a block's prefill into chunks that are appended one after another gives
    the outputs and the cache of the prefill in one piece (the full score matrix)."""
    lay = _small_layer(rng, moe)
    L = 11
    x = rng.standard_normal((L, 64))
    whole = lay.prefill_block(x, pos0=3)
    K = np.zeros((0, lay.Hkv, lay.hd))
    V = np.zeros((0, lay.Hkv, lay.hd))
    ys, a = [], 0
    for c in cuts + [L - sum(cuts)]:
        if c == 0:
            continue
        st = lay.extend_block(x[a:a + c], K, V, pos0=3)
        K, V = st["K"], st["V"]
        ys.append(st["y"])
        a += c
    np.testing.assert_allclose(np.concatenate(ys), whole["y"], rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(K, whole["K"], rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(V, whole["V"], rtol=1e-12, atol=1e-14)


def test_a_chunk_of_one_token_is_a_decode_step(rng):
    lay = _small_layer(rng)
    x = rng.standard_normal((7, 64))
    pre = lay.prefill_block(x[:6], pos0=2)
    a = lay.extend_block(x[6:7], pre["K"], pre["V"], pos0=2)
    b = lay.decode_block(x[6], pre["K"], pre["V"], pos0=2)
    np.testing.assert_array_equal(a["y"][0], b["y"])
    np.testing.assert_array_equal(a["K"], b["K"])


def test_chunk_rows_subset_and_causality_inside_a_chunk(rng):
    lay = _small_layer(rng)
    x = rng.standard_normal((9, 64))
    pre = lay.prefill_block(x[:4])
    full = lay.extend_block(x[4:], pre["K"], pre["V"])
    sub = lay.extend_block(x[4:], pre["K"], pre["V"], rows=[0, 3])
    np.testing.assert_array_equal(sub["y"], full["y"][[0, 3]])
    x2 = x.copy()
    x2[7] += 1.0                                  # chunk row 3
    pert = lay.extend_block(x2[4:], pre["K"], pre["V"])
    np.testing.assert_array_equal(pert["y"][:3], full["y"][:3])
    assert np.abs(pert["y"][3:] - full["y"][3:]).max() > 1e-4


# ---------------------------------------------------------------------------
# block-scaled 4-bit weights ("mxfp4 weights", paper Sec. IV-B; OCP MX v1.0)
# ---------------------------------------------------------------------------
def test_fp4_code_values_match_the_specification_table():
    from oracle import mxfp4 as Q
    rows = [ln.split() for ln in open(os.path.join(HERE, "golden", "fp4_e2m1_values.txt")) if ln.strip() and not ln.startswith("#")]
    assert len(rows) == 16
    for bits, val in rows:
        got = Q.e2m1_value(int(bits, 2))
        assert got == float(val) and np.signbit(got) == np.signbit(float(val)), bits


def test_e8m0_scales_are_powers_of_two():
    from oracle import mxfp4 as Q
    assert Q.e8m0_value(127) == 1.0 and Q.e8m0_value(126) == 0.5 and Q.e8m0_value(130) == 8.0
    assert Q.e8m0_value(0) == 2.0 ** -127 and Q.e8m0_value(254) == 2.0 ** 127
    with pytest.raises(ValueError):
        Q.e8m0_value(255)


def test_mxfp4_packing_order_and_block_scales_by_planting_single_codes():
    """One non-zero code at a time: element k must come out at index k, scaled by the
    scale byte of block k // 32 only."""
    from oracle import mxfp4 as Q
    K = 96
    for k in (0, 1, 2, 31, 32, 33, 63, 64, 95):
        codes = np.zeros((2, K // 2), dtype=np.uint8)
        scales = np.full((2, K // 32), 127, dtype=np.uint8)
        codes[1, k // 2] = 0x7 << (4 * (k % 2))          # +6.0 at element k of row 1
        scales[1, k // 32] = 125                         # x 1/4 for that block only
        scales[0, k // 32] = 140                         # another row's scale must not matter
        w = Q.dequantize(codes, scales)
        expect = np.zeros((2, K))
        expect[1, k] = 1.5
        np.testing.assert_array_equal(w, expect)


def test_mxfp4_dequantize_is_exact_on_representable_matrices(rng):
    """Build a matrix from values of the form (+-){0,.5,1,1.5,2,3,4,6} * 2^s per block of 32, encode it by
    searching the sixteen codes (brute force), and get the same matrix back."""
    from oracle import mxfp4 as Q
    vals = np.array([0, .5, 1, 1.5, 2, 3, 4, 6])
    R, K = 5, 128
    mag = rng.integers(0, 8, size=(R, K))
    sgn = rng.integers(0, 2, size=(R, K))
    exps = rng.integers(-12, 5, size=(R, K // 32))
    w = np.where(sgn == 1, -1.0, 1.0) * vals[mag] * np.repeat(2.0 ** exps, 32, axis=1)
    codes = np.zeros((R, K // 2), dtype=np.uint8)
    for r in range(R):
        for k in range(K):
            target = w[r, k] / 2.0 ** exps[r, k // 32]
            c = [c for c in range(16) if Q.e2m1_value(c) == target and np.signbit(Q.e2m1_value(c)) == (sgn[r, k] == 1)][0]
            codes[r, k // 2] |= c << (4 * (k % 2))
    scales = (exps + 127).astype(np.uint8)
    np.testing.assert_array_equal(Q.dequantize(codes, scales), w)


def test_stack_prefix_aware_worker_equals_a_lone_stack_run_on_its_truncated_history(rng):
    """Through the whole depth, worker k of the prefix-aware layout equals an ordinary
    single-block stack run on the history cut after block k (a different code path:
    private caches per layer, no shared cache)."""
    cfg = small_cfg()
    ws = [small_weights(cfg, rng) for _ in range(3)]
    st = O.Stack(cfg, ws)
    lens = [5, 3, 6]
    cu = np.concatenate([[0], np.cumsum(lens)])
    x = rng.standard_normal((cu[-1], 32))
    xd = rng.standard_normal((3, 3, 32))
    yd, shared, Kt, Vt = st.forward_prefix(x, cu, xd)
    for b in range(3):
        T_b = int(cu[b + 1])
        _, yd1, Ks1, Vs1 = st.forward(x[:T_b], [0, T_b], xd[:, b:b + 1])
        np.testing.assert_allclose(yd[:, b], yd1[:, 0], rtol=1e-10, atol=1e-12)
        for li in range(3):
            np.testing.assert_allclose(Kt[li][b], Ks1[li][0][T_b:], rtol=1e-10, atol=1e-12)
            np.testing.assert_allclose(shared[li][0][:T_b], Ks1[li][0][:T_b], rtol=1e-10, atol=1e-12)
