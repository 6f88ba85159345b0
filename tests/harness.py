"""Runs the HIP library and the fp64 checker on the same seeded inputs.
Used by the GPU parity tests, the smoke check and the benchmark's baseline leg.
No layer arithmetic lives here."""
import numpy as np
import torch

from oracle import layer as O
from paper_2605_23296_amd import binding as B
from paper_2605_23296_amd.workloads import to_numpy_f64


def oracle_layer(inp):
    w = {k: to_numpy_f64(v) for k, v in inp.weights.items()}
    return O.Layer(inp.layer.as_dict(), w)


def gpu_layer(inp, device="cuda"):
    w = {k: v.to(device).contiguous() for k, v in inp.weights.items()}
    return B.Layer(inp.layer, w)


def gpu_forward(inp, lay=None, device="cuda", extra_capacity=0, pos_offset=None, want_prefill=True):
    """compact_layer_forward on the whole workload.  Returns numpy float64 views
    of y_prefill [T,d], y_last [N,d], y_decode [S,N,d], and per-block K, V."""
    lay = lay or gpu_layer(inp, device)
    layer = inp.layer
    dt = lay.torch_dtype
    N, S, T = len(inp.block_lens), inp.x_decode.shape[0], inp.cu_seqlens[-1]
    kv = B.KVCache(layer, [L + S + extra_capacity for L in inp.block_lens], device, dt, pos_offset)
    lay.ensure_workspace(T, N, max(inp.block_lens) + S, device)
    x = inp.x_prefill.to(device)
    xd = inp.x_decode.to(device).contiguous()
    y_pre = torch.empty(T, layer.d_model, dtype=dt, device=device) if want_prefill else None
    y_last = torch.empty(N, layer.d_model, dtype=dt, device=device)
    y_dec = torch.empty(S, N, layer.d_model, dtype=dt, device=device)
    lay.compact_layer_forward(inp.cu_seqlens, x, xd if S > 0 else None, kv, y_pre, y_last, y_dec if S > 0 else None)
    torch.cuda.synchronize()
    out = dict(y_last=to_numpy_f64(y_last), y_decode=to_numpy_f64(y_dec),
               K=[to_numpy_f64(kv.block_k(b)) for b in range(N)],
               V=[to_numpy_f64(kv.block_v(b)) for b in range(N)], lens=kv.lens(), kv=kv, lay=lay)
    if want_prefill:
        out["y_prefill"] = to_numpy_f64(y_pre)
    return out


def oracle_forward(inp, rows=None, pos_offset=None):
    lay = oracle_layer(inp)
    x = to_numpy_f64(inp.x_prefill)
    xd = to_numpy_f64(inp.x_decode)
    pre, y_dec, Ks, Vs, routes = lay.forward(x, inp.cu_seqlens, xd, pos_offset=pos_offset, rows=rows)
    return dict(pre=pre, y_decode=y_dec, K=Ks, V=Vs, routes=routes)


def gpu_forward_steps(inp, device="cuda", pos_offset=None):
    """The same pass through compact_prefill + compact_decode_step, capturing
    the routing tables of MoE layers."""
    lay = gpu_layer(inp, device)
    layer = inp.layer
    dt = lay.torch_dtype
    N, S, T = len(inp.block_lens), inp.x_decode.shape[0], inp.cu_seqlens[-1]
    moe = layer.n_experts > 0
    kv = B.KVCache(layer, [L + S for L in inp.block_lens], device, dt, pos_offset)
    lay.ensure_workspace(T, N, max(inp.block_lens) + S, device)
    x = inp.x_prefill.to(device)
    y_pre = torch.empty(T, layer.d_model, dtype=dt, device=device)
    route = None
    if moe:
        route = (torch.empty(T, layer.top_k, dtype=torch.int32, device=device),
                 torch.empty(T, layer.top_k, dtype=torch.float32, device=device))
    lay.compact_prefill(inp.cu_seqlens, x, kv, y_pre, route)
    y_dec = torch.empty(S, N, layer.d_model, dtype=dt, device=device)
    droutes = []
    for s in range(S):
        r = None
        if moe:
            r = (torch.empty(N, layer.top_k, dtype=torch.int32, device=device),
                 torch.empty(N, layer.top_k, dtype=torch.float32, device=device))
            droutes.append(r)
        lay.compact_decode_step(inp.x_decode[s].to(device).contiguous(), kv, y_dec[s], r)
    torch.cuda.synchronize()
    out = dict(y_prefill=to_numpy_f64(y_pre), y_decode=to_numpy_f64(y_dec),
               K=[to_numpy_f64(kv.block_k(b)) for b in range(N)],
               V=[to_numpy_f64(kv.block_v(b)) for b in range(N)], lens=kv.lens())
    if moe:
        out["idx_prefill"] = route[0].cpu().numpy()
        out["gate_prefill"] = route[1].cpu().numpy()
        out["idx_decode"] = [r[0].cpu().numpy() for r in droutes]
        out["gate_decode"] = [r[1].cpu().numpy() for r in droutes]
    return out


def check_routing(idx_gpu, logits_ref, k, margin_rel, gate_gpu=None):
    """Checks the routing table of a routed layer against the checker's logits, row by row.

    The GPU routes from its own (storage-rounded) activations, the checker from
    unrounded fp64 ones, so two experts whose logits are closer than `margin`
    (margin_rel * max|logit|: a bound on that rounding noise) may legitimately
    swap.  Hence, per row:
      * the GPU's k experts are distinct and each one's checker logit is within
        margin of the checker's k-th largest (a valid choice);
      * if the k-th and (k+1)-th logits are further apart than margin, the
        expert SET is the checker's;
      * if moreover all gaps inside the top k exceed margin, the ORDER is too;
      * the gates are the softmax over the chosen logits (within margin).
    Returns the number of rows whose set was not forced by the margin.  Values
    are compared afterwards for EVERY row, with the checker's feed-forward
    evaluated for the GPU's (validated) choice."""
    idx_gpu = np.asarray(idx_gpu).reshape(-1, k)
    logits_ref = np.asarray(logits_ref).reshape(idx_gpu.shape[0], -1)
    order = np.argsort(-logits_ref, axis=-1, kind="stable")
    srt = np.take_along_axis(logits_ref, order, axis=-1)
    if srt.shape[1] == k:       # every expert is chosen: no runner-up
        srt = np.concatenate([srt, np.full((srt.shape[0], 1), -np.inf)], axis=1)
    margin = margin_rel * np.abs(logits_ref).max()
    gaps = srt[:, :k] - srt[:, 1:k + 1]                    # gap j: between the j-th and (j+1)-th largest
    set_safe = gaps[:, k - 1] > margin
    order_safe = np.all(gaps > margin, axis=1)
    chosen = np.take_along_axis(logits_ref, idx_gpu.astype(np.int64), axis=-1)
    for r in range(idx_gpu.shape[0]):
        assert len(set(idx_gpu[r].tolist())) == k, ("repeated expert", r, idx_gpu[r])
        assert np.all((idx_gpu[r] >= 0) & (idx_gpu[r] < logits_ref.shape[1]))
        assert np.all(chosen[r] >= srt[r, k - 1] - margin), ("expert outside the margin", r, idx_gpu[r], order[r, :k + 1])
        if set_safe[r]:
            assert set(idx_gpu[r].tolist()) == set(order[r, :k].tolist()), ("expert set", r, idx_gpu[r], order[r, :k])
        if order_safe[r]:
            assert np.array_equal(idx_gpu[r], order[r, :k]), ("expert order", r, idx_gpu[r], order[r, :k])
    if gate_gpu is not None:
        e = np.exp(chosen - chosen.max(-1, keepdims=True))
        want = e / e.sum(-1, keepdims=True)
        got = np.asarray(gate_gpu, dtype=np.float64).reshape(want.shape)
        assert np.abs(got.sum(-1) - 1).max() < 1e-5
        assert np.abs(got - want).max() <= max(margin, 1e-6), np.abs(got - want).max()
    return int(np.sum(~set_safe))


def routing_candidates(logits_row, k, margin):
    """Every expert set that is a valid top-k choice for one row when logits closer than
    margin may swap: the experts clearly above the k-th logit, completed by every
    combination of those within margin of it.  For entry points that do not report
    their routing tables."""
    import itertools
    order = np.argsort(-logits_row, kind="stable")
    kth = logits_row[order[k - 1]]
    sure = [int(e) for e in order if logits_row[e] > kth + margin]
    maybe = [int(e) for e in order if abs(logits_row[e] - kth) <= margin]
    return [sure + list(c) for c in itertools.combinations(maybe, k - len(sure))]
