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
    return out


def routed_rows_match(idx_gpu, idx_ref, logits_ref, k, margin_rel):
    """Which rows can be compared value by value in a routed layer.

    The GPU routes from its own (storage-rounded) activations, the checker from
    unrounded fp64 ones, so calls closer than the rounding noise may
    legitimately differ.  A row is `safe` when the checker's k-th and (k+1)-th
    logits are further apart than margin; there the expert SETS must agree.
    On the other rows every expert the GPU picked must lie within margin of
    the checker's k-th logit.  Returns (safe mask, n_rows_not_safe)."""
    srt = -np.sort(-logits_ref, axis=-1)
    margin = margin_rel * np.abs(logits_ref).max()
    safe = (srt[:, k - 1] - srt[:, k]) > margin
    same = np.array([set(a) == set(b) for a, b in zip(idx_gpu, idx_ref)])
    assert np.all(same[safe]), "expert sets differ on rows with a clear margin"
    for r in np.nonzero(~safe)[0]:
        assert len(set(idx_gpu[r])) == k
        assert np.all(logits_ref[r, idx_gpu[r]] >= srt[r, k - 1] - margin)
    return safe & same, int(np.sum(~safe))
