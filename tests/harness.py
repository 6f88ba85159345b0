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
