#!/usr/bin/env python3
"""Benchmark of the batched block-compaction layer on one MI355X.

One "step" = one whole compaction pass of one layer over one batch of blocks:
varlen prefill of every block, then S batched decode steps (compact_layer_forward).
Workload = the dense 8B-shaped bf16 layer, a 32 k-token history cut into 8 blocks
of 4096 tokens, 256 decoded tokens per block (synthetic seeded Gaussians).

Prints ONE JSON line.  `value` is the compaction throughput in the paper's sense
(Sec. V: decode tokens produced per second of compaction time, prefill
included); prefill and decode rates are reported beside it, as are the
per-kernel-class times, the roofline figure of the dominant kernel, the
one-block-at-a-time run and the CPU checker timed on the host cores.
"""
import argparse
import json
import os
import sys
import time

import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from paper_2605_23296_amd import binding as B                       # noqa: E402
from paper_2605_23296_amd.workloads import WORKLOADS, make_inputs, make_mxfp4_experts, make_stack_weights  # noqa: E402

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E
SEQ_REPS = 3                # timed repetitions of every one-block pass of the sequential leg


def event_pair_overhead_us(n=200):
    """What a pair of HIP events on the launch stream reads with nothing between them (median of n): the part of a
    per-launch bracket that is not kernel time.  Reported beside the per-launch figures; never subtracted from them."""
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
    torch.cuda.synchronize()
    for a, b in ev:
        a.record()
        b.record()
    torch.cuda.synchronize()
    us = sorted(a.elapsed_time(b) * 1e3 for a, b in ev)
    return us[len(us) // 2]


def layer_params(layer):
    d, F = layer.d_model, layer.ffn_dim
    attn = (layer.Dq + 2 * layer.Dkv) * d + d * layer.Dq
    if layer.n_experts == 0:
        return attn + 3 * F * d
    return attn + layer.n_experts * d + layer.top_k * 3 * F * d      # parameters touched per token


def algorithmic_work(layer, lens, S, distinct_experts_per_step=None, expert_bits=16.0):
    """Work the method must do, per pass (each weight once per call, the causal
    half of attention, each cached KV byte once per decode step).  For a routed
    layer a decode step must read the weights of every expert that some row of
    the step was routed to, once: distinct_experts_per_step (measured on the
    same inputs) gives their number per step."""
    T, N = sum(lens), len(lens)
    P = layer_params(layer)
    w = {}
    w["gemm_flops"] = 2.0 * P * T
    w["attn_prefill_flops"] = sum(L * (L + 1) / 2 for L in lens) * 4.0 * layer.head_dim * layer.n_q_heads
    kv_tok = 2 * layer.Dkv * 2                                       # bytes per cached token (K and V, bf16)
    w["attn_decode_bytes"] = float(sum(sum((L + s + 1) * kv_tok for L in lens) for s in range(S)))
    if layer.n_experts == 0:
        w["skinny_bytes"] = float(S) * P * 2                         # every weight once per step
    else:
        d, F = layer.d_model, layer.ffn_dim
        attn = (layer.Dq + 2 * layer.Dkv) * d + d * layer.Dq
        experts = sum(distinct_experts_per_step) if distinct_experts_per_step else S * min(layer.n_experts, N * layer.top_k)
        # the router (E x d) runs through the prefill-size GEMM class and is not counted here
        w["skinny_bytes"] = 2.0 * S * attn + experts * 3 * F * d * expert_bits / 8.0
    return w


def distinct_experts(lay, inp, kv, bufs):
    """Experts touched by each decode step of a routed layer (one untimed pass
    through compact_prefill + compact_decode_step with the routing read back)."""
    layer, dev = inp.layer, bufs["x"].device
    N, S, T = len(inp.block_lens), inp.x_decode.shape[0], inp.cu_seqlens[-1]
    lay.compact_prefill(inp.cu_seqlens, bufs["x"], kv, bufs["y_pre"])
    idx = torch.empty(S, N, layer.top_k, dtype=torch.int32, device=dev)
    gate = torch.empty(S, N, layer.top_k, dtype=torch.float32, device=dev)
    for s in range(S):
        lay.compact_decode_step(bufs["xd"][s], kv, bufs["y_dec"][s], (idx[s], gate[s]))
    torch.cuda.synchronize()
    return [int(torch.unique(idx[s]).numel()) for s in range(S)]


def recorded_traffic(workload, kernel_class):
    """HBM bytes per launch from the committed rocprofv3 counter summary, or None
    when there is none for this kernel class or its source changed since."""
    import hashlib
    path = os.path.join(ROOT, "profiles", "hbm_traffic_%s.json" % workload)
    try:
        rec = json.load(open(path))
        if rec.get("kernel_class") != kernel_class:
            return None
        blob = b"".join(open(os.path.join(ROOT, f), "rb").read() for f in rec["sources"])
        if hashlib.sha256(blob).hexdigest() != rec["sources_sha256"]:
            return None
        return rec["traffic_bytes_per_launch"]
    except (OSError, ValueError, KeyError):
        return None


def run_pass(lay, inp, kv, bufs, n_steps=None):
    S = inp.x_decode.shape[0] if n_steps is None else n_steps
    lay.compact_layer_forward(inp.cu_seqlens, bufs["x"], bufs["xd"][:S] if S > 0 else None, kv,
                              bufs["y_pre"], bufs["y_last"], bufs["y_dec"] if S > 0 else None)


def timed(fn, reps):
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / reps


def cpu_baseline(inp, n_blocks=2, n_dec=32):
    """The fp64 checker as it stands, on the host cores: prefill of n_blocks whole blocks
    (the first and the last) and n_dec decode steps of each, extrapolated linearly over the
    independent blocks and steps (exact in work, not in cache behaviour)."""
    import numpy as np
    from oracle import layer as O
    from paper_2605_23296_amd.workloads import to_numpy_f64
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    w = {}
    for k, v in inp.weights.items():
        if k.endswith(("_q", "_s")):
            continue
        w[k] = to_numpy_f64(v)
    lay = O.Layer(inp.layer.as_dict(), w)
    N, S = len(inp.block_lens), inp.x_decode.shape[0]
    blocks = sorted(set([0, N - 1]))[:n_blocks]
    n_dec = min(n_dec, S)
    t_pre = t_dec = 0.0
    tok = 0
    for b in blocks:
        x = to_numpy_f64(inp.x_prefill[inp.cu_seqlens[b]:inp.cu_seqlens[b + 1]])
        t0 = time.perf_counter()
        pre = lay.prefill_block(x)
        t_pre += time.perf_counter() - t0
        tok += x.shape[0]
        K, V = pre["K"], pre["V"]
        xd = to_numpy_f64(inp.x_decode[:n_dec, b])
        t0 = time.perf_counter()
        for s in range(n_dec):
            st = lay.decode_block(xd[s], K, V)
            K, V = st["K"], st["V"]
        t_dec += time.perf_counter() - t0
    T = inp.cu_seqlens[-1]
    per_tok_pre, per_step = t_pre / tok, t_dec / max(n_dec * len(blocks), 1)
    total = T * per_tok_pre + N * S * per_step
    return {
        "value": N * S / total, "unit": "decode tokens/s (prefill time included)",
        "cores": int(cores), "kind": "oracle",
        "sample": "fp64 numpy checker: full prefill of %d of %d blocks (%d tokens, %.1f s) + %d of %d decode steps of each "
                  "(%.3f s/step); extrapolated linearly in prefill tokens and decode steps" % (len(blocks), N, tok, t_pre, n_dec, S, per_step),
        "prefill_tokens_per_s": 1.0 / per_tok_pre, "decode_tokens_per_s": 1.0 / per_step,
    }


def prefix_aware_pass(args, wl, inp, lay, bufs):
    """Prefix-aware layout: every layer prefills the whole history as ONE block into a shared cache, then S
    decode steps in which worker b attends the first cu[b+1] rows of that cache plus its own tail
    (compact_prefix_stack_forward; --stack L for a depth of L layers, else one layer).  Algorithmic KV bytes
    per step and layer: every shared row once (not once per worker) plus the tails.  With --stack the
    sequential baseline (one block, N * S decode tokens one after another) is timed beside it."""
    layer, dev = inp.layer, bufs["x"].device
    lens, S, N, T = inp.block_lens, inp.x_decode.shape[0], len(inp.block_lens), inp.cu_seqlens[-1]
    dt = lay.torch_dtype
    L = max(1, args.stack)
    weights = make_stack_weights(wl, L, device=dev, gen_device=dev) if args.stack > 0 else [inp.weights]
    shared = [B.KVCache(layer, [T], dev, dt) for _ in range(L)]
    need = lay.prefix_stack_workspace_bytes(T, N, S + 8)
    if args.stack > 0:
        need = max(need, lay.stack_workspace_bytes(T, 1, T + N * S))
    lay.ws = torch.empty(need, dtype=torch.uint8, device=dev)
    prefix = [int(c) for c in inp.cu_seqlens[1:]]

    def one_pass(n_steps):
        tails = [B.KVCache(layer, [S + 8] * N, dev, dt) for _ in range(L)]
        lay.compact_prefix_stack_forward(weights, prefix, bufs["x"], bufs["xd"][:n_steps] if n_steps else None, shared, tails,
                                         bufs["y_dec"] if n_steps else None)

    for _ in range(max(1, args.warmup)):
        one_pass(S)
    t_pass = timed(lambda: one_pass(S), args.steps)
    t_prefill = timed(lambda: one_pass(0), max(1, args.steps // 2))
    t_decode = max(t_pass - t_prefill, 1e-9)
    kv_tok = 2 * layer.Dkv * 2
    shared_once = float(L * sum((max(prefix) + N * (s + 1)) * kv_tok for s in range(S)))
    per_worker = float(L * sum((sum(prefix) + N * (s + 1)) * kv_tok for s in range(S)))
    lay.compact_profile_select(B.K_ATTN_DECODE)
    one_pass(S)
    torch.cuda.synchronize()
    n, ms = lay.compact_profile_read()
    lay.compact_profile_select(B.K_NONE)
    attn = dict(bound="hbm", launches_per_pass=n, avg_launch_us=ms * 1e3 / max(n, 1), achieved=shared_once / (ms / 1e3) / 1e9,
                peak=PEAK_HBM_GBS, unit="GB/s", frac=shared_once / (ms / 1e3) / 1e9 / PEAK_HBM_GBS,
                note="algorithmic bytes = every shared cache row once per step for all workers together + the tails; "
                     "reading each worker's prefix separately would move %.1fx as much" % (per_worker / shared_once))
    out = {
        "metric": "compaction_decode_tokens_per_s", "value": N * S / t_pass, "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": max(1, args.warmup), "ms_per_step": t_pass * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": layer.dtype, "data": "synthetic",
        "config": {"workload": "%s, prefix-aware target-at-end layout, %d layer(s): one %d-token prefill, %d workers with "
                               "prefixes %d..%d, %d decode steps each" % (wl.name, L, T, N, prefix[0], prefix[-1], S),
                   "total_prefill_tokens": T, "decode_tokens": N * S, "n_layers": L},
        "prefill_tokens_per_s": T / t_prefill, "decode_tokens_per_s": N * S / t_decode, "ms_prefill": t_prefill * 1e3,
        "ms_decode": t_decode * 1e3, "us_per_decode_step_per_layer": t_decode * 1e6 / max(S, 1) / L,
        "ms_per_decode_token": t_pass * 1e3 / (N * S),
        "roofline": dict(kernel="attn_decode_prefix", **attn), "kernels": {"attn_decode_prefix": attn},
    }
    if args.stack > 0:
        del shared
        Ls = args.seq_layers if args.seq_layers > 0 else L
        kv1 = [B.KVCache(layer, [T + N * S], dev, dt) for _ in range(Ls)]
        xd1 = bufs["xd"].reshape(S * N, 1, layer.d_model)
        yd1 = torch.empty_like(xd1)
        seq = lambda steps: lay.compact_stack_forward(weights[:Ls], [0, T], bufs["x"], xd1[:steps] if steps else None, kv1,
                                                      bufs["y_last"][:1], yd1 if steps else None)
        seq(8)
        t_seq = timed(lambda: seq(S * N), 1) * L / Ls
        t_seq_pre = timed(lambda: seq(0), 1) * L / Ls
        out["sequential_single_block"] = {
            "what": "the whole %d-token history as one block, the same %d decode tokens one after another" % (T, N * S),
            "layers_measured": Ls, "scaled_to_layers": L, "ms_per_step": t_seq * 1e3, "ms_prefill": t_seq_pre * 1e3,
            "ms_decode": (t_seq - t_seq_pre) * 1e3, "ms_per_decode_token": t_seq * 1e3 / (N * S),
            "parallel_speedup": t_seq / t_pass}
    return out


def mixed_pass(args, wl, inp, lay, kv, bufs):
    """The pass under a token budget per step (chunked prefill interleaved with decode) and, beside it,
    the plain pass (all prefill, then S batched steps) on the same inputs."""
    layer, dev = inp.layer, bufs["x"].device
    lens, S, N, T = inp.block_lens, inp.x_decode.shape[0], len(inp.block_lens), inp.cu_seqlens[-1]
    plain_ws = lay.ws
    for _ in range(max(1, args.warmup)):
        run_pass(lay, inp, kv, bufs)
    t_plain = timed(lambda: run_pass(lay, inp, kv, bufs), args.steps)
    need = lay.mixed_workspace_bytes(args.mixed, N, max(lens) + S)
    lay.ws = torch.empty(need, dtype=torch.uint8, device=dev)
    mixed = lambda: lay.compact_mixed_forward(inp.cu_seqlens, bufs["x"], bufs["xd"], kv, args.mixed, bufs["y_last"], bufs["y_dec"])
    for _ in range(max(1, args.warmup)):
        mixed()
    t_mixed = timed(mixed, args.steps)
    return {
        "metric": "compaction_decode_tokens_per_s", "value": N * S / t_mixed, "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": max(1, args.warmup), "ms_per_step": t_mixed * 1e3, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": layer.dtype, "data": "synthetic",
        "config": {"workload": "%s under a budget of %d rows per step (prefill chunks + decode tokens in one batch)"
                               % (wl.name, args.mixed), "total_prefill_tokens": T, "decode_tokens": N * S},
        "workspace_bytes": need,
        "plain_pass": {"ms_per_step": t_plain * 1e3, "value": N * S / t_plain, "workspace_bytes": plain_ws.numel(),
                       "mixed_over_plain_time": t_mixed / t_plain},
    }


def stack_pass(args, wl, inp, lay, bufs):
    """L layers deep: the parallel pass (N blocks, S batched steps) and the sequential
    baseline at matched decode volume (one block = the whole history, N * S steps)."""
    layer, dev, dt = inp.layer, bufs["x"].device, lay.torch_dtype
    lens, S, N, T = inp.block_lens, inp.x_decode.shape[0], len(inp.block_lens), inp.cu_seqlens[-1]
    L = args.stack
    weights = make_stack_weights(wl, L, device=dev, gen_device=dev)
    need = max(lay.stack_workspace_bytes(T, N, max(lens) + S), lay.stack_workspace_bytes(T, 1, T + N * S))
    lay.ws = torch.empty(need, dtype=torch.uint8, device=dev)

    kvs = [B.KVCache(layer, [n + S for n in lens], dev, dt) for _ in range(L)]
    par = lambda steps: lay.compact_stack_forward(weights, inp.cu_seqlens, bufs["x"], bufs["xd"][:steps] if steps else None,
                                                  kvs, bufs["y_last"], bufs["y_dec"] if steps else None)
    par(min(S, 8))
    t_par = timed(lambda: par(S), max(1, args.steps))
    t_par_pre = timed(lambda: par(0), 1)
    del kvs

    Ls = args.seq_layers if args.seq_layers > 0 else L
    kv1 = [B.KVCache(layer, [T + N * S], dev, dt) for _ in range(Ls)]
    xd1 = bufs["xd"].reshape(S * N, 1, layer.d_model)
    yd1 = torch.empty_like(xd1)
    seq = lambda steps: lay.compact_stack_forward(weights[:Ls], [0, T], bufs["x"], xd1[:steps] if steps else None, kv1,
                                                  bufs["y_last"][:1], yd1 if steps else None)
    seq(8)
    t_seq = timed(lambda: seq(S * N), 1) * L / Ls
    t_seq_pre = timed(lambda: seq(0), 1) * L / Ls
    return {
        "metric": "compaction_decode_tokens_per_s", "value": N * S / t_par, "unit": "tokens/s", "n_gpus": 1,
        "steps": max(1, args.steps), "warmup": 1, "ms_per_step": t_par * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": layer.dtype, "data": "synthetic",
        "config": {"workload": "%s, %d layers deep (random weights per layer): %d blocks x %d tokens prefill + %d decode "
                               "steps/block" % (wl.name, L, N, lens[0], S), "total_prefill_tokens": T, "decode_tokens": N * S,
                   "n_layers": L},
        "ms_prefill": t_par_pre * 1e3, "ms_decode": (t_par - t_par_pre) * 1e3,
        "us_per_decode_step_per_layer": (t_par - t_par_pre) * 1e6 / max(S, 1) / L,
        "ms_per_decode_token": t_par * 1e3 / (N * S),
        "sequential_single_block": {
            "what": "the whole %d-token history as one block, the same %d decode tokens one after another" % (T, N * S),
            "layers_measured": Ls, "scaled_to_layers": L, "ms_per_step": t_seq * 1e3, "ms_prefill": t_seq_pre * 1e3,
            "ms_decode": (t_seq - t_seq_pre) * 1e3, "ms_per_decode_token": t_seq * 1e3 / (N * S),
            "parallel_speedup": t_seq / t_par},
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="dense_8x4096")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sequential", action="store_true")
    ap.add_argument("--prefix-aware", action="store_true",
                    help="time the prefix-aware target-at-end layout instead (paper Sec. IV, Dispatch): the history is "
                         "prefilled once as one block, every worker then decodes against its prefix of that shared cache")
    ap.add_argument("--mxfp4", action="store_true",
                    help="routed workloads: the experts come as block-scaled 4-bit arrays (paper Sec. IV-B, mxfp4 weights); "
                         "decode steps stream those, the prefill reads their exact bf16 expansion")
    ap.add_argument("--mixed", type=int, default=0, metavar="TOKENS",
                    help="time the token-budgeted mixed schedule instead (compact_mixed_forward: prefill chunks and decode "
                         "tokens in one batch, at most TOKENS rows per step) beside the plain prefill-then-decode pass")
    ap.add_argument("--stack", type=int, default=0, metavar="L",
                    help="time a depth of L layers instead (compact_stack_forward; per-layer weights and caches), and "
                         "beside it the paper's sequential baseline: the whole history as ONE block, the same number of "
                         "decode tokens one after another (Sec. V, Tables VII-IX)")
    ap.add_argument("--seq-layers", type=int, default=0,
                    help="layers of the sequential baseline under --stack (default: all L; every layer costs the same, "
                         "so fewer layers are scaled up and labelled so)")
    ap.add_argument("--copy-probe-mib", type=int, default=0,
                    help="first run one plain device copy of this many MiB (a kernel of known HBM traffic, "
                         "used to scale rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: the library runs on ONE GPU (blocks are independent; sharding across GPUs is a design note, "
              "not code). Re-run with --gpus 1.", file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)

    wl = WORKLOADS[args.workload]
    dev = "cuda"
    if args.copy_probe_mib > 0:
        src = torch.ones(args.copy_probe_mib << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    inp = make_inputs(wl, device=dev, gen_device=dev)
    layer = inp.layer
    if args.mxfp4:
        if layer.n_experts == 0:
            print("bench.py: --mxfp4 needs a routed workload (--workload moe_16x8192)", file=sys.stderr)
            sys.exit(2)
        gen = torch.Generator(device=dev)
        gen.manual_seed(wl.seed + 77)
        q4 = make_mxfp4_experts(layer, gen, dev)
        lay0 = B.Layer(layer, None)
        for name in ("w_exp_gate_up", "w_exp_down"):       # the 16-bit copy = the exact expansion of the 4-bit arrays
            lay0.compact_mxfp4_dequant(q4[name + "_q"], q4[name + "_s"], inp.weights[name])
        inp.weights.update(q4)
        torch.cuda.synchronize()
    lens, S, N, T = inp.block_lens, inp.x_decode.shape[0], len(inp.block_lens), inp.cu_seqlens[-1]
    lay = B.Layer(layer, inp.weights)
    dt = lay.torch_dtype
    kv = B.KVCache(layer, [L + S for L in lens], dev, dt)
    lay.ensure_workspace(T, N, max(lens) + S, dev)
    bufs = dict(x=inp.x_prefill, xd=inp.x_decode.contiguous(),
                y_pre=torch.empty(T, layer.d_model, dtype=dt, device=dev),
                y_last=torch.empty(N, layer.d_model, dtype=dt, device=dev),
                y_dec=torch.empty(S, N, layer.d_model, dtype=dt, device=dev))

    if args.prefix_aware:
        print(json.dumps(prefix_aware_pass(args, wl, inp, lay, bufs)))
        return
    if args.stack > 0:
        del kv
        print(json.dumps(stack_pass(args, wl, inp, lay, bufs)))
        return
    if args.mixed > 0:
        print(json.dumps(mixed_pass(args, wl, inp, lay, kv, bufs)))
        return

    for _ in range(args.warmup):
        run_pass(lay, inp, kv, bufs)
    t_pass = timed(lambda: run_pass(lay, inp, kv, bufs), args.steps)

    # split of the pass (extra, untimed for `value`): prefill-only passes
    t_prefill = timed(lambda: run_pass(lay, inp, kv, bufs, 0), max(2, args.steps // 2))
    t_decode = max(t_pass - t_prefill, 1e-9)

    # per-kernel-class durations from HIP events on the launch stream, one class per extra pass
    n_distinct = distinct_experts(lay, inp, kv, bufs) if layer.n_experts > 0 else None
    work = algorithmic_work(layer, lens, S, n_distinct, 4.25 if args.mxfp4 else 16.0)
    classes = {
        "gemm_bf16": (B.K_GEMM, "mfma", work["gemm_flops"], PEAK_BF16_TFLOPS),
        "attn_prefill": (B.K_ATTN_PREFILL, "mfma", work["attn_prefill_flops"], PEAK_BF16_TFLOPS),
        "attn_decode": (B.K_ATTN_DECODE, "hbm", work["attn_decode_bytes"], PEAK_HBM_GBS),
        "gemm_skinny": (B.K_GEMM_SKINNY, "hbm", work["skinny_bytes"], PEAK_HBM_GBS),
    }
    kernels = {}
    reps = max(1, min(3, args.steps))
    for name, (klass, bound, units, peak) in classes.items():
        lay.compact_profile_select(klass)
        for _ in range(reps):
            run_pass(lay, inp, kv, bufs)
        torch.cuda.synchronize()
        n, ms = lay.compact_profile_read()
        lay.compact_profile_select(B.K_NONE)
        if n == 0:
            continue
        per_pass_s = ms / 1e3 / reps
        achieved = units / per_pass_s / (1e12 if bound == "mfma" else 1e9)
        kernels[name] = dict(bound=bound, launches_per_pass=n // reps, ms_per_pass=per_pass_s * 1e3,
                             avg_launch_us=ms * 1e3 / n, achieved=achieved, peak=peak,
                             unit="TFLOP/s" if bound == "mfma" else "GB/s", frac=achieved / peak)
    dom = max(kernels, key=lambda k: kernels[k]["ms_per_pass"])
    roofline = dict(kernel=dom, bound=kernels[dom]["bound"], achieved=kernels[dom]["achieved"], peak=kernels[dom]["peak"],
                    unit=kernels[dom]["unit"], frac=kernels[dom]["frac"], traffic=recorded_traffic(wl.name, dom),
                    avg_launch_us=kernels[dom]["avg_launch_us"], launches_per_pass=kernels[dom]["launches_per_pass"],
                    event_pair_overhead_us=event_pair_overhead_us())

    out = {
        "metric": "compaction_decode_tokens_per_s", "value": N * S / t_pass, "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": t_pass * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": layer.dtype, "data": "synthetic",
        "config": {"workload": "%s: %d blocks x %s tokens prefill + %d decode steps/block, d_model %d, %dq/%dkv heads x %d, "
                               "FFN %d%s, one layer" % (wl.name, N, str(lens[0]) if min(lens) == max(lens) else
                                                        "%d..%d" % (min(lens), max(lens)), S, layer.d_model,
                                                        layer.n_q_heads, layer.n_kv_heads, layer.head_dim, layer.ffn_dim,
                                                        "" if layer.n_experts == 0 else
                                                        " x %d experts top-%d%s" % (layer.n_experts, layer.top_k,
                                                                                    ", 4-bit block-scaled experts in decode" if args.mxfp4 else "")),
                   "total_prefill_tokens": T, "decode_tokens": N * S},
        "prefill_tokens_per_s": T / t_prefill, "decode_tokens_per_s": N * S / t_decode,
        "ms_prefill": t_prefill * 1e3, "ms_decode": t_decode * 1e3, "us_per_decode_step": t_decode * 1e6 / max(S, 1),
        "roofline": roofline, "kernels": kernels,
    }

    if not args.no_sequential:
        # the same decode volume, one block at a time (N calls with one block each)
        import copy
        seq_t = seq_pre = 0.0
        for b in range(N):
            one = copy.copy(inp)
            one.block_lens, one.cu_seqlens = [lens[b]], [0, lens[b]]
            kv1 = B.KVCache(layer, [lens[b] + S], dev, dt)
            b1 = dict(x=inp.x_prefill[inp.cu_seqlens[b]:inp.cu_seqlens[b + 1]], xd=inp.x_decode[:, b:b + 1].contiguous(),
                      y_pre=bufs["y_pre"][:lens[b]], y_last=bufs["y_last"][:1],
                      y_dec=torch.empty(S, 1, layer.d_model, dtype=dt, device=dev))
            run_pass(lay, one, kv1, b1)
            seq_t += timed(lambda: run_pass(lay, one, kv1, b1), SEQ_REPS)
            seq_pre += timed(lambda: run_pass(lay, one, kv1, b1, 0), SEQ_REPS)
        seq_dec = max(seq_t - seq_pre, 1e-9)
        out["sequential_one_block_at_a_time"] = {
            "repetitions_per_block": SEQ_REPS, "ms_per_step": seq_t * 1e3, "value": N * S / seq_t, "batched_speedup": seq_t / t_pass,
            "decode_tokens_per_s": N * S / seq_dec, "batched_decode_speedup": seq_dec / t_decode,
            "prefill_tokens_per_s": T / seq_pre}

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(inp)

    print(json.dumps(out))


if __name__ == "__main__":
    main()
