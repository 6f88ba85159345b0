"""Seeded synthetic workloads: layer shapes, block partitions and Gaussian
tensors.  This module holds none of the layer's arithmetic; it only draws
numbers, so that the HIP library and the CPU checker can be fed identical bits.

The shapes stand in for the paper's workloads (Sec. V: compaction threshold
96 k tokens, block sizes 2 k-16 k, 6-48 concurrent workers, Llama-3.1-8B-like
dense and gpt-oss-120B-like MoE backbones): histories of 32 k-128 k tokens cut
into N = ceil(|X| / B) contiguous blocks (Sec. IV, snapshot & partition), a few
hundred decoded summary tokens per block.  Values are Gaussians; no dataset
item is reproduced.

Draw order for one workload (one torch.Generator, seed given):
  1. ragged block lengths (ragged workloads only)
  2. x_prefill [T, d] ~ N(0, 1)
  3. w_qkv, w_o, then w_gate_up, w_down (dense) or w_router, w_exp_gate_up,
     w_exp_down (MoE), each ~ N(0, 0.02)
  4. x_decode [S, N, d] ~ N(0, 1)
RMSNorm gains are all-ones in the named workloads (a N(0, 0.02) gain would
scale activations to nothing); tests that exercise the gain draw 1 + N(0, 0.02).
Every tensor is rounded once to the workload dtype; those bits go to both sides.
"""
from dataclasses import dataclass, field, asdict
from typing import List, Optional

import torch


@dataclass
class LayerConfig:
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn_dim: int
    n_experts: int = 0          # 0 = dense SwiGLU
    top_k: int = 0
    rms_eps: float = 1e-5
    rope_theta: float = 10000.0
    dtype: str = "bf16"         # "fp32" | "bf16"

    @property
    def Dq(self):
        return self.n_q_heads * self.head_dim

    @property
    def Dkv(self):
        return self.n_kv_heads * self.head_dim

    def as_dict(self):
        return asdict(self)


@dataclass
class Workload:
    name: str
    layer: LayerConfig
    block_lens: Optional[List[int]]      # None => ragged, drawn from the seed
    n_blocks: int
    decode_steps: int
    ragged_range: Optional[tuple] = None
    seed: int = 0
    note: str = ""


DENSE_8B = dict(d_model=4096, n_q_heads=32, n_kv_heads=8, head_dim=128,
                ffn_dim=14336, rope_theta=500000.0, dtype="bf16")

WORKLOADS = {
    # tiny fp32 layer, checked in full against the fp64 checker
    "tiny_fp32": Workload(
        "tiny_fp32",
        LayerConfig(d_model=256, n_q_heads=4, n_kv_heads=2, head_dim=64, ffn_dim=1024,
                    rope_theta=10000.0, dtype="fp32"),
        [128] * 4, 4, 16),
    # 32 k history in 8 blocks of 4 k: the headline prefill + B=8 decode case
    "dense_8x4096": Workload("dense_8x4096", LayerConfig(**DENSE_8B), [4096] * 8, 8, 256),
    # the paper's own operating point (Sec. V: threshold 96 k tokens, 4 k blocks => 24 workers)
    "dense_24x4096": Workload("dense_24x4096", LayerConfig(**DENSE_8B), [4096] * 24, 24, 256),
    # 128 k history in 64 blocks of 2 k: decode attention over 64 caches
    "dense_64x2048": Workload("dense_64x2048", LayerConfig(**DENSE_8B), [2048] * 64, 64, 128),
    # 32 ragged blocks, lengths uniform on [512, 8192] inclusive
    "dense_ragged32": Workload("dense_ragged32", LayerConfig(**DENSE_8B), None, 32, 192,
                               ragged_range=(512, 8192)),
    # MoE, 128 experts, top-4, 16 blocks of 8 k
    "moe_16x8192": Workload(
        "moe_16x8192",
        LayerConfig(d_model=2880, n_q_heads=64, n_kv_heads=8, head_dim=64, ffn_dim=2880,
                    n_experts=128, top_k=4, rope_theta=500000.0, dtype="bf16"),
        [8192] * 16, 16, 256),
}


def torch_dtype(name):
    return {"fp32": torch.float32, "bf16": torch.bfloat16}[name]


def partition(total_tokens, block_size):
    """Snapshot & partition (paper Sec. IV): N = ceil(|X| / B) contiguous
    blocks of B tokens, the last possibly shorter."""
    n = -(-total_tokens // block_size)
    lens = [block_size] * n
    lens[-1] = total_tokens - block_size * (n - 1)
    return lens


def cu_seqlens(block_lens):
    cu = [0]
    for L in block_lens:
        cu.append(cu[-1] + int(L))
    return cu


def _normal(shape, std, gen, device, dtype):
    # drawn in fp32 on the generator's device, rounded once to the workload dtype
    t = torch.randn(shape, generator=gen, device=gen.device, dtype=torch.float32)
    if std != 1.0:
        t.mul_(std)
    return t.to(dtype).to(device)


def draw_block_lens(wl, gen):
    if wl.block_lens is not None:
        return list(wl.block_lens)
    lo, hi = wl.ragged_range
    lens = torch.randint(lo, hi + 1, (wl.n_blocks,), generator=gen, device=gen.device)
    return [int(v) for v in lens.cpu()]


def make_weights(layer, gen, device="cpu", gain_jitter=False):
    """Weights in the library's layout ([out, in] row-major)."""
    dt = torch_dtype(layer.dtype)
    d, F = layer.d_model, layer.ffn_dim
    w = {}
    w["w_qkv"] = _normal((layer.Dq + 2 * layer.Dkv, d), 0.02, gen, device, dt)
    w["w_o"] = _normal((d, layer.Dq), 0.02, gen, device, dt)
    if layer.n_experts == 0:
        w["w_gate_up"] = _normal((2 * F, d), 0.02, gen, device, dt)
        w["w_down"] = _normal((d, F), 0.02, gen, device, dt)
    else:
        E = layer.n_experts
        w["w_router"] = _normal((E, d), 0.02, gen, device, dt)
        gu = torch.empty((E, 2 * F, d), dtype=dt, device=device)
        dn = torch.empty((E, d, F), dtype=dt, device=device)
        for e in range(E):          # per expert, to bound the fp32 staging buffer
            gu[e] = _normal((2 * F, d), 0.02, gen, device, dt)
        for e in range(E):
            dn[e] = _normal((d, F), 0.02, gen, device, dt)
        w["w_exp_gate_up"], w["w_exp_down"] = gu, dn
    if gain_jitter:
        w["g_attn"] = (1.0 + _normal((d,), 0.02, gen, device, torch.float32)).to(dt)
        w["g_ffn"] = (1.0 + _normal((d,), 0.02, gen, device, torch.float32)).to(dt)
    else:
        w["g_attn"] = torch.ones(d, dtype=dt, device=device)
        w["g_ffn"] = torch.ones(d, dtype=dt, device=device)
    return w


@dataclass
class Inputs:
    layer: LayerConfig
    block_lens: List[int]
    cu_seqlens: List[int]
    x_prefill: torch.Tensor
    weights: dict
    x_decode: torch.Tensor
    meta: dict = field(default_factory=dict)


def make_inputs(wl, device="cpu", gen_device=None, block_lens=None, decode_steps=None,
                gain_jitter=False):
    """Draw one workload.  `gen_device` = where the random numbers are drawn
    (defaults to CPU; large workloads may draw on the GPU and copy samples
    back).  `block_lens` / `decode_steps` override the named shape for reduced
    test cases; the draw order is unchanged."""
    gen_device = gen_device or "cpu"
    gen = torch.Generator(device=gen_device)
    gen.manual_seed(wl.seed)
    lens = draw_block_lens(wl, gen) if block_lens is None else list(block_lens)
    S = wl.decode_steps if decode_steps is None else decode_steps
    layer = wl.layer
    dt = torch_dtype(layer.dtype)
    T = sum(lens)
    x = _normal((T, layer.d_model), 1.0, gen, device, dt)
    w = make_weights(layer, gen, device, gain_jitter)
    xd = _normal((S, len(lens), layer.d_model), 1.0, gen, device, dt)
    return Inputs(layer, lens, cu_seqlens(lens), x, w, xd,
                  meta=dict(workload=wl.name, seed=wl.seed, gen_device=str(gen_device)))


def make_mxfp4_experts(layer, gen, device="cpu", scale_spread=0):
    """Random block-scaled 4-bit expert weights (drawn, not quantised from anything):
    uniform 4-bit codes, two per byte, and one scale byte per 32 elements drawn from
    {119, 120} (2^-8, 2^-7), which puts the weights' rms near the 0.02 of the 16-bit
    workloads.  Returns uint8 tensors w_exp_gate_up_q [E, 2F, d/2], w_exp_gate_up_s
    [E, 2F, d/32], w_exp_down_q [E, d, F/2], w_exp_down_s [E, d, F/32].

    scale_spread = s > 0 spreads the scale bytes over a wide range while every expert's
    output stays O(1): expert e's gate/up scales are shifted by t_e (evenly spaced over
    -s .. s) and drawn from a window of four bytes, its down scales by -2 t_e (the SwiGLU
    intermediate is quadratic in the gate/up scale where silu is linear or the identity)."""
    E, d, F = layer.n_experts, layer.d_model, layer.ffn_dim

    def draw(shape, lo, hi):
        return torch.randint(lo, hi, shape, generator=gen, device=gen.device, dtype=torch.uint8).to(device)

    if not scale_spread:
        return dict(w_exp_gate_up_q=draw((E, 2 * F, d // 2), 0, 256), w_exp_gate_up_s=draw((E, 2 * F, d // 32), 119, 121),
                    w_exp_down_q=draw((E, d, F // 2), 0, 256), w_exp_down_s=draw((E, d, F // 32), 119, 121))
    t = torch.linspace(-scale_spread, scale_spread, E).round().to(torch.int32).view(E, 1, 1).to(device)
    gu_s = (draw((E, 2 * F, d // 32), 118, 122).to(torch.int32) + t).to(torch.uint8)
    dn_s = (draw((E, d, F // 32), 118, 122).to(torch.int32) - 2 * t).to(torch.uint8)
    return dict(w_exp_gate_up_q=draw((E, 2 * F, d // 2), 0, 256), w_exp_gate_up_s=gu_s,
                w_exp_down_q=draw((E, d, F // 2), 0, 256), w_exp_down_s=dn_s)


def make_stack_weights(wl, n_layers, device="cpu", gen_device=None, gain_jitter=False):
    """Weights of a depth of n_layers layers of the workload's shape: layer l is drawn
    by make_weights' recipe from a generator of its own, seeded wl.seed + 1000 * (l + 1)."""
    gen_device = gen_device or "cpu"
    out = []
    for l in range(n_layers):
        gen = torch.Generator(device=gen_device)
        gen.manual_seed(wl.seed + 1000 * (l + 1))
        out.append(make_weights(wl.layer, gen, device, gain_jitter))
    return out


def to_numpy_f64(t):
    """Exact widening of a (bf16 / fp32) tensor to a float64 numpy array."""
    return t.detach().to("cpu").to(torch.float64).numpy()
