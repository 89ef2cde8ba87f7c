"""Seeded synthetic inputs shaped like the paper's workloads.

This module only draws random numbers and states shapes.  It contains none of
the method's arithmetic (no quantisation, routing or FFN code) and is the one
module that both the HIP path's tests/bench and the CPU oracle's tests use, so
both sides see identical arrays.

The paper evaluates DeepSeek-V2-Lite and Qwen1.5-MoE-A2.7B on a public
benchmark (Section 6.1 item 1); neither the weights nor the benchmark are available
here, so every tensor below is a synthetic stand-in with the same shapes:
weights ~ N(0, 0.02^2), activations ~ N(0, 1), router logits as each workload
states.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np
import torch


@dataclass(frozen=True)
class LayerShape:
    d_model: int
    n_experts: int
    d_ff: int
    top_k: int
    group: int
    n_shared: int = 0
    shared_d_ff: int = 0
    shared_gate: bool = False          # sigmoid gate on the shared expert (Qwen shape)
    act: str = "bf16"                  # activation / scale dtype: "f32" or "bf16"
    b_high: int = 8                    # bits of the full code and of its upper (low-bit) part: 8/4 or 4/2
    b_low: int = 4
    symmetric: bool = False            # symmetric quantiser (zero-point at mid-range) instead of min-max


@dataclass(frozen=True)
class Workload:
    name: str
    layer: LayerShape
    n_layers: int = 1
    steps: int = 16
    seed: int = 0
    dense_first_d_ff: int = 0          # >0: layer 0 is a dense SwiGLU of that width
    prefill_tokens: int = 0


TINY = Workload("tiny-fp32", LayerShape(256, 8, 128, 2, 64, act="f32"), steps=16)
DSV2_LAYER = Workload("dsv2lite-layer", LayerShape(2048, 64, 1408, 6, 128, n_shared=2, shared_d_ff=1408),
                      steps=1024)
QWEN_STACK = Workload("qwen15-moe-24l", LayerShape(2048, 60, 1408, 4, 128, n_shared=1, shared_d_ff=5632,
                                                   shared_gate=True), n_layers=24, steps=256)
DSV2_STACK = Workload("dsv2lite-26l", LayerShape(2048, 64, 1408, 6, 128, n_shared=2, shared_d_ff=1408),
                      n_layers=26, steps=512, dense_first_d_ff=10944)
QWEN_PREFILL = Workload("qwen15-moe-prefill", LayerShape(2048, 60, 1408, 4, 128), n_layers=24,
                        prefill_tokens=2048)

WORKLOADS = {1: TINY, 2: DSV2_LAYER, 3: QWEN_STACK, 4: DSV2_STACK, 5: QWEN_PREFILL}


def _subseed(seed: int, *tags: int) -> int:
    h = (seed * 0x9E3779B1 + 0x7F4A7C15) & 0xFFFFFFFFFFFF
    for t in tags:
        h = ((h ^ (t + 0x632BE5AB)) * 0x100000001B3) & 0xFFFFFFFFFFFF
    return h


def _gen(seed: int, device="cpu") -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def torch_dtype(name: str):
    return {"f32": torch.float32, "bf16": torch.bfloat16}[name]


def expert_weights(seed: int, layer: int, expert: int, d_model: int, d_ff: int,
                   dtype: str = "f32", device="cpu", std: float = 0.02):
    """(w_gate[d_ff,d_model], w_up[d_ff,d_model], w_down[d_model,d_ff]) ~ N(0, std^2).

    Drawn in fp32 from a generator seeded by (seed, layer, expert), so any one
    expert can be regenerated alone; rounded to `dtype` when that is bf16.
    `expert` >= 1000 is used for shared experts, layer-level tag 2000 for a dense FFN.
    """
    g = _gen(_subseed(seed, layer, expert), device)
    out = []
    for shape in ((d_ff, d_model), (d_ff, d_model), (d_model, d_ff)):
        w = torch.randn(shape, generator=g, device=device, dtype=torch.float32) * std
        out.append(w.to(torch_dtype(dtype)))
    return tuple(out)


def router_weight(seed: int, layer: int, n_experts: int, d_model: int, std: float = 0.02) -> torch.Tensor:
    return torch.randn((n_experts, d_model), generator=_gen(_subseed(seed, layer, 3001)), dtype=torch.float32) * std


def shared_gate_weight(seed: int, layer: int, d_model: int, dtype: str, std: float = 0.02) -> torch.Tensor:
    w = torch.randn((d_model,), generator=_gen(_subseed(seed, layer, 3002)), dtype=torch.float32) * std
    return w.to(torch_dtype(dtype))


def activations(seed: int, n: int, d_model: int, dtype: str) -> torch.Tensor:
    """x[n, d_model] ~ N(0, 1), rounded to the activation dtype."""
    x = torch.randn((n, d_model), generator=_gen(_subseed(seed, 4001)), dtype=torch.float32)
    return x.to(torch_dtype(dtype))


def normal_logits(seed: int, n: int, n_experts: int) -> torch.Tensor:
    return torch.randn((n, n_experts), generator=_gen(_subseed(seed, 4002)), dtype=torch.float32)


def bernoulli_masks(seed: int, steps: int, n_experts: int, p_high: float = 0.5) -> np.ndarray:
    """Tiny workload: per step, per expert, mask 3 (both slices) w.p. p_high else 1 (MSB only)."""
    u = torch.rand((steps, n_experts), generator=_gen(_subseed(seed, 4003)))
    return np.where(u.numpy() < p_high, 3, 1).astype(np.uint8)


def cached_set_mask(seed: int, n_experts: int, n_cached: int, n_high: int, beta: float = 1.0):
    """DeepSeek-V2-Lite-shaped layer: a fixed random set of `n_cached` experts has the MSB slice
    resident (bias +beta); `n_high` of them also hold the LSB slice (mask 3); the rest mask 0."""
    perm = torch.randperm(n_experts, generator=_gen(_subseed(seed, 4004))).numpy()
    mask = np.zeros(n_experts, np.uint8)
    mask[perm[:n_cached]] = 1
    mask[perm[:n_high]] = 3
    bias = np.where(mask & 1, np.float32(beta), np.float32(0)).astype(np.float32)
    return mask, bias


def fraction_masks(seed: int, n_layers: int, epoch: int, n_experts: int, frac_high: float = 0.3) -> np.ndarray:
    """Qwen-shaped stack: per layer exactly round(frac*E) experts at mask 3, the rest 1;
    `epoch` = step // 32 selects the redraw."""
    n_high = int(round(frac_high * n_experts))
    out = np.ones((n_layers, n_experts), np.uint8)
    for l in range(n_layers):
        perm = torch.randperm(n_experts, generator=_gen(_subseed(seed, 4005, l, epoch))).numpy()
        out[l, perm[:n_high]] = 3
    return out


def zipf_logits(seed: int, layer: int, steps: int, n_experts: int, s: float = 1.1, period: int = 64) -> torch.Tensor:
    """z[t, e] = -s * ln(rank_pi(e)) + n,  n ~ N(0,1), rank 1..E under a permutation pi that is
    redrawn every `period` steps (a popularity skew whose hot set drifts)."""
    noise = torch.randn((steps, n_experts), generator=_gen(_subseed(seed, 4006, layer)), dtype=torch.float32)
    z = torch.empty_like(noise)
    base = -s * torch.log(torch.arange(1, n_experts + 1, dtype=torch.float32))
    for ep in range((steps + period - 1) // period):
        perm = torch.randperm(n_experts, generator=_gen(_subseed(seed, 4007, layer, ep)))
        rows = slice(ep * period, min(steps, (ep + 1) * period))
        z[rows] = base[perm][None, :] + noise[rows]
    return z


def heavy_tailed_activations(seed: int, n: int, d_model: int, dtype: str) -> torch.Tensor:
    """x[n, d_model] with the structure of transformer hidden states instead of plain N(0, 1): row 0
    has one 100x outlier in every 32-element chunk; row 1 keeps a few fixed outlier channels (x300)
    and has every fourth chunk all zero; row 2 lets every chunk span twenty-four binades (magnitudes
    2^-20 .. 2^4 within a chunk); further rows cycle through the three kinds with fresh draws."""
    g = _gen(_subseed(seed, 4008))
    x = torch.randn((n, d_model), generator=g, dtype=torch.float32)
    n_chunks = d_model // 32
    for r in range(n):
        kind = r % 3
        if kind == 0:
            pos = torch.randint(0, 32, (n_chunks,), generator=g)
            x[r, torch.arange(n_chunks) * 32 + pos] *= 100.0
        elif kind == 1:
            chan = torch.randperm(d_model, generator=g)[: max(1, d_model // 256)]
            x[r, chan] *= 300.0
            x[r].view(n_chunks, 32)[::4] = 0.0
        else:
            e = torch.randint(-20, 5, (d_model,), generator=g).to(torch.float32)
            x[r] = torch.sign(x[r]) * (1.0 + x[r].abs().clamp(max=0.99)) * torch.exp2(e)
    return x.to(torch_dtype(dtype))
