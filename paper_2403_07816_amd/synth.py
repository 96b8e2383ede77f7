"""Seeded synthetic inputs for the MoE feed-forward layer.

This module only draws random tensors; it holds none of the layer's arithmetic
(no routing, no expert FFN, no averaging).  Both the HIP path and the CPU
oracle are fed the very arrays produced here, so neither has to reproduce the
other's random numbers.

Recipe (stands in for the Llama-2-7B MoE-finetuning workload of the paper's
experimental setup: sequences of 4096 tokens, 4 branched experts):
  x[T,d]        N(0,1); optionally every row divided by its RMS (what a
                pre-FF RMSNorm without gain would hand to the layer)
  seed W1,W3    N(0, 1/d)       [d,f]
  seed W2       N(0, 1/f)       [f,d]
  expert e      seed + independent N(0, (0.1/sqrt(fan_in))^2): experts that
                drifted from one seed model during the branch-and-train stage
  W_router      N(0, 0.02^2)    [d,E] fp32
  dY[T,d]       N(0, 1e-2)      (variance 1e-2, i.e. std 0.1)
  U[T]          uniform [0,1) fp32 (sample-top-1 routing only)
All tensors are drawn in fp32 and rounded once (RNE) to the storage dtype.
"""
from __future__ import annotations

import math
from typing import Dict, Optional, Sequence

import torch

BASE_SEED = 20240312

# One stream id per tensor so that changing one shape never shifts another
# tensor's random numbers.
_STREAM = {"x": 1, "seed_w1": 2, "seed_w3": 3, "seed_w2": 4, "pert_w1": 100,
           "pert_w3": 200, "pert_w2": 300, "router": 5, "dY": 6, "U": 7,
           "merge_base": 8, "merge_pert": 400}


def _generator(seed: int, stream: int, device: str) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed((seed * 1000003 + stream) & 0x7FFFFFFFFFFFFFFF)
    return g


def _randn(shape: Sequence[int], std: float, seed: int, stream: int, device: str) -> torch.Tensor:
    g = _generator(seed, stream, device)
    return torch.randn(*shape, generator=g, device=device, dtype=torch.float32) * std


def make_layer(T: int, d: int, f: int, E: int, *, dtype: torch.dtype = torch.float32,
               seed: int = BASE_SEED, device: str = "cpu", unit_rms: bool = False,
               router_E: Optional[int] = None, router_bias: Optional[Sequence[float]] = None,
               with_dY: bool = False, with_U: bool = False, with_gumbel: bool = False,
               identical_experts: bool = False, expert_spread: float = 0.1) -> Dict[str, Optional[torch.Tensor]]:
    """Draw one layer's inputs and parameters.

    E is the number of seed-shaped expert FFNs (each [d,f]); router_E is the
    number of router columns (differs from E only when the caller will split
    every FFN into chunks afterwards).  identical_experts=True leaves out the
    per-expert perturbation (the sparse-upcycling initialisation); expert_spread
    is the perturbation's std in units of the seed's (0.1 in the workload recipe;
    1.0 makes the experts nearly unrelated).  with_U draws the uniforms [T] of inverse-CDF
    sampling, with_gumbel standard Gumbel noise [T, router_E] (both stored under "U").
    """
    router_E = E if router_E is None else router_E
    x = _randn((T, d), 1.0, seed, _STREAM["x"], device)
    if unit_rms:
        x = x / x.pow(2).mean(dim=1, keepdim=True).sqrt()
    out: Dict[str, Optional[torch.Tensor]] = {"x": x.to(dtype)}

    for name, shape, fan_in in (("w1", (d, f), d), ("w3", (d, f), d), ("w2", (f, d), f)):
        base = _randn(shape, 1.0 / math.sqrt(fan_in), seed, _STREAM["seed_" + name], device)
        stacked = torch.empty((E,) + shape, dtype=dtype, device=device)
        for e in range(E):
            if identical_experts:
                stacked[e] = base.to(dtype)
            else:
                pert = _randn(shape, expert_spread / math.sqrt(fan_in), seed, _STREAM["pert_" + name] + e, device)
                stacked[e] = (base + pert).to(dtype)
                del pert
        out["W" + name[1]] = stacked
        del base

    out["W_router"] = _randn((d, router_E), 0.02, seed, _STREAM["router"], device)
    out["b_router"] = (None if router_bias is None else
                       torch.tensor(list(router_bias), dtype=torch.float32, device=device))
    out["dY"] = _randn((T, d), 0.1, seed, _STREAM["dY"], device).to(dtype) if with_dY else None
    if with_gumbel:
        g = _generator(seed, _STREAM["U"], device)
        u = torch.rand((T, router_E), generator=g, device=device, dtype=torch.float32).clamp_(1e-7, 1.0 - 1e-7)
        out["U"] = -torch.log(-torch.log(u))
    elif with_U:
        g = _generator(seed, _STREAM["U"], device)
        out["U"] = torch.rand(T, generator=g, device=device, dtype=torch.float32)
    else:
        out["U"] = None
    return out


def make_merge_set(shapes: Sequence[Sequence[int]], n_copies: int, *, dtype: torch.dtype = torch.bfloat16,
                   seed: int = BASE_SEED, device: str = "cpu"):
    """n_copies perturbed copies of every tensor in `shapes` (the non-FF
    parameters of n_copies branched models): base N(0,1/fan_in) plus an
    independent N(0,(0.1/sqrt(fan_in))^2) per copy.  Returns a list (one entry
    per shape) of lists (one tensor per copy)."""
    result = []
    for i, shape in enumerate(shapes):
        fan_in = shape[-1]
        base = _randn(shape, 1.0 / math.sqrt(fan_in), seed, _STREAM["merge_base"] + 1000 * i, device)
        copies = []
        for n in range(n_copies):
            pert = _randn(shape, 0.1 / math.sqrt(fan_in), seed, _STREAM["merge_pert"] + 1000 * i + n, device)
            copies.append((base + pert).to(dtype))
        result.append(copies)
    return result
