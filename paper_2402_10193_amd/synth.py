"""Seeded synthetic inputs shaped like the paper's workloads.

This module draws random tensors and nothing else: none of the method's
arithmetic (delta, sign, packing, scale, products) lives here, so both the GPU
library's tests and the CPU oracle can be fed from it.

The paper serves Llama-2-7B fine-tunes (Sec. 4.3); those weights are not
available, so the stand-ins are dense Gaussian tensors with the layer shapes of
Llama-2-7B / 70B:  base weights fp16 ~ N(0, 0.02^2), a fine-tuning delta
~ N(0, sigma^2) with sigma = 0.002 (7B) or 0.001 (70B) drawn in fp16, the
fine-tuned weight W_ft = fp16(f32(W_base) + f32(delta)), activations fp16
~ N(0, 1).  Real deltas are dense and high rank (Fig. 2), so iid signs are a
fair stand-in for the kernels.
"""
from __future__ import annotations

import zlib
from typing import Dict, List, Tuple

import torch

DEFAULT_SEED = 20240210

# (out, in) of the seven block linears, in the order they run in a decoder layer
LLAMA2_7B_LAYER: List[Tuple[str, int, int]] = [
    ("q", 4096, 4096), ("k", 4096, 4096), ("v", 4096, 4096), ("o", 4096, 4096),
    ("gate", 11008, 4096), ("up", 11008, 4096), ("down", 4096, 11008),
]
LLAMA2_70B_LAYER: List[Tuple[str, int, int]] = [
    ("q", 8192, 8192), ("k", 1024, 8192), ("v", 1024, 8192), ("o", 8192, 8192),
    ("gate", 28672, 8192), ("up", 28672, 8192), ("down", 8192, 28672),
]


def _gen(device, seed: int, *tags) -> torch.Generator:
    h = zlib.crc32(repr(tags).encode()) & 0x7FFFFFFF
    g = torch.Generator(device=device)
    g.manual_seed((int(seed) * 1000003 + h) % (2**63 - 1))
    return g


def base_weight(out: int, inn: int, *, seed: int = DEFAULT_SEED, tag=("base",), device="cpu",
                std: float = 0.02) -> torch.Tensor:
    g = _gen(device, seed, "w_base", tag)
    w = torch.empty((out, inn), dtype=torch.float32, device=device).normal_(0.0, std, generator=g)
    return w.to(torch.float16)


def finetune_delta(out: int, inn: int, *, sigma: float = 0.002, seed: int = DEFAULT_SEED, tag=("delta",),
                   device="cpu") -> torch.Tensor:
    g = _gen(device, seed, "delta", tag)
    d = torch.empty((out, inn), dtype=torch.float32, device=device).normal_(0.0, sigma, generator=g)
    return d.to(torch.float16)


def finetuned_weight(w_base: torch.Tensor, *, sigma: float = 0.002, seed: int = DEFAULT_SEED, tag=("ft",),
                     ) -> torch.Tensor:
    """A stand-in fine-tuned matrix: the base plus a dense Gaussian perturbation, stored in fp16."""
    out, inn = w_base.shape
    d = finetune_delta(out, inn, sigma=sigma, seed=seed, tag=tag, device=w_base.device)
    return (w_base.to(torch.float32) + d.to(torch.float32)).to(torch.float16)


def activations(T: int, inn: int, *, seed: int = DEFAULT_SEED, tag=("x",), device="cpu",
                std: float = 1.0) -> torch.Tensor:
    g = _gen(device, seed, "x", tag)
    x = torch.empty((T, inn), dtype=torch.float32, device=device).normal_(0.0, std, generator=g)
    return x.to(torch.float16)


def one_token_per_tenant(B: int) -> List[int]:
    """The paper's serving setting: every model receives one distinct request (Sec. 4.3)."""
    return list(range(B))


def mixed_batch(n_tenants: int, T: int, *, seed: int = DEFAULT_SEED) -> List[int]:
    """Continuous-batching shape: T tokens spread unevenly over tenants, unsorted, some tenants idle."""
    g = torch.Generator().manual_seed(seed)
    return torch.randint(0, n_tenants, (T,), generator=g).tolist()


def layer_bytes(shapes, B: int) -> Dict[str, float]:
    """Weight bytes one decode step streams through one layer: fp16 base once + B one-bit deltas."""
    P = sum(o * i for _, o, i in shapes)
    return {"params": P, "base_bytes": 2.0 * P, "delta_bytes": B * P / 8.0, "total": 2.0 * P + B * P / 8.0}
