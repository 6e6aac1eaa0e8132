"""Seeded synthetic inputs: model shapes and value generators.

This module holds NO arithmetic of the method (no Adam, no rounding to bf16
by hand, no partition layout).  It only says which tensors a model of a given
shape has and draws seeded random values, so that the CPU oracle's tests and
the HIP path's tests can be fed the same inputs.  It imports neither of them.

Shapes stand in for the paper's workloads (Experimental settings: Llama-3 70B
and Mixtral 8x7B, "47B"; 140 GB and 94 GB in bf16).  Weights are random, not
the trained checkpoints, and no dataset is used.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Tuple

import numpy as np

WORLD = 8  # ranks the paper's shards are "one of"


@dataclass(frozen=True)
class ModelShape:
    name: str
    layers: int
    d_model: int
    ffn: int
    q_heads: int
    kv_heads: int
    vocab: int
    experts: int = 0  # 0 = dense FFN
    head_dim: int = 128


LLAMA3_8B = ModelShape("llama3_8b", 32, 4096, 14336, 32, 8, 128256)
LLAMA3_70B = ModelShape("llama3_70b", 80, 8192, 28672, 64, 8, 128256)
MIXTRAL_8X7B = ModelShape("mixtral_8x7b", 32, 4096, 14336, 32, 8, 32000, experts=8)
SHAPES = {s.name: s for s in (LLAMA3_8B, LLAMA3_70B, MIXTRAL_8X7B)}


def tensor_list(shape: ModelShape) -> List[Tuple[str, Tuple[int, ...]]]:
    """(name, dims) of every weight in canonical order.

    embed; per layer q, k, v, o, [router], FFN matrices (per expert for MoE),
    two norm vectors; final norm; untied LM head.
    """
    d, hd = shape.d_model, shape.head_dim
    out: List[Tuple[str, Tuple[int, ...]]] = [("embed", (shape.vocab, d))]
    for l in range(shape.layers):
        pre = f"layers.{l}."
        out.append((pre + "attn.q", (shape.q_heads * hd, d)))
        out.append((pre + "attn.k", (shape.kv_heads * hd, d)))
        out.append((pre + "attn.v", (shape.kv_heads * hd, d)))
        out.append((pre + "attn.o", (d, shape.q_heads * hd)))
        if shape.experts:
            out.append((pre + "moe.router", (shape.experts, d)))
            for e in range(shape.experts):
                out.append((pre + f"moe.experts.{e}.w1", (shape.ffn, d)))
                out.append((pre + f"moe.experts.{e}.w2", (d, shape.ffn)))
                out.append((pre + f"moe.experts.{e}.w3", (shape.ffn, d)))
        else:
            out.append((pre + "mlp.gate", (shape.ffn, d)))
            out.append((pre + "mlp.up", (shape.ffn, d)))
            out.append((pre + "mlp.down", (d, shape.ffn)))
        out.append((pre + "norm1", (d,)))
        out.append((pre + "norm2", (d,)))
    out.append(("final_norm", (d,)))
    out.append(("lm_head", (shape.vocab, d)))
    return out


def tensor_numels(shape: ModelShape) -> List[int]:
    return [int(np.prod(dims, dtype=np.int64)) for _, dims in tensor_list(shape)]


def total_params(shape: ModelShape) -> int:
    return sum(tensor_numels(shape))


TINY_TENSORS = [(f"w{i}", (512, 512)) for i in range(4)]  # 1,048,576 elements
TINY_N = 4 * 512 * 512

# Hyper-parameters of every benchmark workload.
HP = dict(lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01)
P_STD = 0.02
G_STD = 1e-3


def host_normal(n: int, std: float, seed: int) -> np.ndarray:
    """Seeded N(0, std) fp32 values on the host."""
    rng = np.random.default_rng(seed)
    return (rng.standard_normal(n, dtype=np.float32) * np.float32(std)).astype(np.float32)


def host_params(n: int, seed: int = 1) -> np.ndarray:
    return host_normal(n, P_STD, seed)


def host_grads_f32(n: int, step: int) -> np.ndarray:
    """Fresh fp32 gradients of step `step` (seed = 1000 + step)."""
    return host_normal(n, G_STD, 1000 + step)


def host_index_hash16(start: int, count: int) -> np.ndarray:
    """16-bit pattern that depends only on the global element index."""
    with np.errstate(over="ignore"):
        i = np.arange(start, start + count, dtype=np.uint64)
        h = i * np.uint64(0x9E3779B97F4A7C15)
        h ^= h >> np.uint64(29)
        return ((h >> np.uint64(17)) & np.uint64(0xFFFF)).astype(np.uint16)


# ---- device-side generators (torch used as a random source and allocator) ----

def _torch():
    import torch
    return torch


def device_normal_(out, std: float, seed: int, chunk: int = 1 << 27) -> None:
    """Fill a device tensor (fp32 or bf16) with seeded N(0, std), chunked so the
    temporary stays small.  The bf16 case draws fp32 and lets torch narrow it;
    the resulting bits are the input, whatever they are."""
    torch = _torch()
    gen = torch.Generator(device=out.device)
    gen.manual_seed(seed)
    flat = out.view(-1)
    n = flat.numel()
    for s in range(0, n, chunk):
        e = min(n, s + chunk)
        tmp = torch.randn(e - s, generator=gen, device=out.device, dtype=torch.float32)
        tmp.mul_(std)
        flat[s:e].copy_(tmp)
        del tmp


def device_index_hash16_(out, start: int = 0, chunk: int = 1 << 27) -> None:
    """Fill an int16/uint16-viewable device tensor with host_index_hash16's pattern."""
    torch = _torch()
    flat = out.view(-1).view(torch.int16)
    n = flat.numel()
    for s in range(0, n, chunk):
        e = min(n, s + chunk)
        flat[s:e].copy_(device_index_hash16_values(start + s, e - s, out.device))


def device_index_hash16_values(start: int, count: int, device):
    """int16 tensor holding host_index_hash16(start, count) bit patterns."""
    torch = _torch()
    i = torch.arange(start, start + count, device=device, dtype=torch.int64)
    h = i * (-7046029254386353131)  # 0x9E3779B97F4A7C15 as signed 64-bit
    # logical right shifts on signed storage: mask off the sign extension
    h = h ^ ((h >> 29) & ((1 << 35) - 1))
    return ((h >> 17) & 0xFFFF).to(torch.int16)
