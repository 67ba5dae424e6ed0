"""Seeded synthetic gradient workloads.

This module only *makes inputs*: tensor-shape lists in the structure of LLM
policy gradients (embedding / attention / MLP / norm tensors per layer) and
seeded random values with a controlled correlation to a reference direction.
It contains none of the arithmetic of Gradient Alignment Control, and it is the
only module that both the GPU library's callers and the CPU oracle's callers
use.

Value recipe (all draws in fp32 from a per-tensor ``torch.Generator``):
    d = std * n1,   z = std * n2,   g = rho * d + sqrt(1 - rho^2) * z
then g and d are cast to the storage dtype.  The AR(1) stream keeps an fp32
master h per tensor:  h_t = phi * h_{t-1} + sqrt(1 - phi^2) * std * n_t,
g_t = cast(h_t).

The gradients of the paper's own runs (Qwen3 / Llama policies under GRPO) are
not available; these lists stand in for them and keep only their shape
structure and a chosen cosine to the previous gradient.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import List, Optional, Sequence, Tuple

import numpy as np
import torch

Shape = Tuple[int, ...]

SEED_BASE = 0x6AC0


@dataclass(frozen=True)
class ModelShape:
    """Dimensions of a decoder-only transformer whose gradient list is mimicked."""
    name: str
    vocab: int
    hidden: int
    kv: int
    ffn: int
    layers: int
    lm_head: bool

    def tensor_shapes(self, layers: Optional[int] = None) -> List[Shape]:
        """Parameter-gradient shapes in registration order: embedding, [lm_head],
        per layer q, k, v, o, gate, up, down, norm, norm; then the final norm."""
        L = self.layers if layers is None else layers
        h, kv, f = self.hidden, self.kv, self.ffn
        out: List[Shape] = [(self.vocab, h)]
        if self.lm_head:
            out.append((self.vocab, h))
        for _ in range(L):
            out += [(h, h), (kv, h), (kv, h), (h, h), (f, h), (f, h), (h, f), (h,), (h,)]
        out.append((h,))
        return out


# The five workload families.  "flat" is a single vector; the others are
# transformer gradient lists of increasing size.
MODEL_05B = ModelShape("0.5B", 151936, 896, 128, 4864, 24, False)
MODEL_15B = ModelShape("1.5B", 151936, 1536, 256, 8960, 28, False)
MODEL_76B = ModelShape("7.6B", 152064, 3584, 512, 18944, 28, True)
MODEL_14B = ModelShape("14B", 152064, 5120, 1024, 13824, 48, True)

FLAT_N = 1_048_576


def numel(shape: Shape) -> int:
    n = 1
    for s in shape:
        n *= int(s)
    return n


def total_numel(shapes: Sequence[Shape]) -> int:
    return sum(numel(s) for s in shapes)


def scaled_down(model: ModelShape, factor: int, layers: int, vocab: int) -> ModelShape:
    """Same tensor structure with every width divided by ``factor`` (kept ragged on
    purpose: no rounding to powers of two), fewer layers and a smaller vocabulary."""
    return ModelShape(model.name + f"/{factor}", vocab, model.hidden // factor,
                      max(1, model.kv // factor), model.ffn // factor, layers, model.lm_head)


def tensor_seed(config_id: int, tensor_index: int, step: int = 0) -> int:
    return SEED_BASE + 1000 * config_id + 10 * tensor_index + step * 100_003


def _storage(t: torch.Tensor, dtype: torch.dtype) -> torch.Tensor:
    return t if dtype == torch.float32 else t.to(dtype)


def correlated_pair(shapes: Sequence[Shape], dtype: torch.dtype, rho: float, std: float,
                    config_id: int, device: str = "cpu") -> Tuple[List[torch.Tensor], List[torch.Tensor]]:
    """(g list, d list) with population correlation ``rho`` between g and d."""
    gs, ds = [], []
    w = math.sqrt(max(0.0, 1.0 - rho * rho))
    for j, shp in enumerate(shapes):
        gen = torch.Generator(device=device)
        gen.manual_seed(tensor_seed(config_id, j))
        d32 = torch.randn(shp, generator=gen, device=device, dtype=torch.float32).mul_(std)
        z32 = torch.randn(shp, generator=gen, device=device, dtype=torch.float32).mul_(std)
        z32.mul_(w).add_(d32, alpha=rho)
        gs.append(_storage(z32, dtype).contiguous())
        ds.append(_storage(d32, dtype).contiguous())
        del d32, z32
    return gs, ds


class AR1Stream:
    """Consecutive gradients g_1, g_2, ... whose neighbours have correlation ``phi``."""

    def __init__(self, shapes: Sequence[Shape], dtype: torch.dtype, phi: float, std: float,
                 config_id: int, device: str = "cpu", master_dtype: torch.dtype = torch.float32):
        self.shapes = list(shapes)
        self.dtype = dtype
        self.phi = phi
        self.std = std
        self.config_id = config_id
        self.device = device
        self.t = 0
        self.h: List[torch.Tensor] = []
        self.master_dtype = master_dtype
        for j, shp in enumerate(self.shapes):
            gen = torch.Generator(device=device)
            gen.manual_seed(tensor_seed(config_id, j, 0))
            h0 = torch.randn(shp, generator=gen, device=device, dtype=torch.float32).mul_(std)
            self.h.append(h0.to(master_dtype))

    def next_into(self, out: Sequence[torch.Tensor]) -> None:
        """Advance one step and write g_t (storage dtype) into the given tensors.
        The first call returns the cast of h_0 advanced once, like every later call."""
        self.t += 1
        w = math.sqrt(1.0 - self.phi * self.phi) * self.std
        for j, shp in enumerate(self.shapes):
            gen = torch.Generator(device=self.device)
            gen.manual_seed(tensor_seed(self.config_id, j, self.t))
            z = torch.randn(shp, generator=gen, device=self.device, dtype=torch.float32)
            z.mul_(w).add_(self.h[j].to(torch.float32), alpha=self.phi)
            self.h[j].copy_(z)
            out[j].copy_(z)
            del z

    def next(self) -> List[torch.Tensor]:
        out = [torch.empty(s, dtype=self.dtype, device=self.device) for s in self.shapes]
        self.next_into(out)
        return out


def to_oracle_array(t: torch.Tensor) -> np.ndarray:
    """Host copy of a tensor in the layout the CPU oracle reads: float32 values, or the
    raw bfloat16 bit patterns as uint16.  Always a flat contiguous array that shares no
    memory with ``t`` (the oracle overwrites state arrays in place)."""
    c = t.detach().to("cpu").contiguous().reshape(-1)
    if not t.is_cuda:
        c = c.clone()
    if c.dtype == torch.bfloat16:
        return c.view(torch.int16).numpy().view(np.uint16)
    if c.dtype == torch.float32:
        return c.numpy()
    raise TypeError(f"unsupported dtype {c.dtype}")


def from_bits(a: np.ndarray, dtype: torch.dtype) -> torch.Tensor:
    """Inverse of ``to_oracle_array``."""
    if dtype == torch.bfloat16:
        return torch.from_numpy(a.view(np.int16).copy()).view(torch.bfloat16)
    return torch.from_numpy(a.copy())
