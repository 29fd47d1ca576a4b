"""Seeded synthetic workloads for the MoE FFN layer.

This module only *draws inputs* (tokens, parameters, a routing choice and
gate weights, the upstream gradient).  It holds none of the layer's own
arithmetic: the router that produces a routing choice R_i(x) is outside the
expert-specific operators (the method takes R as an input; Sec. 3.1 and the
symbol table of App. A), so drawing top-k indices and gates here is input
generation, not part of the path under test.  Both the CPU oracle and the HIP
library are fed from the tensors this module returns.

The five named workloads stand in for the paper's Swin-Transformer-MoE
training batches (Sec. 4 "Experimental setup"), which need a dataset and a
trained router that are not available; "32x32 patches" means 1024 tokens per
image.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace
from typing import Dict

import torch


@dataclass(frozen=True)
class MoEWorkload:
    name: str
    T: int          # tokens (the paper's N)
    d_model: int    # D_i = D_o of the FFN
    d_ff: int       # hidden size between the two MLPs
    E: int          # global experts
    k: int          # top-k
    dtype: str      # "f32" | "bf16" | "f16"
    routing: str    # recipe name, see _route()
    seed: int

    @property
    def A(self) -> int:
        return self.T * self.k

    @property
    def useful_flop(self) -> float:
        """2 GEMMs forward + 4 backward, 2*A*d*f each."""
        return 12.0 * self.A * self.d_model * self.d_ff


_SEED0 = 0x48455841  # "HEXA"

WORKLOADS: Dict[str, MoEWorkload] = {
    "C1": MoEWorkload("C1", 256, 64, 256, 4, 1, "f32", "uniform_top1", _SEED0 + 1),
    "C2": MoEWorkload("C2", 4096, 384, 1536, 8, 2, "bf16", "topk", _SEED0 + 2),
    "C3": MoEWorkload("C3", 32768, 768, 3072, 16, 2, "bf16", "zipf", _SEED0 + 3),
    "C4": MoEWorkload("C4", 65536, 1024, 4096, 32, 1, "bf16", "forced", _SEED0 + 4),
    "C5": MoEWorkload("C5", 131072, 2048, 8192, 64, 2, "bf16", "bias", _SEED0 + 5),
}

C4_EMPTY_EXPERTS = (1, 15, 16, 31)


def workload(name: str, **overrides) -> MoEWorkload:
    w = WORKLOADS[name]
    return replace(w, **overrides) if overrides else w


def _randn(shape, gen, device, std=1.0):
    t = torch.randn(shape, generator=gen, device=device, dtype=torch.float32)
    if std != 1.0:
        t.mul_(std)
    return t


def _topk_stable(logits: torch.Tensor, k: int):
    """Top-k by value; equal logits resolve to the lower expert id."""
    order = torch.sort(logits, dim=1, descending=True, stable=True).indices[:, :k]
    return order, torch.gather(logits, 1, order)


def _route(w: MoEWorkload, gen, device):
    """Returns (topk_idx int32 [T,k], gate f32 [T,k])."""
    T, E, k = w.T, w.E, w.k
    logits = _randn((T, E), gen, device)
    if w.routing == "uniform_top1":
        # expert uniform per token; gate = full softmax evaluated at that expert
        assert k == 1
        idx = torch.randint(0, E, (T, 1), generator=gen, device=device)
        gate = torch.gather(torch.softmax(logits, dim=1), 1, idx)
    elif w.routing == "forced":
        # half the tokens (a random half) go to expert 0, a fixed set of experts
        # receives nothing, the rest is uniform over the remaining experts
        assert k == 1
        order = torch.randperm(T, generator=gen, device=device)
        allowed = torch.tensor(
            [e for e in range(1, E) if e not in C4_EMPTY_EXPERTS],
            device=device, dtype=torch.int64)
        pick = torch.randint(0, allowed.numel(), (T,), generator=gen, device=device)
        idx = allowed[pick]
        idx[order[: T // 2]] = 0
        idx = idx.view(T, 1)
        gate = torch.gather(torch.softmax(logits, dim=1), 1, idx)
    else:
        if w.routing == "zipf":
            p = torch.arange(1, E + 1, device=device, dtype=torch.float64).pow(-1.2)
            p = p / p.sum()
            logits = logits + p.log().to(torch.float32)[None, :]
        elif w.routing == "bias":
            beta = _randn((E,), gen, device, std=0.5)
            logits = logits + beta[None, :]
        elif w.routing != "topk":
            raise ValueError(w.routing)
        idx, sel = _topk_stable(logits, k)
        gate = torch.softmax(sel, dim=1)          # renormalised over the k selected
    return idx.to(torch.int32).contiguous(), gate.to(torch.float32).contiguous()


def generate(w: MoEWorkload, device="cpu") -> Dict[str, torch.Tensor]:
    """Draw one batch.  Same (workload, device type) -> same tensors.

    Standard deviations: x, dY ~ N(0,1); weights ~ N(0,0.02); biases ~ N(0,0.01).
    Tensors come back in the workload's dtype (gate is always f32, topk_idx i32).
    """
    device = torch.device(device)
    gen = torch.Generator(device=device)
    gen.manual_seed(w.seed)
    tdt = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[w.dtype]
    out = {}
    out["topk_idx"], out["gate"] = _route(w, gen, device)
    out["x"] = _randn((w.T, w.d_model), gen, device).to(tdt)
    out["dY"] = _randn((w.T, w.d_model), gen, device).to(tdt)
    out["b1"] = _randn((w.E, w.d_ff), gen, device, 0.01).to(tdt)
    out["b2"] = _randn((w.E, w.d_model), gen, device, 0.01).to(tdt)
    # the two big ones last, one expert at a time to bound the fp32 temporary
    for name, shape in (("W1", (w.d_model, w.d_ff)), ("W2", (w.d_ff, w.d_model))):
        full = torch.empty((w.E,) + shape, device=device, dtype=tdt)
        for e in range(w.E):
            full[e] = _randn(shape, gen, device, 0.02).to(tdt)
        out[name] = full
    return out
