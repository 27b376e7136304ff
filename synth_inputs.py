"""Seeded synthetic inputs shared by the tests, the benchmark and the smoke check.

This module holds shapes and random-number recipes only: none of the optimizer's
arithmetic lives here.  The parameter sets are transformer-shaped stand-ins for the
paper's models (per layer: four d x d attention matrices, one d x f and one f x d
feed-forward matrix; embeddings, norms and the output layer are routed to AdamW by
the paper's Sec. 5 "MuLoCo" paragraph and are therefore absent).  Values are i.i.d.
Gaussians whose standard deviations follow the workload descriptions: parameters
0.02, gradients 1e-3, pseudogradient displacements 1e-2.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Tuple

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    layers: int
    d_model: int
    d_ffn: int
    K: int                 # worker replicas resident on the GPU
    H: int                 # inner steps per outer step
    param_dtype: str       # "f32" | "bf16"
    beta: float = 0.9      # Muon momentum (paper Sec. 5 "MuLoCo": 0.9)
    eta_in: float = 6.25e-2
    weight_decay: float = 1.25e-3
    eta_out: float = 0.7
    mu: float = 0.9
    quant_bits: int = 0

    def shape_groups(self) -> List[Tuple[int, int, int]]:
        """(count, m, n) for every group of same-shape 2-D matrices."""
        L, d, f = self.layers, self.d_model, self.d_ffn
        return [(4 * L, d, d), (L, d, f), (L, f, d)]

    def n_params(self) -> int:
        return sum(c * m * n for c, m, n in self.shape_groups())


# Hyper-parameters not fixed by the workload descriptions are taken from the paper's
# table of optimal MuLoCo hyper-parameters (150M rows): K=1 -> eta_in 6.25e-2,
# lambda 1.25e-3; K=8 -> eta_in 1.25e-1, lambda 6.25e-4, eta_out 0.9, mu 0.8;
# K=4 -> eta_in 8.84e-2, lambda 6.25e-4, eta_out 0.9, mu 0.8.
WORKLOADS: Dict[str, Workload] = {
    "tiny": Workload("tiny", 2, 128, 512, K=1, H=8, param_dtype="f32", beta=0.95,
                     eta_out=0.7, mu=0.9),
    "150m": Workload("150m", 12, 768, 3072, K=8, H=30, param_dtype="bf16",
                     eta_in=1.25e-1, weight_decay=6.25e-4, eta_out=0.9, mu=0.8),
    "1.76b": Workload("1.76b", 24, 2048, 8192, K=1, H=30, param_dtype="bf16"),
    "3.1b": Workload("3.1b", 32, 2560, 10240, K=4, H=30, param_dtype="bf16",
                     eta_in=8.84e-2, weight_decay=6.25e-4, eta_out=0.9, mu=0.8,
                     quant_bits=4),
    "15b": Workload("15b", 48, 5120, 20480, K=1, H=30, param_dtype="bf16"),
}

PARAM_STD = 0.02
GRAD_STD = 1e-3
DELTA_STD = 1e-2


def _generator(seed: int, stream: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    # distinct, reproducible sub-streams: one per (seed, stream id)
    g.manual_seed((int(seed) * 1_000_003 + int(stream) * 7919 + 12345) % (2 ** 63 - 1))
    return g


def normal(shape, std: float, seed: int, stream: int, device="cpu",
           dtype=torch.float32) -> torch.Tensor:
    """std * N(0,1) of the given shape, drawn in fp32 then cast to `dtype`.

    The same (seed, stream) gives the same values on the same device type; CPU and
    GPU streams differ, so a parity test draws on one device and copies."""
    g = _generator(seed, stream, device)
    x = torch.randn(shape, generator=g, device=device, dtype=torch.float32)
    return (x * std).to(dtype)


def torch_dtype(name: str):
    return {"f32": torch.float32, "bf16": torch.bfloat16}[name]
