"""The five synthetic workloads (graph + features + parameters), as inputs only.

Each builder returns a `Workload` whose tensors live on the requested device.
Where a workload asks for degree-ordered vertex ids, the permutation is not
computed here: the caller passes `reorder(off, col) -> new_of_old` (the GPU
library's routine in the benchmark, the CPU checker's in CPU tests), and this
module only applies it.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Callable, List, Optional

import torch

from . import (EdgeSource, LayerParams, build_csr, features, layer_params, permute_rows, rmat_graph,
               uniform_graph)

SEED0 = 0x5EED0000


@dataclass
class Workload:
    name: str
    model: str                 # "sage" | "gcn" | "gat" | "gin"
    off: torch.Tensor          # int64 [n+1]
    col: torch.Tensor          # int32 [E]
    X: torch.Tensor            # [n, d0], storage dtype
    layers: List[LayerParams]  # fp64 masters rounded to the storage dtype
    dims: List[int]
    chunk: int
    store: torch.dtype
    act: str
    heads: int = 1
    new_of_old: Optional[torch.Tensor] = None
    notes: dict = field(default_factory=dict)

    @property
    def n(self) -> int:
        return self.off.numel() - 1

    @property
    def e(self) -> int:
        return self.col.numel()


Reorder = Callable[[torch.Tensor, torch.Tensor], torch.Tensor]


def _short(store: torch.dtype) -> str:
    return {torch.bfloat16: "bf16", torch.float16: "f16", torch.float32: "fp32"}[store]


def _finish(name, model, g: EdgeSource, seed, dims, chunk, feat, store, act, device, heads=1,
            reorder: Optional[Reorder] = None) -> Workload:
    off, col = build_csr(g, device)
    new_of_old = None
    if reorder is not None:
        new_of_old = reorder(off, col).to(torch.int64)
        del off, col
        g = g.with_relabel(new_of_old)
        off, col = build_csr(g, device)
    X = features(seed, g.n, dims[0], feat, store, device)
    if new_of_old is not None:
        X = permute_rows(X, new_of_old)
    layers = [layer_params(seed, li, model, dims[li], dims[li + 1], heads).rounded(store)
              for li in range(len(dims) - 1)]
    return Workload(name, model, off, col, X, layers, dims, chunk, store, act, heads, new_of_old)


def config1(device="cpu") -> Workload:
    """Tiny GraphSAGE-mean, fp32: 10,000 vertices, 100,000 uniform edges."""
    seed = SEED0 + 1
    return _finish("config1_tiny_sage_fp32", "sage", uniform_graph(seed, 10_000, 100_000, device), seed,
                   [64, 64, 16], 1024, "uniform", torch.float32, "relu", device)


def config2(device="cpu", scale: int = 20, reorder: Optional[Reorder] = None, chunk: Optional[int] = None) -> Workload:
    """GCN on R-MAT, fp32, random ids, one self-loop per vertex; optional degree ordering."""
    seed = SEED0 + 2
    g = rmat_graph(seed, scale, 16, random_ids=True, self_loops=True, device=device)
    return _finish("config2_gcn_rmat%d_fp32" % scale, "gcn", g, seed, [128, 128, 64],
                   chunk or max(64, (1 << scale) // 16), "normal", torch.float32, "relu", device, reorder=reorder)


def config3(device="cpu", scale: int = 22, chunk: Optional[int] = None) -> Workload:
    """GraphSAGE-mean on R-MAT, bf16 storage, d = 256, three layers."""
    seed = SEED0 + 3
    g = rmat_graph(seed, scale, 25, device=device)
    return _finish("config3_sage_rmat%d_bf16" % scale, "sage", g, seed, [256, 256, 256, 128],
                   chunk or max(64, (1 << scale) // 16), "uniform", torch.bfloat16, "relu", device)


def config4(device="cpu", scale: int = 22, chunk: Optional[int] = None) -> Workload:
    """GAT, 4 heads x 32, fp32, two layers."""
    seed = SEED0 + 4
    g = rmat_graph(seed, scale, 16, device=device)
    return _finish("config4_gat_rmat%d_fp32" % scale, "gat", g, seed, [128, 128, 128],
                   chunk or max(64, (1 << scale) // 16), "normal", torch.float32, "elu", device, heads=4)


def config5(device="cpu", scale: int = 26, reorder: Optional[Reorder] = None, chunk: Optional[int] = None,
            edge_factor: int = 32, model: str = "sage", store: torch.dtype = torch.bfloat16) -> Workload:
    """Large GraphSAGE-mean on R-MAT, bf16, d = 128, degree-ordered ids
    (model="gin": the same graph and widths through GIN layers; store=float16:
    IEEE half storage, the format of the paper's larger feature sets)."""
    seed = SEED0 + 5
    g = rmat_graph(seed, scale, edge_factor, device=device)
    return _finish("config5_%s_rmat%d_%s" % (model, scale, _short(store)), model, g, seed, [128, 128, 128, 64],
                   chunk or max(64, (1 << scale) // 16), "uniform", store, "relu", device, reorder=reorder)


def wide(device="cpu", scale: int = 22, d_in: int = 512, reorder: Optional[Reorder] = None,
         chunk: Optional[int] = None, store: torch.dtype = torch.bfloat16) -> Workload:
    """Wide 16-bit input features into a narrow hidden layer, the shape of the first
    layer on the paper's MAG240M / IGB feature sets (768 / 1024 wide, Sec. 4.1):
    GraphSAGE-mean d_in -> 128 -> 128 on R-MAT, bf16, edge factor 16."""
    seed = SEED0 + 6
    g = rmat_graph(seed, scale, 16, device=device)
    return _finish("wide%d_sage_rmat%d_%s" % (d_in, scale, _short(store)), "sage", g, seed, [d_in, 128, 128],
                   chunk or max(64, (1 << scale) // 16), "uniform", store, "relu", device, reorder=reorder)
