"""Autograd glue for one MaxK aggregation: Y = A * MaxK_k(H)  (training dataflow of Sec. 3.2, Eq. 2).

Forward : maxk_topk_cbsr -> maxk_spgemm_fwd.
Backward: maxk_sspmm_bwd (gradient only at the CBSR support) -> maxk_cbsr_scatter back to dense.
Every step runs in the HIP kernels; torch provides tensors, the stream and the autograd tape.
"""
from __future__ import annotations

import torch

from . import binding as _b


class MaxKAggregate(torch.autograd.Function):
    @staticmethod
    def forward(ctx, H: torch.Tensor, graph: _b.MaxKGraph, k: int, index_bytes: int = 0):
        N, dim = H.shape
        ib = index_bytes or (1 if dim <= 256 else 2 if dim <= 65536 else 4)
        H = H.contiguous()
        sp_data = torch.empty((N, k), dtype=torch.float32, device=H.device)
        sp_index = torch.empty((N, k), dtype=_b.index_dtype(ib), device=H.device)
        Y = torch.empty((N, dim), dtype=torch.float32, device=H.device)
        _b.maxk_topk_cbsr(H, k, sp_data, sp_index)
        _b.maxk_spgemm_fwd(graph, sp_data, sp_index, dim, Y)
        ctx.graph, ctx.dim, ctx.k = graph, dim, k
        ctx.save_for_backward(sp_index)
        return Y

    @staticmethod
    def backward(ctx, dY: torch.Tensor):
        (sp_index,) = ctx.saved_tensors
        N = sp_index.shape[0]
        dXs = torch.empty((N, ctx.k), dtype=torch.float32, device=dY.device)
        dH = torch.empty((N, ctx.dim), dtype=torch.float32, device=dY.device)
        _b.maxk_sspmm_bwd(ctx.graph, dY.contiguous(), sp_index, dXs)
        _b.maxk_cbsr_scatter(dXs, sp_index, dH)
        return dH, None, None, None


def maxk_aggregate(H: torch.Tensor, graph: _b.MaxKGraph, k: int) -> torch.Tensor:
    """Y = A * MaxK_k(H), differentiable with respect to H."""
    return MaxKAggregate.apply(H, graph, k)
