"""torch.autograd wrapper around the C-ABI operator (Sec. 3.3 of arXiv 2511.13645:
``save_indices`` records the sampled IDs in forward and replays them in backward, so that
gradients reach the same sampled neighborhoods).

Only glue: forward calls ``fsa_sample_mean_fwd``, backward calls ``fsa_mean_bwd`` on the IDs
saved by that forward.  IDs are emitted only when the feature table needs a gradient (or the
caller asks for them), as in the paper's optional flag.
"""
from __future__ import annotations

from typing import Optional, Sequence, Tuple

import torch

from . import binding


class _FusedSampleMean(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, indptr, indices, seeds, fanouts, seed, want_h1, save_indices):
        fan = [int(k) for k in fanouts]
        need_ids = bool(save_indices or x.requires_grad)
        out, h1, ids1, ids2 = binding.fsa_sample_mean_fwd(indptr, indices, x, seeds, fan, seed,
                                                          emit_h1=bool(want_h1) and len(fan) == 2,
                                                          emit_ids=need_ids)
        ctx.shape = tuple(x.shape)
        ctx.x_dtype = x.dtype
        ctx.hops = len(fan)
        ctx.save_for_backward(*(t for t in (ids1, ids2) if t is not None))
        ctx.mark_non_differentiable(*(t for t in (ids1, ids2) if t is not None))
        empty = x.new_empty(0)
        return (out,
                h1 if h1 is not None else empty,
                ids1 if ids1 is not None else empty.to(torch.int32),
                ids2 if ids2 is not None else empty.to(torch.int32))

    @staticmethod
    def backward(ctx, g_out, g_h1, _g_ids1, _g_ids2):
        saved = ctx.saved_tensors
        if not saved:
            raise RuntimeError("backward needs the sampled IDs: call with save_indices=True or a table that requires grad")
        ids1 = saved[0]
        ids2 = saved[1] if ctx.hops == 2 else None
        if ctx.x_dtype != torch.float32:
            raise RuntimeError("the backward pass accumulates into an fp32 table only")
        grad_x = torch.zeros(ctx.shape, dtype=torch.float32, device=g_out.device)
        gh = None
        if ctx.hops == 2 and g_h1 is not None and g_h1.numel() > 0:
            gh = g_h1.contiguous().float()
        binding.fsa_mean_bwd(g_out.contiguous().float(), ids1, ids2, gh, grad_x=grad_x)
        return grad_x, None, None, None, None, None, None, None


def fused_sample_mean(x: torch.Tensor, indptr: torch.Tensor, indices: torch.Tensor, seeds: torch.Tensor,
                      fanouts: Sequence[int], seed: int, *, want_h1: bool = False, save_indices: bool = False
                      ) -> Tuple[torch.Tensor, Optional[torch.Tensor], Optional[torch.Tensor], Optional[torch.Tensor]]:
    """Differentiable fused sample + mean.  Returns (out, out_h1 | None, ids1 | None, ids2 | None)."""
    out, h1, ids1, ids2 = _FusedSampleMean.apply(x, indptr, indices, seeds, tuple(fanouts), int(seed),
                                                 bool(want_h1), bool(save_indices))
    return (out, h1 if h1.numel() or (want_h1 and len(fanouts) == 2 and seeds.numel() == 0) else None,
            ids1 if ids1.numel() else None, ids2 if ids2.numel() else None)
