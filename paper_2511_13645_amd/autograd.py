"""torch.autograd wrapper around the C-ABI operator (Sec. 3.3 of arXiv 2511.13645:
``save_indices`` records the sampled IDs in forward and replays them in backward, so that
gradients reach the same sampled neighborhoods).

Only glue: forward calls ``fsa_sample_mean_fwd``, backward calls ``fsa_mean_bwd`` (fp32) or
``fsa_mean_bwd_lp`` (16-bit tables or gradients) on the IDs saved by that forward.  IDs are
emitted only when the feature table needs a gradient (or the caller asks for them), as in the
paper's optional flag.

A bf16 / fp16 table gets its gradient in its own type, added with packed 16-bit atomics, or --
when the caller passes ``master_grad``, an fp32 [N,D] tensor -- the backward accumulates into
that master gradient instead and leaves ``x.grad`` unset.  ``workspace`` (any contiguous GPU
tensor, optional) goes to ``fsa_mean_bwd_ws``: wide-row 2-hop backward passes over an fp32 table
then update every destination row once instead of once per sampled leaf.
"""
from __future__ import annotations

from typing import Optional, Sequence, Tuple

import torch

from . import binding


class _FusedSampleMean(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, indptr, indices, seeds, fanouts, seed, want_h1, save_indices, master_grad, workspace):
        fan = [int(k) for k in fanouts]
        need_ids = bool(save_indices or x.requires_grad)
        out, h1, ids1, ids2 = binding.fsa_sample_mean_fwd(indptr, indices, x, seeds, fan, seed,
                                                          emit_h1=bool(want_h1) and len(fan) == 2,
                                                          emit_ids=need_ids)
        ctx.shape = tuple(x.shape)
        ctx.x_dtype = x.dtype
        ctx.hops = len(fan)
        ctx.master_grad = master_grad
        ctx.workspace = workspace
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
        gh = None
        if ctx.hops == 2 and g_h1 is not None and g_h1.numel() > 0:
            gh = g_h1.contiguous()
        g_out = g_out.contiguous()
        if ctx.master_grad is not None:
            binding.fsa_mean_bwd_lp(g_out, ids1, ids2, gh, grad_x=ctx.master_grad)
            return (None,) * 10
        if ctx.x_dtype == torch.float32:
            grad_x = torch.zeros(ctx.shape, dtype=torch.float32, device=g_out.device)
            binding.fsa_mean_bwd_ws(g_out.float(), ids1, ids2, None if gh is None else gh.float(), grad_x=grad_x,
                                    workspace=ctx.workspace)
        elif ctx.shape[1] % 2 == 0:
            grad_x = torch.zeros(ctx.shape, dtype=ctx.x_dtype, device=g_out.device)
            binding.fsa_mean_bwd_lp(g_out, ids1, ids2, gh, grad_x=grad_x)
        else:                                   # packed atomics take element pairs: odd D goes through fp32
            master = torch.zeros(ctx.shape, dtype=torch.float32, device=g_out.device)
            binding.fsa_mean_bwd_lp(g_out, ids1, ids2, gh, grad_x=master)
            grad_x = master.to(ctx.x_dtype)
        return (grad_x,) + (None,) * 9


def fused_sample_mean(x: torch.Tensor, indptr: torch.Tensor, indices: torch.Tensor, seeds: torch.Tensor,
                      fanouts: Sequence[int], seed: int, *, want_h1: bool = False, save_indices: bool = False,
                      master_grad: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None
                      ) -> Tuple[torch.Tensor, Optional[torch.Tensor], Optional[torch.Tensor], Optional[torch.Tensor]]:
    """Differentiable fused sample + mean.  Returns (out, out_h1 | None, ids1 | None, ids2 | None).
    `master_grad` (fp32 [N,D], optional): backward accumulates the table's gradient into it.
    `workspace` (optional, see binding.fsa_mean_bwd_workspace_bytes): lets the fp32 backward own its rows."""
    if master_grad is not None and (master_grad.dtype != torch.float32 or tuple(master_grad.shape) != tuple(x.shape)):
        raise ValueError("master_grad must be an fp32 tensor of the table's shape")
    out, h1, ids1, ids2 = _FusedSampleMean.apply(x, indptr, indices, seeds, tuple(fanouts), int(seed),
                                                 bool(want_h1), bool(save_indices), master_grad, workspace)
    return (out, h1 if h1.numel() or (want_h1 and len(fanouts) == 2 and seeds.numel() == 0) else None,
            ids1 if ids1.numel() else None, ids2 if ids2.numel() else None)
