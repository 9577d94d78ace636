"""The boundary transform as one differentiable PyTorch operation.

The paper's boundary communicator is an autograd-aware operation: its forward
materialises the source module's activation in the destination layout and its
backward applies the reverse transform (Method, paragraph on boundary edges).
This module only strings the library's calls together for torch.autograd -
every tensor element is still moved by the HIP kernels behind hp_forward,
hp_backward and hp_zero_image_rows:

    outs = boundary_transform(plan, src_bufs, text_bufs)

`text_bufs` are the destination buffers already holding the text embeddings;
they are modified in place (the image-token rows are overwritten) and returned.
Backward gives, for every source buffer, the TP-summed gradient of its rows (all
TP copies of a source rank receive the same gradient) and, for every text
buffer, the incoming gradient with the image-token rows set to zero.
"""
from __future__ import annotations

from typing import List, Sequence

import torch

from .binding import Plan


class _BoundaryTransform(torch.autograd.Function):
    @staticmethod
    def forward(ctx, plan: Plan, n_src: int, *bufs):
        src, dst = list(bufs[:n_src]), list(bufs[n_src:])
        stream = torch.cuda.current_stream()
        plan.forward([t.detach() if t is not None else None for t in src], [t.detach() for t in dst], stream)
        ctx.plan, ctx.n_src = plan, n_src
        ctx.src_meta = [(tuple(t.shape), t.dtype, t.device) for t in src]
        ctx.mark_dirty(*dst)
        return tuple(dst)

    @staticmethod
    def backward(ctx, *grad_dst):
        plan, stream = ctx.plan, torch.cuda.current_stream()
        grads = [g.contiguous() for g in grad_dst]
        src_grads: List[torch.Tensor] = [torch.empty(shape, dtype=dtype, device=device)
                                         for shape, dtype, device in ctx.src_meta]
        plan.backward(grads, src_grads, stream)
        # gradient with respect to the text embeddings: the rows forward replaced carry none
        text_grads = [g.clone() for g in grads]
        plan.zero_image_rows(text_grads, stream)
        return (None, None, *src_grads, *text_grads)


def boundary_transform(plan: Plan, src_bufs: Sequence[torch.Tensor], text_bufs: Sequence[torch.Tensor]):
    """Differentiable hp_forward: returns the destination buffers (the same
    tensors as `text_bufs`, modified in place) as a tuple.  Every source buffer
    must be a tensor (empty ranks: a [0, hidden] tensor).  Runs on torch's
    current stream."""
    if len(src_bufs) != plan.info.n_src_bufs or len(text_bufs) != plan.info.n_dst_bufs:
        raise ValueError("wrong number of buffers for this plan")
    return _BoundaryTransform.apply(plan, len(src_bufs), *src_bufs, *text_bufs)
