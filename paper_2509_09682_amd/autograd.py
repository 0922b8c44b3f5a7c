"""torch.autograd front end of the C ABI: the loss as a differentiable function of the hidden states and the item table.

Nothing of the method is computed here: forward() calls cce_neg_forward, backward() calls cce_neg_backward with the
upstream gradient of the per-position loss vector (the paper's grad-LSE, Sec. 3.3), and the scalar reduction of Eq. 3
is ordinary torch arithmetic on that vector, so its 1/N reaches the kernels through autograd as `grad_loss`.
"""
from __future__ import annotations

import collections
from typing import Optional

import torch

from . import binding as B

_workspaces: "collections.OrderedDict" = collections.OrderedDict()   # least recently used first
_last_forward: dict = {}      # workspace key -> serial number of the forward call that filled it last
_serial = 0
MAX_CACHED_WORKSPACES = 4     # shapes in use at a time (training + evaluation batch shapes); older ones are released


def clear_workspaces() -> None:
    """Releases every cached workspace (they are re-created on demand)."""
    _workspaces.clear()
    _last_forward.clear()


def _workspace(desc: B.CceDesc, device):
    """One workspace per descriptor shape, device and stream; forward and backward of a step share it.  At most
    MAX_CACHED_WORKSPACES are kept; a pending backward call holds its own reference, so eviction never pulls a
    workspace from under it."""
    key = (desc.N, desc.V, desc.d, desc.K, desc.in_dtype, desc.dH_dtype, desc.neg_mode, desc.mask_target_collisions,
           desc.validate_indices, desc.algo, desc.fuse_dH, str(device), int(torch.cuda.current_stream(device).cuda_stream))
    ws = _workspaces.pop(key, None)
    if ws is None:
        ws = B.new_workspace(desc, device=device)
    _workspaces[key] = ws          # most recently used last
    while len(_workspaces) > MAX_CACHED_WORKSPACES:
        old, _ = _workspaces.popitem(last=False)
        _last_forward.pop(old, None)
    return key, ws


class _CceNegLoss(torch.autograd.Function):
    @staticmethod
    def forward(ctx, H, E, tgt, neg, mask, neg_mode, mask_target_collisions, filter_eps, sampler, n_neg, grad_E_out):
        if H.dtype != E.dtype or H.dtype not in (torch.float32, torch.bfloat16):
            raise TypeError("H and E must both be float32 or both be bfloat16")
        N, d = H.shape
        V = E.shape[0]
        if sampler is not None:
            K = int(n_neg)
        else:
            K = 0 if neg is None or neg_mode == B.CCE_NEG_FULL else int(neg.shape[-1])
        dt = B.CCE_F32 if H.dtype == torch.float32 else B.CCE_BF16
        # fuse_dH: the forward call also forms the hidden-state gradient short of grad_loss (one pass over the candidates
        # less per step); only worth it when a backward call will follow, and not with gradient filtering
        wants_grad = ctx.needs_input_grad[0] or ctx.needs_input_grad[1] or grad_E_out is not None
        fuse = 1 if (wants_grad and not filter_eps > 0) else 0
        if grad_E_out is not None and (grad_E_out.dtype != torch.float32 or tuple(grad_E_out.shape) != tuple(E.shape)
                                       or not grad_E_out.is_contiguous() or grad_E_out.device != E.device):
            raise ValueError("grad_E_out must be a contiguous float32 tensor of E's shape on E's device")
        ctx.grad_E_out = grad_E_out
        kw = dict(dH_dtype=dt, mask_target_collisions=1 if mask_target_collisions else 0, fuse_dH=fuse)
        desc = B.make_desc(N, V, d, K, dt, neg_mode, **kw)
        B.check_step_args(desc, H, E, tgt, neg, mask, sampled=sampler is not None)   # before anything touches the device
        global _serial
        key, ws = _workspace(desc, H.device)
        _serial += 1
        _last_forward[key] = ctx.serial = _serial
        ctx.key = key
        H, E = H.contiguous(), E.contiguous()
        loss = torch.empty(N, device=H.device, dtype=torch.float32)
        lse = torch.empty(N, device=H.device, dtype=torch.float32)
        if sampler is not None:
            B.cce_neg_forward_sampled(desc, sampler, H, E, tgt, mask, loss, lse, ws)
        else:
            B.cce_neg_forward(desc, H, E, tgt, neg, mask, loss, lse, ws)
        ctx.sampler = sampler   # the backward call draws the same ids again
        ctx.save_for_backward(H, E, tgt, neg, mask, lse)
        ctx.bwd = (N, V, d, K, dt, neg_mode, filter_eps, kw)
        ctx.ws = ws
        return loss

    @staticmethod
    def backward(ctx, grad_loss):
        H, E, tgt, neg, mask, lse = ctx.saved_tensors
        dH = torch.empty_like(H)
        # The library accumulates dE into an fp32 [V,d] buffer and touches only the rows that were indexed.  A caller
        # that holds such a buffer (grad_E_out: its own fp32 gradient accumulator) gets the rows added in place and no
        # gradient tensor for E from autograd; otherwise a dense buffer is zeroed, filled and converted to E's dtype,
        # which for a large table costs more than the loss itself.
        own = ctx.grad_E_out is None
        dE = torch.zeros(E.shape, device=E.device, dtype=torch.float32) if own else ctx.grad_E_out
        g = grad_loss.contiguous().to(torch.float32)
        N, V, d, K, dt, neg_mode, filter_eps, kw = ctx.bwd
        # the compaction the forward call left in the workspace is reused unless another forward call of the same
        # shape has overwritten it since (two loss terms in one graph)
        reuse = 1 if _last_forward.get(ctx.key) == ctx.serial else 0
        if not reuse:
            _last_forward[ctx.key] = None   # this call rewrites the workspace: it no longer holds any forward call's state
        desc = B.make_desc(N, V, d, K, dt, neg_mode, reuse_forward_prep=reuse, filter_eps=filter_eps, **kw)
        if ctx.sampler is not None:
            B.cce_neg_backward_sampled(desc, ctx.sampler, H, E, tgt, mask, lse, g, dH, dE, ctx.ws)
        else:
            B.cce_neg_backward(desc, H, E, tgt, neg, mask, lse, g, dH, dE, ctx.ws)
        return dH, (dE.to(E.dtype) if own else None), None, None, None, None, None, None, None, None, None


def cce_neg_loss(H: torch.Tensor, E: torch.Tensor, tgt: torch.Tensor, neg: Optional[torch.Tensor] = None,
                 mask: Optional[torch.Tensor] = None, *, neg_mode: int = B.CCE_NEG_SHARED, reduction: str = "mean",
                 mask_target_collisions: bool = True, filter_eps: float = 0.0, sampler: Optional[B.CceSampler] = None,
                 n_neg: int = 0, grad_E_out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Cross-entropy with negative sampling (Eq. 3-5), or over the full catalogue with neg_mode = CCE_NEG_FULL (Eq. 1-2).

    H [N,d] hidden states, E [V,d] item table (both float32 or both bfloat16, CUDA), tgt [N] int32, neg [K] or [N,K]
    int32, mask [N] uint8 (1 = valid).  reduction: "none" (per-position vector, 0 at padded positions), "sum", or
    "mean" over the valid positions (Eq. 3).  Gradients flow to H and E.

    sampler (binding.make_sampler) with n_neg = K instead of neg: the negatives are drawn inside the kernels, in the
    forward and again in the backward pass, and no index tensor exists; give the sampler another `stream` every step.

    grad_E_out: a float32 [V,d] tensor held by the caller (a gradient accumulator for the item table).  The backward
    pass then ADDS the table gradient into it, touching only the rows of the targets and negatives of this batch (the
    gradient of the classifier is non-zero only at the indexed columns, Sec. 3.3), and autograd delivers no gradient
    for E.  Without it the backward pass zeroes and converts a dense [V,d] tensor every step.  Mixed precision: an
    upstream gradient scaled by a loss scale (torch.amp.GradScaler) passes through unchanged in fp32, so both gradients
    carry the scale exactly; inf / NaN from an overflowed scale reach dH and the touched rows of dE, where the scaler's
    check finds them.
    """
    if sampler is not None:
        sampler = B.CceSampler(sampler.kind, sampler.stream, sampler.seed, sampler.alias_thresh, sampler.alias_id)  # frozen copy
    loss = _CceNegLoss.apply(H, E, tgt, neg, mask, neg_mode, mask_target_collisions, filter_eps, sampler, n_neg, grad_E_out)
    if reduction == "none":
        return loss
    if reduction == "sum":
        return loss.sum()
    if reduction == "mean":
        n_valid = loss.numel() if mask is None else mask.to(torch.float32).sum().clamp_min(1.0)
        return loss.sum() / n_valid
    raise ValueError(reduction)
