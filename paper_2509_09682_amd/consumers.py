"""Other consumers of the indexed log-sum-exp kernels (marshalling only: every score, softmax and gradient comes from the
C-ABI calls).

bucketed_step: losses whose candidate sets are chosen per BUCKET of positions rather than per batch or per position.
The paper's Sec. 5 ("Comparison Sampling Strategies") names the Scalable Cross-Entropy loss as a case in point: it
groups positions into buckets, picks for each bucket the catalogue items with the largest scores under a cheap proxy,
and takes the cross-entropy of every position over its bucket's items plus its own correct item; the paper notes that
such a loss could run on kernels that need nothing but the indices of the correct and the selected items.  That is the
shared-negatives mode of this library applied bucket by bucket: the positions are brought into bucket order once (a
row gather of H, plain data movement), each bucket is one forward and one backward call on its contiguous slice with its
own candidate list, the table gradient of all buckets accumulates into the same buffer, and the per-position results
are put back in batch order.  How the buckets and their candidates are chosen is the caller's business.
"""
from __future__ import annotations

from typing import Optional, Sequence

import torch

from . import binding as B


def bucketed_step(H: torch.Tensor, E: torch.Tensor, tgt: torch.Tensor, order: torch.Tensor, bucket_ptr: Sequence[int],
                  bucket_neg: torch.Tensor, grad_loss: Optional[torch.Tensor], dE: torch.Tensor, *,
                  mask_target_collisions: bool = True):
    """Forward + backward of the loss with one candidate list per bucket of positions.

    H [N,d], E [V,d] (both float32 or both bfloat16), tgt [N] int32.
    order      [M] int64: the positions that take part, sorted by bucket (positions left out, e.g. padding, get
               loss = lse = 0 and a zero dH row);
    bucket_ptr B + 1 offsets into `order` (host integers): bucket b owns order[bucket_ptr[b]:bucket_ptr[b+1]];
    bucket_neg [B, Kb] int32: the candidate items of every bucket (a position's own correct item is scored besides);
    grad_loss  [N] float32 upstream gradient of the per-position loss, or None for 1;
    dE         [V,d] float32, ACCUMULATED INTO.
    Returns (loss [N], lse [N], dH [N,d]) in batch order, dH in H's dtype.
    """
    N, d = H.shape
    V = E.shape[0]
    n_buckets, Kb = bucket_neg.shape
    if len(bucket_ptr) != n_buckets + 1 or bucket_ptr[0] != 0 or bucket_ptr[-1] != order.numel():
        raise ValueError("bucket_ptr must hold B + 1 offsets covering `order`")
    dt = B.CCE_F32 if H.dtype == torch.float32 else B.CCE_BF16
    Hs = H.index_select(0, order).contiguous()          # positions in bucket order: slices are contiguous
    ts = tgt.index_select(0, order).contiguous()
    gs = None if grad_loss is None else grad_loss.index_select(0, order).contiguous()
    M = order.numel()
    loss_s = torch.empty(M, device=H.device, dtype=torch.float32)
    lse_s = torch.empty(M, device=H.device, dtype=torch.float32)
    dH_s = torch.empty((M, d), device=H.device, dtype=H.dtype)
    largest = max((bucket_ptr[b + 1] - bucket_ptr[b] for b in range(n_buckets)), default=0)
    ws = None
    if largest > 0:
        ws = B.new_workspace(B.make_desc(largest, V, d, Kb, dt, B.CCE_NEG_SHARED, dH_dtype=dt,
                                         mask_target_collisions=int(mask_target_collisions), fuse_dH=1), device=H.device)
    for b in range(n_buckets):
        b0, b1 = int(bucket_ptr[b]), int(bucket_ptr[b + 1])
        if b1 == b0:
            continue
        kw = dict(dH_dtype=dt, mask_target_collisions=int(mask_target_collisions), fuse_dH=1)
        desc = B.make_desc(b1 - b0, V, d, Kb, dt, B.CCE_NEG_SHARED, **kw)
        desc_b = B.make_desc(b1 - b0, V, d, Kb, dt, B.CCE_NEG_SHARED, reuse_forward_prep=1, **kw)
        neg = bucket_neg[b]
        B.cce_neg_forward(desc, Hs[b0:b1], E, ts[b0:b1], neg, None, loss_s[b0:b1], lse_s[b0:b1], ws)
        B.cce_neg_backward(desc_b, Hs[b0:b1], E, ts[b0:b1], neg, None, lse_s[b0:b1], None if gs is None else gs[b0:b1],
                           dH_s[b0:b1], dE, ws)
    loss = torch.zeros(N, device=H.device, dtype=torch.float32)
    lse = torch.zeros(N, device=H.device, dtype=torch.float32)
    dH = torch.zeros((N, d), device=H.device, dtype=H.dtype)
    loss.index_copy_(0, order, loss_s)
    lse.index_copy_(0, order, lse_s)
    dH.index_copy_(0, order, dH_s)
    return loss, lse, dH
