"""Moves a seeded workload (workloads.Workload: numpy arrays) into device memory and runs it through the C ABI.

Argument marshalling only, for the tests, the smoke check and the benchmark; no arithmetic of the method lives here.
"""
from __future__ import annotations

from typing import Optional

import numpy as np
import torch

from . import binding as P


def to_device(w):
    dev = "cuda"
    if w.in_dtype == "f32":
        H = torch.from_numpy(w.H).to(dev)
        E = torch.from_numpy(w.E).to(dev)
    else:  # uint16 bit patterns -> same bits in device memory
        H = torch.from_numpy(w.H.view(np.int16)).to(dev)
        E = torch.from_numpy(w.E.view(np.int16)).to(dev)
    tgt = torch.from_numpy(w.tgt).to(dev)
    neg = None if w.neg is None else torch.from_numpy(np.ascontiguousarray(w.neg)).to(dev)
    mask = None if w.mask is None else torch.from_numpy(w.mask).to(dev)
    return H, E, tgt, neg, mask


def run_hip(w, *, g: Optional[np.ndarray] = "workload", algo=P.CCE_ALGO_AUTO, dH_dtype=P.CCE_F32, validate=0,
            use_mask=True, dE_init: Optional[np.ndarray] = None, repeat_backward: int = 1, reuse_prep: bool = False,
            filter_eps: float = 0.0, fuse_dH: bool = False):
    """Forward + backward on cuda:0.  Returns dict(loss, lse, dH (float32), dE (float32), status)."""
    H, E, tgt, neg, mask = to_device(w)
    if not use_mask:
        mask = None
    desc = P.make_desc(w.N, w.V, w.d, w.K, P.CCE_F32 if w.in_dtype == "f32" else P.CCE_BF16, w.neg_mode,
                       dH_dtype=dH_dtype, mask_target_collisions=w.mask_collisions, validate_indices=validate, algo=algo,
                       fuse_dH=1 if fuse_dH else 0)
    desc_bwd = P.make_desc(w.N, w.V, w.d, w.K, P.CCE_F32 if w.in_dtype == "f32" else P.CCE_BF16, w.neg_mode,
                           dH_dtype=dH_dtype, mask_target_collisions=w.mask_collisions, validate_indices=validate,
                           algo=algo, reuse_forward_prep=1 if reuse_prep else 0, filter_eps=filter_eps,
                           fuse_dH=1 if fuse_dH else 0)
    ws = P.new_workspace(desc)
    loss = torch.full((w.N,), float("nan"), device="cuda")
    lse = torch.full((w.N,), float("nan"), device="cuda")
    P.cce_neg_forward(desc, H, E, tgt, neg, mask, loss, lse, ws)
    if isinstance(g, str):
        g_t = torch.from_numpy(w.g).to("cuda")
    elif g is None:
        g_t = None
    else:
        g_t = torch.from_numpy(np.asarray(g, np.float32)).to("cuda")
    if dH_dtype == P.CCE_BF16:
        dH = torch.full((w.N, w.d), float("nan"), device="cuda", dtype=torch.bfloat16)
    else:
        dH = torch.full((w.N, w.d), float("nan"), device="cuda")
    dE = torch.zeros((w.V, w.d), device="cuda") if dE_init is None else torch.from_numpy(dE_init).to("cuda")
    for _ in range(repeat_backward):
        P.cce_neg_backward(desc_bwd, H, E, tgt, neg, mask, lse, g_t, dH, dE, ws)
    status = P.cce_neg_index_status(ws)
    torch.cuda.synchronize()
    return dict(loss=loss.cpu().numpy(), lse=lse.cpu().numpy(), dH=dH.float().cpu().numpy(), dE=dE.cpu().numpy(),
                status=status)


def device_sampler(kind, seed, stream, thresh=None, alias=None):
    """Sampler descriptor plus the device tensors it borrows (keep the tuple alive while the sampler is used)."""
    keep = []
    th = al = None
    if thresh is not None:
        th = torch.from_numpy(thresh.view(np.int32)).to("cuda")   # same 32-bit words
        al = torch.from_numpy(alias).to("cuda")
        keep = [th, al]
    return P.make_sampler(kind, seed, stream, th, al), keep


def sample_hip(w, smp):
    """The ids the library's sampler denotes for the workload's shape: numpy int32 [K] or [N,K]."""
    desc = P.make_desc(w.N, w.V, w.d, w.K, P.CCE_F32 if w.in_dtype == "f32" else P.CCE_BF16, w.neg_mode)
    shape = (w.K,) if w.neg_mode == P.CCE_NEG_SHARED else (w.N, w.K)
    out = torch.full(shape, -7, dtype=torch.int32, device="cuda")
    P.cce_neg_sample(desc, smp, out)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def run_hip_sampled(w, smp, *, algo=P.CCE_ALGO_AUTO, dH_dtype=P.CCE_F32, fuse_dH: bool = False):
    """Forward + backward through the *_sampled calls (w.neg is ignored).  Same result dict as run_hip.
    fuse_dH: the forward call also forms the hidden-state gradient; the backward call reuses what it left."""
    H, E, tgt, _, mask = to_device(w)
    desc = P.make_desc(w.N, w.V, w.d, w.K, P.CCE_F32 if w.in_dtype == "f32" else P.CCE_BF16, w.neg_mode,
                       dH_dtype=dH_dtype, mask_target_collisions=w.mask_collisions, algo=algo,
                       fuse_dH=1 if fuse_dH else 0)
    desc_bwd = P.make_desc(w.N, w.V, w.d, w.K, P.CCE_F32 if w.in_dtype == "f32" else P.CCE_BF16, w.neg_mode,
                           dH_dtype=dH_dtype, mask_target_collisions=w.mask_collisions, algo=algo,
                           fuse_dH=1 if fuse_dH else 0, reuse_forward_prep=1 if fuse_dH else 0)
    ws = P.new_workspace(desc)
    loss = torch.full((w.N,), float("nan"), device="cuda")
    lse = torch.full((w.N,), float("nan"), device="cuda")
    P.cce_neg_forward_sampled(desc, smp, H, E, tgt, mask, loss, lse, ws)
    g_t = torch.from_numpy(w.g).to("cuda")
    dH = torch.full((w.N, w.d), float("nan"), device="cuda", dtype=torch.bfloat16 if dH_dtype == P.CCE_BF16 else torch.float32)
    dE = torch.zeros((w.V, w.d), device="cuda")
    P.cce_neg_backward_sampled(desc_bwd, smp, H, E, tgt, mask, lse, g_t, dH, dE, ws)
    status = P.cce_neg_index_status(ws)
    torch.cuda.synchronize()
    return dict(loss=loss.cpu().numpy(), lse=lse.cpu().numpy(), dH=dH.float().cpu().numpy(), dE=dE.cpu().numpy(),
                status=status)
