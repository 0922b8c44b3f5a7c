"""The torch.autograd front end (cce_neg_loss) against the fp64 oracle: the scalar loss of Eq. 3 and the gradients that
reach H and E through autograd, on seeded workloads of every negative mode."""
import dataclasses

import numpy as np
import pytest

from oracle import cce_oracle as O
from oracle.compare import tensor_rel
from workloads import NEG_FULL, NEG_PER_POSITION, NEG_SHARED, config, make_workload  # noqa: F401

pytestmark = pytest.mark.gpu


def _leaves(w):
    import torch

    if w.in_dtype == "f32":
        H = torch.from_numpy(w.H).cuda()
        E = torch.from_numpy(w.E).cuda()
    else:
        H = torch.from_numpy(w.H.view(np.int16)).cuda().view(torch.bfloat16)
        E = torch.from_numpy(w.E.view(np.int16)).cuda().view(torch.bfloat16)
    H.requires_grad_(True)
    E.requires_grad_(True)
    tgt = torch.from_numpy(w.tgt).cuda()
    neg = None if w.neg is None else torch.from_numpy(np.ascontiguousarray(w.neg)).cuda()
    mask = torch.from_numpy(w.mask).cuda()
    return H, E, tgt, neg, mask


@pytest.mark.parametrize("idx,scale,tol", [(1, 1.0, 1e-5), (2, 0.03, 2e-2), (3, 0.02, 2e-2), (4, 0.05, 2e-2), (5, 0.006, 2e-2)])
def test_mean_loss_and_its_gradients(idx, scale, tol):
    import paper_2509_09682_amd as P

    w = config(idx, scale=scale, g_kind="mean")       # w.g = 1 / (number of valid positions): the gradient of the mean
    H, E, tgt, neg, mask = _leaves(w)
    loss = P.cce_neg_loss(H, E, tgt, neg, mask, neg_mode=w.neg_mode, reduction="mean",
                          mask_target_collisions=bool(w.mask_collisions))
    loss.backward()
    ref = O.run_workload(w, g=w.g.astype(np.float64))
    valid = w.mask != 0
    ref_mean = float(ref.loss[valid].mean())
    assert abs(float(loss.detach()) - ref_mean) <= tol * max(abs(ref_mean), float(np.abs(ref.lse[valid]).mean()))
    assert H.grad.dtype == H.dtype and E.grad.dtype == E.dtype
    e_dH = tensor_rel(H.grad.float().cpu().numpy(), ref.dH)
    e_dE = tensor_rel(E.grad.float().cpu().numpy(), ref.dE)
    print(w.name, f"loss {float(loss):.6f} ref {ref_mean:.6f} dH {e_dH:.2e} dE {e_dE:.2e}")
    assert e_dH <= tol and e_dE <= tol


def test_two_losses_of_one_shape_in_one_graph():
    """Two forward calls of the same shape share a workspace; the backward call of the first must not reuse the
    second one's compaction.  Total = loss_a + 2 loss_b with different negatives, targets and masks."""
    import torch

    import paper_2509_09682_amd as P

    wa = config(2, scale=0.03, g_kind="mean")
    wb_src = make_workload("b", wa.batch, wa.seq_len, wa.d, wa.V, wa.K, "bf16", NEG_SHARED, 777, tgt_dist="zipf",
                           pad="bernoulli", pad_p=0.3)
    wb = dataclasses.replace(wb_src, H=wa.H, E=wa.E)
    H, E, tgt_a, neg_a, mask_a = _leaves(wa)
    tgt_b, neg_b, mask_b = (torch.from_numpy(x).cuda() for x in (wb.tgt, wb.neg, wb.mask))
    la = P.cce_neg_loss(H, E, tgt_a, neg_a, mask_a, reduction="sum")
    lb = P.cce_neg_loss(H, E, tgt_b, neg_b, mask_b, reduction="sum")
    (la + 2.0 * lb).backward()
    ra = O.run_workload(wa, g=np.ones(wa.N))
    rb = O.run_workload(wb, g=np.full(wb.N, 2.0))
    assert abs(float(la) - ra.loss[wa.mask != 0].sum()) <= 2e-2 * abs(ra.lse).sum()
    assert abs(float(lb) - rb.loss[wb.mask != 0].sum()) <= 2e-2 * abs(rb.lse).sum()
    e_dH = tensor_rel(H.grad.float().cpu().numpy(), ra.dH + rb.dH)
    e_dE = tensor_rel(E.grad.float().cpu().numpy(), ra.dE + rb.dE)
    print(f"dH {e_dH:.2e} dE {e_dE:.2e}")
    assert e_dH <= 2e-2 and e_dE <= 2e-2


def test_backward_order_against_forward_order():
    """Forward a, forward b, then backward a BEFORE backward b: a's backward call rewrites the shared workspace, so
    b's must not trust it either."""
    import torch

    import paper_2509_09682_amd as P

    wa = config(2, scale=0.03, g_kind="mean")
    wb_src = make_workload("b", wa.batch, wa.seq_len, wa.d, wa.V, wa.K, "bf16", NEG_SHARED, 778, tgt_dist="zipf",
                           pad="bernoulli", pad_p=0.3)
    wb = dataclasses.replace(wb_src, H=wa.H, E=wa.E)
    H, E, tgt_a, neg_a, mask_a = _leaves(wa)
    tgt_b, neg_b, mask_b = (torch.from_numpy(x).cuda() for x in (wb.tgt, wb.neg, wb.mask))
    la = P.cce_neg_loss(H, E, tgt_a, neg_a, mask_a, reduction="sum")
    lb = P.cce_neg_loss(H, E, tgt_b, neg_b, mask_b, reduction="sum")
    la.backward()
    lb.backward()
    ra = O.run_workload(wa, g=np.ones(wa.N))
    rb = O.run_workload(wb, g=np.ones(wb.N))
    assert tensor_rel(H.grad.float().cpu().numpy(), ra.dH + rb.dH) <= 2e-2
    assert tensor_rel(E.grad.float().cpu().numpy(), ra.dE + rb.dE) <= 2e-2


def test_reductions_agree():
    import paper_2509_09682_amd as P

    w = config(1, g_kind="mean")
    H, E, tgt, neg, mask = _leaves(w)
    vec = P.cce_neg_loss(H, E, tgt, neg, mask, reduction="none")
    total = P.cce_neg_loss(H, E, tgt, neg, mask, reduction="sum")
    mean = P.cce_neg_loss(H, E, tgt, neg, mask, reduction="mean")
    n_valid = int(w.mask.sum())
    assert vec.shape == (w.N,)
    assert float(vec[mask == 0].abs().max()) == 0.0
    assert abs(float(vec.sum()) - float(total)) <= 1e-6 * abs(float(total))
    assert abs(float(total) / n_valid - float(mean)) <= 1e-6 * abs(float(mean))


@pytest.mark.parametrize("idx,scale,tol", [(2, 0.03, 2e-2), (3, 0.02, 2e-2)])
def test_loss_with_negatives_sampled_in_the_kernels(idx, scale, tol):
    """cce_neg_loss with a sampler against the oracle run on the reference sampler's ids; the sampler object may be
    changed by the caller between forward and backward (the loss keeps its own copy)."""
    import paper_2509_09682_amd as P
    from oracle import sampler as S

    w = config(idx, scale=scale, g_kind="mean")
    H, E, tgt, _, mask = _leaves(w)
    smp = P.make_sampler(P.CCE_SAMPLER_UNIFORM, 31337, 4)
    loss = P.cce_neg_loss(H, E, tgt, None, mask, neg_mode=w.neg_mode, reduction="mean", sampler=smp, n_neg=w.K)
    smp.stream = 5            # next step's number: must not reach the pending backward call
    loss.backward()
    ids = S.sample_negatives(S.UNIFORM, 31337, 4, w.N, w.K, w.V, per_position=(w.neg_mode == NEG_PER_POSITION))
    ref = O.run_workload(dataclasses.replace(w, neg=ids), g=w.g.astype(np.float64))
    valid = w.mask != 0
    ref_mean = float(ref.loss[valid].mean())
    assert abs(float(loss.detach()) - ref_mean) <= tol * max(abs(ref_mean), float(np.abs(ref.lse[valid]).mean()))
    assert tensor_rel(H.grad.float().cpu().numpy(), ref.dH) <= tol
    assert tensor_rel(E.grad.float().cpu().numpy(), ref.dE) <= tol
