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


def test_table_gradient_added_into_a_caller_held_buffer():
    """grad_E_out: the backward pass adds the table gradient into the caller's fp32 buffer, touches only indexed rows,
    and autograd returns no gradient for E; two steps accumulate."""
    import torch

    import paper_2509_09682_amd as P

    w = config(2, scale=0.03, g_kind="mean")
    H, E, tgt, neg, mask = _leaves(w)
    P.cce_neg_loss(H, E, tgt, neg, mask, reduction="mean").backward()
    dense_dH, dense_dE = H.grad.clone(), E.grad.float().clone()
    H.grad = E.grad = None
    acc = torch.full(E.shape, 0.25, device="cuda", dtype=torch.float32)
    for step in range(2):
        P.cce_neg_loss(H, E, tgt, neg, mask, reduction="mean", grad_E_out=acc).backward()
    assert E.grad is None
    assert torch.equal(H.grad, 2 * dense_dH)                 # dH has no atomics: bitwise the same each step
    ref = O.run_workload(w, g=w.g.astype(np.float64))
    got = (acc - 0.25).cpu().numpy() / 2
    assert tensor_rel(got, ref.dE) <= 2e-2
    rows = O.touched_rows(w.tgt, w.neg, w.mask, w.neg_mode, w.V, mask_collisions=w.mask_collisions)
    untouched = np.setdiff1d(np.arange(w.V), rows)
    assert np.all(acc.cpu().numpy()[untouched] == 0.25)       # rows nobody indexed keep their content bit for bit
    # E frozen (no requires_grad): the buffer is still filled
    E2 = E.detach()
    acc2 = torch.zeros(E.shape, device="cuda", dtype=torch.float32)
    P.cce_neg_loss(H, E2, tgt, neg, mask, reduction="mean", grad_E_out=acc2).backward()
    assert tensor_rel(acc2.cpu().numpy(), ref.dE) <= 2e-2
    with pytest.raises(ValueError):
        P.cce_neg_loss(H, E, tgt, neg, mask, grad_E_out=acc.to(torch.bfloat16))


@pytest.mark.parametrize("idx,scale", [(2, 0.03), (3, 0.01), (1, 1.0)])
def test_loss_scaling_of_mixed_precision_training_passes_through(idx, scale):
    """The paper trains in fp16 mixed precision (Sec. 4.3, Training Details), where the loss is multiplied by a large
    power of two before backward() and the gradients are divided by it afterwards.  The upstream gradient reaches the
    kernels in fp32 and multiplies every term once, so a power-of-two scale must come out of both gradients exactly
    (dE: up to the order of its atomics), and an overflowed scale must show up as inf / NaN where the scaler looks."""
    import torch

    import paper_2509_09682_amd as P

    w = config(idx, scale=scale, g_kind="mean")
    H, E, tgt, neg, mask = _leaves(w)
    kw = dict(neg_mode=w.neg_mode, reduction="mean", mask_target_collisions=bool(w.mask_collisions))
    P.cce_neg_loss(H, E, tgt, neg, mask, **kw).backward()
    dH0, dE0 = H.grad.float().clone(), E.grad.float().clone()
    H.grad = E.grad = None
    S = 65536.0
    (P.cce_neg_loss(H, E, tgt, neg, mask, **kw) * S).backward()
    assert torch.equal(H.grad.float() / S, dH0)
    assert tensor_rel((E.grad.float() / S).cpu().numpy(), dE0.cpu().numpy()) <= (2e-3 if H.dtype == torch.bfloat16 else 1e-5)
    H.grad = E.grad = None
    (P.cce_neg_loss(H, E, tgt, neg, mask, **kw) * float("inf")).backward()
    valid = torch.from_numpy(w.mask != 0).cuda()
    assert not torch.isfinite(H.grad.float()[valid]).all() and not torch.isfinite(E.grad.float()).all()
    assert torch.all(H.grad.float()[~valid] == 0)          # padded rows stay exactly zero even then


def test_workspace_cache_is_bounded_and_can_be_cleared():
    import paper_2509_09682_amd as P
    from paper_2509_09682_amd import autograd as A

    P.clear_workspaces()
    for n in range(A.MAX_CACHED_WORKSPACES + 3):
        w = make_workload(f"cache{n}", 1, 20 + n, 32, 100, 8, "f32", NEG_SHARED, 60 + n)
        H, E, tgt, neg, mask = _leaves(w)
        P.cce_neg_loss(H, E, tgt, neg, mask).backward()
    assert len(A._workspaces) == A.MAX_CACHED_WORKSPACES
    P.clear_workspaces()
    assert len(A._workspaces) == 0 and len(A._last_forward) == 0


def test_large_workload_through_autograd_costs_little_more_than_the_raw_calls():
    """Workload c5 (204,800 positions, 5 M items, d 256, K 4096): forward + backward through cce_neg_loss with a
    caller-held gradient buffer against the two C-ABI calls on the same inputs.  Results must agree (they run the same
    kernels) and the autograd step must stay within a quarter of the raw step's time (target 15 %; the bound leaves
    room for timer noise); the dense default (zero + convert a 5 GB tensor per step) is timed for comparison."""
    import torch

    import paper_2509_09682_amd as P

    w = config(5)
    H, E, tgt, neg, mask = _leaves(w)
    g = torch.from_numpy(w.g).cuda()
    desc = P.make_desc(w.N, w.V, w.d, w.K, P.CCE_BF16, w.neg_mode, dH_dtype=P.CCE_BF16, mask_target_collisions=w.mask_collisions, fuse_dH=1)
    desc_b = P.make_desc(w.N, w.V, w.d, w.K, P.CCE_BF16, w.neg_mode, dH_dtype=P.CCE_BF16, mask_target_collisions=w.mask_collisions, fuse_dH=1,
                         reuse_forward_prep=1)
    ws = P.new_workspace(desc)
    loss = torch.empty(w.N, device="cuda")
    lse = torch.empty(w.N, device="cuda")
    dH = torch.empty((w.N, w.d), device="cuda", dtype=torch.bfloat16)
    dE = torch.zeros((w.V, w.d), device="cuda")
    Hd, Ed = H.detach(), E.detach()

    def raw():
        P.cce_neg_forward(desc, Hd, Ed, tgt, neg, mask, loss, lse, ws)
        P.cce_neg_backward(desc_b, Hd, Ed, tgt, neg, mask, lse, g, dH, dE, ws)

    acc = torch.zeros((w.V, w.d), device="cuda")

    def through_autograd(buffer):
        H.grad = None
        E.grad = None
        out = P.cce_neg_loss(H, E, tgt, neg, mask, neg_mode=w.neg_mode, reduction="none", grad_E_out=buffer)
        out.backward(g)

    def timed(fn, reps=5):
        for _ in range(2):
            fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    t_raw = timed(raw)
    t_auto = timed(lambda: through_autograd(acc))
    t_dense = timed(lambda: through_autograd(None), reps=3)
    print(f"c5 step: raw calls {t_raw:.3f} ms, cce_neg_loss with a gradient buffer {t_auto:.3f} ms, dense default {t_dense:.3f} ms")
    assert t_auto <= 1.25 * t_raw
    dE.zero_()
    acc.zero_()
    raw()
    through_autograd(acc)
    torch.cuda.synchronize()
    assert torch.equal(H.grad, dH)
    rows = torch.from_numpy(O.touched_rows(w.tgt, w.neg, w.mask, w.neg_mode, w.V, mask_collisions=w.mask_collisions)).cuda()
    a_rows, r_rows = acc[rows], dE[rows]
    assert float((a_rows - r_rows).abs().max()) <= 1e-4 * float(r_rows.abs().max())      # same terms, other atomics order
