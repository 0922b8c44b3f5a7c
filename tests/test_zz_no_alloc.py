"""cce_neg_forward_noalloc (the entry point for callers that cannot allocate or pass a workspace) against
cce_neg_forward: same inputs, same loss and lse, through the C ABI, twice in a row, the second call on a smaller
input, so that what the first call left in the library's fixed scratch array must not leak into the second."""
import numpy as np
import pytest

from workloads import NEG_FULL, NEG_PER_POSITION, NEG_SHARED, make_workload

pytestmark = pytest.mark.gpu


def _both(w):
    import torch

    import paper_2509_09682_amd as P
    from paper_2509_09682_amd.runner import to_device

    H, E, tgt, neg, mask = to_device(w)
    desc = P.make_desc(w.N, w.V, w.d, w.K, P.CCE_F32 if w.in_dtype == "f32" else P.CCE_BF16, w.neg_mode,
                       mask_target_collisions=w.mask_collisions)
    out = {}
    for name in ("workspace", "noalloc"):
        loss = torch.full((w.N,), float("nan"), device="cuda")
        lse = torch.full((w.N,), float("nan"), device="cuda")
        if name == "workspace":
            ws = P.new_workspace(desc)
            P.cce_neg_forward(desc, H, E, tgt, neg, mask, loss, lse, ws)
        else:
            P.cce_neg_forward_noalloc(desc, H, E, tgt, neg, mask, loss, lse)
        torch.cuda.synchronize()
        out[name] = (loss.cpu().numpy(), lse.cpu().numpy())
    return out


def _check(w):
    out = _both(w)
    for k in (0, 1):
        a, b = out["workspace"][k], out["noalloc"][k]
        assert np.all(np.isfinite(b))
        # the forward pass has no atomics: the two entry points run the same kernels and agree bit for bit
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32)), ("loss", "lse")[k]
    assert np.all(out["noalloc"][0][w.mask == 0] == 0)


@pytest.mark.parametrize("mode,dtype,d", [(NEG_SHARED, "bf16", 64), (NEG_FULL, "bf16", 256), (NEG_PER_POSITION, "bf16", 128),
                                          (NEG_SHARED, "f32", 40)])
def test_noalloc_forward_equals_forward_on_two_calls_in_a_row(mode, dtype, d):
    K = 0 if mode == NEG_FULL else 150
    big = make_workload("noalloc_big", 9, 120, d, 3000, K, dtype, mode, 600 + d, pad="bernoulli", pad_p=0.3, g_kind="random",
                        e_sigma=0.1, tgt_dist="zipf")
    small = make_workload("noalloc_small", 2, 37, d, 700, 0 if mode == NEG_FULL else 33, dtype, mode, 700 + d, pad="right",
                          pad_len_lo=5, g_kind="random", e_sigma=0.1, tgt_dist="zipf")
    _check(big)
    _check(small)   # fewer positions, fewer candidates, another padding pattern: nothing of the first call may show


def test_noalloc_forward_refuses_what_does_not_fit_and_what_it_cannot_report():
    import torch

    import paper_2509_09682_amd as P

    # at least 20 bytes of scratch per position on the matrix-core path: 2,000,000 positions do not fit in 32 MiB
    desc = P.make_desc(2_000_000, 1000, 64, 256, P.CCE_BF16, P.CCE_NEG_SHARED)
    one = torch.zeros(16, device="cuda")
    L = P.binding.lib()
    import ctypes

    p = ctypes.c_void_p(one.data_ptr())   # never dereferenced: the call must fail on the host
    assert L.cce_neg_forward_noalloc(ctypes.byref(desc), p, p, p, p, None, p, p, None) == P.CCE_ERR_WORKSPACE
    desc = P.make_desc(1000, 1000, 64, 256, P.CCE_BF16, P.CCE_NEG_SHARED, validate_indices=1)
    assert L.cce_neg_forward_noalloc(ctypes.byref(desc), p, p, p, p, None, p, p, None) == P.CCE_ERR_UNSUPPORTED
    assert L.cce_neg_forward_noalloc(ctypes.byref(desc), None, p, p, p, None, p, p, None) == P.CCE_ERR_NULL
