"""Other consumers of the kernels: candidate sets per bucket of positions (the shape of the Scalable Cross-Entropy loss
the paper compares with and names as a future user of index-only kernels), a masked-position batch in the style of
BERT4Rec (the paper's appendix on BERT4Rec: only the masked positions carry a loss, scattered over the sequence), and the
hidden size 320 of the paper's matrix-multiplication timing table."""
import dataclasses

import numpy as np
import pytest

from oracle import cce_oracle as O
from oracle.compare import per_position_rel, tensor_rel
from test_gpu_parity import TOL_BF16, check_against_oracle
from workloads import NEG_PER_POSITION, NEG_SHARED, make_workload

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype,d", [("bf16", 64), ("bf16", 256), ("f32", 40)])
def test_candidates_per_bucket_of_positions(dtype, d):
    """Positions are dealt into buckets at random, every bucket has its own candidate list; the oracle sees the same
    problem as per-position negatives (row i = the list of i's bucket)."""
    import torch

    import paper_2509_09682_amd as P
    from paper_2509_09682_amd.runner import to_device

    n_buckets, Kb = 13, 150
    w = make_workload(f"buckets_{dtype}_d{d}", 6, 150, d, 4000, Kb, dtype, NEG_PER_POSITION, 900 + d, g_kind="random",
                      pad="bernoulli", pad_p=0.15, e_sigma=0.1, tgt_dist="zipf")
    rng = np.random.default_rng(12)
    bucket_of = rng.integers(0, n_buckets, size=w.N)
    bucket_neg = rng.integers(0, w.V, size=(n_buckets, Kb)).astype(np.int32)
    bucket_neg[:, :5] = w.tgt[rng.integers(0, w.N, size=(n_buckets, 5))]      # some candidates are somebody's correct item
    w = dataclasses.replace(w, neg=bucket_neg[bucket_of])
    valid = np.flatnonzero(w.mask != 0)
    order = valid[np.argsort(bucket_of[valid], kind="stable")]
    counts = np.bincount(bucket_of[valid], minlength=n_buckets)
    ptr = np.concatenate([[0], np.cumsum(counts)]).tolist()
    H, E, tgt, _, _ = to_device(w)
    if dtype == "bf16":
        H, E = H.view(torch.bfloat16), E.view(torch.bfloat16)
    dE = torch.zeros((w.V, w.d), device="cuda")
    loss, lse, dH = P.bucketed_step(H, E, tgt, torch.from_numpy(order).cuda(), ptr, torch.from_numpy(bucket_neg).cuda(),
                                    torch.from_numpy(w.g).cuda(), dE, mask_target_collisions=bool(w.mask_collisions))
    torch.cuda.synchronize()
    out = dict(loss=loss.cpu().numpy(), lse=lse.cpu().numpy(), dH=dH.float().cpu().numpy(), dE=dE.cpu().numpy())
    on_tiles = dtype == "bf16"
    check_against_oracle(w, out, TOL_BF16 if on_tiles else 1e-5, dH_tol=TOL_BF16 if on_tiles else None)


@pytest.mark.parametrize("mode", [NEG_SHARED, NEG_PER_POSITION])
def test_masked_position_batch(mode):
    """A fifth of the positions, scattered over every sequence, carry a loss; the rest is masked out and must cost
    nothing and change nothing (their ids are poisoned to show that they are never read)."""
    w = make_workload(f"masked_lm_m{mode}", 64, 200, 64, 20000, 256, "bf16", mode, 4100 + mode, g_kind="random",
                      pad="bernoulli", pad_p=0.8, e_sigma=0.05, tgt_dist="zipf")
    assert 0.15 < w.mask.mean() < 0.25
    w.tgt[w.mask == 0] = -12345
    if mode == NEG_PER_POSITION:
        w.neg[w.mask == 0] = 1 << 30
    from hip_harness import run_hip

    for fuse in (False, True):
        out = run_hip(w, fuse_dH=fuse, reuse_prep=fuse)
        check_against_oracle(w, out, TOL_BF16 if mode == NEG_SHARED else 2e-5)


@pytest.mark.parametrize("mode,dtype", [(NEG_SHARED, "bf16"), (NEG_PER_POSITION, "bf16"), (NEG_SHARED, "f32")])
def test_hidden_size_320(mode, dtype):
    """d = 320 has no matrix-core instantiation (64, 128, 256 do): the row-gather kernels take it, in fp32 arithmetic."""
    w = make_workload(f"d320_m{mode}_{dtype}", 16, 50, 320, 30000, 200, dtype, mode, 3200 + mode, g_kind="random", pad="right",
                      pad_len_lo=30, e_sigma=0.05, tgt_dist="zipf")
    from hip_harness import run_hip

    check_against_oracle(w, run_hip(w), 2e-5)
