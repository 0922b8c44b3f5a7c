"""The forward call that also forms the hidden-state gradient (fuse_dH = 1: one pass over the candidates for lse and
for U = sum_j p_ij E_j - E_tgt, an online softmax; the backward call scales U by grad_loss and recomputes the scores
for dE only) against the fp64 oracle, on the shapes that exercise its parts: split candidate ranges and their merge,
the last-round split at hidden size 256, ragged tiles, collisions, padded positions, bf16 dH, a NULL grad_loss, repeated
backward calls, and scores that outgrow the block's reference (the restart in the exact form)."""
import numpy as np
import pytest

from oracle import cce_oracle as O
from oracle.compare import tensor_rel
from test_gpu_parity import (FULL_SIZE_BARS, TOL_BF16, check_against_oracle, rounding_model_excess)
from workloads import NEG_FULL, NEG_PER_POSITION, NEG_SHARED, config, make_workload

pytestmark = pytest.mark.gpu


def _run(w, **kw):
    from hip_harness import run_hip
    import paper_2509_09682_amd as P

    kw.setdefault("algo", P.CCE_ALGO_TILE)
    return run_hip(w, fuse_dH=True, reuse_prep=True, **kw)


@pytest.mark.parametrize("d", [64, 128, 256])
@pytest.mark.parametrize("mode", [NEG_SHARED, NEG_FULL])
def test_fused_ragged_shapes_collisions_and_duplicates(d, mode):
    import paper_2509_09682_amd as P

    K = 0 if mode == NEG_FULL else 203
    V = 1003 if mode == NEG_FULL else 157
    w = make_workload(f"fused_ragged_d{d}_m{mode}", 7, 61, d, V, K, "bf16", mode, 500 + d + mode, pad="right",
                      pad_len_lo=20, g_kind="random", e_sigma=0.1, tgt_dist="zipf")
    for collide in ((0, 1) if mode == NEG_SHARED else (1,)):
        w.mask_collisions = collide
        check_against_oracle(w, _run(w), TOL_BF16)
    out = _run(w, dH_dtype=P.CCE_BF16, use_mask=False, g=None)      # NULL grad_loss, no mask, bf16 dH
    w.mask[:] = 1
    check_against_oracle(w, out, TOL_BF16, g=None, dH_tol=TOL_BF16)


@pytest.mark.parametrize("idx,scale", [(2, 0.03), (4, 0.05), (5, 0.006)])
def test_fused_reduced_configs(idx, scale):
    w = config(idx, scale=scale, g_kind="random")
    check_against_oracle(w, _run(w), TOL_BF16)


def test_fused_equals_the_separate_passes_closely():
    """Same inputs through both forms: lse to fp32 rounding, gradients to the rounding of the probabilities."""
    from hip_harness import run_hip
    import paper_2509_09682_amd as P

    w = make_workload("fused_vs_plain", 9, 83, 64, 211, 190, "bf16", NEG_SHARED, 4242, pad="bernoulli", pad_p=0.35,
                      g_kind="random", e_sigma=0.1, tgt_dist="zipf")
    a = _run(w)
    b = run_hip(w, algo=P.CCE_ALGO_TILE, reuse_prep=True)
    assert np.max(np.abs(a["lse"] - b["lse"])) <= 2e-6 * np.max(np.abs(b["lse"]))
    assert np.max(np.abs(a["loss"] - b["loss"])) <= 4e-6 * np.max(np.abs(b["lse"]))
    assert tensor_rel(a["dH"], b["dH"]) <= 8e-3 and tensor_rel(a["dE"], b["dE"]) <= 1e-5   # dE: same kernels, same inputs
    assert np.all(a["dH"][w.mask == 0] == 0)


@pytest.mark.parametrize("d", [64, 128, 256])
def test_fused_two_backward_calls_after_one_forward(d):
    """U, the coefficients and the exponent offsets survive a backward call: a second one adds the same gradient again
    (few positions, many candidates: the candidate range is split and merged)."""
    w = make_workload(f"fused_twice_d{d}", 7, 90, d, 6000, 0, "bf16", NEG_FULL, 99 + d, pad="bernoulli", pad_p=0.2,
                      g_kind="random", e_sigma=0.1, tgt_dist="zipf")
    out = _run(w, repeat_backward=2)
    out["dE"] = out["dE"] * 0.5
    check_against_oracle(w, out, TOL_BF16)


@pytest.mark.parametrize("batch,pad", [(357, "right"), (264, "none"), (460, "bernoulli"), (400, "none")])
def test_fused_last_round_of_position_blocks_splits_the_candidates(batch, pad):
    import paper_2509_09682_amd as P

    w = make_workload("fused_tail", batch, 256, 256, 3000, 70, "bf16", NEG_SHARED, 41 + batch, g_kind="random", tgt_dist="zipf",
                      pad=pad, pad_p=0.25, pad_len_lo=200)
    assert w.n_valid > 65536
    check_against_oracle(w, _run(w), TOL_BF16)
    check_against_oracle(w, _run(w, dH_dtype=P.CCE_BF16), TOL_BF16, dH_tol=TOL_BF16)


@pytest.mark.parametrize("d,mode", [(64, NEG_FULL), (128, NEG_SHARED), (256, NEG_FULL)])
def test_fused_scores_that_outgrow_the_reference_by_hundreds_of_nats(d, mode):
    """The fast form takes its reference from the first 32 candidates; here the scores climb (or fall) by several
    hundred nats along the candidate index, so blocks overflow and start over in the exact form."""
    from workloads import bf16_bits_from_f32

    V, K = 3000, 1500
    w = make_workload(f"fused_steep_d{d}", 3, 111, d, V, 0 if mode == NEG_FULL else K, "bf16", mode, 7 + d, pad="bernoulli",
                      pad_p=0.1, g_kind="random", neg_dist="uniform")
    rng = np.random.default_rng(d)
    u = rng.standard_normal(d).astype(np.float32)
    u /= np.linalg.norm(u)
    slope = rng.uniform(-1.5, 1.5, size=w.N).astype(np.float32)
    H = slope[:, None] * u[None, :] + 0.01 * rng.standard_normal((w.N, d)).astype(np.float32)
    ramp = np.arange(V, dtype=np.float32) / V
    if mode == NEG_SHARED:
        order = np.full(V, 0.5, np.float32)
        order[w.neg] = np.arange(K, dtype=np.float32) / K
        ramp = order
    E = 400.0 * ramp[:, None] * u[None, :] + 0.01 * rng.standard_normal((V, d)).astype(np.float32)
    w.H = bf16_bits_from_f32(H.astype(np.float32))
    w.E = bf16_bits_from_f32(E.astype(np.float32))
    out = _run(w)
    assert np.all(np.isfinite(out["loss"])) and np.all(np.isfinite(out["dH"]))
    ref = O.run_workload(w, g=w.g.astype(np.float64), want_p=True)
    assert np.abs(ref.lse).max() > 300
    check_against_oracle(w, out, TOL_BF16, row_tol=1.0)
    ex_H, ex_E = rounding_model_excess(w, out, ref)
    print(w.name, f"excess over the bf16 rounding model: dH {ex_H:.2e} dE {ex_E:.2e}")
    assert ex_H <= 0 and ex_E <= 0


@pytest.mark.parametrize("seed", range(18))
def test_fused_random_medium_shapes(seed):
    import paper_2509_09682_amd as P

    rng = np.random.default_rng(7000 + seed)
    mode = NEG_SHARED if seed % 2 == 0 else NEG_FULL
    d = [64, 128, 256][seed % 3]
    batch, seq = int(rng.integers(2, 40)), int(rng.integers(20, 160))
    V = int(rng.integers(600, 9000))
    K = 0 if mode == NEG_FULL else int(rng.integers(100, 1600))
    pad = ["none", "bernoulli", "right"][int(rng.integers(0, 3))]
    w = make_workload(f"fused_med{seed}", batch, seq, d, V, K, "bf16", mode, 8000 + seed, g_kind="random", pad=pad, pad_p=0.2,
                      pad_len_lo=seq // 2, tgt_dist="zipf", e_sigma=0.1, mask_collisions=int(rng.integers(0, 2)))
    dH_bf16 = bool(rng.integers(0, 2))
    print(dict(mode=mode, d=d, N=w.N, V=V, K=K, pad=pad, collide=w.mask_collisions, dH_bf16=dH_bf16))
    out = _run(w, dH_dtype=P.CCE_BF16 if dH_bf16 else P.CCE_F32)
    check_against_oracle(w, out, TOL_BF16, dH_tol=TOL_BF16 if dH_bf16 else None)


def test_fused_edge_cases():
    """One position; one candidate; every position padded; a backward call that cannot reuse (falls back to the dH pass)."""
    from hip_harness import run_hip
    import paper_2509_09682_amd as P

    w = make_workload("fused_n1", 1, 1, 64, 50, 5, "bf16", NEG_SHARED, 8)
    check_against_oracle(w, _run(w), TOL_BF16)
    w = make_workload("fused_k1", 2, 40, 128, 50, 1, "bf16", NEG_SHARED, 9, g_kind="random")
    check_against_oracle(w, _run(w), TOL_BF16)
    w = make_workload("fused_all_masked", 2, 80, 256, 400, 60, "bf16", NEG_SHARED, 10)
    w.mask[:] = 0
    out = _run(w)
    assert np.all(out["loss"] == 0) and np.all(out["dH"] == 0) and np.all(out["dE"] == 0)
    w = make_workload("fused_no_reuse", 5, 70, 64, 900, 130, "bf16", NEG_SHARED, 11, g_kind="random", pad="bernoulli", pad_p=0.2)
    out = run_hip(w, algo=P.CCE_ALGO_TILE, fuse_dH=True, reuse_prep=False)     # the flag alone changes the forward pass only
    check_against_oracle(w, out, TOL_BF16)


def test_fused_full_size_c2_against_full_oracle():
    w = config(2)
    errs = check_against_oracle(w, _run(w, algo=0), TOL_BF16)
    b = FULL_SIZE_BARS[2]
    assert errs["dH"] <= b[0] and errs["dE"] <= b[1] and errs["dH_row"] <= b[2] and errs["dE_row"] <= b[3], (errs, b)


# ---- the same flag on the row-gather kernels (fp32 inputs, other hidden sizes, per-position negatives): the forward
#      call sums the weighted candidate rows while it has them for the score; the backward call gathers none for dH

def _run_gather(w, **kw):
    from hip_harness import run_hip
    import paper_2509_09682_amd as P

    kw.setdefault("algo", P.CCE_ALGO_GATHER)
    return run_hip(w, fuse_dH=True, reuse_prep=True, **kw)


@pytest.mark.parametrize("mode", [NEG_SHARED, NEG_PER_POSITION, NEG_FULL])
@pytest.mark.parametrize("dtype,d", [("f32", 40), ("f32", 64), ("bf16", 128), ("bf16", 320)])
def test_fused_row_gather_family(mode, dtype, d):
    import paper_2509_09682_amd as P

    K = 0 if mode == NEG_FULL else 203
    V = 1003 if mode == NEG_FULL else 157
    w = make_workload(f"fused_gather_m{mode}_{dtype}_d{d}", 7, 61, d, V, K, dtype, mode, 900 + d + mode, pad="right",
                      pad_len_lo=20, g_kind="random", e_sigma=0.1, tgt_dist="zipf")
    for collide in ((0, 1) if mode != NEG_FULL else (1,)):
        w.mask_collisions = collide
        check_against_oracle(w, _run_gather(w), 2e-5)
    out = _run_gather(w, dH_dtype=P.CCE_BF16 if dtype == "bf16" else P.CCE_F32, use_mask=False, g=None, repeat_backward=2)
    out["dE"] = out["dE"] * 0.5                                   # U and p+ - 1 survive a backward call
    w.mask[:] = 1
    check_against_oracle(w, out, 2e-5, g=None, dH_tol=TOL_BF16 if dtype == "bf16" else None)


def test_fused_row_gather_reduced_c3_and_c1():
    for idx, scale in ((3, 0.05), (1, 1.0)):
        w = config(idx, scale=scale, g_kind="random")
        check_against_oracle(w, _run_gather(w), 2e-5)


def test_fused_row_gather_scores_that_outgrow_the_first_reference():
    """Every lane group takes its first live score as reference; here later candidates score up to 150 nats higher, the
    sums leave the float range and the wavefront walks its candidates again against the true maximum."""
    d, K = 64, 300
    w = make_workload("fused_gather_climb", 3, 40, d, 2000, K, "f32", NEG_PER_POSITION, 77, pad="bernoulli", pad_p=0.1,
                      g_kind="random", e_sigma=0.05)
    rng = np.random.default_rng(5)
    E = w.E.reshape(w.V, d).copy()
    H = w.H.reshape(w.N, d)
    neg = w.neg.reshape(w.N, K)
    for i in range(0, w.N, 3):                       # a third of the positions get a steep candidate late in the list
        j = int(rng.integers(K // 2, K))
        v = int(neg[i, j])
        h = H[i].astype(np.float64)
        E[v] = (150.0 * h / float(h @ h)).astype(np.float32)   # <h_i, e_v> = 150
    w.E = E.reshape(w.E.shape)
    errs = check_against_oracle(w, _run_gather(w), 2e-5)
    assert errs["lse"] <= 2e-5


def test_fused_row_gather_equals_the_separate_passes():
    from hip_harness import run_hip
    import paper_2509_09682_amd as P

    w = make_workload("fused_gather_vs_plain", 9, 83, 128, 4000, 97, "bf16", NEG_PER_POSITION, 4243, pad="bernoulli",
                      pad_p=0.35, g_kind="random", e_sigma=0.1, tgt_dist="zipf")
    a = _run_gather(w)
    b = run_hip(w, algo=P.CCE_ALGO_GATHER)
    assert np.max(np.abs(a["lse"] - b["lse"])) <= 2e-6 * np.max(np.abs(b["lse"]))
    assert tensor_rel(a["dH"], b["dH"]) <= 1e-5 and tensor_rel(a["dE"], b["dE"]) <= 1e-5
    assert np.all(a["dH"][w.mask == 0] == 0)


@pytest.mark.parametrize("mode,dtype,d", [(NEG_PER_POSITION, "bf16", 128), (NEG_PER_POSITION, "f32", 40), (NEG_SHARED, "f32", 64),
                                          (NEG_SHARED, "bf16", 256)])
def test_fused_sampled_calls(mode, dtype, d):
    """Negatives drawn inside the kernels, with the fused forward pass: the row-gather kernels redraw the ids in the one
    pass that is left; shared lists (drawn once into the workspace) follow the stored-list paths of either family."""
    import dataclasses

    from hip_harness import device_sampler, run_hip_sampled
    from oracle import sampler as S

    w = make_workload(f"fused_sampled_m{mode}_{dtype}_d{d}", 9, 37, d, 3000, 130, dtype, mode, 1234 + d, pad="bernoulli",
                      pad_p=0.2, g_kind="random", e_sigma=0.1, tgt_dist="zipf")
    smp, keep = device_sampler(S.UNIFORM, 777, 3)
    ids = S.sample_negatives(S.UNIFORM, 777, 3, w.N, w.K, w.V, per_position=(mode == NEG_PER_POSITION))
    w_ref = dataclasses.replace(w, neg=ids)
    out = run_hip_sampled(w, smp, fuse_dH=True)
    assert out["status"] == 0
    check_against_oracle(w_ref, out, TOL_BF16 if (dtype == "bf16" and mode == NEG_SHARED) else 2e-5)
