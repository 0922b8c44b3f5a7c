"""Element-by-element parity of the HIP path (through the C ABI) against the fp64 oracle on seeded inputs."""
import numpy as np
import pytest

from oracle import cce_oracle as O
from oracle.compare import per_position_rel, row_rel, tensor_rel
from workloads import NEG_FULL, NEG_PER_POSITION, NEG_SHARED, config, make_workload  # noqa: F401

pytestmark = pytest.mark.gpu

TOL_F32 = 1e-5    # fp32 path: relative error on loss, lse and gradients
TOL_BF16 = 2e-2   # bf16 path
# Measured bars, held IN ADDITION to the contract tolerances above so that a regression is noticed long before the
# contract breaks.  Per tensor: max|x - ref| / max|ref|.  Per row (oracle.compare.row_rel): every dH row and every
# touched dE row against its own largest entry, floor 1e-3 of the tensor's.
#   loss / lse, matrix-core path: fp32 accumulation of exact bf16 products, hardware exp2 / log2; worst seen 3.7e-7.
#   gradients, fp32 arithmetic (row-gather path, fp32 inputs): worst seen 2e-6 per tensor, 3.2e-5 per row.
#   gradients, matrix-core path: the probabilities are rounded to bf16 before the second product, half an ulp = 2^-9 =
#   2e-3 relative per term.  Small cases with few candidates sit right at that figure (worst seen 3.4e-3 per tensor,
#   4.6e-3 per row), so their bar cannot be ten times the observation without passing the contract; it is about twice.
#   The full-size workloads average over thousands of terms and get bars of their own, ten times what they show.
FWD_BAR_TILE = 4e-6
GRAD_BAR_TILE = 8e-3
ROW_BAR_TILE = 1.2e-2
ROW_BAR_FP32_MATH = 3e-4
FULL_SIZE_BARS = {   # workload: (dH, dE, dH per row, dE per row) = 10 x the errors measured on the MI355X
    2: (7e-4, 1.2e-4, 1.5e-3, 8e-3),
    3: (7e-6, 4e-6, 1.2e-5, 1e-5),
    4: (6e-5, 1e-6, 1e-4, 9e-4),
    5: (3e-4, 2e-5, 5e-4, 1.7e-2),
}


def rounding_model_excess(w, out, ref):
    """Largest amount by which a gradient row leaves the error the bf16 rounding of the probabilities allows.

    On the matrix-core path every term G_ij e_j (dH) or G_ij h_i (dE) carries the probability rounded to bf16, a
    relative error of at most 2^-9 of p_ij; the correct item's -g_i is exact.  A row may therefore be off by at most
    2^-9 sum |g_i| p_ij max|e_j| (the sum running over the row's own terms), whatever cancels inside the row: this is
    the per-row check for inputs whose rows nearly cancel (a peaked softmax: p of the correct item close to 1).  The
    bound is doubled for the fp32 accumulation and the hardware exponential.  ref must carry p (want_p)."""
    from workloads import f32_from_bf16_bits

    valid = np.flatnonzero(w.mask != 0)
    E_inf = np.abs(f32_from_bf16_bits(w.E).astype(np.float64)).max(1)
    H_inf = np.abs(f32_from_bf16_bits(w.H).astype(np.float64)).max(1)
    g = np.abs(np.asarray(w.g, np.float64))
    p = ref.p[valid]
    if w.neg_mode == NEG_FULL:
        cand = np.broadcast_to(np.arange(w.V), p.shape)
    else:
        cand = np.concatenate([w.tgt[valid, None], np.broadcast_to(w.neg, (valid.size, w.K))], 1)
    bound_H = 2.0 ** -8 * g[valid] * (p * E_inf[cand]).sum(1)
    bound_E = np.zeros(w.V)
    np.add.at(bound_E, cand.ravel(), (2.0 ** -8 * (g[valid] * H_inf[valid])[:, None] * p).ravel())
    dev_H = np.abs(out["dH"][valid].astype(np.float64) - ref.dH[valid]).max(1)
    dev_E = np.abs(out["dE"].astype(np.float64) - ref.dE).max(1)
    tiny_H, tiny_E = 1e-6 * np.abs(ref.dH).max(), 1e-6 * np.abs(ref.dE).max()
    return float(np.max(dev_H - bound_H - tiny_H)), float(np.max(dev_E - bound_E - tiny_E))


def check_against_oracle(w, out, tol, *, g="workload", dE_init=None, dH_tol=None, row_tol=None):
    g_np = w.g if isinstance(g, str) else g
    g64 = np.ones(w.N) if g_np is None else np.asarray(g_np, np.float64)   # a NULL grad_loss means 1
    ref = O.run_workload(w, g=g64)
    valid = w.mask != 0
    # masked positions: exactly +0.0
    for name in ("loss", "lse"):
        assert np.all(out[name][~valid] == 0) and not np.any(np.signbit(out[name][~valid])), name
    assert np.all(out["dH"][~valid] == 0)
    e_loss = per_position_rel(out["loss"][valid], ref.loss[valid], ref.lse[valid], ref.loss[valid])
    e_lse = per_position_rel(out["lse"][valid], ref.loss[valid], ref.lse[valid], ref.lse[valid])
    e_dH = tensor_rel(out["dH"], ref.dH)
    rows = O.touched_rows(w.tgt, w.neg, w.mask, w.neg_mode, w.V, mask_collisions=w.mask_collisions)
    base = np.zeros_like(out["dE"]) if dE_init is None else dE_init
    e_dE = tensor_rel((out["dE"].astype(np.float64) - base)[rows], ref.dE[rows])
    # rows nobody indexes are untouched bit for bit
    untouched = np.setdiff1d(np.arange(w.V), rows)
    assert np.array_equal(out["dE"][untouched].view(np.uint32), base[untouched].view(np.uint32))
    # every touched row whose oracle gradient is non-zero changed
    changed = np.flatnonzero(np.any(out["dE"] != base, axis=1))
    ref_nonzero = rows[np.any(ref.dE[rows] != 0, axis=1)]
    assert np.array_equal(np.intersect1d(changed, ref_nonzero), ref_nonzero)
    assert np.all(np.isin(changed, rows))
    # every row against its own size: dH rows of valid positions, dE rows the oracle touched
    r_dH = row_rel(out["dH"][valid], ref.dH[valid])
    r_dE = row_rel((out["dE"].astype(np.float64) - base)[rows], ref.dE[rows])
    errs = dict(loss=e_loss, lse=e_lse, dH=e_dH, dE=e_dE, dH_row=r_dH, dE_row=r_dE)
    print(w.name, {k: f"{v:.2e}" for k, v in errs.items()})
    assert e_loss <= tol and e_lse <= tol, errs
    assert e_dH <= (tol if dH_tol is None else dH_tol) and e_dE <= tol, errs
    if row_tol is None:    # the measured bar of the path that ran: fp32 arithmetic unless the tolerance is the bf16 one
        row_tol = ROW_BAR_TILE if tol >= TOL_BF16 else ROW_BAR_FP32_MATH
    if dE_init is None:
        assert r_dE <= row_tol, errs
    assert r_dH <= max(row_tol, 0.0 if dH_tol is None else dH_tol), errs
    if tol >= TOL_BF16 and dE_init is None:       # matrix-core path: the measured per-tensor bars
        assert e_loss <= FWD_BAR_TILE and e_lse <= FWD_BAR_TILE, errs
        assert e_dE <= GRAD_BAR_TILE and (dH_tol is not None or e_dH <= GRAD_BAR_TILE), errs
    return errs


def _run(w, **kw):
    from hip_harness import run_hip

    return run_hip(w, **kw)


def test_c1_tiny_fp32_shared_full_size():
    w = config(1, g_kind="random")
    assert ((w.neg[None, :] == w.tgt[:, None]) & (w.mask[:, None] != 0)).sum() > 0  # the collision path is exercised
    check_against_oracle(w, _run(w), TOL_F32)


@pytest.mark.parametrize("idx,scale", [(2, 0.02), (3, 0.02), (4, 0.03), (5, 0.004)])
def test_reduced_configs_gather_path(idx, scale):
    import paper_2509_09682_amd as P

    w = config(idx, scale=scale, g_kind="random")
    out = _run(w, algo=P.CCE_ALGO_GATHER)
    # the gather path computes in fp32 from the exact bf16 inputs: hold it to a much tighter bar than the bf16 target
    check_against_oracle(w, out, 2e-5)


@pytest.mark.parametrize("idx,scale", [(2, 0.03), (4, 0.05), (5, 0.006)])
def test_reduced_configs_tile_path(idx, scale):
    import paper_2509_09682_amd as P

    w = config(idx, scale=scale, g_kind="random")
    out = _run(w, algo=P.CCE_ALGO_TILE)
    check_against_oracle(w, out, TOL_BF16)


@pytest.mark.parametrize("d", [64, 128, 256])
@pytest.mark.parametrize("mode", [NEG_SHARED, NEG_FULL])
def test_tile_path_ragged_shapes_collisions_and_duplicates(d, mode):
    """Sizes that are no multiple of any tile edge, a catalogue so small that negatives repeat and hit targets."""
    import paper_2509_09682_amd as P

    K = 0 if mode == NEG_FULL else 203
    V = 1003 if mode == NEG_FULL else 157
    w = make_workload(f"tile_ragged_d{d}_m{mode}", 7, 61, d, V, K, "bf16", mode, 500 + d + mode, pad="right",
                      pad_len_lo=20, g_kind="random", e_sigma=0.1, tgt_dist="zipf")
    if mode == NEG_SHARED:
        dup = (w.neg[None, :] == w.tgt[:, None]).sum(1)
        assert dup.max() >= 2          # some target appears several times among the negatives
    for collide in ((0, 1) if mode == NEG_SHARED else (1,)):
        w.mask_collisions = collide
        out = _run(w, algo=P.CCE_ALGO_TILE)
        check_against_oracle(w, out, TOL_BF16)
    out = _run(w, algo=P.CCE_ALGO_TILE, dH_dtype=P.CCE_BF16, use_mask=False, g=None)
    w.mask[:] = 1
    check_against_oracle(w, out, TOL_BF16, g=None)


@pytest.mark.parametrize("d", [64, 256])
def test_backward_reusing_the_forward_preparation(d):
    """reuse_forward_prep = 1: the backward call skips the compaction / collision pass and must give the same result
    (masked rows of dH still exactly zero, collisions still masked)."""
    import paper_2509_09682_amd as P

    w = make_workload(f"tile_reuse_prep_d{d}", 9, 83, d, 211, 190, "bf16", NEG_SHARED, 4242 + d, pad="bernoulli", pad_p=0.35,
                      g_kind="random", e_sigma=0.1, tgt_dist="zipf")
    assert ((w.neg[None, :] == w.tgt[:, None]).sum(1)[w.mask != 0]).max() >= 1   # collisions on valid positions
    a = _run(w, algo=P.CCE_ALGO_TILE, reuse_prep=True)
    check_against_oracle(w, a, TOL_BF16)
    b = _run(w, algo=P.CCE_ALGO_TILE, reuse_prep=False)
    assert np.array_equal(a["dH"], b["dH"]) and np.array_equal(a["loss"], b["loss"])
    assert tensor_rel(a["dE"], b["dE"]) <= 1e-5      # atomics: same terms, order may differ


@pytest.mark.parametrize("d", [64, 128, 256])
def test_two_backward_calls_reuse_one_forward_preparation(d):
    """What the forward call files for the backward pass survives a backward call: a second one on the same workspace
    (few positions and many candidates: the dH role splits and merges) adds the same gradient again."""
    import paper_2509_09682_amd as P

    w = make_workload(f"twice_d{d}", 7, 90, d, 6000, 0, "bf16", NEG_FULL, 99 + d, pad="bernoulli", pad_p=0.2, g_kind="random",
                      e_sigma=0.1, tgt_dist="zipf")
    out = _run(w, algo=P.CCE_ALGO_TILE, reuse_prep=True, repeat_backward=2)
    out["dE"] = out["dE"] * 0.5
    check_against_oracle(w, out, TOL_BF16)


@pytest.mark.parametrize("d", [64, 256])
def test_forward_and_dH_are_bitwise_reproducible(d):
    """No atomics feed loss, lse or dH: two runs on the same inputs must agree bit for bit (a vector instruction that
    read a matrix-instruction result too early once showed up here as last-bit noise)."""
    import paper_2509_09682_amd as P

    w = make_workload(f"tile_repro_d{d}", 60, 200, d, 211, 96, "bf16", NEG_SHARED, 99 + d, pad="none", g_kind="random",
                      e_sigma=0.1, tgt_dist="zipf")
    a = _run(w, algo=P.CCE_ALGO_TILE)
    for _ in range(3):
        b = _run(w, algo=P.CCE_ALGO_TILE)
        for name in ("loss", "lse", "dH"):
            assert np.array_equal(a[name].view(np.uint32), b[name].view(np.uint32)), name


def test_tile_path_many_positions_splits_the_dE_pass():
    import paper_2509_09682_amd as P

    w = make_workload("tile_split_de", 40, 77, 64, 5000, 130, "bf16", NEG_SHARED, 777, pad="bernoulli", pad_p=0.3,
                      g_kind="random", e_sigma=0.05, tgt_dist="zipf", zipf_s=1.2)
    out = _run(w, algo=P.CCE_ALGO_TILE)
    check_against_oracle(w, out, TOL_BF16)


def test_tile_path_index_validation_reports_and_stays_in_bounds():
    import paper_2509_09682_amd as P

    w = make_workload("tile_validate", 3, 50, 64, 300, 96, "bf16", NEG_SHARED, 41, g_kind="random")
    assert _run(w, algo=P.CCE_ALGO_TILE, validate=1)["status"] == P.CCE_OK
    w.neg[5] = 300
    w.neg[17] = -3
    w.tgt[11] = 1 << 20
    out = _run(w, algo=P.CCE_ALGO_TILE, validate=1)
    assert out["status"] == P.CCE_ERR_INDEX   # outputs of a flagged call are unspecified; it must only not fault


@pytest.mark.parametrize("d", [8, 24, 72, 320, 512])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_hidden_sizes_and_ragged_tail(d, dtype):
    w = make_workload(f"ragged_d{d}_{dtype}", 1, 37, d, 301, 19, dtype, NEG_PER_POSITION, 99 + d, pad="bernoulli",
                      pad_p=0.2, g_kind="random", e_sigma=0.3)
    check_against_oracle(w, _run(w), 2e-5)


def test_edge_cases_k0_single_position_all_masked_no_mask_no_g():
    import paper_2509_09682_amd as P

    w = make_workload("k0", 1, 9, 16, 50, 0, "f32", NEG_SHARED, 7, g_kind="random")
    out = _run(w)
    assert np.all(out["loss"] == 0)
    check_against_oracle(w, out, TOL_F32)

    w = make_workload("n1", 1, 1, 64, 50, 5, "bf16", NEG_SHARED, 8)
    check_against_oracle(w, _run(w, algo=P.CCE_ALGO_GATHER), 2e-5)
    check_against_oracle(w, _run(w, algo=P.CCE_ALGO_TILE), TOL_BF16)

    w = make_workload("all_masked", 2, 8, 32, 40, 6, "f32", NEG_PER_POSITION, 9)
    w.mask[:] = 0
    w.tgt[:] = -5            # never read
    w.neg[:] = 1 << 30
    out = _run(w)
    assert np.all(out["loss"] == 0) and np.all(out["dH"] == 0) and np.all(out["dE"] == 0)

    w = make_workload("nomask_nog", 2, 13, 64, 200, 17, "bf16", NEG_SHARED, 10)
    w.mask[:] = 1
    check_against_oracle(w, _run(w, g=None, use_mask=False, algo=P.CCE_ALGO_GATHER), 2e-5, g=None)
    check_against_oracle(w, _run(w, g=None, use_mask=False), TOL_BF16, g=None)

    w = make_workload("dup_collide", 2, 16, 32, 12, 30, "f32", NEG_PER_POSITION, 11, g_kind="random", e_sigma=0.5)
    for collide in (0, 1):   # V=12 < K: duplicates and collisions everywhere
        w.mask_collisions = collide
        check_against_oracle(w, _run(w), TOL_F32)

    # FULL mode in fp32
    w = make_workload("full_f32", 1, 21, 40, 333, 0, "f32", NEG_FULL, 12, g_kind="random", e_sigma=0.2)
    check_against_oracle(w, _run(w), TOL_F32)
    assert P.CCE_OK == 0


def test_dE_is_accumulated_into_and_dH_bf16_output():
    import paper_2509_09682_amd as P

    w = make_workload("accum", 2, 25, 64, 500, 33, "bf16", NEG_SHARED, 21, g_kind="random", pad="right", pad_len_lo=10)
    init = np.random.default_rng(1).standard_normal((w.V, w.d)).astype(np.float32)
    for algo, tol in ((P.CCE_ALGO_GATHER, 2e-5), (P.CCE_ALGO_TILE, TOL_BF16)):
        out = _run(w, dE_init=init.copy(), algo=algo)
        # the gradient is small next to the N(0,1) initial content: the difference carries the rounding of the sum
        check_against_oracle(w, out, max(tol, 1e-3), dE_init=init, dH_tol=tol)
        out = _run(w, dH_dtype=P.CCE_BF16, algo=algo)
        check_against_oracle(w, out, tol, dH_tol=max(tol, 2 ** -8))   # dH rounded to bf16: half an ulp = 2^-9


def test_index_validation_skips_bad_ids_and_reports():
    import paper_2509_09682_amd as P

    w = make_workload("validate", 2, 10, 32, 100, 8, "f32", NEG_PER_POSITION, 31, g_kind="random")
    clean = _run(w, validate=1)
    assert clean["status"] == P.CCE_OK
    bad = make_workload("validate", 2, 10, 32, 100, 8, "f32", NEG_PER_POSITION, 31, g_kind="random")
    bad.neg[3, 2] = 100            # == V: out of range
    bad.neg[5, 0] = -1
    bad.tgt[7] = 12345
    out = _run(bad, validate=1)
    assert out["status"] == P.CCE_ERR_INDEX
    # the oracle on the sanitised problem: bad negatives dropped = replaced by a collision, bad target = masked
    ref = make_workload("validate", 2, 10, 32, 100, 8, "f32", NEG_PER_POSITION, 31, g_kind="random")
    ref.neg[3, 2] = ref.tgt[3]
    ref.neg[5, 0] = ref.tgt[5]
    ref.mask[7] = 0
    check_against_oracle(ref, out, TOL_F32)


@pytest.mark.parametrize("idx", [2, 3])
def test_full_size_configs_against_full_oracle(idx):
    """The benchmark shapes, every output element held against the oracle (the oracle finishes these in seconds)."""
    w = config(idx)
    out = _run(w, reuse_prep=True)   # as bench.py runs it: the backward call reuses the forward call's preparation
    tol = TOL_BF16
    errs = check_against_oracle(w, out, tol)
    b = FULL_SIZE_BARS[idx]
    assert errs["dH"] <= b[0] and errs["dE"] <= b[1] and errs["dH_row"] <= b[2] and errs["dE_row"] <= b[3], (errs, b)
    # zero column sum of dE: sum_v dE[v,:] = sum_i g_i (sum_j p_ij - 1) h_i = 0
    scale = np.abs(out["dE"]).sum(0).max()
    assert np.abs(out["dE"].astype(np.float64).sum(0)).max() <= 1e-3 * scale, errs


def _peaked_full_workload(d, V, seed):
    """Full-catalogue workload with a concentrated softmax: hidden states point at their target's row."""
    from workloads import bf16_bits_from_f32, f32_from_bf16_bits

    w = make_workload(f"filter_d{d}", 5, 77, d, V, 0, "bf16", NEG_FULL, seed, pad="bernoulli", pad_p=0.25, g_kind="random",
                      e_sigma=1.0 / np.sqrt(d), tgt_dist="zipf")
    rng = np.random.default_rng(seed + 1)
    E = f32_from_bf16_bits(w.E)
    H = 9.0 * E[w.tgt] + 0.5 * rng.standard_normal((w.N, d)).astype(np.float32)
    w.H = bf16_bits_from_f32(H.astype(np.float32))
    return w


@pytest.mark.parametrize("d,V", [(64, 1500), (128, 700), (256, 900)])
def test_gradient_filtering_of_the_full_catalogue_mode(d, V):
    """filter_eps > 0: 32 x 32 blocks of the softmax matrix whose largest probability is below the threshold add nothing
    to dH and dE; loss and lse stay exact.  Held against the oracle's block reading at a threshold that no block
    maximum comes near (the two sides compute the probabilities in different precisions)."""
    import paper_2509_09682_amd as P

    w = _peaked_full_workload(d, V, 900 + d)
    _, valid, p = O.run_workload_filtered(w, 1e-3)
    # the threshold goes into the widest gap between block maxima around their median, so that about half of the blocks
    # are dropped and every verdict is clear-cut
    nr, nc = p.shape
    big = np.pad(p, ((0, -nr % 32), (0, -nc % 32))).reshape((nr + -nr % 32) // 32, 32, (nc + -nc % 32) // 32, 32).max(axis=(1, 3))
    srt = np.sort(big.ravel())
    cand = srt[int(0.3 * srt.size):int(0.7 * srt.size)]
    gaps = cand[1:] / cand[:-1]
    k = int(np.argmax(gaps))
    assert gaps[k] > 1.01
    eps = float(np.sqrt(cand[k] * cand[k + 1]))
    ref, valid, p = O.run_workload_filtered(w, eps)
    dropped = 1.0 - O.filter_blocks(p, eps).mean()
    assert 0.2 < dropped < 0.999, dropped            # most blocks go, some stay
    out = _run(w, algo=P.CCE_ALGO_TILE, filter_eps=eps)
    plain = _run(w, algo=P.CCE_ALGO_TILE)
    assert np.array_equal(out["loss"], plain["loss"]) and np.array_equal(out["lse"], plain["lse"])   # forward untouched
    assert np.all(out["dH"][w.mask == 0] == 0)
    e_dH = tensor_rel(out["dH"][valid], ref.dH)
    e_dE = tensor_rel(out["dE"], ref.dE)
    # the filtered gradient differs from the exact one by more than the tolerance: the test can tell them apart
    exact = O.run_workload(w)
    d_dH = tensor_rel(exact.dH[valid], ref.dH)
    print(w.name, f"eps {eps:.3e} dropped {dropped:.3f} dH {e_dH:.2e} dE {e_dE:.2e} (filtered vs exact oracle dH {d_dH:.2e})")
    assert e_dH <= TOL_BF16 and e_dE <= TOL_BF16, (e_dH, e_dE)


@pytest.mark.parametrize("d,V,eps", [(64, 1500, 1e-3), (128, 700, 1e-4), (256, 900, 1e-2)])
def test_gradient_filtering_against_the_unfiltered_definition(d, V, eps):
    """Evidence that does not lean on any block structure: only the paper's statement that values below the threshold
    are disregarded in the backward pass (Sec. 3.1, last paragraph).

    (i)  A threshold so small that nothing falls below it gives the gradients of the plain call.
    (ii) For eps > 0 the filtered gradient may differ from the UNFILTERED oracle gradient only by terms whose
         probability is below eps.  With p the oracle's softmax, position i may lose at most
         B_i = |g_i| sum_{j: p_ij < eps} p_ij max_t|E_jt| in any entry of dH_i, and item v at most
         C_v = sum_{i: p_iv < eps} |g_i| p_iv max_t|H_it| in any entry of dE_v: dropping one probability >= eps
         anywhere breaks the bound of its row.  loss and lse are exact.
    """
    import paper_2509_09682_amd as P
    from workloads import f32_from_bf16_bits

    w = _peaked_full_workload(d, V, 300 + d)
    plain = _run(w, algo=P.CCE_ALGO_TILE)
    tiny = _run(w, algo=P.CCE_ALGO_TILE, filter_eps=1e-37)
    assert np.array_equal(tiny["loss"], plain["loss"]) and np.array_equal(tiny["lse"], plain["lse"])
    assert tensor_rel(tiny["dH"], plain["dH"]) <= 1e-6 and tensor_rel(tiny["dE"], plain["dE"]) <= 1e-5

    out = _run(w, algo=P.CCE_ALGO_TILE, filter_eps=eps)
    assert np.array_equal(out["loss"], plain["loss"]) and np.array_equal(out["lse"], plain["lse"])
    valid = np.flatnonzero(w.mask != 0)
    exact = O.run_workload(w, sel=valid.astype(np.int64), want_p=True)           # the unfiltered definition
    p, g = exact.p, np.abs(w.g[valid].astype(np.float64))
    small = np.where(p < eps, p, 0.0)
    E_inf = np.abs(f32_from_bf16_bits(w.E).astype(np.float64)).max(1)
    H_inf = np.abs(f32_from_bf16_bits(w.H).astype(np.float64)).max(1)[valid]
    B = g * (small @ E_inf)                                                        # [n_valid]
    C = (small * (g * H_inf)[:, None]).sum(0)                                      # [V]
    # rounding of the kept terms: every probability enters the second product rounded to bf16 (2^-9 relative, doubled
    # here for the fp32 accumulation), whatever cancels inside a row
    slack_H = 2.0 ** -8 * g * (p @ E_inf) + 1e-6 * np.abs(exact.dH).max()
    slack_E = 2.0 ** -8 * (p * (g * H_inf)[:, None]).sum(0) + 1e-6 * np.abs(exact.dE).max()
    dev_H = np.abs(out["dH"][valid].astype(np.float64) - exact.dH).max(1)
    dev_E = np.abs(out["dE"].astype(np.float64) - exact.dE).max(1)
    frac_small = float((p < eps).mean())
    moved = float((dev_H > slack_H).mean())
    print(w.name, f"eps {eps:g}: {frac_small:.3f} of the probabilities are below it; dH rows beyond rounding {moved:.3f};",
          f"worst dH excess {np.max(dev_H - B - slack_H):.2e}, worst dE excess {np.max(dev_E - C - slack_E):.2e}")
    assert frac_small > 0.4
    assert np.all(dev_H <= B + slack_H) and np.all(dev_E <= C + slack_E)


def test_gradient_filtering_with_a_block_on_the_threshold():
    """A threshold within half a percent of one block's largest probability: the two sides compute that probability
    in different precisions, so either verdict on that block is right; every position must agree with one of the two
    oracle outcomes, and positions outside that block with both."""
    import paper_2509_09682_amd as P

    d, V = 64, 1500
    w = _peaked_full_workload(d, V, 700)
    _, valid, p = O.run_workload_filtered(w, 1e-3)
    nr, nc = p.shape
    big = np.pad(p, ((0, -nr % 32), (0, -nc % 32))).reshape((nr + -nr % 32) // 32, 32, (nc + -nc % 32) // 32, 32).max(axis=(1, 3))
    flat = np.sort(big.ravel())
    mid = flat[int(0.2 * flat.size):int(0.8 * flat.size)]
    # a block maximum with no other block maximum within 3 % of it
    lonely = np.flatnonzero((mid[1:-1] / mid[:-2] > 1.03) & (mid[2:] / mid[1:-1] > 1.03))
    assert lonely.size > 0
    m_star = float(mid[1 + lonely[lonely.size // 2]])
    eps = m_star * 1.004                      # by exact arithmetic the block is dropped
    ref_drop, _, _ = O.run_workload_filtered(w, eps)
    ref_keep, _, _ = O.run_workload_filtered(w, m_star * 0.996)
    bi = int(np.argwhere(big == m_star)[0][0])
    in_block = np.zeros(nr, bool)
    in_block[bi * 32:(bi + 1) * 32] = True
    assert np.array_equal(ref_drop.dH[~in_block], ref_keep.dH[~in_block])    # the two outcomes differ in that block only
    out = _run(w, algo=P.CCE_ALGO_TILE, filter_eps=eps)
    dH = out["dH"][valid].astype(np.float64)

    # per position: within the bf16 rounding of its kept probabilities (2^-8 |g_i| sum_j p_ij max|e_j|) of one outcome
    from workloads import f32_from_bf16_bits

    E_inf = np.abs(f32_from_bf16_bits(w.E).astype(np.float64)).max(1)
    bound = 2.0 ** -8 * np.abs(w.g[valid].astype(np.float64)) * (p @ E_inf) + 1e-6 * np.abs(ref_drop.dH).max()
    dev = np.minimum(np.abs(dH - ref_drop.dH).max(1), np.abs(dH - ref_keep.dH).max(1))
    both = np.maximum(np.abs(dH - ref_drop.dH).max(1), np.abs(dH - ref_keep.dH).max(1))
    print(w.name, f"threshold {eps:.4e} at block row {bi}: worst excess over the rounding model {np.max(dev - bound):.2e}")
    assert np.all(dev <= bound) and np.all(both[~in_block] <= bound[~in_block])
    assert min(tensor_rel(out["dE"], ref_drop.dE), tensor_rel(out["dE"], ref_keep.dE)) <= GRAD_BAR_TILE


def test_item_table_beyond_4_gib_uses_64_bit_load_addresses():
    """The tile kernels address streamed rows with 32-bit offsets below 4 GiB and with 64-bit addresses above:
    a 4.4 GB item table with negatives spread over all of it takes the second path."""
    import torch

    import paper_2509_09682_amd as P
    from hip_harness import to_device

    w = make_workload("tile_wide_table", 6, 200, 256, 8_600_000, 300, "bf16", NEG_SHARED, 31337, pad="right", pad_len_lo=120,
                      g_kind="random", e_sigma=0.05, tgt_dist="uniform")
    assert int(w.V) * w.d * 2 > 2 ** 32 and int(w.neg.max()) * w.d * 2 > 2 ** 32
    H, E, tgt, neg, mask = to_device(w)
    desc = P.make_desc(w.N, w.V, w.d, w.K, P.CCE_BF16, w.neg_mode, mask_target_collisions=w.mask_collisions, algo=P.CCE_ALGO_TILE)
    ws = P.new_workspace(desc)
    loss = torch.full((w.N,), float("nan"), device="cuda")
    lse = torch.full((w.N,), float("nan"), device="cuda")
    dH = torch.full((w.N, w.d), float("nan"), device="cuda")
    dE = torch.zeros((w.V, w.d), device="cuda")
    P.cce_neg_forward(desc, H, E, tgt, neg, mask, loss, lse, ws)
    P.cce_neg_backward(desc, H, E, tgt, neg, mask, lse, torch.from_numpy(w.g).cuda(), dH, dE, ws)
    torch.cuda.synchronize()
    S = np.flatnonzero(w.mask).astype(np.int64)
    ref = O.run_workload(w, sel=S, want_dE="compact")
    e_loss = per_position_rel(loss.cpu().numpy()[S], ref.loss, ref.lse, ref.loss)
    e_lse = per_position_rel(lse.cpu().numpy()[S], ref.loss, ref.lse, ref.lse)
    e_dH = tensor_rel(dH.cpu().numpy()[S], ref.dH)
    rows = torch.from_numpy(ref.dE_rows).cuda()
    e_dE = tensor_rel(dE[rows].cpu().numpy(), ref.dE)
    other = torch.ones(w.V, dtype=torch.bool, device="cuda")
    other[rows] = False
    assert float(dE[other].abs().max()) == 0.0
    errs = dict(loss=e_loss, lse=e_lse, dH=e_dH, dE=e_dE)
    print(w.name, {k: f"{v:.2e}" for k, v in errs.items()})
    assert all(v <= TOL_BF16 for v in errs.values()), errs


@pytest.mark.parametrize("idx,n_sample", [(4, 512), (5, 1280)])
def test_full_size_large_configs_on_sampled_positions(idx, n_sample):
    """The benchmark shapes the oracle cannot finish in seconds, in the launch configuration bench.py times.

    Forward: loss and lse of EVERY valid position are held against the oracle (forward only, about a minute of host time).
    Run 1: grad_loss is non-zero on a sample S of valid positions only: the first 64 and the last 256 valid positions
    (first block; last round of blocks and its split tail) and a random draw from the rest.  dH and dE are linear in
    grad_loss, so the oracle needs just the positions of S: dH rows of S and the whole dE are held against it, dH rows
    outside S must be zero and dE rows that S does not index must stay zero.
    Run 2: the benchmark's own grad_loss; properties that hold at any size: the zero column sum of dE and the exact set
    of changed rows for the sampled modes.
    """
    import torch

    import paper_2509_09682_amd as P
    from hip_harness import to_device

    w = config(idx)
    rng = np.random.default_rng(1234 + idx)
    valid_idx = np.flatnonzero(w.mask)
    head, tail = valid_idx[:64], valid_idx[-256:]
    middle = rng.choice(valid_idx[64:-256], size=n_sample - 320, replace=False)
    S = np.sort(np.concatenate([head, middle, tail])).astype(np.int64)
    g = np.zeros(w.N, np.float32)
    g[S] = rng.standard_normal(n_sample).astype(np.float32)

    H, E, tgt, neg, mask = to_device(w)
    desc = P.make_desc(w.N, w.V, w.d, w.K, P.CCE_BF16, w.neg_mode, mask_target_collisions=w.mask_collisions)
    desc_bwd = P.make_desc(w.N, w.V, w.d, w.K, P.CCE_BF16, w.neg_mode, mask_target_collisions=w.mask_collisions,
                           reuse_forward_prep=1)   # as in bench.py
    ws = P.new_workspace(desc)
    loss = torch.full((w.N,), float("nan"), device="cuda")
    lse = torch.full((w.N,), float("nan"), device="cuda")
    dH = torch.full((w.N, w.d), float("nan"), device="cuda")
    dE = torch.zeros((w.V, w.d), device="cuda")
    P.cce_neg_forward(desc, H, E, tgt, neg, mask, loss, lse, ws)
    P.cce_neg_backward(desc_bwd, H, E, tgt, neg, mask, lse, torch.from_numpy(g).cuda(), dH, dE, ws)
    torch.cuda.synchronize()

    # ---- forward, every valid position
    print(w.name, "oracle forward on all", valid_idx.size, "valid positions ...", flush=True)
    allv = valid_idx.astype(np.int64)
    fwd = O.run_workload(w, sel=allv, want_dE="none", want_dH=False)
    loss_all, lse_all = loss.cpu().numpy(), lse.cpu().numpy()
    e_loss_all = per_position_rel(loss_all[allv], fwd.loss, fwd.lse, fwd.loss)
    e_lse_all = per_position_rel(lse_all[allv], fwd.loss, fwd.lse, fwd.lse)
    print(w.name, "all positions", dict(loss=f"{e_loss_all:.2e}", lse=f"{e_lse_all:.2e}"), flush=True)
    assert e_loss_all <= TOL_BF16 and e_lse_all <= TOL_BF16
    assert e_loss_all <= FWD_BAR_TILE and e_lse_all <= FWD_BAR_TILE

    print(w.name, "oracle forward + backward on", S.size, "sampled positions ...", flush=True)
    ref = O.run_workload(w, g=g.astype(np.float64), sel=S, want_dE="compact")
    assert np.all(loss_all[w.mask == 0] == 0) and np.all(lse_all[w.mask == 0] == 0)
    assert np.all(np.isfinite(loss_all)) and np.all(np.isfinite(lse_all))
    dH_S = dH[torch.from_numpy(S).cuda()].cpu().numpy()
    e_dH, r_dH = tensor_rel(dH_S, ref.dH), row_rel(dH_S, ref.dH)
    rest = torch.ones(w.N, dtype=torch.bool, device="cuda")
    rest[torch.from_numpy(S).cuda()] = False
    assert float(dH[rest].abs().max()) == 0.0
    rows = torch.from_numpy(ref.dE_rows).cuda()
    dE_rows = dE[rows].cpu().numpy()
    e_dE, r_dE = tensor_rel(dE_rows, ref.dE), row_rel(dE_rows, ref.dE)
    other = torch.ones(w.V, dtype=torch.bool, device="cuda")
    other[rows] = False
    assert float(dE[other].abs().max()) == 0.0 if bool(other.any()) else True
    errs = dict(dH=e_dH, dE=e_dE, dH_row=r_dH, dE_row=r_dE)
    print(w.name, "sampled", {k: f"{v:.2e}" for k, v in errs.items()}, flush=True)
    b = FULL_SIZE_BARS[idx]
    assert e_dH <= b[0] and e_dE <= b[1] and r_dH <= b[2] and r_dE <= b[3], (errs, b)

    # ---- run 2: the benchmark's grad_loss
    dE.zero_()
    P.cce_neg_backward(desc_bwd, H, E, tgt, neg, mask, lse, torch.from_numpy(w.g).cuda(), dH, dE, ws)
    torch.cuda.synchronize()
    col = dE.double().sum(0).abs().max().item()
    scale = dE.double().abs().sum(0).max().item()
    assert col <= 2e-3 * scale, (col, scale)
    if w.neg_mode != NEG_FULL:
        touched = O.touched_rows(w.tgt, w.neg, w.mask, w.neg_mode, w.V, mask_collisions=w.mask_collisions)
        changed = torch.nonzero((dE != 0).any(1)).flatten().cpu().numpy()
        assert np.all(np.isin(changed, touched))
        # every row of a target or negative normally receives a non-zero gradient; allow exact cancellations
        assert changed.size >= 0.999 * touched.size


@pytest.mark.parametrize("case", ["all_hot", "zipf_head"])
def test_per_position_negatives_with_items_sampled_very_often(case):
    """Items with more pairs than one lane group walks are cut into chunks and added by the work-list kernel."""
    import dataclasses

    from workloads import zipf_ids

    if case == "all_hot":      # 50 items, 600 x 64 pairs: every item has several hundred pairs
        w = make_workload("hot", 600, 1, 128, 50, 64, "bf16", NEG_PER_POSITION, 31, g_kind="random", pad="bernoulli", pad_p=0.1)
    else:                      # power-law negatives: the head is hot, the tail is sampled once or never
        w = make_workload("hot", 900, 1, 64, 3000, 128, "bf16", NEG_PER_POSITION, 32, g_kind="random")
        rng = np.random.default_rng(5)
        ids, _ = zipf_ids(rng, rng, w.N * w.K, w.V, 1.3)
        w = dataclasses.replace(w, neg=ids.reshape(w.N, w.K))
    counts = np.bincount(w.neg[w.mask != 0].ravel(), minlength=w.V)
    assert counts.max() > 600 and (case == "all_hot" or (counts <= 4).sum() > 100)   # one lane group walks 256 pairs
    check_against_oracle(w, _run(w), 2e-5)


@pytest.mark.parametrize("batch,pad", [(357, "right"), (264, "none"), (460, "bernoulli"), (400, "none")])
def test_last_round_of_position_blocks_splits_the_candidates(batch, pad):
    """d = 256 with more position blocks than the chip holds at once: the blocks of the last, partly filled round split
    the candidate range and a merge adds the partial dH rows (planned on the device from the count of valid positions).
    Cases: last rounds of 63, 8 and 88 blocks on 256 slots (split 4, 4 and 2 ways; with 70 candidates = 3 tiles some
    splits are empty), and one of 144 blocks, which stays whole."""
    w = make_workload("tail", batch, 256, 256, 3000, 70, "bf16", NEG_SHARED, 41 + batch, g_kind="random", tgt_dist="zipf",
                      pad=pad, pad_p=0.25, pad_len_lo=200)
    assert w.n_valid > 65536
    print("valid positions", w.n_valid, "position blocks", -(-w.n_valid // 256))
    check_against_oracle(w, _run(w), TOL_BF16)
    out = _run(w, reuse_prep=True, dH_dtype=__import__("paper_2509_09682_amd").CCE_BF16)
    check_against_oracle(w, out, TOL_BF16)


@pytest.mark.parametrize("d,mode", [(64, NEG_FULL), (128, NEG_SHARED), (256, NEG_FULL)])
def test_scores_that_outgrow_the_running_maximum_by_hundreds_of_nats(d, mode):
    """The forward pass sums a tile's exponentials against the maximum it knew when the tile began and repeats the tile
    exactly when that overflowed.  Here the scores of a position climb (or fall) by several hundred nats along the
    candidate index, far beyond the range of a float exponential relative to a stale maximum."""
    from workloads import bf16_bits_from_f32

    V, K = 3000, 1500
    w = make_workload(f"steep_d{d}", 3, 111, d, V, 0 if mode == NEG_FULL else K, "bf16", mode, 7 + d, pad="bernoulli", pad_p=0.1,
                      g_kind="random", neg_dist="uniform")
    rng = np.random.default_rng(d)
    u = rng.standard_normal(d).astype(np.float32)
    u /= np.linalg.norm(u)
    slope = rng.uniform(-1.5, 1.5, size=w.N).astype(np.float32)               # climbing and falling positions
    H = slope[:, None] * u[None, :] + 0.01 * rng.standard_normal((w.N, d)).astype(np.float32)
    ramp = np.arange(V, dtype=np.float32) / V
    if mode == NEG_SHARED:                                                     # make the ramp follow the candidate order
        order = np.empty(V, np.float32)
        order[:] = 0.5
        order[w.neg] = np.arange(K, dtype=np.float32) / K
        ramp = order
    E = 400.0 * ramp[:, None] * u[None, :] + 0.01 * rng.standard_normal((V, d)).astype(np.float32)
    w.H = bf16_bits_from_f32(H.astype(np.float32))
    w.E = bf16_bits_from_f32(E.astype(np.float32))
    out = _run(w)
    assert np.all(np.isfinite(out["loss"])) and np.all(np.isfinite(out["dH"]))
    ref = O.run_workload(w, g=w.g.astype(np.float64), want_p=True)
    assert np.abs(ref.lse).max() > 300
    # a few candidates at the end of the ramp carry the whole softmax, so rows nearly cancel (p of one candidate close
    # to 1 against the correct item's -1): the per-row check is the rounding model, not the row's own size
    check_against_oracle(w, out, TOL_BF16, row_tol=1.0)
    ex_H, ex_E = rounding_model_excess(w, out, ref)
    print(w.name, f"excess over the bf16 rounding model: dH {ex_H:.2e} dE {ex_E:.2e}")
    assert ex_H <= 0 and ex_E <= 0


@pytest.mark.parametrize("seed", range(72))
def test_random_small_shapes_every_mode(seed):
    """Seeded random draws of shape, mode, dtype, padding, collision flag, algorithm, dH dtype and the reuse flag."""
    import paper_2509_09682_amd as P

    rng = np.random.default_rng(9000 + seed)
    mode = [NEG_SHARED, NEG_PER_POSITION, NEG_FULL][seed % 3]
    dtype = "bf16" if rng.random() < 0.7 else "f32"
    d = int(rng.choice([64, 128, 256])) if (dtype == "bf16" and rng.random() < 0.7) else int(8 * rng.integers(1, 41))
    batch, seq = int(rng.integers(1, 9)), int(rng.integers(1, 90))
    V = int(rng.integers(40, 2500))
    K = 0 if mode == NEG_FULL else int(rng.integers(1, 400))
    pad = ["none", "bernoulli", "right"][int(rng.integers(0, 3))]
    w = make_workload(f"rand{seed}", batch, seq, d, V, K, dtype, mode, 5000 + seed, g_kind="random", pad=pad, pad_p=0.3,
                      pad_len_lo=0, tgt_dist="zipf" if rng.random() < 0.5 else "uniform", e_sigma=0.2,
                      mask_collisions=int(rng.integers(0, 2)))
    tile_ok = dtype == "bf16" and mode != NEG_PER_POSITION and d in (64, 128, 256)
    algo = P.CCE_ALGO_AUTO if (tile_ok and rng.random() < 0.7) else P.CCE_ALGO_GATHER
    on_tiles = tile_ok and algo == P.CCE_ALGO_AUTO
    dH_dtype = P.CCE_BF16 if (dtype == "bf16" and rng.random() < 0.4) else P.CCE_F32
    reuse = bool(rng.integers(0, 2))
    print(dict(mode=mode, dtype=dtype, d=d, N=w.N, V=V, K=K, pad=pad, collide=w.mask_collisions, tiles=on_tiles,
               dH_bf16=dH_dtype == P.CCE_BF16, reuse=reuse))
    out = _run(w, algo=algo, dH_dtype=dH_dtype, reuse_prep=reuse, use_mask=True)
    tol = TOL_BF16 if on_tiles else (TOL_F32 if dtype == "f32" else 2e-5)
    check_against_oracle(w, out, tol, dH_tol=max(tol, 8e-3) if dH_dtype == P.CCE_BF16 else None)


@pytest.mark.parametrize("seed", range(18))
def test_random_medium_shapes_on_the_matrix_core_path(seed):
    """Several tiles, ragged tails, split and unsplit grids: bf16, shared negatives or full catalogue, d in {64,128,256}."""
    import paper_2509_09682_amd as P

    rng = np.random.default_rng(7000 + seed)
    mode = NEG_SHARED if seed % 2 == 0 else NEG_FULL
    d = [64, 128, 256][seed % 3]
    batch, seq = int(rng.integers(2, 40)), int(rng.integers(20, 160))
    V = int(rng.integers(600, 9000))
    K = 0 if mode == NEG_FULL else int(rng.integers(100, 1600))
    pad = ["none", "bernoulli", "right"][int(rng.integers(0, 3))]
    w = make_workload(f"med{seed}", batch, seq, d, V, K, "bf16", mode, 8000 + seed, g_kind="random", pad=pad, pad_p=0.2,
                      pad_len_lo=seq // 2, tgt_dist="zipf", e_sigma=0.1, mask_collisions=int(rng.integers(0, 2)))
    reuse = bool(rng.integers(0, 2))
    print(dict(mode=mode, d=d, N=w.N, V=V, K=K, pad=pad, collide=w.mask_collisions, reuse=reuse))
    check_against_oracle(w, _run(w, algo=P.CCE_ALGO_TILE, reuse_prep=reuse), TOL_BF16)


@pytest.mark.parametrize("case", ["ordinary_buckets", "one_crowded_bucket", "power_law"])
def test_per_position_index_built_in_slices(case):
    """More (position, negative) pairs than one slice of the inverted index holds (2^22): the index is built and used
    up slice by slice over the item-id range.  ordinary_buckets: uniform ids over 147 buckets, two slices.
    one_crowded_bucket: a catalogue of 1000 items, so all 8.4 M pairs fall into one bucket of 2048 ids, more than a
    eighth of the budget: the bucket stays out of the index and its pairs are added with atomics.  power_law: the
    head item's bucket is crowded, the others are sliced."""
    import dataclasses

    from workloads import zipf_ids

    if case == "ordinary_buckets":
        w = make_workload("slices", 100, 200, 64, 300_000, 300, "bf16", NEG_PER_POSITION, 77, g_kind="random", pad="bernoulli",
                          pad_p=0.1, tgt_dist="zipf")
    elif case == "one_crowded_bucket":
        w = make_workload("slices_hot", 128, 128, 64, 1000, 512, "bf16", NEG_PER_POSITION, 78, g_kind="random", pad="none")
    else:
        w = make_workload("slices_zipf", 100, 200, 64, 50_000, 300, "bf16", NEG_PER_POSITION, 79, g_kind="random", pad="right",
                          pad_len_lo=150)
        rng = np.random.default_rng(6)
        ids, _ = zipf_ids(rng, rng, w.N * w.K, w.V, 1.3)
        w = dataclasses.replace(w, neg=ids.reshape(w.N, w.K))
    assert w.N * w.K > (1 << 22)
    counts = np.bincount((w.neg[w.mask != 0].ravel() >> 11), minlength=(w.V + 2047) >> 11)
    print(case, "pairs", w.N * w.K, "buckets", counts.size, "largest bucket", int(counts.max()))
    if case != "ordinary_buckets":
        assert counts.max() > (1 << 19)      # beyond an eighth of the budget
    if case == "power_law":
        # the head item's dE row is a sum of over a million terms of both signs, taken by fp32 atomics in arrival order:
        # its rounding error is that of the summation (about sqrt(n) * 2^-24 of the sum of magnitudes), not of the terms
        check_against_oracle(w, _run(w), 2e-3, row_tol=2e-3)
    else:
        check_against_oracle(w, _run(w), 2e-5)
