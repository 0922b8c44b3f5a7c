"""Pins of the fp64 oracle against things other than itself (CPU only).

Each test names what fixes the expected value: a library routine on explicitly
materialised logits, a closed form, an invariant of softmax cross-entropy, finite
differences, or the paper's listings restated step by step.
"""
import math
import os

import numpy as np
import pytest
import torch

from oracle import cce_oracle as O
from workloads import bf16_bits_from_f32, f32_from_bf16_bits

SH, PP, FULL = O.NEG_SHARED, O.NEG_PER_POSITION, O.NEG_FULL


def _rand(seed, N=7, V=23, d=5, K=6, e_sigma=0.7):
    r = np.random.default_rng(seed)
    H = r.standard_normal((N, d)).astype(np.float32)
    E = (e_sigma * r.standard_normal((V, d))).astype(np.float32)
    tgt = r.integers(0, V, N).astype(np.int32)
    return r, H, E, tgt


def _torch_ce_on_logits(logits64, pos_col):
    """Library routine: per-row cross entropy and logsumexp on materialised logits."""
    t = torch.from_numpy(logits64)
    lse = torch.logsumexp(t, dim=1).numpy()
    ce = torch.nn.functional.cross_entropy(t, torch.from_numpy(np.asarray(pos_col, dtype=np.int64)), reduction="none").numpy()
    return ce, lse


# ---- P1: full-catalogue mode against brute-force softmax over all items ---------------------------------------
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_full_mode_equals_bruteforce_cross_entropy(seed):
    _, H, E, tgt = _rand(seed, N=8, V=64, d=8)
    res = O.run(H, E, tgt, None, None, None, in_dtype="f32", neg_mode=FULL, want_p=True)
    logits = H.astype(np.float64) @ E.astype(np.float64).T
    ce, lse = _torch_ce_on_logits(logits, tgt)
    np.testing.assert_allclose(res.loss, ce, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(res.lse, lse, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(res.p, torch.softmax(torch.from_numpy(logits), 1).numpy(), rtol=1e-12, atol=1e-15)


# ---- P2: sampled modes reduce to the full catalogue --------------------------------------------------------------
def test_per_position_all_other_items_equals_full_cross_entropy():
    _, H, E, tgt = _rand(3, N=9, V=31, d=6)
    V = E.shape[0]
    neg = np.stack([np.delete(np.arange(V, dtype=np.int32), t) for t in tgt])  # K = V-1, every id but the target
    res = O.run(H, E, tgt, neg, None, None, in_dtype="f32", neg_mode=PP, mask_collisions=0)
    full = O.run(H, E, tgt, None, None, None, in_dtype="f32", neg_mode=FULL)
    ce, lse = _torch_ce_on_logits(H.astype(np.float64) @ E.astype(np.float64).T, tgt)
    np.testing.assert_allclose(res.loss, ce, rtol=1e-13)
    np.testing.assert_allclose(res.lse, lse, rtol=1e-13)
    np.testing.assert_allclose(res.dH, full.dH, rtol=1e-11, atol=1e-14)
    np.testing.assert_allclose(res.dE, full.dE, rtol=1e-11, atol=1e-14)


def test_shared_all_items_with_collision_mask_equals_full_cross_entropy():
    r, H, E, tgt = _rand(4, N=10, V=29, d=4)
    V = E.shape[0]
    neg = r.permutation(V).astype(np.int32)  # every id once: each position's own target collides and is dropped
    g = r.standard_normal(H.shape[0])
    res = O.run(H, E, tgt, neg, None, g, in_dtype="f32", neg_mode=SH, mask_collisions=1)
    full = O.run(H, E, tgt, None, None, g, in_dtype="f32", neg_mode=FULL)
    np.testing.assert_allclose(res.loss, full.loss, rtol=1e-13)
    np.testing.assert_allclose(res.dH, full.dH, rtol=1e-11, atol=1e-14)
    np.testing.assert_allclose(res.dE, full.dE, rtol=1e-11, atol=1e-14)
    # without the collision mask the target is counted twice: LSE must grow by exactly log(1 + p_target)
    res0 = O.run(H, E, tgt, neg, None, g, in_dtype="f32", neg_mode=SH, mask_collisions=0)
    p_t = np.exp(-full.loss)
    np.testing.assert_allclose(res0.lse - full.lse, np.log1p(p_t), rtol=1e-11)


# ---- P10: torch fp64 logsumexp / autograd on explicitly gathered [N, 1+K] logits -----------------------------------
@pytest.mark.parametrize("mode", [SH, PP])
@pytest.mark.parametrize("collide", [0, 1])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_against_torch_autograd_on_gathered_logits(mode, collide, dtype):
    r, H, E, tgt = _rand(10 + mode * 2 + collide, N=12, V=17, d=8, K=9)
    N, V, K = H.shape[0], E.shape[0], 9
    if dtype == "bf16":
        Hs, Es = bf16_bits_from_f32(H), bf16_bits_from_f32(E)
        H, E = f32_from_bf16_bits(Hs), f32_from_bf16_bits(Es)
    else:
        Hs, Es = H, E
    neg = r.integers(0, V, (K,) if mode == SH else (N, K)).astype(np.int32)  # V small: duplicates and collisions occur
    mask = (r.random(N) > 0.25).astype(np.uint8)
    g = r.standard_normal(N)
    assert ((neg if mode == PP else neg[None, :].repeat(N, 0)) == tgt[:, None]).any()

    res = O.run(Hs, Es, tgt, neg, mask, g, in_dtype=dtype, neg_mode=mode, mask_collisions=collide)

    Ht = torch.tensor(H, dtype=torch.float64, requires_grad=True)
    Et = torch.tensor(E, dtype=torch.float64, requires_grad=True)
    negm = torch.from_numpy((neg if mode == PP else np.broadcast_to(neg, (N, K))).astype(np.int64))
    inds = torch.cat([torch.from_numpy(tgt.astype(np.int64))[:, None], negm], dim=1)
    logits = torch.einsum("nd,nkd->nk", Ht, Et[inds])
    if collide:
        dead = torch.zeros_like(logits, dtype=torch.bool)
        dead[:, 1:] = negm == inds[:, :1]
        logits = logits.masked_fill(dead, float("-inf"))
    ce = torch.nn.functional.cross_entropy(logits, torch.zeros(N, dtype=torch.int64), reduction="none")
    lse = torch.logsumexp(logits, dim=1)
    mt = torch.from_numpy(mask.astype(np.float64))
    (ce * mt * torch.from_numpy(g)).sum().backward()

    v = mask != 0
    np.testing.assert_allclose(res.loss[v], ce.detach().numpy()[v], rtol=1e-12)
    np.testing.assert_allclose(res.lse[v], lse.detach().numpy()[v], rtol=1e-12)
    assert np.all(res.loss[~v] == 0) and np.all(res.lse[~v] == 0) and np.all(res.dH[~v] == 0)
    np.testing.assert_allclose(res.dH, Ht.grad.numpy(), rtol=1e-10, atol=1e-13)
    np.testing.assert_allclose(res.dE, Et.grad.numpy(), rtol=1e-10, atol=1e-13)


# ---- P3: central finite differences of sum_i g_i loss_i -----------------------------------------------------------
@pytest.mark.parametrize("mode", [SH, PP, FULL])
def test_gradients_match_finite_differences(mode):
    r, H, E, tgt = _rand(20 + mode, N=5, V=11, d=3, K=4)
    N, V, K = 5, 11, 4
    neg = None if mode == FULL else r.integers(0, V, (K,) if mode == SH else (N, K)).astype(np.int32)
    g = r.standard_normal(N)
    mask = np.array([1, 1, 0, 1, 1], np.uint8)

    def total(Hx, Ex):
        o = O.run(Hx, Ex, tgt, neg, mask, g, in_dtype="f32", neg_mode=mode, want_dH=False, want_dE="none")
        return float(np.sum(g * o.loss))

    res = O.run(H, E, tgt, neg, mask, g, in_dtype="f32", neg_mode=mode)
    # float32 storage: use steps that are exactly representable around each value
    h = 2.0 ** -10
    for (arr, grad, name) in ((H, res.dH, "dH"), (E, res.dE, "dE")):
        num = np.zeros_like(grad)
        for idx in np.ndindex(arr.shape):
            a0 = arr[idx]
            hi, lo = np.float32(a0 + h), np.float32(a0 - h)
            arr[idx] = hi
            fp = total(H, E)
            arr[idx] = lo
            fm = total(H, E)
            arr[idx] = a0
            num[idx] = (fp - fm) / (float(hi) - float(lo))
        np.testing.assert_allclose(grad, num, rtol=2e-5, atol=2e-6, err_msg=name)


# ---- P4 / P5 / P6: softmax rows, closed-form dH from p, zero column sum of dE --------------------------------------
@pytest.mark.parametrize("mode", [SH, PP, FULL])
def test_softmax_rows_sum_to_one_and_closed_form_dH_and_zero_column_sum(mode):
    r, H, E, tgt = _rand(30 + mode, N=16, V=40, d=8, K=12)
    N, V, K = 16, 40, 12
    neg = None if mode == FULL else r.integers(0, V, (K,) if mode == SH else (N, K)).astype(np.int32)
    g = r.standard_normal(N)
    mask = (r.random(N) > 0.2).astype(np.uint8)
    res = O.run(H, E, tgt, neg, mask, g, in_dtype="f32", neg_mode=mode, want_p=True)
    v = mask != 0
    np.testing.assert_allclose(res.p[v].sum(1), 1.0, atol=1e-14)
    assert np.all(res.p[~v] == 0)
    # dH_i = g_i * sum_j (p_ij - y_ij) e_ij, rebuilt here from the returned p
    E64 = E.astype(np.float64)
    for i in range(N):
        if mode == FULL:
            cand, pos = np.arange(V), int(tgt[i])
        else:
            cand = np.concatenate([[tgt[i]], neg if mode == SH else neg[i]])
            pos = 0
        y = np.zeros(len(cand))
        y[pos] = 1.0
        want = g[i] * ((res.p[i] - y * (mask[i] != 0))[:, None] * E64[cand]).sum(0)
        np.testing.assert_allclose(res.dH[i], want, rtol=1e-11, atol=1e-14)
    # sum over items of dE = sum_i g_i (sum_j p_ij - 1) h_i = 0
    assert np.abs(res.dE.sum(0)).max() < 1e-13
    # rows that no valid position indexes stay exactly zero
    rows = O.touched_rows(tgt, neg, mask, mode, V)
    untouched = np.setdiff1d(np.arange(V), rows)
    assert np.all(res.dE[untouched] == 0)


# ---- P7: closed forms -----------------------------------------------------------------------------------------------
def _golden():
    path = os.path.join(os.path.dirname(__file__), "golden", "closed_forms.txt")
    out = {}
    for line in open(path):
        if line.strip() and not line.startswith("#"):
            name, n, val = line.split()
            out[name] = (int(n), float(val))
    return out


def test_zero_hidden_gives_log_of_live_count():
    gold = _golden()
    r = np.random.default_rng(5)
    for name, K, V in (("zero_hidden_K128", 128, 4096), ("zero_hidden_K1", 1, 10), ("zero_hidden_K1024", 1024, 50000)):
        n_live, val = gold[name]
        assert n_live == K + 1 and abs(val - math.log(n_live)) < 1e-15
        E = r.standard_normal((V, 4)).astype(np.float32)
        H = np.zeros((3, 4), np.float32)
        tgt = np.array([0, 1, 2], np.int32)
        neg = np.arange(3, 3 + K, dtype=np.int32)  # no collisions
        res = O.run(H, E, tgt, neg, None, None, in_dtype="f32", neg_mode=SH, want_p=True)
        np.testing.assert_allclose(res.loss, val, rtol=1e-15)
        np.testing.assert_allclose(res.lse, val, rtol=1e-15)
        np.testing.assert_allclose(res.p, 1.0 / n_live, rtol=1e-14)
    n_live, val = gold["zero_hidden_full_V64"]
    E = r.standard_normal((64, 4)).astype(np.float32)
    res = O.run(np.zeros((2, 4), np.float32), E, np.array([5, 9], np.int32), None, None, None, in_dtype="f32", neg_mode=FULL)
    np.testing.assert_allclose(res.loss, val, rtol=1e-15)
    # a collision removes one live candidate: log(K) instead of log(K+1)
    neg = np.array([0, 7, 8, 9], np.int32)
    res = O.run(np.zeros((1, 4), np.float32), E, np.array([0], np.int32), neg, None, None, in_dtype="f32", neg_mode=SH)
    np.testing.assert_allclose(res.loss, math.log(4), rtol=1e-15)
    res = O.run(np.zeros((1, 4), np.float32), E, np.array([0], np.int32), neg, None, None, in_dtype="f32", neg_mode=SH, mask_collisions=0)
    np.testing.assert_allclose(res.loss, math.log(5), rtol=1e-15)


def test_no_negatives_gives_zero_loss_and_zero_gradients():
    _, H, E, tgt = _rand(6)
    res = O.run(H, E, tgt, None, None, None, in_dtype="f32", neg_mode=SH, K=0)
    assert np.all(res.loss == 0) and np.all(res.dH == 0) and np.all(res.dE == 0)
    np.testing.assert_allclose(res.lse, np.einsum("nd,nd->n", H.astype(np.float64), E[tgt].astype(np.float64)), rtol=1e-14)


def test_dominant_and_extreme_scores():
    d = 4
    E = np.zeros((6, d), np.float32)
    E[0, 0] = 1.0   # item 0 scores +s, item 1 scores -s, the rest 0
    E[1, 0] = -1.0
    for s in (50.0, 200.0, 700.0):
        H = np.zeros((2, d), np.float32)
        H[:, 0] = s
        neg = np.array([1, 2, 3], np.int32)
        # target = dominant item: loss = log(1 + 2 e^-s + e^-2s) -> ~0 ; lse -> s
        res = O.run(H, E, np.array([0, 0], np.int32), neg, None, None, in_dtype="f32", neg_mode=SH)
        assert np.all(np.isfinite(res.loss)) and np.all(np.isfinite(res.dH)) and np.all(np.isfinite(res.dE))
        # loss = lse - o+ cancels to rounding level of s (about 1e-14) when the target dominates
        np.testing.assert_allclose(res.loss, np.log1p(2 * math.exp(-s) + math.exp(-2 * s)), rtol=1e-12, atol=2e-13)
        np.testing.assert_allclose(res.lse, s + np.log1p(2 * math.exp(-s) + math.exp(-2 * s)), rtol=1e-14)
        # target = a zero-score item while item 0 dominates among the negatives: loss = s + log(1 + 2e^-s + e^-2s)
        res = O.run(H, E, np.array([4, 4], np.int32), np.array([0, 1, 2], np.int32), None, None, in_dtype="f32", neg_mode=SH)
        np.testing.assert_allclose(res.loss, s + np.log1p(2 * math.exp(-s) + math.exp(-2 * s)), rtol=1e-14)
        assert np.all(np.isfinite(res.dH))


# ---- P8: invariances ------------------------------------------------------------------------------------------------
def test_permutation_duplicates_shift_and_bounds():
    r, H, E, tgt = _rand(40, N=6, V=50, d=6, K=10)
    N, K = 6, 10
    neg = r.integers(0, 50, (N, K)).astype(np.int32)
    g = r.standard_normal(N)
    base = O.run(H, E, tgt, neg, None, g, in_dtype="f32", neg_mode=PP, want_p=True)
    # order of negatives is irrelevant
    perm = r.permutation(K)
    res = O.run(H, E, tgt, neg[:, perm], None, g, in_dtype="f32", neg_mode=PP)
    np.testing.assert_allclose(res.loss, base.loss, rtol=1e-13)
    np.testing.assert_allclose(res.dH, base.dH, rtol=1e-10, atol=1e-14)
    np.testing.assert_allclose(res.dE, base.dE, rtol=1e-10, atol=1e-14)
    # a repeated negative counts twice: lse' = log(e^lse + e^o_dup) = lse + log(1 + p_dup)
    dup = np.concatenate([neg, neg[:, 3:4]], axis=1)
    res = O.run(H, E, tgt, dup, None, g, in_dtype="f32", neg_mode=PP)
    live = base.p[:, 4] > 0
    np.testing.assert_allclose((res.lse - base.lse)[live], np.log1p(base.p[live, 4]), rtol=1e-10)
    # max o <= lse <= max o + log(#live)
    scores = np.einsum("nd,nkd->nk", H.astype(np.float64), E[np.concatenate([tgt[:, None], neg], 1)].astype(np.float64))
    livem = np.concatenate([np.ones((N, 1), bool), neg != tgt[:, None]], 1)
    mx = np.where(livem, scores, -np.inf).max(1)
    assert np.all(base.lse >= mx - 1e-12) and np.all(base.lse <= mx + np.log(livem.sum(1)) + 1e-12)
    # softmax shift invariance: adding a vector u to every item row adds <h_i,u> to every score, loss unchanged
    u = r.standard_normal(6).astype(np.float32)
    res = O.run(H, (E.astype(np.float64) + u).astype(np.float64).astype(np.float32), tgt, neg, None, g, in_dtype="f32", neg_mode=PP)
    np.testing.assert_allclose(res.loss, base.loss, rtol=1e-5, atol=1e-6)  # E+u is re-rounded to float32


# ---- P9: the online-softmax identity the forward algorithm rests on (Alg. 1), and Eq. 6 as sparse matrix products -----
@pytest.mark.parametrize("seed", [1, 4, 5])
def test_lse_of_random_partitions_merged_in_random_order_and_sparse_matrix_gradients(seed):
    """Any way of cutting a position's candidates into parts, taking (max, sum of exponentials) per part and merging the
    pairs in any order must reproduce the two-pass LSE of the definition: that associativity is what lets Alg. 1 walk
    the candidates block by block with a running maximum.  The gradients of Eq. 6 are held against scipy's sparse
    matrix product of the coefficient matrix with H (dE) and a dense product with the gathered rows (dH)."""
    import scipy.sparse as sp

    r, H, E, tgt = _rand(50 + seed, N=11, V=37, d=7, K=13)
    N, K, V = 11, 13, 37
    neg = r.integers(0, V, (N, K)).astype(np.int32)
    cand = np.concatenate([tgt[:, None], neg], 1).astype(np.int64)
    res = O.run(H, E, tgt, neg, None, None, in_dtype="f32", neg_mode=PP, mask_collisions=0)
    H64, E64 = H.astype(np.float64), E.astype(np.float64)
    for i in range(N):
        o = E64[cand[i]] @ H64[i]
        order = r.permutation(K + 1)
        cuts = np.sort(r.choice(np.arange(1, K + 1), size=int(r.integers(1, 6)), replace=False))
        pairs = [(float(o[part].max()), float(np.exp(o[part] - o[part].max()).sum())) for part in np.split(order, cuts)]
        while len(pairs) > 1:                      # merge two random pairs until one is left
            a = pairs.pop(int(r.integers(len(pairs))))
            b = pairs.pop(int(r.integers(len(pairs))))
            M = max(a[0], b[0])
            pairs.append((M, a[1] * math.exp(a[0] - M) + b[1] * math.exp(b[0] - M)))
        assert abs(pairs[0][0] + math.log(pairs[0][1]) - res.lse[i]) <= 1e-13 * max(1.0, abs(res.lse[i]))
    g = r.standard_normal(N)
    resg = O.run(H, E, tgt, neg, None, g, in_dtype="f32", neg_mode=PP, mask_collisions=0)
    scores = np.einsum("nkd,nd->nk", E64[cand], H64)
    G = g[:, None] * np.exp(scores - resg.lse[:, None])
    G[:, 0] -= g                                    # the correct item sits in column 0
    dH = np.einsum("nk,nkd->nd", G, E64[cand])
    rows = np.repeat(np.arange(N), K + 1)
    dE = (sp.coo_matrix((G.ravel(), (cand.ravel(), rows)), shape=(V, N)).tocsr() @ H64)   # duplicates add up
    np.testing.assert_allclose(resg.dH, dH, rtol=1e-10, atol=1e-14)
    np.testing.assert_allclose(resg.dE, np.asarray(dE), rtol=1e-10, atol=1e-14)


# ---- masks, selections, bookkeeping -----------------------------------------------------------------------------------
def test_masked_positions_never_read_their_ids_and_selection_matches_full_run():
    r, H, E, tgt = _rand(60, N=20, V=30, d=4, K=5)
    N, K = 20, 5
    neg = r.integers(0, 30, (N, K)).astype(np.int32)
    mask = (r.random(N) > 0.3).astype(np.uint8)
    g = r.standard_normal(N)
    ref = O.run(H, E, tgt, neg, mask, g, in_dtype="f32", neg_mode=PP)
    tgt2, neg2 = tgt.copy(), neg.copy()
    tgt2[mask == 0] = 2_000_000_000  # out of range on purpose: must not be touched
    neg2[mask == 0] = -7
    res = O.run(H, E, tgt2, neg2, mask, g, in_dtype="f32", neg_mode=PP)
    assert np.array_equal(res.loss, ref.loss) and np.array_equal(res.dH, ref.dH)
    np.testing.assert_allclose(res.dE, ref.dE, rtol=1e-12, atol=1e-15)
    # an out-of-range id on a valid position is an error
    tgt3 = tgt.copy()
    tgt3[np.flatnonzero(mask)[0]] = 30
    with pytest.raises(RuntimeError):
        O.run(H, E, tgt3, neg, mask, g, in_dtype="f32", neg_mode=PP)
    # a selection returns the same rows, and its compact dE equals the dense dE of the same positions
    sel = np.array([3, 0, 17, 9], np.int64)
    part = O.run(H, E, tgt, neg, mask, g, in_dtype="f32", neg_mode=PP, sel=sel, want_dE="compact")
    assert np.array_equal(part.loss, ref.loss[sel]) and np.array_equal(part.dH, ref.dH[sel])
    gsel = np.zeros(N)
    gsel[sel] = g[sel]
    only = O.run(H, E, tgt, neg, mask, gsel, in_dtype="f32", neg_mode=PP)
    np.testing.assert_allclose(part.dE, only.dE[part.dE_rows], rtol=1e-12, atol=1e-15)
    rest = np.setdiff1d(np.arange(30), part.dE_rows)
    assert np.all(only.dE[rest] == 0)


def test_bf16_inputs_are_widened_exactly():
    r, H, E, tgt = _rand(70, N=6, V=20, d=8, K=4)
    neg = r.integers(0, 20, 4).astype(np.int32)
    Hb, Eb = bf16_bits_from_f32(H), bf16_bits_from_f32(E)
    a = O.run(Hb, Eb, tgt, neg, None, None, in_dtype="bf16", neg_mode=SH)
    b = O.run(f32_from_bf16_bits(Hb), f32_from_bf16_bits(Eb), tgt, neg, None, None, in_dtype="f32", neg_mode=SH)
    assert np.array_equal(a.loss, b.loss) and np.array_equal(a.dH, b.dH)
    # the rounding helper itself: round-to-nearest-even on the 16 dropped bits
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 3.140625], np.float32)  # 1+2^-8 ties to even (1.0); 1+3*2^-8 ties up
    assert np.array_equal(f32_from_bf16_bits(bf16_bits_from_f32(x)), np.array([1.0, 1.0, 1.015625, -2.5, 3.140625], np.float32))


# ---- P11: gradient filtering (block reading) -------------------------------------------------------------------
def _peaked_full_case(seed, N=70, V=150, d=8, frac_masked=0.2):
    """Full-catalogue case whose softmax is concentrated: hidden states point at their target's row."""
    r = np.random.default_rng(seed)
    E = r.standard_normal((V, d)).astype(np.float32)
    tgt = r.integers(0, V, N).astype(np.int32)
    H = (2.5 * E[tgt] + 0.3 * r.standard_normal((N, d))).astype(np.float32)
    mask = (r.random(N) >= frac_masked).astype(np.uint8)
    g = r.standard_normal(N)
    return H, E, tgt, mask, g


def test_filter_with_zero_threshold_changes_nothing_and_with_huge_threshold_leaves_the_one_hot_term():
    H, E, tgt, mask, g = _peaked_full_case(5)
    valid = np.flatnonzero(mask).astype(np.int64)
    base = O.run(H, E, tgt, None, mask, g, in_dtype="f32", neg_mode=FULL, sel=valid, want_p=True)
    keep_all = O.filter_blocks(base.p, 0.0, 32)
    assert keep_all.all()
    same = O.run(H, E, tgt, None, mask, g, in_dtype="f32", neg_mode=FULL, sel=valid, p_keep=keep_all)
    assert np.array_equal(same.dH, base.dH) and np.array_equal(same.loss, base.loss)
    np.testing.assert_allclose(same.dE, base.dE, rtol=1e-13, atol=1e-15)   # threads add in any order
    none = O.filter_blocks(base.p, 2.0, 32)          # no probability reaches 2
    assert not none.any()
    only = O.run(H, E, tgt, None, mask, g, in_dtype="f32", neg_mode=FULL, sel=valid, p_keep=none)
    # closed form: G = -g on the target column only; loss and lse are those of the unfiltered run
    assert np.array_equal(only.loss, base.loss) and np.array_equal(only.lse, base.lse)
    np.testing.assert_allclose(only.dH, -g[valid, None] * E[tgt[valid]].astype(np.float64), rtol=1e-13, atol=1e-13)
    dE = np.zeros((E.shape[0], E.shape[1]))
    np.add.at(dE, tgt[valid], -g[valid, None] * H[valid].astype(np.float64))
    np.testing.assert_allclose(only.dE, dE, rtol=1e-13, atol=1e-13)


@pytest.mark.parametrize("block,eps", [(8, 1e-2), (8, 0.2), (16, 0.9)])
def test_filter_against_dense_matrix_products(block, eps):
    """Library routines on materialised matrices: scipy softmax, block maxima by reshaping a padded copy, and the
    gradients as two matrix products with the filtered softmax."""
    from scipy.special import softmax

    H, E, tgt, mask, g = _peaked_full_case(11)
    valid = np.flatnonzero(mask)
    Hv, gv, tv = H[valid].astype(np.float64), g[valid], tgt[valid]
    P = softmax(Hv @ E.astype(np.float64).T, axis=1)
    nr, nc = P.shape
    pr, pc = -nr % block, -nc % block
    big = np.pad(P, ((0, pr), (0, pc))).reshape((nr + pr) // block, block, (nc + pc) // block, block).max(axis=(1, 3))
    keep = np.repeat(np.repeat(big >= eps, block, axis=0), block, axis=1)[:nr, :nc]
    assert 0 < keep.mean() < 1                       # the case exercises both outcomes
    Pf = np.where(keep, P, 0.0)
    Y = np.zeros_like(P)
    Y[np.arange(nr), tv] = 1.0
    G = gv[:, None] * (Pf - Y)
    got, sel, p = _filtered(H, E, tgt, mask, g, eps, block)
    assert np.array_equal(sel, valid)
    np.testing.assert_allclose(p, P, rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(got.dH, G @ E.astype(np.float64), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(got.dE, G.T @ Hv, rtol=1e-11, atol=1e-12)
    # every dropped probability is below the threshold, every probability at or above it survives
    marks = O.filter_blocks(p, eps, block).astype(bool)
    assert np.array_equal(marks, keep) and (p[~marks] < eps).all() and marks[p >= eps].all()


def _filtered(H, E, tgt, mask, g, eps, block):
    class W:  # the few fields run_workload_filtered reads
        pass
    w = W()
    w.H, w.E, w.tgt, w.neg, w.mask, w.g = H, E, tgt, None, mask, g
    w.in_dtype, w.neg_mode, w.mask_collisions, w.K = "f32", FULL, 1, 0
    return O.run_workload_filtered(w, eps, block=block)
