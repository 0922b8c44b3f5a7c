"""Negative sampling inside the kernels: the ids against the reference sampler bit for bit, and the *_sampled calls
against the fp64 oracle run on the reference sampler's ids."""
import dataclasses

import numpy as np
import pytest

from oracle import sampler as S
from workloads import NEG_PER_POSITION, NEG_SHARED, alias_table, config, make_workload, popularity_weights

pytestmark = pytest.mark.gpu

TOL_F32 = 1e-5
TOL_BF16 = 2e-2


def _table(V, seed=3):
    r2i = np.random.default_rng(seed).permutation(V).astype(np.int32)
    return alias_table(popularity_weights(r2i, 1.2, 0.75))


def _shape(N, K, V, mode, d=64, dtype="f32", seed=11, **kw):
    return make_workload("sampler", N, 1, d, V, K, dtype, mode, seed, g_kind="random", **kw)


def _reference_ids(w, kind, seed, stream, table):
    th, al = table if table is not None else (None, None)
    return S.sample_negatives(kind, seed, stream, w.N, w.K, w.V, per_position=(w.neg_mode == NEG_PER_POSITION),
                              thresh=th, alias=al)


@pytest.mark.parametrize("kind", [S.UNIFORM, S.ALIAS])
@pytest.mark.parametrize("N,K,V,mode", [(300, 257, 1000, NEG_PER_POSITION), (64, 1, 5_000_000, NEG_PER_POSITION),
                                        (5, 1023, 77, NEG_PER_POSITION), (1, 1024, 50_000, NEG_SHARED),
                                        (9, 4096, 5_000_000, NEG_SHARED), (2048, 64, 1_000_000, NEG_PER_POSITION)])
def test_sampled_ids_equal_the_reference_sampler(kind, N, K, V, mode):
    from hip_harness import device_sampler, sample_hip

    table = _table(V) if kind == S.ALIAS else None
    w = _shape(N, K, V, mode)
    for seed, stream in ((0, 0), (0x0123_4567_89AB_CDEF, 3), (1 << 63, 0xFFFFFFFF)):
        smp, keep = device_sampler(kind, seed, stream, *(table or ()))
        got = sample_hip(w, smp)
        want = _reference_ids(w, kind, seed, stream, table)
        assert got.shape == want.shape and np.array_equal(got, want), (seed, stream)


def _check(w_ref, out, tol):
    from test_gpu_parity import check_against_oracle

    return check_against_oracle(w_ref, out, tol)


@pytest.mark.parametrize("kind", [S.UNIFORM, S.ALIAS])
@pytest.mark.parametrize("case", ["c3_reduced", "f32_K37_masked", "f32_K600", "bf16_d256_K300"])
def test_per_position_sampled_calls_against_the_oracle(kind, case):
    """Forward, dH (row-gather pass) and dE (inverted index built from redrawn ids) with no index matrix anywhere."""
    from hip_harness import device_sampler, run_hip_sampled

    if case == "c3_reduced":
        w, tol = config(3, scale=0.02, g_kind="random"), 2e-5
    elif case == "f32_K37_masked":
        w, tol = _shape(333, 37, 900, NEG_PER_POSITION, d=64, pad="bernoulli", pad_p=0.3), TOL_F32
    elif case == "f32_K600":
        w, tol = _shape(70, 600, 5000, NEG_PER_POSITION, d=40), TOL_F32      # several windows of draws per position
    else:
        w, tol = _shape(150, 300, 3000, NEG_PER_POSITION, d=256, dtype="bf16", tgt_dist="zipf"), 2e-5
    table = _table(w.V) if kind == S.ALIAS else None
    smp, keep = device_sampler(kind, 20250909, 5, *(table or ()))
    w_ref = dataclasses.replace(w, neg=_reference_ids(w, kind, 20250909, 5, table))
    if case != "f32_K600":
        hits = (w_ref.neg == w_ref.tgt[:, None]) & (w_ref.mask[:, None] != 0)
        print("collisions with own target:", int(hits.sum()))
    out = run_hip_sampled(w, smp)
    assert out["status"] == 0
    _check(w_ref, out, tol)


@pytest.mark.parametrize("kind", [S.UNIFORM, S.ALIAS])
@pytest.mark.parametrize("idx,scale,tol", [(1, 1.0, TOL_F32), (2, 0.03, TOL_BF16), (5, 0.006, TOL_BF16)])
def test_shared_sampled_calls_against_the_oracle(kind, idx, scale, tol):
    from hip_harness import device_sampler, run_hip_sampled

    w = config(idx, scale=scale, g_kind="random")
    table = _table(w.V) if kind == S.ALIAS else None
    smp, keep = device_sampler(kind, 99, 1, *(table or ()))
    w_ref = dataclasses.replace(w, neg=_reference_ids(w, kind, 99, 1, table))
    out = run_hip_sampled(w, smp)
    _check(w_ref, out, tol)


def test_sampled_calls_equal_the_plain_calls_on_the_materialised_ids():
    """Same kernels, same order of summation: loss, lse and dH agree bit for bit, dE (inverted index, one
    read-modify-write per row) as well."""
    from hip_harness import device_sampler, run_hip, run_hip_sampled, sample_hip

    w = config(3, scale=0.02, g_kind="random")
    smp, keep = device_sampler(S.UNIFORM, 4242, 9)
    ids = sample_hip(w, smp)
    a = run_hip_sampled(w, smp)
    b = run_hip(dataclasses.replace(w, neg=ids))
    for name in ("loss", "lse", "dH"):
        assert np.array_equal(a[name].view(np.uint32), b[name].view(np.uint32)), name
    assert np.allclose(a["dE"], b["dE"], rtol=1e-5, atol=1e-7)


def test_other_stream_other_negatives():
    from hip_harness import device_sampler, run_hip_sampled

    w = config(3, scale=0.01, g_kind="random")
    a = run_hip_sampled(w, device_sampler(S.UNIFORM, 1, 0)[0])
    b = run_hip_sampled(w, device_sampler(S.UNIFORM, 1, 1)[0])
    assert np.mean(a["loss"] != b["loss"]) > 0.99


def test_sampled_calls_edge_cases():
    """K = 0 (nothing to draw: loss 0, gradients 0), every position padded, and a single position."""
    from hip_harness import device_sampler, run_hip_sampled

    smp, _ = device_sampler(S.UNIFORM, 5, 0)
    w = _shape(40, 0, 500, NEG_PER_POSITION, d=64, dtype="bf16")
    out = run_hip_sampled(w, smp)
    assert np.all(out["loss"] == 0) and np.all(out["dH"] == 0) and np.all(out["dE"] == 0)

    w = _shape(50, 33, 500, NEG_PER_POSITION, d=64, dtype="bf16")
    w.mask[:] = 0
    out = run_hip_sampled(w, smp)
    assert np.all(out["loss"] == 0) and np.all(out["lse"] == 0) and np.all(out["dH"] == 0) and np.all(out["dE"] == 0)

    for mode in (NEG_PER_POSITION, NEG_SHARED):
        w = _shape(1, 19, 500, mode, d=128, dtype="bf16")
        w_ref = dataclasses.replace(w, neg=_reference_ids(w, S.UNIFORM, 5, 0, None))
        _check(w_ref, run_hip_sampled(w, smp), TOL_BF16)
