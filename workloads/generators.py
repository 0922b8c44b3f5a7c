"""Seeded generators for the five benchmark workloads and for reduced test cases.

The paper trains on six public interaction datasets (its dataset table); none of
them is used here.  The generators below produce synthetic stand-ins that keep
what matters to the loss kernel: N = batch * sequence positions, hidden size d,
catalogue size V, number of negatives K, a power-law (Zipf) popularity of the
target ids, uniform or popularity-weighted negative ids, and right-padded
sequences.  All values are drawn on the host with numpy's PCG64 and rounded once
to the storage dtype, so every consumer sees identical bits.

Nothing in this file computes scores, softmax, losses or gradients.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np

BASE_SEED = 250909682

NEG_SHARED = 0
NEG_PER_POSITION = 1
NEG_FULL = 2

CONFIG_NAMES = {
    1: "c1_tiny_f32_shared",
    2: "c2_mid_bf16_shared",
    3: "c3_per_position_bf16",
    4: "c4_full_catalog_bf16",
    5: "c5_large_bf16_shared_popularity",
}


def bf16_bits_from_f32(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even) and return the uint16 bit patterns."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def f32_from_bf16_bits(bits: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns exactly to float32."""
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _normal_table(rng: np.random.Generator, rows: int, d: int, sigma: float, dtype: str) -> np.ndarray:
    """[rows, d] ~ N(0, sigma) in storage form: float32 array, or uint16 bf16 bit patterns."""
    out = np.empty((rows, d), dtype=np.float32 if dtype == "f32" else np.uint16)
    chunk = max(1, (1 << 26) // max(d, 1))  # ~64M values per chunk keeps the temporary small
    for r0 in range(0, rows, chunk):
        r1 = min(rows, r0 + chunk)
        x = rng.standard_normal((r1 - r0, d), dtype=np.float32)
        if sigma != 1.0:
            x *= np.float32(sigma)
        out[r0:r1] = x if dtype == "f32" else bf16_bits_from_f32(x)
    return out


def zipf_ids(rng: np.random.Generator, perm_rng: np.random.Generator, n: int, V: int, s: float):
    """n ids from a Zipf(s) law bounded to ranks 1..V, by inverse CDF.

    A seeded permutation maps rank -> id so that popular rows are scattered over
    the table instead of sitting next to each other.  Returns (ids, rank_to_id).
    """
    ranks = np.arange(1, V + 1, dtype=np.float64)
    cdf = np.cumsum(ranks ** (-s))
    u = rng.random(n) * cdf[-1]
    r = np.searchsorted(cdf, u, side="right")
    np.clip(r, 0, V - 1, out=r)
    rank_to_id = perm_rng.permutation(V).astype(np.int32)
    return rank_to_id[r].astype(np.int32), rank_to_id


def popularity_negatives(rng: np.random.Generator, rank_to_id: np.ndarray, K: int, s: float, power: float) -> np.ndarray:
    """K distinct ids drawn with probability proportional to count**power, count ~ rank**(-s).

    Weighted sampling without replacement through exponential keys: the K smallest
    of Exp(1)/w_r are a draw without replacement with weights w_r.
    """
    V = rank_to_id.shape[0]
    w = np.arange(1, V + 1, dtype=np.float64) ** (-s * power)
    keys = rng.standard_exponential(V) / w
    pick = np.argpartition(keys, K)[:K]
    pick = pick[np.argsort(keys[pick], kind="stable")]
    return rank_to_id[pick].astype(np.int32)


def popularity_weights(rank_to_id: np.ndarray, s: float, power: float) -> np.ndarray:
    """Unnormalised sampling weight per item id: count**power with count ~ rank**(-s) (the law of popularity_negatives)."""
    V = rank_to_id.shape[0]
    w = np.empty(V, dtype=np.float64)
    w[rank_to_id] = np.arange(1, V + 1, dtype=np.float64) ** (-s * power)
    return w


def alias_table(weights: np.ndarray):
    """Alias table of a discrete law (Walker / Vose): V columns of equal mass 1/V, column c keeps id c with probability
    thresh[c] / 2^32 and yields alias[c] otherwise.  Returns (thresh uint32 [V], alias int32 [V]).

    Input data for the on-device sampler and for its reference alike: the table is handed to both, neither builds it.
    """
    w = np.asarray(weights, dtype=np.float64)
    V = w.shape[0]
    q = w * (V / w.sum())                 # mean 1: the share of its own column an id fills
    alias = np.arange(V, dtype=np.int64)
    small = [int(x) for x in np.flatnonzero(q < 1.0)]
    large = [int(x) for x in np.flatnonzero(q >= 1.0)]
    q = q.copy()
    while small and large:
        lo = small.pop()
        hi = large[-1]
        alias[lo] = hi                     # the rest of column lo is filled from hi
        q[hi] -= 1.0 - q[lo]
        if q[hi] < 1.0:
            large.pop()
            small.append(hi)
    for c in small + large:                # leftovers are full columns up to rounding
        q[c] = 1.0
    thresh = np.minimum(np.floor(q * 2.0 ** 32), 2.0 ** 32 - 1).astype(np.uint32)
    return thresh, alias.astype(np.int32)


@dataclass
class Workload:
    name: str
    N: int
    V: int
    d: int
    K: int
    in_dtype: str            # "f32" | "bf16"
    neg_mode: int            # NEG_SHARED | NEG_PER_POSITION | NEG_FULL
    mask_collisions: int
    H: np.ndarray            # [N, d] float32, or uint16 bf16 bits
    E: np.ndarray            # [V, d] same storage as H
    tgt: np.ndarray          # [N] int32
    neg: Optional[np.ndarray]  # [K] | [N, K] int32 | None (full catalogue)
    mask: np.ndarray         # [N] uint8, 1 = valid position
    g: np.ndarray            # [N] float32 upstream gradient of the per-position loss
    batch: int = 0
    seq_len: int = 0
    notes: dict = field(default_factory=dict)

    @property
    def n_valid(self) -> int:
        return int(self.mask.sum())

    def H_f32(self) -> np.ndarray:
        return self.H if self.in_dtype == "f32" else f32_from_bf16_bits(self.H)

    def E_f32(self) -> np.ndarray:
        return self.E if self.in_dtype == "f32" else f32_from_bf16_bits(self.E)


def make_workload(
    name: str,
    batch: int,
    seq_len: int,
    d: int,
    V: int,
    K: int,
    in_dtype: str,
    neg_mode: int,
    seed: int,
    *,
    tgt_dist: str = "uniform",      # "uniform" | "zipf"
    zipf_s: float = 1.1,
    neg_dist: str = "uniform",      # "uniform" (with replacement) | "uniform_distinct" | "popularity"
    pad: str = "none",              # "none" | "bernoulli" | "right"
    pad_p: float = 0.1,
    pad_len_lo: int = 0,
    mask_collisions: int = 1,
    h_sigma: float = 1.0,
    e_sigma: float = 0.02,
    g_kind: str = "mean",           # "mean": 1/N_valid ; "random": N(0,1)
) -> Workload:
    """Build one seeded workload.  Independent child streams feed H, E, targets, negatives, mask, permutation, g."""
    ss = np.random.SeedSequence(seed)
    r_h, r_e, r_t, r_n, r_m, r_p, r_g = [np.random.Generator(np.random.PCG64(c)) for c in ss.spawn(7)]
    N = batch * seq_len
    H = _normal_table(r_h, N, d, h_sigma, in_dtype)
    E = _normal_table(r_e, V, d, e_sigma, in_dtype)

    rank_to_id = None
    if tgt_dist == "uniform":
        tgt = r_t.integers(0, V, size=N, dtype=np.int32)
    elif tgt_dist == "zipf":
        tgt, rank_to_id = zipf_ids(r_t, r_p, N, V, zipf_s)
    else:
        raise ValueError(tgt_dist)

    if neg_mode == NEG_FULL:
        neg = None
    else:
        shape = (K,) if neg_mode == NEG_SHARED else (N, K)
        if neg_dist == "uniform":
            neg = r_n.integers(0, V, size=shape, dtype=np.int32)
        elif neg_dist == "uniform_distinct":
            if neg_mode != NEG_SHARED:
                raise ValueError("distinct negatives are generated for the shared mode only")
            neg = r_n.choice(V, size=K, replace=False).astype(np.int32)
        elif neg_dist == "popularity":
            if neg_mode != NEG_SHARED:
                raise ValueError("popularity negatives are generated for the shared mode only")
            if rank_to_id is None:
                rank_to_id = r_p.permutation(V).astype(np.int32)
            neg = popularity_negatives(r_n, rank_to_id, K, zipf_s, 0.75)
        else:
            raise ValueError(neg_dist)

    if pad == "none":
        mask = np.ones(N, dtype=np.uint8)
    elif pad == "bernoulli":
        mask = (r_m.random(N) >= pad_p).astype(np.uint8)
    elif pad == "right":
        lens = r_m.integers(pad_len_lo, seq_len + 1, size=batch)
        mask = (np.arange(seq_len)[None, :] < lens[:, None]).astype(np.uint8).reshape(N)
    else:
        raise ValueError(pad)

    nv = max(int(mask.sum()), 1)
    if g_kind == "mean":
        g = np.full(N, 1.0 / nv, dtype=np.float32)
    elif g_kind == "random":
        g = r_g.standard_normal(N, dtype=np.float32)
    else:
        raise ValueError(g_kind)

    return Workload(name, N, V, d, K if neg_mode != NEG_FULL else 0, in_dtype, neg_mode, mask_collisions,
                    H, E, tgt, neg, mask, g, batch=batch, seq_len=seq_len,
                    notes={"seed": seed, "tgt_dist": tgt_dist, "zipf_s": zipf_s, "neg_dist": neg_dist, "pad": pad})


def config(idx: int, *, scale: float = 1.0, g_kind: str = "mean") -> Workload:
    """The five benchmark workloads.  `scale` < 1 shrinks batch (and V, K for the big ones) for quick tests."""
    seed = BASE_SEED + idx
    sb = lambda b: max(1, int(round(b * scale)))  # noqa: E731
    if idx == 1:
        return make_workload(CONFIG_NAMES[1], sb(16), 32, 64, 4096, 128, "f32", NEG_SHARED, seed,
                             tgt_dist="uniform", neg_dist="uniform_distinct", pad="bernoulli", pad_p=0.1, g_kind=g_kind)
    if idx == 2:
        return make_workload(CONFIG_NAMES[2], sb(256), 200, 64, 50_000, 1024, "bf16", NEG_SHARED, seed,
                             tgt_dist="zipf", zipf_s=1.1, neg_dist="uniform", pad="right", pad_len_lo=120, g_kind=g_kind)
    if idx == 3:
        V = 1_000_000 if scale >= 1.0 else max(4096, int(1_000_000 * scale))
        return make_workload(CONFIG_NAMES[3], sb(128), 200, 128, V, 256, "bf16", NEG_PER_POSITION, seed,
                             tgt_dist="zipf", zipf_s=1.1, neg_dist="uniform", pad="none", g_kind=g_kind)
    if idx == 4:
        V = 100_000 if scale >= 1.0 else max(2048, int(100_000 * scale))
        return make_workload(CONFIG_NAMES[4], sb(64), 200, 64, V, 0, "bf16", NEG_FULL, seed,
                             tgt_dist="zipf", zipf_s=1.1, pad="none", g_kind=g_kind)
    if idx == 5:
        V = 5_000_000 if scale >= 1.0 else max(8192, int(5_000_000 * scale))
        K = 4096 if scale >= 1.0 else max(256, int(4096 * scale))
        return make_workload(CONFIG_NAMES[5], sb(1024), 200, 256, V, K, "bf16", NEG_SHARED, seed,
                             tgt_dist="zipf", zipf_s=1.2, neg_dist="popularity", pad="right", pad_len_lo=100, g_kind=g_kind)
    raise ValueError(f"unknown config {idx}")
