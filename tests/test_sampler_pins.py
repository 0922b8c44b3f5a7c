"""Pins of the reference negative sampler (CPU only): the generator against its published known-answer vectors, the
range mapping against exact integer arithmetic, both laws against chi-square bounds, the alias table against the law
it was built from, and the structural properties the fused kernels rely on (pure function of seed, stream, position,
slot; shared negatives = draws of position 0)."""
import os

import numpy as np
import pytest

from oracle import sampler as S
from workloads import alias_table, popularity_weights

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def test_generator_reproduces_the_published_vectors():
    rows = [ln.split() for ln in open(GOLDEN) if ln.strip() and not ln.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        w = [int(x, 16) for x in r]
        out = S.philox4x32_10(*[np.array([x]) for x in w[0:4]], w[4], w[5])
        assert [int(o[0]) for o in out] == w[6:10]


def test_generator_is_a_bijection_of_the_counter_on_a_sample():
    """A keyed permutation of the counter space never maps two counters to one output."""
    c = np.arange(1 << 16, dtype=np.uint64)
    out = S.philox4x32_10(c, 0 * c + 7, 0 * c, 0 * c + 3, 11, 13)
    packed = np.stack(out, 1)
    assert np.unique(packed, axis=0).shape[0] == c.shape[0]


@pytest.mark.parametrize("V", [1, 2, 7, 4096, 1_000_000, 5_000_000])
def test_uniform_ids_follow_exact_integer_scaling(V):
    """id = floor(r V / 2^32) with r the selected output word: checked with Python integers, and the range is [0, V)."""
    pos = np.array([0, 1, 5, 2**33 + 9], np.uint64)
    j = np.arange(1, 42, dtype=np.uint64)
    ids = S.draw(S.UNIFORM, 0x1234_5678_9ABC_DEF0, 3, pos[:, None], j[None, :], V)
    assert ids.min() >= 0 and ids.max() < V
    for a, p in enumerate(pos):
        for b, jj in enumerate(j):
            words = S.philox4x32_10(np.array([int(jj) >> 2]), np.array([int(p) & 0xFFFFFFFF]), np.array([int(p) >> 32]),
                                    np.array([3]), 0x9ABCDEF0, 0x12345678)
            r = int(words[int(jj) & 3][0])
            assert int(ids[a, b]) == (r * V) >> 32


def test_uniform_law_chi_square():
    V, N, K = 1000, 500, 256
    ids = S.sample_negatives(S.UNIFORM, 42, 0, N, K, V, per_position=True)
    cnt = np.bincount(ids.ravel(), minlength=V)
    chi = ((cnt - N * K / V) ** 2 / (N * K / V)).sum()
    assert abs(chi - (V - 1)) < 6 * np.sqrt(2 * (V - 1))       # six sigma of a chi-square with V-1 degrees
    # slots of one position and positions of one slot are uncorrelated draws
    a = ids.astype(np.float64)
    assert abs(np.corrcoef(a[:, 0], a[:, 1])[0, 1]) < 0.2 and abs(np.corrcoef(a[0], a[1])[0, 1]) < 0.25


def _table(V, seed=5):
    r2i = np.random.default_rng(seed).permutation(V).astype(np.int32)
    w = popularity_weights(r2i, 1.2, 0.75)
    return w, alias_table(w)


@pytest.mark.parametrize("V", [1, 2, 3, 1000, 65_537])
def test_alias_table_encodes_the_law_it_was_built_from(V):
    w, (thresh, alias) = _table(V)
    assert thresh.dtype == np.uint32 and alias.dtype == np.int32 and alias.min() >= 0 and alias.max() < V
    law = S.alias_law(thresh, alias)
    assert abs(law.sum() - 1.0) < 1e-12
    assert np.abs(law - w / w.sum()).max() < 2.0 ** -31            # fixed-point thresholds: one unit of 2^-32 per column


def test_alias_law_on_a_hand_made_table():
    """Three columns; column 0 keeps half of its mass and gives the rest to id 2: law = (1/6, 1/3, 1/2)."""
    thresh = np.array([2 ** 31, 2 ** 32 - 1, 2 ** 32 - 1], np.uint32)
    alias = np.array([2, 1, 2], np.int32)
    assert np.allclose(S.alias_law(thresh, alias), [1 / 6, 1 / 3, 1 / 2], atol=1e-9)
    ids = S.sample_negatives(S.ALIAS, 9, 1, 3000, 64, 3, per_position=True, thresh=thresh, alias=alias)
    f = np.bincount(ids.ravel(), minlength=3) / ids.size
    assert np.abs(f - [1 / 6, 1 / 3, 1 / 2]).max() < 5e-3


def test_alias_draw_chi_square():
    V, N, K = 800, 1000, 256
    w, (thresh, alias) = _table(V)
    ids = S.sample_negatives(S.ALIAS, 77, 2, N, K, V, per_position=True, thresh=thresh, alias=alias)
    e = N * K * w / w.sum()
    big = e >= 5
    chi = ((np.bincount(ids.ravel(), minlength=V)[big] - e[big]) ** 2 / e[big]).sum()
    dof = int(big.sum()) - 1
    assert abs(chi - dof) < 6 * np.sqrt(2 * dof)


def test_alias_draw_uses_its_own_two_words():
    """Draws 2q and 2q+1 share a counter and take words (0,1) and (2,3): restated with Python integers."""
    V = 50
    w, (thresh, alias) = _table(V)
    for j in range(1, 20):
        words = S.philox4x32_10(np.array([j >> 1]), np.array([4]), np.array([0]), np.array([6]), 21, 0)
        r0, r1 = int(words[2 * (j & 1)][0]), int(words[2 * (j & 1) + 1][0])
        col = (r0 * V) >> 32
        want = col if r1 < int(thresh[col]) else int(alias[col])
        assert int(S.draw(S.ALIAS, 21, 6, 4, j, V, thresh, alias)) == want


def test_ids_are_a_pure_function_of_seed_stream_position_slot():
    V, N, K = 5000, 40, 33
    a = S.sample_negatives(S.UNIFORM, 1, 0, N, K, V, per_position=True)
    assert np.array_equal(a, S.sample_negatives(S.UNIFORM, 1, 0, N, K, V, per_position=True))
    # a longer list or more positions extend, never reshuffle
    b = S.sample_negatives(S.UNIFORM, 1, 0, N + 7, K + 30, V, per_position=True)
    assert np.array_equal(b[:N, :K], a)
    # other seed / other stream: other ids
    assert (S.sample_negatives(S.UNIFORM, 2, 0, N, K, V, per_position=True) != a).mean() > 0.99
    assert (S.sample_negatives(S.UNIFORM, 1, 1, N, K, V, per_position=True) != a).mean() > 0.99
    assert (S.sample_negatives(S.UNIFORM, 1 + (1 << 32), 0, N, K, V, per_position=True) != a).mean() > 0.99
    # shared negatives are the draws of position 0
    assert np.array_equal(S.sample_negatives(S.UNIFORM, 1, 0, N, K, V, per_position=False), a[0])
    # positions differ from each other
    assert (a[0] != a[1]).mean() > 0.99
