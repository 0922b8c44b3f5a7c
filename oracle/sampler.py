"""Reference negative sampler: which item ids a (seed, stream) pair denotes.  TEST INFRASTRUCTURE ONLY.

The paper draws the negatives of a step on the host (global uniform sampling, and popularity-based sampling through a
multinomial over the whole catalogue; Sec. "Comparison Sampling Strategies") and hands the loss an index matrix, whose
memory it names as the overhead of CCE- over CCE (Sec. 5, "What is better").  A sampler fused into the loss kernels
needs ids that are a pure function of (seed, stream, position, slot), so that the forward pass, the backward pass and
the index build all see the same multiset without storing it.  The paper fixes no generator; this file states the one
used here, as plainly as possible (numpy, 64-bit integers, no tricks):

  * generator: Philox4x32-10 (Salmon, Moraes, Dror, Shaw, "Parallel random numbers: as easy as 1, 2, 3", SC'11), key =
    the two halves of the 64-bit seed, counter = (q, position low word, position high word, stream);
  * slot s of a position (s = 0 .. K-1) is draw number j = s + 1 (draw 0 is left to the correct item's column);
  * uniform: q = j >> 2, r = output word j & 3, id = floor(r * V / 2^32);
  * popularity (alias method, Walker 1977 / Vose 1991, table given by the caller): q = j >> 1, (r0, r1) = output words
    2(j & 1), 2(j & 1) + 1, column c = floor(r0 * V / 2^32), id = c if r1 < thresh[c] else alias[c];
  * shared negatives are the draws of position 0.

Draws are independent: sampling is with replacement, a slot may repeat an id or hit the position's own target (the loss
handles both: multiset semantics, collision weight).

parity pins: known-answer vectors of the generator, exact range mapping, chi-square of both laws, reconstruction of
the target law from an alias table (tests/test_sampler_pins.py).
"""
from __future__ import annotations

from typing import Optional, Tuple

import numpy as np

UNIFORM, ALIAS = 1, 2

_M0, _M1 = np.uint64(0xD2511F53), np.uint64(0xCD9E8D57)
_W0, _W1 = np.uint64(0x9E3779B9), np.uint64(0xBB67AE85)
_LO = np.uint64(0xFFFFFFFF)
_S32 = np.uint64(32)


def philox4x32_10(c0, c1, c2, c3, k0, k1) -> Tuple[np.ndarray, np.ndarray, np.ndarray, np.ndarray]:
    """Ten rounds of Philox-4x32 on arrays of 32-bit words held in uint64 (so that the 32x32 -> 64 bit products are exact)."""
    c0, c1, c2, c3 = (np.asarray(x, np.uint64) & _LO for x in (c0, c1, c2, c3))
    k0 = np.uint64(k0) & _LO
    k1 = np.uint64(k1) & _LO
    for rnd in range(10):
        p0 = _M0 * c0            # < 2^64: both factors are below 2^32
        p1 = _M1 * c2
        c0, c1, c2, c3 = ((p1 >> _S32) ^ c1 ^ k0) & _LO, p1 & _LO, ((p0 >> _S32) ^ c3 ^ k1) & _LO, p0 & _LO
        if rnd < 9:
            k0 = (k0 + _W0) & _LO
            k1 = (k1 + _W1) & _LO
    return c0, c1, c2, c3


def _select(words, which):
    out = words[0].copy()
    for w in (1, 2, 3):
        out = np.where(which == w, words[w], out)
    return out


def draw(kind: int, seed: int, stream: int, pos, j, V: int, thresh: Optional[np.ndarray] = None,
         alias: Optional[np.ndarray] = None) -> np.ndarray:
    """Item id of draw number j (>= 1) of position pos; pos and j broadcast against each other.  int32 result."""
    pos = np.asarray(pos, np.uint64)
    j = np.asarray(j, np.uint64)
    pos, j = np.broadcast_arrays(pos, j)
    k0, k1 = seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF
    st = np.uint64(stream & 0xFFFFFFFF)
    Vq = np.uint64(V)
    if kind == UNIFORM:
        words = philox4x32_10(j >> np.uint64(2), pos & _LO, pos >> _S32, st, k0, k1)
        r = _select(words, j & np.uint64(3))
        return ((r * Vq) >> _S32).astype(np.int32)
    if kind == ALIAS:
        words = philox4x32_10(j >> np.uint64(1), pos & _LO, pos >> _S32, st, k0, k1)
        odd = (j & np.uint64(1)) == 1
        r0 = np.where(odd, words[2], words[0])
        r1 = np.where(odd, words[3], words[1])
        col = ((r0 * Vq) >> _S32).astype(np.int64)
        keep = r1 < np.asarray(thresh, np.uint64)[col]
        return np.where(keep, col, np.asarray(alias, np.int64)[col]).astype(np.int32)
    raise ValueError(kind)


def sample_negatives(kind: int, seed: int, stream: int, N: int, K: int, V: int, *, per_position: bool,
                     thresh: Optional[np.ndarray] = None, alias: Optional[np.ndarray] = None) -> np.ndarray:
    """The index array the loss would have been handed: [N, K] (per position) or [K] (shared = draws of position 0)."""
    j = np.arange(1, K + 1, dtype=np.uint64)
    if per_position:
        out = np.empty((N, K), np.int32)
        step = max(1, (1 << 22) // max(K, 1))
        for a in range(0, N, step):      # bounded temporaries
            b = min(N, a + step)
            out[a:b] = draw(kind, seed, stream, np.arange(a, b, dtype=np.uint64)[:, None], j[None, :], V, thresh, alias)
        return out
    return draw(kind, seed, stream, np.uint64(0), j, V, thresh, alias)


def alias_law(thresh: np.ndarray, alias: np.ndarray) -> np.ndarray:
    """The exact law an alias table encodes under the draw above, as fp64 probabilities (for pins)."""
    V = thresh.shape[0]
    t = thresh.astype(np.float64) / 2.0 ** 32         # P(r1 < thresh) = thresh / 2^32
    p = t.copy()
    np.add.at(p, alias.astype(np.int64), 1.0 - t)
    return p / V                                       # columns: uniform up to the floor(r0 V / 2^32) granularity
