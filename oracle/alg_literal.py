"""The paper's two listings restated step by step in fp64 numpy, for small inputs.  TEST INFRASTRUCTURE ONLY.

`lse_online` follows the forward algorithm (memory-efficient linear-log-sum-exp with
negative sampling): per block of positions, walk over the candidate columns j,
load the indexed classifier rows, take the scalar products over the whole hidden
dimension, and keep a running maximum m and a running sum d of exponentials that is
rescaled whenever the maximum grows; LSE = m + log d at the end.

`grads_blockwise` follows the backward algorithm: for every (position block,
candidate column) pair reload the rows, recompute the scalar products, form the
softmax block S = exp(o - LSE), scale by the upstream gradient of LSE, and add the
rank-one updates into the hidden-state gradient and (indexed) into the classifier
gradient.

Two readings of garbled spots in the listings (both recorded in the design notes):
the scalar product uses the row that was just loaded (the listing's subscript names
the target row), and the rescale factor of the running sum is exp(m_old - m_new)
(the listing prints the opposite sign, which would turn the first step into 0*inf).

Inds is the [N, 1+K] candidate matrix whose first column holds the correct items.
These functions cover only what the listings cover: the LSE term and its gradients.
The correct-logit term (first term of Eq. 4) is handled by the caller.
"""
from __future__ import annotations

import numpy as np


def lse_online(Hm: np.ndarray, Em: np.ndarray, Inds: np.ndarray, block: int = 4) -> np.ndarray:
    N, _ = Hm.shape
    Vs = Inds.shape[1]
    LSE = np.full(N, -np.inf)
    for n0 in range(0, N, block):
        n1 = min(N, n0 + block)
        Hn = Hm[n0:n1].astype(np.float64)
        m = np.full(n1 - n0, -np.inf)
        dsum = np.zeros(n1 - n0)
        j = 0
        while j < Vs:
            c_n = Em[Inds[n0:n1, j]].astype(np.float64)      # indexed load
            o_n = np.sum(Hn * c_n, axis=1)                   # scalar product over the full hidden dim
            m_new = np.maximum(m, o_n)
            dsum = dsum * np.exp(m - m_new) + np.exp(o_n - m_new)
            m = m_new
            j += 1
        LSE[n0:n1] = m + np.log(dsum)
    return LSE


def grads_blockwise(Hm: np.ndarray, Em: np.ndarray, Inds: np.ndarray, LSE: np.ndarray, gLSE: np.ndarray, block: int = 4):
    """Returns (dH [N,d], dE [V,d]) of sum_i gLSE_i * LSE_i."""
    N, d = Hm.shape
    Vs = Inds.shape[1]
    dH = np.zeros((N, d))
    dE = np.zeros((Em.shape[0], d))
    for n0 in range(0, N, block):
        n1 = min(N, n0 + block)
        Hn = Hm[n0:n1].astype(np.float64)
        for j in range(Vs):
            idx = Inds[n0:n1, j]
            c_n = Em[idx].astype(np.float64)
            o_n = np.sum(Hn * c_n, axis=1)
            S = np.exp(o_n - LSE[n0:n1])
            SG = S * gLSE[n0:n1]
            dH[n0:n1] += SG[:, None] * c_n
            np.add.at(dE, idx, SG[:, None] * Hn)             # indexed update; repeated ids accumulate
    return dH, dE
