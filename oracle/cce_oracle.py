"""ctypes front end of the C oracle (oracle/cce_oracle.c).  TEST INFRASTRUCTURE ONLY.

Marshals numpy arrays into cce_oracle_run and returns fp64 results.  No arithmetic
of the method lives here; see the C file for the definition and its citations.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional

import numpy as np

from . import build as _build

_LIB = None

F32, BF16 = 0, 1
NEG_SHARED, NEG_PER_POSITION, NEG_FULL = 0, 1, 2


def _lib():
    global _LIB
    if _LIB is None:
        path = _build.LIB
        if not os.path.exists(path) or os.path.getmtime(path) < os.path.getmtime(_build.SRC):
            _build.build()
        lib = ctypes.CDLL(path)
        lib.cce_oracle_run.restype = ctypes.c_int
        lib.cce_oracle_run.argtypes = [
            ctypes.c_int64, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
            ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
        ]
        lib.cce_oracle_filter_blocks.restype = ctypes.c_int
        lib.cce_oracle_filter_blocks.argtypes = [ctypes.c_int64, ctypes.c_int64, ctypes.c_int32, ctypes.c_double,
                                                 ctypes.c_void_p, ctypes.c_void_p]
        lib.cce_oracle_num_threads.restype = ctypes.c_int
        _LIB = lib
    return _LIB


def num_threads() -> int:
    return int(_lib().cce_oracle_num_threads())


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


@dataclass
class OracleResult:
    loss: np.ndarray               # [n_out] fp64
    lse: np.ndarray                # [n_out] fp64
    dH: Optional[np.ndarray]       # [n_out, d] fp64
    dE: Optional[np.ndarray]       # dense [V, d] or compact [R, d] fp64
    dE_rows: Optional[np.ndarray]  # ids of the compact dE rows (None when dense)
    p: Optional[np.ndarray]        # [n_out, n_cand] softmax


def touched_rows(tgt, neg, mask, neg_mode: int, V: int, sel=None, mask_collisions: int = 1) -> np.ndarray:
    """Sorted unique ids whose dE row receives at least one update (index bookkeeping only)."""
    tgt = np.asarray(tgt)
    valid = np.ones(tgt.shape[0], bool) if mask is None else (np.asarray(mask) != 0)
    if sel is not None:
        keep = np.zeros_like(valid)
        keep[np.asarray(sel)] = True
        valid &= keep
    if not valid.any():
        return np.zeros(0, np.int64)
    if neg_mode == NEG_FULL:
        return np.arange(V, dtype=np.int64)
    parts = [tgt[valid].astype(np.int64)]
    if neg is not None and np.asarray(neg).size:
        neg = np.asarray(neg)
        if neg_mode == NEG_SHARED:
            if mask_collisions:
                # a shared negative is touched if at least one valid position does not collide with it
                tv = np.unique(tgt[valid])
                if tv.size == 1:
                    parts.append(neg[neg != tv[0]].astype(np.int64))
                else:
                    parts.append(neg.astype(np.int64))
            else:
                parts.append(neg.astype(np.int64))
        else:
            nv = neg[valid]
            if mask_collisions:
                nv = nv[nv != tgt[valid][:, None]]
            parts.append(nv.reshape(-1).astype(np.int64))
    return np.unique(np.concatenate(parts))


def run(H, E, tgt, neg, mask, g, *, in_dtype: str, neg_mode: int, mask_collisions: int = 1, K: Optional[int] = None,
        sel=None, want_dH: bool = True, want_dE: str = "dense", want_p: bool = False, p_keep=None) -> OracleResult:
    """H, E: float32 arrays (in_dtype 'f32') or uint16 bf16 bit patterns ('bf16').

    want_dE: "none" | "dense" ([V,d]) | "compact" (rows = touched_rows(...)).
    p_keep: optional [n_out, n_cand] uint8 marks of the gradient filter (filter_blocks).
    """
    lib = _lib()
    H = np.ascontiguousarray(H)
    E = np.ascontiguousarray(E)
    N, d = H.shape
    V = E.shape[0]
    assert E.shape[1] == d
    dt = F32 if in_dtype == "f32" else BF16
    assert H.dtype == (np.float32 if dt == F32 else np.uint16) and E.dtype == H.dtype
    tgt = np.ascontiguousarray(tgt, dtype=np.int32)
    if neg_mode == NEG_FULL:
        neg_a, K_ = None, 0
    else:
        neg_a = None if neg is None else np.ascontiguousarray(neg, dtype=np.int32)
        if K is None:
            K = 0 if neg_a is None else (neg_a.shape[0] if neg_mode == NEG_SHARED else neg_a.shape[1])
        K_ = int(K)
        if neg_mode == NEG_PER_POSITION and neg_a is not None:
            assert neg_a.shape == (N, K_)
    mask_a = None if mask is None else np.ascontiguousarray(mask, dtype=np.uint8)
    g_a = None if g is None else np.ascontiguousarray(g, dtype=np.float64)
    sel_a = None if sel is None else np.ascontiguousarray(sel, dtype=np.int64)
    n_out = N if sel_a is None else sel_a.shape[0]
    n_cand = V if neg_mode == NEG_FULL else K_ + 1

    loss = np.zeros(n_out, np.float64)
    lse = np.zeros(n_out, np.float64)
    dH = np.zeros((n_out, d), np.float64) if want_dH else None
    p = np.zeros((n_out, n_cand), np.float64) if want_p else None
    dE = rows = slot = None
    if want_dE == "dense":
        dE = np.zeros((V, d), np.float64)
    elif want_dE == "compact":
        rows = touched_rows(tgt, neg_a, mask_a, neg_mode, V, sel=sel_a, mask_collisions=mask_collisions)
        slot = np.full(V, -1, np.int64)
        slot[rows] = np.arange(rows.shape[0])
        dE = np.zeros((rows.shape[0], d), np.float64)
    elif want_dE != "none":
        raise ValueError(want_dE)

    keep_a = None
    if p_keep is not None:
        keep_a = np.ascontiguousarray(p_keep, dtype=np.uint8)
        assert keep_a.shape == (n_out, n_cand)
    rc = lib.cce_oracle_run(N, V, d, K_, dt, neg_mode, int(mask_collisions), _ptr(H), _ptr(E), _ptr(tgt), _ptr(neg_a),
                            _ptr(mask_a), _ptr(g_a), n_out, _ptr(sel_a), _ptr(loss), _ptr(lse), _ptr(dH), _ptr(slot),
                            _ptr(dE), _ptr(p), _ptr(keep_a))
    if rc != 0:
        raise RuntimeError(f"cce_oracle_run failed with status {rc}")
    return OracleResult(loss, lse, dH, dE, rows, p)


def run_workload(w, *, g=None, sel=None, want_dE: str = "dense", want_p: bool = False, want_dH: bool = True) -> OracleResult:
    """Convenience: run on a workloads.Workload."""
    return run(w.H, w.E, w.tgt, w.neg, w.mask, w.g if g is None else g, in_dtype=w.in_dtype, neg_mode=w.neg_mode,
               mask_collisions=w.mask_collisions, K=w.K, sel=sel, want_dH=want_dH, want_dE=want_dE, want_p=want_p)


def filter_blocks(p: np.ndarray, eps: float, block: int = 32) -> np.ndarray:
    """Marks of the gradient filter for the softmax p [n_valid, n_cand] of the valid positions in batch order."""
    p = np.ascontiguousarray(p, dtype=np.float64)
    keep = np.zeros(p.shape, np.uint8)
    rc = _lib().cce_oracle_filter_blocks(p.shape[0], p.shape[1], int(block), float(eps), _ptr(p), _ptr(keep))
    if rc != 0:
        raise RuntimeError(f"cce_oracle_filter_blocks failed with status {rc}")
    return keep


def run_workload_filtered(w, eps: float, *, g=None, block: int = 32, want_dE: str = "dense"):
    """Forward + filtered backward on a workload.  Returns (result over the valid positions in batch order, their
    indices, the unfiltered softmax of those positions)."""
    valid = np.flatnonzero(np.asarray(w.mask) != 0).astype(np.int64)
    first = run_workload(w, g=g, sel=valid, want_dE="none", want_p=True, want_dH=False)
    keep = filter_blocks(first.p, eps, block)
    res = run(w.H, w.E, w.tgt, w.neg, w.mask, w.g if g is None else g, in_dtype=w.in_dtype, neg_mode=w.neg_mode,
              mask_collisions=w.mask_collisions, K=w.K, sel=valid, want_dE=want_dE, p_keep=keep)
    return res, valid, first.p
