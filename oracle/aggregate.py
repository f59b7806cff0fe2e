"""KV aggregation of a sync block (Phase II, global KV matrix).

TEST INFRASTRUCTURE; never used by the GPU library.

[K V] = sum_n Pi_n [k_n v_n]: Pi_n's columns are basis vectors at participant
n's global positions, so the sum places row r of k_n at global row i_n^r and
touches every global row exactly once.  With contiguous index sets that is the
concatenation of the local matrices in participant order.
"""
from __future__ import annotations

from typing import Sequence, Tuple

import numpy as np


def selection_matrix(seg_offsets, n: int) -> np.ndarray:
    """Pi_n in {0,1}^{L x L_n} (Section IV-A)."""
    seg_offsets = np.asarray(seg_offsets)
    L = int(seg_offsets[-1])
    s, e = int(seg_offsets[n]), int(seg_offsets[n + 1])
    pi = np.zeros((L, e - s))
    pi[np.arange(s, e), np.arange(e - s)] = 1.0
    return pi


def aggregate_kv(k_locals: Sequence[np.ndarray], v_locals: Sequence[np.ndarray],
                 seg_offsets) -> Tuple[np.ndarray, np.ndarray]:
    """Global K, V [L,Hkv,D] from the participants' local [L_n,Hkv,D] matrices."""
    seg_offsets = np.asarray(seg_offsets)
    L = int(seg_offsets[-1])
    shape = (L,) + tuple(k_locals[0].shape[1:])
    K = np.zeros(shape, dtype=k_locals[0].dtype)
    V = np.zeros(shape, dtype=v_locals[0].dtype)
    for n, (kn, vn) in enumerate(zip(k_locals, v_locals)):
        s, e = int(seg_offsets[n]), int(seg_offsets[n + 1])
        assert kn.shape[0] == e - s and vn.shape[0] == e - s
        K[s:e] = kn
        V[s:e] = vn
    return K, V


def aggregate_kv_by_definition(k_locals, v_locals, seg_offsets):
    """The same through the literal sum of Pi_n products (tiny inputs only)."""
    seg_offsets = np.asarray(seg_offsets)
    L = int(seg_offsets[-1])
    tail = tuple(k_locals[0].shape[1:])
    K = np.zeros((L, int(np.prod(tail))))
    V = np.zeros_like(K)
    for n, (kn, vn) in enumerate(zip(k_locals, v_locals)):
        pi = selection_matrix(seg_offsets, n)
        K += pi @ np.asarray(kn, dtype=np.float64).reshape(kn.shape[0], K.shape[1])
        V += pi @ np.asarray(vn, dtype=np.float64).reshape(vn.shape[0], V.shape[1])
    return K.reshape((L,) + tail), V.reshape((L,) + tail)
