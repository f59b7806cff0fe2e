"""Brute-force route of the oracle: dense visibility matrix, dense scores, dense
softmax, all in numpy float64.  Only for tiny inputs (memory is Hq * L * L).

TEST INFRASTRUCTURE; never used by the GPU library.  Written separately from
the row-by-row C program so that the two can check each other.
"""
from __future__ import annotations

import math
from typing import Optional, Tuple

import numpy as np


def visibility(seg_offsets, *, is_sync: bool, causal: bool = True, keep_tok=None) -> np.ndarray:
    """Boolean [L, L]: entry (i, j) says whether query i may attend to key j.

    Causal order (Section III-B, read as "self and preceding tokens"), own
    segment always (Phase I), remote segments only in a sync block (Phase II)
    and, under sparse KV exchange, only the remote rows that were sent."""
    seg_offsets = np.asarray(seg_offsets, dtype=np.int64)
    L = int(seg_offsets[-1])
    owner = np.repeat(np.arange(len(seg_offsets) - 1), np.diff(seg_offsets))
    same = owner[:, None] == owner[None, :]
    if is_sync:
        sent = np.ones(L, dtype=bool) if keep_tok is None else np.asarray(keep_tok).astype(bool)
        vis = same | sent[None, :]
    else:
        vis = same.copy()
    if causal:
        idx = np.arange(L)
        vis &= idx[None, :] <= idx[:, None]
    return vis


def attention(q, k, v, seg_offsets, *, is_sync: bool, causal: bool = True,
              scale: Optional[float] = None, keep_tok=None) -> Tuple[np.ndarray, np.ndarray]:
    """(out [L,Hq,D], prob [Hq,L,L]) with the additive 0 / -inf mask of Section
    III-B applied to the full score matrix.  KV heads are repeated Hq/Hkv times
    (GQA written out as plain multi-head attention)."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    L, Hq, D = q.shape
    group = Hq // k.shape[1]
    k = np.repeat(k, group, axis=1)
    v = np.repeat(v, group, axis=1)
    sc = (1.0 / math.sqrt(D)) if scale is None else float(scale)
    vis = visibility(seg_offsets, is_sync=is_sync, causal=causal, keep_tok=keep_tok)
    mask = np.where(vis, 0.0, -np.inf)
    out = np.zeros((L, Hq, D))
    prob = np.zeros((Hq, L, L))
    for h in range(Hq):
        s = sc * (q[:, h, :] @ k[:, h, :].T) + mask
        mx = s.max(axis=1, keepdims=True) if L else s
        mx = np.where(np.isfinite(mx), mx, 0.0)
        e = np.exp(s - mx)
        den = e.sum(axis=1, keepdims=True)
        p = np.divide(e, den, out=np.zeros_like(e), where=den > 0)
        prob[h] = p
        out[:, h, :] = p @ v[:, h, :]
    return out, prob


def decode(q, k_cache, v_cache, seg_offsets, seg_lens, *, is_sync: bool, remote_lens=None,
           scale: Optional[float] = None) -> np.ndarray:
    """[N,Hq,D]: one query per participant over the cached rows it may see
    (Section IV-C)."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k_cache, dtype=np.float64)
    v = np.asarray(v_cache, dtype=np.float64)
    N, Hq, D = q.shape
    group = Hq // k.shape[1]
    sc = (1.0 / math.sqrt(D)) if scale is None else float(scale)
    seg_offsets = np.asarray(seg_offsets)
    remote = seg_lens if remote_lens is None else remote_lens
    out = np.zeros((N, Hq, D))
    for n in range(N):
        idx = []
        for m in range(N):
            if m == n:
                idx.append(np.arange(seg_offsets[m], seg_offsets[m] + seg_lens[m]))
            elif is_sync:
                idx.append(np.arange(seg_offsets[m], seg_offsets[m] + remote[m]))
        idx = np.concatenate(idx) if idx else np.zeros(0, dtype=np.int64)
        if idx.size == 0:
            continue
        for h in range(Hq):
            g = h // group
            s = sc * (k[idx, g, :] @ q[n, h, :])
            e = np.exp(s - s.max())
            out[n, h] = (e / e.sum()) @ v[idx, g, :]
    return out
