"""Algorithm 1 (FedAttn) applied to the attention operator of a block stack.

TEST INFRASTRUCTURE; never used by the GPU library.

The hot path is the attention alone, so the Q, K, V of every block are inputs
(in a model they come from the QKV projection of the hidden state).  The walk
keeps the algorithm's order and notation: rounds t = 0..T-1; in each round
local forwards h = 1..H-1 where every participant runs Attention(q_n, k_n, v_n)
on its own slice (Phase I), then local forward h = H where the participants'
k_n, v_n are aggregated into the global K, V and every participant runs
Attention(q_n, K, V) (Phase II).  Block index m = H t + h (1-based).  Blocks
left over when H does not divide M are local forwards of an unfinished round.
"""
from __future__ import annotations

from typing import List, Optional, Sequence

import numpy as np

from .aggregate import aggregate_kv
from .rowwise import attend_block, attend_rows


def _local_forward(q, k, v, seg, causal, scale):
    """Phase I: each participant alone, on its own slice, as a one-participant
    problem (no shared mask logic with the sync path)."""
    total, Hq, D = q.shape
    out = np.zeros((total, Hq, D))
    for n in range(len(seg) - 1):
        s, e = int(seg[n]), int(seg[n + 1])
        if e > s:
            out[s:e] = attend_block(q[s:e], k[s:e], v[s:e], [0, e - s], is_sync=False,
                                    causal=causal, scale=scale)
    return out


def _global_forward(q, k, v, seg, causal, scale, keep_tok):
    """Phase II: aggregate, then every participant's queries over the global KV."""
    total, Hq, D = q.shape
    k_loc = [k[int(seg[n]):int(seg[n + 1])] for n in range(len(seg) - 1)]
    v_loc = [v[int(seg[n]):int(seg[n + 1])] for n in range(len(seg) - 1)]
    K, V = aggregate_kv(k_loc, v_loc, seg)
    out = np.zeros((total, Hq, D))
    for n in range(len(seg) - 1):
        s, e = int(seg[n]), int(seg[n + 1])
        if e <= s:
            continue
        rows = np.repeat(np.arange(s, e, dtype=np.int32), Hq)
        heads = np.tile(np.arange(Hq, dtype=np.int32), e - s)
        o = attend_rows(q, K, V, seg, rows, heads, is_sync=True, causal=causal, scale=scale,
                        keep_tok=keep_tok)
        out[s:e] = o.reshape(e - s, Hq, D)
    return out


def run_stack(q_blocks: Sequence[np.ndarray], k_blocks: Sequence[np.ndarray],
              v_blocks: Sequence[np.ndarray], seg_offsets, H: int, *, causal: bool = True,
              scale: Optional[float] = None,
              keep_tok_per_round: Optional[Sequence[Optional[np.ndarray]]] = None) -> List[np.ndarray]:
    """Attention outputs of all M blocks, in block order."""
    M = len(q_blocks)
    seg = np.asarray(seg_offsets, dtype=np.int64)
    outs: List[Optional[np.ndarray]] = [None] * M
    if H <= 0:
        T, rest = 0, M
    else:
        T, rest = M // H, M % H
    for t in range(T):
        for h in range(1, H):
            m = H * t + h
            outs[m - 1] = _local_forward(q_blocks[m - 1], k_blocks[m - 1], v_blocks[m - 1],
                                         seg, causal, scale)
        m = H * t + H
        keep = None if keep_tok_per_round is None else keep_tok_per_round[t]
        outs[m - 1] = _global_forward(q_blocks[m - 1], k_blocks[m - 1], v_blocks[m - 1],
                                      seg, causal, scale, keep)
    for h in range(1, rest + 1):
        m = (H * T if H > 0 else 0) + h
        outs[m - 1] = _local_forward(q_blocks[m - 1], k_blocks[m - 1], v_blocks[m - 1],
                                     seg, causal, scale)
    return outs  # type: ignore[return-value]
