"""Host-side planning helpers: where to synchronise, and what a plan costs.

No arithmetic of the attention path lives here; these helpers only produce the
`sync_override` flags that fedattn_prefill / fedattn_decode take, and the
analytic per-participant cost figures the paper's evaluation reports beside the
measured ones (Section VII-A, evaluation metrics: bits transmitted per
participant for the KV exchange; FLOPs and peak memory per participant).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Sequence

import numpy as np


def uniform_schedule(n_blocks: int, sync_interval: int) -> List[bool]:
    """Algorithm 1: block m = H t + h (1-based) synchronises iff h = H; H <= 0 never."""
    return [sync_interval >= 1 and (b + 1) % sync_interval == 0 for b in range(n_blocks)]


def _spread(lo: int, hi: int, count: int) -> List[int]:
    """`count` distinct block indices spread evenly over [lo, hi), each at the end of its share."""
    span = hi - lo
    count = max(0, min(count, span))
    return [lo + ((i + 1) * span + count - 1) // count - 1 for i in range(count)]


def sync_schedule(name: str, n_blocks: int, n_syncs: int) -> List[bool]:
    """The alternative placements of the global-attention blocks compared in Section VII-B
    (where to synchronise), for a budget of `n_syncs` global blocks among `n_blocks`.

    The paper names the schemes without printing block positions; the readings here:
      uniform      equal intervals (Algorithm 1 with H = n_blocks / n_syncs when that divides)
      shallow-half all global blocks spread over the first half of the stack
      deep-half    all global blocks spread over the second half
      progressive  intervals that grow with depth: 1, 2, 3, ... local forwards more each time,
                   scaled to the stack (global blocks concentrate in shallow layers)
      regressive   the mirror image: intervals shrink with depth
    Returns one flag per block (True = global attention).
    """
    M, T = int(n_blocks), int(n_syncs)
    if M < 0 or T < 0 or T > M:
        raise ValueError("need 0 <= n_syncs <= n_blocks")
    flags = [False] * M
    if T == 0:
        return flags
    half = max(T, M // 2)
    if name == "uniform":
        idx = _spread(0, M, T)
    elif name == "shallow-half":
        idx = _spread(0, half, T)
    elif name == "deep-half":
        idx = _spread(M - half, M, T)
    elif name in ("progressive", "regressive"):
        # the i-th interval (local forwards up to and including a global block) is proportional
        # to i: it ends at block ceil(M (1 + ... + i) / (1 + ... + T)); collisions on short
        # stacks are pushed apart
        tri = T * (T + 1) // 2
        ends = [(M * (i * (i + 1) // 2) + tri - 1) // tri - 1 for i in range(1, T + 1)]
        for i in range(1, T):
            ends[i] = max(ends[i], ends[i - 1] + 1)
        for i in range(T - 1, -1, -1):
            ends[i] = min(ends[i], M - 1 - (T - 1 - i))
        if name == "progressive":
            idx = ends
        else:
            gaps = [ends[0] + 1] + [ends[i] - ends[i - 1] for i in range(1, T)]
            idx, pos = [], -1
            for g in reversed(gaps):
                pos += g
                idx.append(pos)
    else:
        raise ValueError("unknown schedule %r" % name)
    for i in idx:
        flags[i] = True
    if sum(flags) != T:
        raise AssertionError("schedule %s placed %d of %d global blocks" % (name, sum(flags), T))
    return flags


@dataclass
class CostReport:
    """Analytic cost of one inference under a synchronisation plan, averaged over participants."""
    n_participants: int
    n_sync_blocks: int
    comm_bits_per_participant: float        # KV exchange during prefill: sent + received
    comm_bits_sent_per_participant: float
    prefill_attn_flops_per_participant: float
    decode_attn_flops_per_participant_step: float
    peak_kv_bytes_per_participant: float    # KV caches kept for decoding (local or global, per block)

    def as_dict(self) -> dict:
        return dict(self.__dict__)


def cost_report(seg_lens: Sequence[int], sync_flags: Sequence[bool], n_q_heads: int, n_kv_heads: int,
                head_dim: int, bytes_per_elem: int = 2, keep_fraction: float = 1.0,
                causal: bool = True, decode_tokens: int = 0) -> CostReport:
    """Per-participant communication, attention FLOPs and KV memory of FedAttn.

    Communication: in every global block a participant sends its (kept) K and V rows once and
    receives every other participant's kept rows (Section IV-B, Phase II; sparse exchange keeps
    the fraction `keep_fraction` of the remote rows).
    FLOPs: 4 D per visible (query, key) pair and query head (Q K^T and P V), pairs counted as
    the attention mask allows them: own segment in local blocks, the global sequence in global
    blocks (own rows complete, remote rows kept).
    Memory: a local block caches the participant's own K, V; a global block caches the global
    K, V it attended to (Section IV-C), plus `decode_tokens` generated rows per block.
    """
    lens = np.asarray(seg_lens, dtype=np.int64)
    N = len(lens)
    flags = [bool(f) for f in sync_flags]
    n_sync = sum(flags)
    n_local = len(flags) - n_sync
    row_bytes = 2 * n_kv_heads * head_dim * bytes_per_elem  # K and V
    kept = np.floor(lens * keep_fraction + 0.5).astype(np.int64) if keep_fraction < 1.0 else lens
    sent = kept * row_bytes * 8.0
    recv = (kept.sum() - kept) * row_bytes * 8.0
    kept_before = np.concatenate([[0], np.cumsum(kept)[:-1]])
    if causal:
        own_pairs = lens * (lens + 1) // 2
        remote_pairs = lens * kept_before
    else:
        own_pairs = lens * lens
        remote_pairs = lens * (kept.sum() - kept)
    fl = 4.0 * head_dim * n_q_heads
    prefill = fl * (len(flags) * own_pairs + n_sync * remote_pairs)
    visible_local = lens + decode_tokens
    visible_sync = lens + decode_tokens + (kept.sum() - kept)
    decode = fl * (n_local * visible_local + n_sync * visible_sync)
    mem = row_bytes * (n_local * (lens + decode_tokens) + n_sync * (lens + decode_tokens + (kept.sum() - kept)))
    return CostReport(N, n_sync, float((sent + recv).mean() * n_sync), float(sent.mean() * n_sync),
                      float(prefill.mean()), float(decode.mean()), float(mem.mean()))
