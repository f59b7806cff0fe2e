"""Seeded synthetic inputs for the FedAttn attention path.

This module serves both the CPU oracle's tests and the GPU path's tests and
benchmark.  It holds no attention arithmetic: only random draws, the rounding of
drawn values to the storage type, segment layouts, keep-lists and row samples.

The inputs stand in for the paper's workload (a few-shot prompt cut into
contiguous per-participant segments, equal or uneven in length, decoded for at
most 256 new tokens with the prefill caches kept; Section "Experimental
Results", Setup).  No item of that workload's dataset is reproduced here:
Q, K and V are i.i.d. normal draws shaped like the projections of a
Llama-style GQA model.

Every array is produced by a counter-based Philox stream keyed by
(seed, workload id) and positioned by (block, tensor id), so any block of any
workload can be regenerated alone.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Tuple

import numpy as np

DEFAULT_SEED = 251102647

# tensor ids (Philox counter word 2)
_T_Q, _T_K, _T_V, _T_LENS, _T_KEEP, _T_ROWS, _T_X, _T_W = range(8)


def stream(seed: int, workload_id: int, block: int, tensor: int) -> np.random.Generator:
    """Independent generator for one (workload, block, tensor)."""
    bitgen = np.random.Philox(key=np.array([seed, workload_id], dtype=np.uint64),
                              counter=np.array([0, 0, tensor, block], dtype=np.uint64))
    return np.random.Generator(bitgen)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even); result is
    float32 holding exactly bf16-representable values."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    r = (u + bias) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def bf16_bits(x_bf16_valued: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of float32 values that are already bf16-representable."""
    u = np.ascontiguousarray(x_bf16_valued, dtype=np.float32).view(np.uint32)
    assert not np.any(u & np.uint32(0xFFFF)), "values are not bf16-representable"
    return (u >> np.uint32(16)).astype(np.uint16)


def bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """float32 values of bf16 bit patterns (exact)."""
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass(frozen=True)
class Workload:
    """Shape of one synthetic workload.  Letters follow the paper: N
    participants, M Transformer blocks, H sync interval, L_n segment lengths."""
    name: str
    wid: int                 # Philox key word
    n_participants: int
    seg_lens: Tuple[int, ...]
    n_blocks: int            # M
    sync_interval: int       # H
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    dtype: str               # "f32" or "bf16"
    sigma: float             # std of Q, K, V draws
    decode_steps: int = 0
    chunk_tokens: int = 0    # sparse KV exchange granularity (0 = dense)
    keep_fraction: float = 1.0

    @property
    def seg_offsets(self) -> np.ndarray:
        return np.concatenate([[0], np.cumsum(self.seg_lens)]).astype(np.int32)

    @property
    def total_tokens(self) -> int:
        return int(sum(self.seg_lens))


def hetero_lens(seed: int = DEFAULT_SEED, n: int = 8, lo: int = 1024, hi: int = 3072) -> Tuple[int, ...]:
    g = stream(seed, 3, 0, _T_LENS)
    return tuple(int(x) for x in g.integers(lo, hi, size=n, endpoint=True))


def workload(name: str, seed: int = DEFAULT_SEED) -> Workload:
    if name == "cfg1_tiny":
        return Workload(name, 1, 2, (32, 32), 4, 2, 2, 2, 64, "f32", 1.0)
    if name == "cfg2_llama8b_prefill":
        return Workload(name, 2, 4, (512,) * 4, 32, 4, 32, 8, 128, "bf16", 0.5)
    if name == "cfg3_hetero_prefill":
        return Workload(name, 3, 8, hetero_lens(seed), 32, 4, 32, 8, 128, "bf16", 1.0)
    if name == "cfg4_decode":
        # seg_lens here is the per-participant cache capacity (prompt + steps)
        return Workload(name, 4, 16, (1280,) * 16, 32, 4, 32, 8, 128, "bf16", 1.0,
                        decode_steps=256)
    if name == "cfg5_sparse_sync":
        return Workload(name, 5, 16, (4096,) * 16, 8, 2, 16, 4, 128, "bf16", 1.0,
                        chunk_tokens=64, keep_fraction=0.25)
    raise KeyError(name)


WORKLOADS = ("cfg1_tiny", "cfg2_llama8b_prefill", "cfg3_hetero_prefill",
             "cfg4_decode", "cfg5_sparse_sync")


def normal_tensor(w: Workload, seed: int, block: int, tensor: int, shape, sigma: Optional[float] = None) -> np.ndarray:
    """float32 N(0, sigma^2) draws, rounded to bf16 when the workload stores bf16."""
    g = stream(seed, w.wid, block, tensor)
    x = g.standard_normal(size=shape, dtype=np.float32)
    s = w.sigma if sigma is None else sigma
    if s != 1.0:
        x *= np.float32(s)
    if w.dtype == "bf16":
        x = round_to_bf16(x)
    return x


def prefill_block(w: Workload, block: int, seed: int = DEFAULT_SEED,
                  total: Optional[int] = None) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Q[total,Hq,D], K[total,Hkv,D], V[total,Hkv,D] of one Transformer block."""
    t = w.total_tokens if total is None else total
    q = normal_tensor(w, seed, block, _T_Q, (t, w.n_q_heads, w.head_dim))
    k = normal_tensor(w, seed, block, _T_K, (t, w.n_kv_heads, w.head_dim))
    v = normal_tensor(w, seed, block, _T_V, (t, w.n_kv_heads, w.head_dim))
    return q, k, v


def hidden_input(w: Workload, d_model: int, seed: int = DEFAULT_SEED, total: Optional[int] = None) -> np.ndarray:
    """x0 [total, d_model] ~ N(0, 1), bf16-valued: the input of the first block of the
    end-to-end configuration."""
    t = w.total_tokens if total is None else total
    return normal_tensor(w, seed, 0, _T_X, (t, d_model), sigma=1.0)


def block_weights(w: Workload, block: int, d_model: int, hidden: int, seed: int = DEFAULT_SEED,
                  sigma: float = 0.02) -> dict:
    """Weights of one decoder block of the end-to-end configuration, y = x @ W layouts, N(0, sigma^2)
    rounded to bf16: qkv [d_model, (Hq + 2 Hkv) D], o [Hq D, d_model], gate_up [d_model, 2 hidden]
    (gate columns first), down [hidden, d_model]."""
    g = stream(seed, w.wid, block, _T_W)
    Hq, Hkv, D = w.n_q_heads, w.n_kv_heads, w.head_dim
    mk = lambda *shape: round_to_bf16((g.standard_normal(size=shape, dtype=np.float32) * np.float32(sigma)))
    return {"qkv": mk(d_model, (Hq + 2 * Hkv) * D), "o": mk(Hq * D, d_model),
            "gate_up": mk(d_model, 2 * hidden), "down": mk(hidden, d_model)}


def decode_cache_block(w: Workload, block: int, seed: int = DEFAULT_SEED) -> Tuple[np.ndarray, np.ndarray]:
    """K and V caches [capacity_total,Hkv,D] of one block, filled for every row
    up to capacity (step s reads the first prompt+s+1 rows of each segment)."""
    t = w.total_tokens
    k = normal_tensor(w, seed, block, _T_K, (t, w.n_kv_heads, w.head_dim))
    v = normal_tensor(w, seed, block, _T_V, (t, w.n_kv_heads, w.head_dim))
    return k, v


def decode_query(w: Workload, step: int, block: int, seed: int = DEFAULT_SEED) -> np.ndarray:
    """Q[N,Hq,D] of decode step `step` in block `block`."""
    return normal_tensor(w, seed, step * w.n_blocks + block, _T_Q,
                         (w.n_participants, w.n_q_heads, w.head_dim))


def chunk_counts(seg_lens, chunk_tokens: int) -> np.ndarray:
    return np.array([(l + chunk_tokens - 1) // chunk_tokens for l in seg_lens], dtype=np.int64)


def keep_chunks(w: Workload, sync_round: int, seed: int = DEFAULT_SEED,
                seg_lens=None, chunk_tokens: Optional[int] = None,
                fraction: Optional[float] = None) -> np.ndarray:
    """uint8 keep flag per KV chunk, participants concatenated.  In every sync
    round, each source participant keeps round(fraction * #chunks) of its
    chunks, drawn without replacement; all receivers see the same subset."""
    lens = w.seg_lens if seg_lens is None else seg_lens
    ct = w.chunk_tokens if chunk_tokens is None else chunk_tokens
    fr = w.keep_fraction if fraction is None else fraction
    g = stream(seed, w.wid, sync_round, _T_KEEP)
    out: List[np.ndarray] = []
    for nc in chunk_counts(lens, ct):
        flags = np.zeros(int(nc), dtype=np.uint8)
        n_keep = int(round(fr * int(nc)))
        if n_keep > 0:
            flags[g.choice(int(nc), size=n_keep, replace=False)] = 1
        out.append(flags)
    return np.concatenate(out) if out else np.zeros(0, dtype=np.uint8)


def sample_rows(seg_offsets: np.ndarray, n_heads: int, n_random: int, seed: int,
                salt: int = 0, tile: int = 64, max_boundary_rows: int = 20000) -> Tuple[np.ndarray, np.ndarray]:
    """(rows, heads) to check at sizes where the oracle cannot do every row: per segment its
    first two and last two rows and the rows on both sides of EVERY `tile`-aligned position
    inside it, counted from the segment start and from token 0 (the two grids on which the
    kernels cut query and key tiles), plus n_random uniform (row, head) pairs.  If the boundary
    rows number more than max_boundary_rows, every k-th of them is kept (segment ends always)."""
    g = stream(seed, 99, salt, _T_ROWS)
    total = int(seg_offsets[-1])
    ends: List[int] = []
    bounds: List[int] = []
    for n in range(len(seg_offsets) - 1):
        s, e = int(seg_offsets[n]), int(seg_offsets[n + 1])
        if e <= s:
            continue
        ends.extend(r for r in (s, s + 1, e - 2, e - 1) if s <= r < e)
        for base in (s, 0):
            first = base + ((s - base) // tile + 1) * tile      # first aligned position > s
            for t in range(first, e, tile):
                bounds.extend((t - 1, t))
    bounds_a = np.array(sorted(set(bounds)), dtype=np.int64)
    if bounds_a.shape[0] > max_boundary_rows:
        step = -(-bounds_a.shape[0] // max_boundary_rows)
        bounds_a = bounds_a[int(g.integers(0, step))::step]
    rows_a = np.array(sorted(set(ends) | set(bounds_a.tolist())), dtype=np.int32)
    heads_a = g.integers(0, n_heads, size=rows_a.shape[0]).astype(np.int32)
    if n_random > 0 and total > 0:
        rr = g.integers(0, total, size=n_random).astype(np.int32)
        hh = g.integers(0, n_heads, size=n_random).astype(np.int32)
        rows_a = np.concatenate([rows_a, rr])
        heads_a = np.concatenate([heads_a, hh])
    return rows_a, heads_a
