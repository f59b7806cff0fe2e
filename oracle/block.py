"""One decoder block of the mini-Transformer that carries FedAttn in the end-to-end
configuration: x += W_O Attn(RoPE(RMSNorm(x) W_QKV)); x += W_down(silu(gate) * up).

TEST INFRASTRUCTURE; never used by the GPU library.

The paper's block (Section III-B, Section IV-B Phase I/II) is attention followed by
a feed-forward network with residual connections and normalisation; the end-to-end
configuration fixes the Llama-style pieces around it: RMSNorm with unit gain,
rotary position embedding on q and k with the token's index in the GLOBAL sequence,
grouped-query attention, an output projection, and a SwiGLU feed-forward network.
Everything is written out in fp64 numpy, step by step.  `round_fn`, when given, is
applied at the tensor interfaces that the GPU path stores in bf16 (inputs of the
matrix products, their outputs, q/k/v, the attention output); the residual stream
stays unrounded.  Conventions the paper does not fix (rotate-half pairing,
theta = 10000, eps = 1e-6) are "parity unpinned" by the paper and pinned here
against the textbook forms only.
"""
from __future__ import annotations

from typing import Callable, Dict, Optional

import numpy as np

from .rowwise import attend_block, attend_rows

Array = np.ndarray


def rmsnorm(x: Array, eps: float = 1e-6) -> Array:
    """x / sqrt(mean(x^2) + eps) over the last axis, unit gain."""
    x = np.asarray(x, dtype=np.float64)
    return x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps)


def rope(x: Array, pos: Array, theta: float = 10000.0) -> Array:
    """Rotary embedding, rotate-half pairing: element i < D/2 is paired with i + D/2 and
    the pair is rotated by the angle pos * theta^(-2 i / D).  x [T, H, D], pos [T]."""
    x = np.asarray(x, dtype=np.float64)
    T, H, D = x.shape
    half = D // 2
    inv_freq = theta ** (-2.0 * np.arange(half, dtype=np.float64) / D)
    ang = np.asarray(pos, dtype=np.float64)[:, None] * inv_freq[None, :]   # [T, D/2]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    a, b = x[..., :half], x[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def swiglu(gate: Array, up: Array) -> Array:
    """silu(gate) * up with silu(z) = z / (1 + exp(-z))."""
    gate = np.asarray(gate, dtype=np.float64)
    return gate / (1.0 + np.exp(-gate)) * np.asarray(up, dtype=np.float64)


def block_forward(x: Array, w: Dict[str, Array], seg_offsets, *, n_q_heads: int, n_kv_heads: int,
                  head_dim: int, is_sync: bool, keep_tok: Optional[Array] = None,
                  pos: Optional[Array] = None, causal: bool = True, eps: float = 1e-6,
                  theta: float = 10000.0, round_fn: Optional[Callable[[Array], Array]] = None) -> Dict[str, Array]:
    """One block.  x [T, d_model]; w: 'qkv' [d_model, (Hq + 2 Hkv) D], 'o' [Hq D, d_model],
    'gate_up' [d_model, 2 F] (gate columns first), 'down' [F, d_model]; y = x @ W.
    Returns the block output and the intermediate tensors the parity tests compare."""
    rd = (lambda a: a) if round_fn is None else (lambda a: np.asarray(round_fn(np.asarray(a, dtype=np.float32)), dtype=np.float64))
    x = np.asarray(x, dtype=np.float64)
    T = x.shape[0]
    Hq, Hkv, D = n_q_heads, n_kv_heads, head_dim
    W = {k: np.asarray(v, dtype=np.float64) for k, v in w.items()}
    if pos is None:
        pos = np.arange(T)          # index in the global sequence
    # attention half
    h = rd(rmsnorm(x, eps))
    qkv = rd(h @ W["qkv"])
    q = qkv[:, :Hq * D].reshape(T, Hq, D)
    k = qkv[:, Hq * D:(Hq + Hkv) * D].reshape(T, Hkv, D)
    v = qkv[:, (Hq + Hkv) * D:].reshape(T, Hkv, D)
    q, k = rd(rope(q, pos, theta)), rd(rope(k, pos, theta))
    # the attention oracle reads its inputs as stored tensors (float32 at most): make that
    # interface explicit here rather than implicit inside it
    q, k, v = (np.asarray(t.astype(np.float32), dtype=np.float64) for t in (q, k, v))
    attn = rd(attend_block(q, k, v, seg_offsets, is_sync=is_sync, causal=causal, keep_tok=keep_tok))
    proj = rd(attn.reshape(T, Hq * D) @ W["o"])
    x1 = x + proj
    # feed-forward half
    h2 = rd(rmsnorm(x1, eps))
    gu = rd(h2 @ W["gate_up"])
    F = W["down"].shape[0]
    act = rd(swiglu(gu[:, :F], gu[:, F:]))
    down = rd(act @ W["down"])
    x2 = x1 + down
    return {"out": x2, "attn": attn, "q": q, "k": k, "v": v, "x_mid": x1, "act": act, "proj": proj, "down": down}


def block_forward_rows(x: Array, w: Dict[str, Array], seg_offsets, rows, *, n_q_heads: int, n_kv_heads: int,
                       head_dim: int, is_sync: bool, keep_tok: Optional[Array] = None,
                       pos: Optional[Array] = None, causal: bool = True, eps: float = 1e-6,
                       theta: float = 10000.0, round_fn: Optional[Callable[[Array], Array]] = None) -> Dict[str, Array]:
    """The block output for the token rows `rows` only, for sizes at which the whole block is out
    of a CPU's reach.  A row of the output needs the whole block only through the keys and values
    its attention sees, so K and V are computed for every token (normalisation, K/V columns of
    the projection, rotary embedding of K) and everything else - the query, the attention of all
    heads, the output projection, the feed-forward half - for the requested rows alone.  Same
    steps, same order and same rounding hook as block_forward; returns 'out' [R, d_model],
    'attn' [R, Hq, D], 'proj' and 'down' [R, d_model] (the two residual updates)."""
    rd = (lambda a: a) if round_fn is None else (lambda a: np.asarray(round_fn(np.asarray(a, dtype=np.float32)), dtype=np.float64))
    x = np.asarray(x, dtype=np.float64)
    rows = np.asarray(rows, dtype=np.int64)
    T, R = x.shape[0], rows.shape[0]
    Hq, Hkv, D = n_q_heads, n_kv_heads, head_dim
    W = {k: np.asarray(v, dtype=np.float64) for k, v in w.items()}
    if pos is None:
        pos = np.arange(T)
    pos = np.asarray(pos)
    # keys and values of every token
    h = rd(rmsnorm(x, eps))
    k = rd(h @ W["qkv"][:, Hq * D:(Hq + Hkv) * D]).reshape(T, Hkv, D)
    v = rd(h @ W["qkv"][:, (Hq + Hkv) * D:]).reshape(T, Hkv, D)
    k = rd(rope(k, pos, theta))
    # queries of the requested rows, scattered into an otherwise empty [T, Hq, D] array (the
    # attention routine addresses queries by token index)
    qr = rd(h[rows] @ W["qkv"][:, :Hq * D]).reshape(R, Hq, D)
    qr = rd(rope(qr, pos[rows], theta))
    q = np.zeros((T, Hq, D), dtype=np.float32)
    q[rows] = qr.astype(np.float32)
    k32, v32 = k.astype(np.float32), v.astype(np.float32)
    rr = np.repeat(rows, Hq).astype(np.int32)
    hh = np.tile(np.arange(Hq, dtype=np.int32), R)
    attn = rd(attend_rows(q, k32, v32, seg_offsets, rr, hh, is_sync=is_sync, causal=causal, keep_tok=keep_tok)).reshape(R, Hq, D)
    proj = rd(attn.reshape(R, Hq * D) @ W["o"])
    x1 = x[rows] + proj
    h2 = rd(rmsnorm(x1, eps))
    gu = rd(h2 @ W["gate_up"])
    F = W["down"].shape[0]
    act = rd(swiglu(gu[:, :F], gu[:, F:]))
    down = rd(act @ W["down"])
    return {"out": x1 + down, "attn": attn, "proj": proj, "down": down, "x_mid": x1}
