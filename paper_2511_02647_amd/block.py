"""The decoder block of the end-to-end configuration on the device: the FedAttn attention
operator with its surroundings.

    x += W_O Attention(RoPE(RMSNorm(x) W_QKV));   x += W_down (silu(gate) * up)

The attention, RMSNorm, rotary embedding + QKV split, SwiGLU and the residual adds run in the
library's kernels; the four matrix products are plain GEMMs and go to the GEMM library through
`torch.matmul` (bf16 operands, fp32 accumulation).  Composition only: no arithmetic of its own.
Residual stream fp32, every other tensor bf16.  Each residual update is applied by the kernel
that normalises the stream for the next matrix product (one pass instead of two): the
attention's update inside the block, the feed-forward's at the start of the next block when the
caller hands it on (`pending`), else by a plain residual add at the end of the block.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, Optional

import torch

from . import (FEDATTN_OP_PREFILL, fedattn_params, fedattn_prefill, fedattn_residual_add, fedattn_residual_add_rmsnorm,
               fedattn_rmsnorm, fedattn_rope_split_qkv, fedattn_swiglu, fedattn_workspace_bytes)


@dataclass
class BlockWeights:
    """y = x @ W layouts: qkv [d_model, (Hq + 2 Hkv) D] (q heads, k heads, v heads), o [Hq D, d_model],
    gate_up [d_model, 2 F] (gate columns first), down [F, d_model]; bf16 device tensors."""
    qkv: torch.Tensor
    o: torch.Tensor
    gate_up: torch.Tensor
    down: torch.Tensor


class BlockBuffers:
    """Activation buffers of one block for `tokens` tokens, allocated once and reused."""

    def __init__(self, params: fedattn_params, tokens: int, d_model: int, hidden: int, chunk_tokens: int = 0):
        Hq, Hkv, D = params.n_q_heads, params.n_kv_heads, params.head_dim
        bf = dict(dtype=torch.bfloat16, device="cuda")
        self.h = torch.empty(tokens, d_model, **bf)
        self.qkv = torch.empty(tokens, (Hq + 2 * Hkv) * D, **bf)
        self.q = torch.empty(tokens, Hq, D, **bf)
        self.k = torch.empty(tokens, Hkv, D, **bf)
        self.v = torch.empty(tokens, Hkv, D, **bf)
        self.attn = torch.empty(tokens, Hq, D, **bf)
        self.proj = torch.empty(tokens, d_model, **bf)
        self.gate_up = torch.empty(tokens, 2 * hidden, **bf)
        self.act = torch.empty(tokens, hidden, **bf)
        nbytes = fedattn_workspace_bytes(params, FEDATTN_OP_PREFILL, tokens, chunk_tokens) if chunk_tokens else 0
        self.workspace = torch.empty(max(nbytes, 16), dtype=torch.uint8, device="cuda")


def block_forward(params: fedattn_params, block_idx: int, x: torch.Tensor, w: BlockWeights, seg_offsets,
                  buf: BlockBuffers, *, keep_chunks: Optional[torch.Tensor] = None, chunk_tokens: int = 0,
                  sync_override: int = -1, pos: Optional[torch.Tensor] = None, eps: float = 1e-6,
                  theta: float = 10000.0, pending: Optional[torch.Tensor] = None,
                  defer_update: bool = False) -> Dict[str, torch.Tensor]:
    """Runs block `block_idx` in place on the fp32 residual stream x [tokens, d_model]; whether the
    block is local or global follows Algorithm 1 (or `sync_override`).  `pending`: the previous
    block's feed-forward update (bf16 [tokens, d_model]) still to be added to x; it is added by this
    block's first kernel.  With defer_update the block's own feed-forward update is not added but
    returned under "pending" for the next call (a stack ends with fedattn_residual_add(x, pending)).
    Returns views of the intermediate tensors (valid until the next call with the same buffers)."""
    T = x.shape[0]
    if pending is None:
        fedattn_rmsnorm(x, buf.h, eps)
    else:
        fedattn_residual_add_rmsnorm(x, pending, buf.h, eps)
    torch.matmul(buf.h, w.qkv, out=buf.qkv)
    fedattn_rope_split_qkv(buf.qkv, pos, buf.q, buf.k, buf.v, theta)
    fedattn_prefill(params, block_idx, buf.q, buf.k, buf.v, buf.attn, seg_offsets, keep_chunks=keep_chunks,
                    chunk_tokens=chunk_tokens, sync_override=sync_override,
                    workspace=buf.workspace if keep_chunks is not None else None)
    torch.matmul(buf.attn.view(T, -1), w.o, out=buf.proj)
    fedattn_residual_add_rmsnorm(x, buf.proj, buf.h, eps)
    torch.matmul(buf.h, w.gate_up, out=buf.gate_up)
    fedattn_swiglu(buf.gate_up, buf.act)
    torch.matmul(buf.act, w.down, out=buf.proj)
    res = {"out": x, "attn": buf.attn, "q": buf.q, "k": buf.k, "v": buf.v, "act": buf.act}
    if defer_update:
        res["pending"] = buf.proj
    else:
        fedattn_residual_add(x, buf.proj)
    return res
