"""Helpers of the GPU parity tests: host arrays -> device tensors, calls through
the C ABI binding, and the error metrics of the parity bar."""
from __future__ import annotations

import sys

import numpy as np
import torch

import paper_2511_02647_amd as fa

BF16_MAX_ABS, BF16_MEAN_ABS = 2e-2, 2e-3   # parity bar for bf16 inputs
F32_MAX_ABS = 1e-5                          # parity bar for fp32 inputs


def say(msg: str) -> None:
    """Name the case before the GPU step runs (kept if the step takes the box down)."""
    print("[gpu-case] " + msg, flush=True)
    sys.stdout.flush()


def dev(x: np.ndarray, dtype: torch.dtype) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to("cuda")
    if dtype == torch.bfloat16:
        t16 = t.to(torch.bfloat16)
        assert torch.equal(t16.float(), t), "input is not bf16-representable"
        return t16.contiguous()
    return t.contiguous()


def host(t: torch.Tensor) -> np.ndarray:
    return t.float().cpu().numpy().astype(np.float64)


def prefill(q, k, v, seg, *, Hq, Hkv, D, H, block, dtype, causal=True, keep_chunks=None,
            chunk_tokens=0, sync_override=-1, scale=0.0):
    """One block through fedattn_prefill; returns the output on the host (float64)."""
    N = len(seg) - 1
    p = fa.make_params(N, Hq, Hkv, D, H, dtype, causal=causal, softmax_scale=scale)
    tq, tk, tv = dev(q, dtype), dev(k, dtype), dev(v, dtype)
    out = torch.full_like(tq, float("nan"))
    kc = ws = None
    if keep_chunks is not None:
        kc = torch.from_numpy(np.ascontiguousarray(keep_chunks, dtype=np.uint8)).to("cuda")
        nbytes = fa.fedattn_workspace_bytes(p, fa.FEDATTN_OP_PREFILL, int(seg[-1]), chunk_tokens)
        ws = torch.empty(max(nbytes, 16), dtype=torch.uint8, device="cuda")
    fa.fedattn_prefill(p, block, tq, tk, tv, out, seg, keep_chunks=kc, chunk_tokens=chunk_tokens,
                       sync_override=sync_override, workspace=ws)
    torch.cuda.synchronize()
    return host(out)


def decode(q, kc, vc, seg, lens, *, Hq, Hkv, D, H, block, dtype, remote_lens=None, sync_override=-1):
    N = len(seg) - 1
    p = fa.make_params(N, Hq, Hkv, D, H, dtype)
    tq, tk, tv = dev(q, dtype), dev(kc, dtype), dev(vc, dtype)
    out = torch.full_like(tq, float("nan"))
    nbytes = fa.fedattn_workspace_bytes(p, fa.FEDATTN_OP_DECODE, int(seg[-1]))
    ws = torch.empty(max(nbytes, 16), dtype=torch.uint8, device="cuda")
    fa.fedattn_decode(p, block, tq, tk, tv, out, seg, lens, remote_lens=remote_lens,
                      sync_override=sync_override, workspace=ws)
    torch.cuda.synchronize()
    return host(out)


def check(got: np.ndarray, ref: np.ndarray, dtype: torch.dtype, what: str) -> None:
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.all(np.isfinite(got)), "%s: non-finite output (rows never written?)" % what
    err = np.abs(got - ref)
    mx, mean = float(err.max()) if err.size else 0.0, float(err.mean()) if err.size else 0.0
    print("[parity] %-60s max-abs %.3e mean-abs %.3e" % (what, mx, mean), flush=True)
    if dtype == torch.bfloat16:
        assert mx <= BF16_MAX_ABS and mean <= BF16_MEAN_ABS, "%s: max %.3e mean %.3e" % (what, mx, mean)
    else:
        assert mx <= F32_MAX_ABS, "%s: max %.3e" % (what, mx)
