"""Python binding of the FedAttn HIP library (argument marshalling only).

Every function has the name and the meaning of the C entry point it calls
(include/fedattn.h); all arithmetic runs in the library's gfx950 kernels.
PyTorch is used for device memory and the stream only.  There is no CPU or
PyTorch fallback: if libfedattn.so is missing or fails to load, importing a
function's result fails loudly.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("FEDATTN_LIB") or os.path.join(_HERE, "libfedattn.so")

FEDATTN_OK, FEDATTN_EINVAL, FEDATTN_EUNSUPPORTED, FEDATTN_EWORKSPACE, FEDATTN_ELAUNCH = range(5)
FEDATTN_BF16, FEDATTN_F32 = 0, 1
FEDATTN_OP_PREFILL, FEDATTN_OP_DECODE, FEDATTN_OP_PREFILL_SYNC_LOCAL_KV = 0, 1, 2
FEDATTN_MAX_PARTICIPANTS = 128

EXPORTS = ("fedattn_is_sync_block", "fedattn_workspace_bytes", "fedattn_prefill", "fedattn_prefill_sync_local_kv",
           "fedattn_prefill_blocks", "fedattn_decode", "fedattn_decode_blocks", "fedattn_decode_blocks_fused",
           "fedattn_decode_static", "fedattn_aggregate_kv",
           "fedattn_rmsnorm", "fedattn_rope_split_qkv", "fedattn_swiglu", "fedattn_residual_add",
           "fedattn_residual_add_rmsnorm", "fedattn_probe_stream", "fedattn_probe_mfma",
           "fedattn_last_error", "fedattn_version")


class fedattn_params(ctypes.Structure):
    _fields_ = [("n_participants", ctypes.c_int32), ("n_q_heads", ctypes.c_int32),
                ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("sync_interval", ctypes.c_int32), ("causal", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("softmax_scale", ctypes.c_float)]


class FedAttnError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__("fedattn status %d: %s" % (status, message))
        self.status = status


_lib = None


def load():
    """Load libfedattn.so (built by paper_2511_02647_amd.build.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("%s not found: build it with `python -m paper_2511_02647_amd.build` "
                           "(there is no fallback path)" % LIB_PATH)
    lib = ctypes.CDLL(LIB_PATH)
    i32, i64, vp, sz = ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p, ctypes.c_size_t
    pp = ctypes.POINTER(fedattn_params)
    lib.fedattn_is_sync_block.argtypes = [i32, i32]
    lib.fedattn_is_sync_block.restype = ctypes.c_int
    lib.fedattn_workspace_bytes.argtypes = [pp, i32, i32, i32]
    lib.fedattn_workspace_bytes.restype = sz
    lib.fedattn_prefill.argtypes = [pp, i32, vp, vp, vp, vp, vp, vp, i32, i32, vp, sz, vp]
    lib.fedattn_prefill.restype = ctypes.c_int
    lib.fedattn_prefill_sync_local_kv.argtypes = [pp, vp, vp, vp, vp, vp, vp, i32, vp, sz, vp]
    lib.fedattn_prefill_sync_local_kv.restype = ctypes.c_int
    lib.fedattn_prefill_blocks.argtypes = [pp, i32, i32, vp, vp, vp, vp, i64, i64, vp, vp]
    lib.fedattn_prefill_blocks.restype = ctypes.c_int
    lib.fedattn_decode.argtypes = [pp, i32, vp, vp, vp, vp, vp, vp, vp, i32, vp, sz, vp]
    lib.fedattn_decode.restype = ctypes.c_int
    lib.fedattn_decode_static.argtypes = [pp, i32, vp, vp, vp, vp, vp, vp, vp, i32, vp]
    lib.fedattn_decode_static.restype = ctypes.c_int
    lib.fedattn_decode_blocks.argtypes = [pp, i32, i32, vp, vp, vp, vp, i64, i64, vp, vp, vp, i32, vp, sz, vp]
    lib.fedattn_decode_blocks.restype = ctypes.c_int
    lib.fedattn_decode_blocks_fused.argtypes = lib.fedattn_decode_blocks.argtypes
    lib.fedattn_decode_blocks_fused.restype = ctypes.c_int
    lib.fedattn_aggregate_kv.argtypes = [pp, vp, vp, vp, vp, vp, vp]
    lib.fedattn_aggregate_kv.restype = ctypes.c_int
    fl = ctypes.c_float
    lib.fedattn_rmsnorm.argtypes = [vp, vp, i64, i32, fl, vp]
    lib.fedattn_rmsnorm.restype = ctypes.c_int
    lib.fedattn_rope_split_qkv.argtypes = [vp, vp, vp, vp, vp, i64, i32, i32, i32, fl, vp]
    lib.fedattn_rope_split_qkv.restype = ctypes.c_int
    lib.fedattn_swiglu.argtypes = [vp, vp, i64, i32, vp]
    lib.fedattn_swiglu.restype = ctypes.c_int
    lib.fedattn_residual_add.argtypes = [vp, vp, i64, vp]
    lib.fedattn_residual_add.restype = ctypes.c_int
    lib.fedattn_residual_add_rmsnorm.argtypes = [vp, vp, vp, i64, i32, fl, vp]
    lib.fedattn_residual_add_rmsnorm.restype = ctypes.c_int
    lib.fedattn_probe_stream.argtypes = [vp, i64, i32, vp, vp]
    lib.fedattn_probe_stream.restype = i64
    lib.fedattn_probe_mfma.argtypes = [vp, i32, vp]
    lib.fedattn_probe_mfma.restype = i64
    lib.fedattn_last_error.restype = ctypes.c_char_p
    lib.fedattn_version.restype = ctypes.c_char_p
    _lib = lib
    return lib


def make_params(n_participants: int, n_q_heads: int, n_kv_heads: int, head_dim: int,
                sync_interval: int, dtype: torch.dtype, causal: bool = True,
                softmax_scale: float = 0.0) -> fedattn_params:
    if dtype == torch.bfloat16:
        dt = FEDATTN_BF16
    elif dtype == torch.float32:
        dt = FEDATTN_F32
    else:
        raise TypeError("dtype must be torch.bfloat16 or torch.float32")
    return fedattn_params(n_participants, n_q_heads, n_kv_heads, head_dim, sync_interval,
                          1 if causal else 0, dt, float(softmax_scale))


def _check(status: int) -> None:
    if status != FEDATTN_OK:
        raise FedAttnError(status, load().fedattn_last_error().decode())


def _dev(t: Optional[torch.Tensor], name: str):
    if t is None:
        return None
    if not t.is_cuda:
        raise TypeError("%s must be a device tensor" % name)
    if not t.is_contiguous():
        raise TypeError("%s must be contiguous" % name)
    return ctypes.c_void_p(t.data_ptr())


def _host_i32(a, name: str) -> np.ndarray:
    arr = np.ascontiguousarray(np.asarray(a), dtype=np.int32)
    if arr.ndim != 1:
        raise TypeError("%s must be one-dimensional" % name)
    return arr


def _stream(stream) -> ctypes.c_void_p:
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def fedattn_version() -> str:
    return load().fedattn_version().decode()


def fedattn_is_sync_block(sync_interval: int, block_idx: int) -> bool:
    return bool(load().fedattn_is_sync_block(int(sync_interval), int(block_idx)))


def fedattn_workspace_bytes(params: fedattn_params, op: int, tokens: int, chunk_tokens: int = 0) -> int:
    return int(load().fedattn_workspace_bytes(ctypes.byref(params), int(op), int(tokens), int(chunk_tokens)))


def fedattn_prefill(params: fedattn_params, block_idx: int, q: torch.Tensor, k: torch.Tensor,
                    v: torch.Tensor, out: torch.Tensor, seg_offsets, keep_chunks: Optional[torch.Tensor] = None,
                    chunk_tokens: int = 0, sync_override: int = -1,
                    workspace: Optional[torch.Tensor] = None, stream=None) -> None:
    seg = _host_i32(seg_offsets, "seg_offsets")
    if seg.shape[0] != params.n_participants + 1:
        raise ValueError("seg_offsets must have n_participants + 1 entries")
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().fedattn_prefill(ctypes.byref(params), int(block_idx), _dev(q, "q"), _dev(k, "k"),
                                  _dev(v, "v"), _dev(out, "out"), seg.ctypes.data_as(ctypes.c_void_p),
                                  _dev(keep_chunks, "keep_chunks"), int(chunk_tokens), int(sync_override),
                                  _dev(workspace, "workspace"), ws_bytes, _stream(stream)))


def _local_ptrs(local: Sequence[Optional[torch.Tensor]], n: int, name: str):
    arr = (ctypes.c_void_p * n)()
    for i in range(n):
        t = local[i]
        if t is None or t.numel() == 0:
            arr[i] = None
        else:
            if not (t.is_cuda and t.is_contiguous()):
                raise TypeError("%s[%d] must be a contiguous device tensor" % (name, i))
            arr[i] = t.data_ptr()
    return arr


def fedattn_prefill_sync_local_kv(params: fedattn_params, q: torch.Tensor, k_local: Sequence[Optional[torch.Tensor]],
                                  v_local: Sequence[Optional[torch.Tensor]], out: torch.Tensor, seg_offsets,
                                  keep_chunks: Optional[torch.Tensor] = None, chunk_tokens: int = 0,
                                  workspace: Optional[torch.Tensor] = None, stream=None) -> None:
    seg = _host_i32(seg_offsets, "seg_offsets")
    n = params.n_participants
    if seg.shape[0] != n + 1 or len(k_local) != n or len(v_local) != n:
        raise ValueError("k_local / v_local / seg_offsets have the wrong length")
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().fedattn_prefill_sync_local_kv(ctypes.byref(params), _dev(q, "q"), _local_ptrs(k_local, n, "k_local"),
                                                _local_ptrs(v_local, n, "v_local"), _dev(out, "out"),
                                                seg.ctypes.data_as(ctypes.c_void_p), _dev(keep_chunks, "keep_chunks"),
                                                int(chunk_tokens), _dev(workspace, "workspace"), ws_bytes,
                                                _stream(stream)))


def fedattn_prefill_blocks(params: fedattn_params, block_idx0: int, n_blocks: int, q: torch.Tensor,
                           k: torch.Tensor, v: torch.Tensor, out: torch.Tensor, q_block_stride: int,
                           kv_block_stride: int, seg_offsets, stream=None) -> None:
    seg = _host_i32(seg_offsets, "seg_offsets")
    if seg.shape[0] != params.n_participants + 1:
        raise ValueError("seg_offsets must have n_participants + 1 entries")
    _check(load().fedattn_prefill_blocks(ctypes.byref(params), int(block_idx0), int(n_blocks), _dev(q, "q"),
                                         _dev(k, "k"), _dev(v, "v"), _dev(out, "out"), int(q_block_stride),
                                         int(kv_block_stride), seg.ctypes.data_as(ctypes.c_void_p),
                                         _stream(stream)))


def fedattn_decode(params: fedattn_params, block_idx: int, q: torch.Tensor, k_cache: torch.Tensor,
                   v_cache: torch.Tensor, out: torch.Tensor, seg_offsets, seg_lens, remote_lens=None,
                   sync_override: int = -1, workspace: Optional[torch.Tensor] = None, stream=None) -> None:
    seg = _host_i32(seg_offsets, "seg_offsets")
    lens = _host_i32(seg_lens, "seg_lens")
    if seg.shape[0] != params.n_participants + 1 or lens.shape[0] != params.n_participants:
        raise ValueError("seg_offsets / seg_lens have the wrong length")
    rl = None
    if remote_lens is not None:
        rl = _host_i32(remote_lens, "remote_lens")
        if rl.shape[0] != params.n_participants:
            raise ValueError("remote_lens has the wrong length")
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().fedattn_decode(ctypes.byref(params), int(block_idx), _dev(q, "q"), _dev(k_cache, "k_cache"),
                                 _dev(v_cache, "v_cache"), _dev(out, "out"),
                                 seg.ctypes.data_as(ctypes.c_void_p), lens.ctypes.data_as(ctypes.c_void_p),
                                 None if rl is None else rl.ctypes.data_as(ctypes.c_void_p),
                                 int(sync_override), _dev(workspace, "workspace"), ws_bytes, _stream(stream)))


FEDATTN_STATIC_SCRATCH_BYTES = 16 << 20


def fedattn_decode_static(params: fedattn_params, block_idx: int, q: torch.Tensor, k_cache: torch.Tensor,
                          v_cache: torch.Tensor, out: torch.Tensor, seg_offsets, seg_lens, remote_lens=None,
                          sync_override: int = -1, stream=None) -> None:
    """fedattn_decode without a workspace (the library's built-in scratch array; allocates nothing)."""
    seg = _host_i32(seg_offsets, "seg_offsets")
    lens = _host_i32(seg_lens, "seg_lens")
    if seg.shape[0] != params.n_participants + 1 or lens.shape[0] != params.n_participants:
        raise ValueError("seg_offsets / seg_lens have the wrong length")
    rl = None
    if remote_lens is not None:
        rl = _host_i32(remote_lens, "remote_lens")
        if rl.shape[0] != params.n_participants:
            raise ValueError("remote_lens has the wrong length")
    _check(load().fedattn_decode_static(ctypes.byref(params), int(block_idx), _dev(q, "q"), _dev(k_cache, "k_cache"),
                                        _dev(v_cache, "v_cache"), _dev(out, "out"),
                                        seg.ctypes.data_as(ctypes.c_void_p), lens.ctypes.data_as(ctypes.c_void_p),
                                        None if rl is None else rl.ctypes.data_as(ctypes.c_void_p),
                                        int(sync_override), _stream(stream)))


def fedattn_decode_blocks(params: fedattn_params, block_idx0: int, n_blocks: int, q: torch.Tensor,
                          k_cache: torch.Tensor, v_cache: torch.Tensor, out: torch.Tensor, q_block_stride: int,
                          cache_block_stride: int, seg_offsets, seg_lens, remote_lens=None, sync_override: int = -1,
                          workspace: Optional[torch.Tensor] = None, stream=None, fused: bool = False) -> None:
    """fused=True calls fedattn_decode_blocks_fused (blocks of one kind share launches)."""
    seg = _host_i32(seg_offsets, "seg_offsets")
    lens = _host_i32(seg_lens, "seg_lens")
    if seg.shape[0] != params.n_participants + 1 or lens.shape[0] != params.n_participants:
        raise ValueError("seg_offsets / seg_lens have the wrong length")
    rl = None
    if remote_lens is not None:
        rl = _host_i32(remote_lens, "remote_lens")
        if rl.shape[0] != params.n_participants:
            raise ValueError("remote_lens has the wrong length")
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    fn = load().fedattn_decode_blocks_fused if fused else load().fedattn_decode_blocks
    _check(fn(ctypes.byref(params), int(block_idx0), int(n_blocks), _dev(q, "q"),
              _dev(k_cache, "k_cache"), _dev(v_cache, "v_cache"), _dev(out, "out"),
              int(q_block_stride), int(cache_block_stride),
              seg.ctypes.data_as(ctypes.c_void_p), lens.ctypes.data_as(ctypes.c_void_p),
              None if rl is None else rl.ctypes.data_as(ctypes.c_void_p),
              int(sync_override), _dev(workspace, "workspace"), ws_bytes, _stream(stream)))


def fedattn_decode_blocks_fused(*args, **kwargs) -> None:
    """Same arguments as fedattn_decode_blocks."""
    fedattn_decode_blocks(*args, fused=True, **kwargs)


def fedattn_aggregate_kv(params: fedattn_params, k_local: Sequence[Optional[torch.Tensor]],
                         v_local: Sequence[Optional[torch.Tensor]], seg_offsets, k_global: torch.Tensor,
                         v_global: torch.Tensor, stream=None) -> None:
    seg = _host_i32(seg_offsets, "seg_offsets")
    n = params.n_participants
    if seg.shape[0] != n + 1 or len(k_local) != n or len(v_local) != n:
        raise ValueError("k_local / v_local / seg_offsets have the wrong length")
    kp, vp = _local_ptrs(k_local, n, "k_local"), _local_ptrs(v_local, n, "v_local")
    _check(load().fedattn_aggregate_kv(ctypes.byref(params), kp, vp, seg.ctypes.data_as(ctypes.c_void_p),
                                       _dev(k_global, "k_global"), _dev(v_global, "v_global"), _stream(stream)))


def fedattn_rmsnorm(x: torch.Tensor, out: torch.Tensor, eps: float = 1e-6, stream=None) -> None:
    """x fp32 [rows, d_model] -> out bf16 [rows, d_model]."""
    if x.dtype != torch.float32 or out.dtype != torch.bfloat16 or x.shape != out.shape or x.dim() != 2:
        raise TypeError("rmsnorm: x fp32 [rows, d_model], out bf16 of the same shape")
    _check(load().fedattn_rmsnorm(_dev(x, "x"), _dev(out, "out"), x.shape[0], x.shape[1], float(eps), _stream(stream)))


def fedattn_rope_split_qkv(qkv: torch.Tensor, pos: Optional[torch.Tensor], q: torch.Tensor, k: torch.Tensor,
                           v: torch.Tensor, theta: float = 10000.0, stream=None) -> None:
    """qkv bf16 [T, (Hq + 2 Hkv) D] -> q [T,Hq,D], k,v [T,Hkv,D] (bf16), q and k rotated; pos int32 [T] or None."""
    T, Hq, D = q.shape
    Hkv = k.shape[1]
    if qkv.shape != (T, (Hq + 2 * Hkv) * D) or k.shape != (T, Hkv, D) or v.shape != (T, Hkv, D):
        raise ValueError("rope: shapes of qkv, q, k, v do not fit together")
    if any(t.dtype != torch.bfloat16 for t in (qkv, q, k, v)):
        raise TypeError("rope: qkv, q, k, v must be bf16")
    if pos is not None and (pos.dtype != torch.int32 or pos.shape != (T,)):
        raise TypeError("rope: pos must be int32 [tokens]")
    _check(load().fedattn_rope_split_qkv(_dev(qkv, "qkv"), _dev(pos, "pos"), _dev(q, "q"), _dev(k, "k"), _dev(v, "v"),
                                         T, Hq, Hkv, D, float(theta), _stream(stream)))


def fedattn_swiglu(gate_up: torch.Tensor, out: torch.Tensor, stream=None) -> None:
    """gate_up bf16 [rows, 2 F] -> out bf16 [rows, F]."""
    if gate_up.dim() != 2 or out.shape != (gate_up.shape[0], gate_up.shape[1] // 2) or gate_up.shape[1] % 2:
        raise ValueError("swiglu: gate_up [rows, 2 F], out [rows, F]")
    if gate_up.dtype != torch.bfloat16 or out.dtype != torch.bfloat16:
        raise TypeError("swiglu: bf16 tensors")
    _check(load().fedattn_swiglu(_dev(gate_up, "gate_up"), _dev(out, "out"), out.shape[0], out.shape[1], _stream(stream)))


def fedattn_residual_add(x: torch.Tensor, y: torch.Tensor, stream=None) -> None:
    """x fp32 += y bf16, same shape."""
    if x.dtype != torch.float32 or y.dtype != torch.bfloat16 or x.shape != y.shape:
        raise TypeError("residual_add: x fp32, y bf16, same shape")
    _check(load().fedattn_residual_add(_dev(x, "x"), _dev(y, "y"), x.numel(), _stream(stream)))


def fedattn_residual_add_rmsnorm(x: torch.Tensor, y: torch.Tensor, out: torch.Tensor, eps: float = 1e-6, stream=None) -> None:
    """x fp32 += y bf16, then out bf16 = rmsnorm(x), one pass; all [rows, d_model]."""
    if x.dtype != torch.float32 or y.dtype != torch.bfloat16 or out.dtype != torch.bfloat16 or x.dim() != 2 \
            or x.shape != y.shape or x.shape != out.shape:
        raise TypeError("residual_add_rmsnorm: x fp32, y and out bf16, all [rows, d_model]")
    _check(load().fedattn_residual_add_rmsnorm(_dev(x, "x"), _dev(y, "y"), _dev(out, "out"), x.shape[0], x.shape[1],
                                               float(eps), _stream(stream)))


def fedattn_probe_stream(src: torch.Tensor, pattern: int, sink: torch.Tensor, stream=None) -> int:
    """One streaming-read kernel over `src` (pattern 0 contiguous, 1 the decode cache layout); returns the bytes read."""
    n = load().fedattn_probe_stream(_dev(src, "src"), src.numel() * src.element_size(), int(pattern), _dev(sink, "sink"),
                                    _stream(stream))
    if n < 0:
        raise FedAttnError(FEDATTN_EINVAL, load().fedattn_last_error().decode())
    return int(n)


def fedattn_probe_mfma(sink: torch.Tensor, iters: int, stream=None) -> int:
    """One MFMA-only kernel; returns the FLOPs it performs."""
    n = load().fedattn_probe_mfma(_dev(sink, "sink"), int(iters), _stream(stream))
    if n < 0:
        raise FedAttnError(FEDATTN_EINVAL, load().fedattn_last_error().decode())
    return int(n)
