"""ctypes front end of the row-by-row fp64 C oracle (fedattn_oracle.c).

TEST INFRASTRUCTURE; never used by the GPU library.
"""
from __future__ import annotations

import ctypes
import math
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fedattn_oracle.c")
_LIB = os.path.join(_HERE, "libfedattn_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (OpenMP over independent rows)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        c_i32, c_i64, c_dbl, vp = ctypes.c_int32, ctypes.c_int64, ctypes.c_double, ctypes.c_void_p
        lib.fedattn_oracle_is_sync.argtypes = [c_i32, c_i32]
        lib.fedattn_oracle_is_sync.restype = ctypes.c_int
        lib.fedattn_oracle_threads.restype = ctypes.c_int
        lib.fedattn_oracle_attend_rows.argtypes = [vp, vp, vp, c_i32, c_i32, c_i32, c_i32, vp, c_i32,
                                                   c_dbl, c_i32, c_i32, vp, vp, vp, c_i64, vp, vp]
        lib.fedattn_oracle_attend_rows.restype = None
        lib.fedattn_oracle_decode.argtypes = [vp, vp, vp, c_i32, c_i32, c_i32, c_i32, vp, vp, vp,
                                              c_dbl, c_i32, vp]
        lib.fedattn_oracle_decode.restype = None
        _lib = lib
    return _lib


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def is_sync_block(H: int, block_idx: int) -> bool:
    """Algorithm 1: block m = Ht + h is the global-attention block iff h = H."""
    return bool(_load().fedattn_oracle_is_sync(int(H), int(block_idx)))


def n_threads() -> int:
    return int(_load().fedattn_oracle_threads())


def expand_keep_chunks(keep_chunks, seg_offsets, chunk_tokens: int) -> np.ndarray:
    """Token-level keep flags from per-chunk flags: chunk c of participant n
    covers tokens seg_off[n] + c*chunk_tokens ... (clipped to the segment)."""
    seg_offsets = np.asarray(seg_offsets)
    total = int(seg_offsets[-1])
    keep_tok = np.zeros(total, dtype=np.uint8)
    c = 0
    for n in range(len(seg_offsets) - 1):
        s, e = int(seg_offsets[n]), int(seg_offsets[n + 1])
        for t in range(s, e, chunk_tokens):
            keep_tok[t:min(t + chunk_tokens, e)] = keep_chunks[c]
            c += 1
    assert c == len(keep_chunks), "keep_chunks length does not match the chunk count"
    return keep_tok


def attend_rows(q, k, v, seg_offsets, rows, heads, *, is_sync: bool, causal: bool = True,
                scale: Optional[float] = None, keep_tok=None,
                return_prob: bool = False):
    """Outputs [n_rows, D] (float64) for the requested (row, head) pairs."""
    q, k, v = _f32(q), _f32(k), _f32(v)
    total, Hq, D = q.shape
    Hkv = k.shape[1]
    assert k.shape == (total, Hkv, D) and v.shape == (total, Hkv, D) and Hq % Hkv == 0
    seg = _i32(seg_offsets)
    assert seg[0] == 0 and seg[-1] == total and np.all(np.diff(seg) >= 0)
    rows, heads = _i32(rows), _i32(heads)
    assert rows.shape == heads.shape
    if rows.size:
        assert rows.min() >= 0 and rows.max() < total and heads.min() >= 0 and heads.max() < Hq
    kt = None
    if keep_tok is not None:
        kt = np.ascontiguousarray(keep_tok, dtype=np.uint8)
        assert kt.shape == (total,)
    sc = (1.0 / math.sqrt(D)) if scale is None else float(scale)
    out = np.zeros((rows.size, D), dtype=np.float64)
    prob = np.zeros((rows.size, total), dtype=np.float64) if return_prob else None
    _load().fedattn_oracle_attend_rows(_ptr(q), _ptr(k), _ptr(v), total, Hq, Hkv, D, _ptr(seg),
                                       len(seg) - 1, sc, int(bool(is_sync)), int(bool(causal)),
                                       _ptr(kt), _ptr(rows), _ptr(heads), rows.size,
                                       _ptr(out), _ptr(prob))
    return (out, prob) if return_prob else out


def attend_block(q, k, v, seg_offsets, *, is_sync: bool, causal: bool = True,
                 scale: Optional[float] = None, keep_tok=None) -> np.ndarray:
    """Full output [total, Hq, D] (float64) of one block."""
    total, Hq, D = np.shape(q)
    rows = np.repeat(np.arange(total, dtype=np.int32), Hq)
    heads = np.tile(np.arange(Hq, dtype=np.int32), total)
    out = attend_rows(q, k, v, seg_offsets, rows, heads, is_sync=is_sync, causal=causal,
                      scale=scale, keep_tok=keep_tok)
    return out.reshape(total, Hq, D)


def decode_step(q, k_cache, v_cache, seg_offsets, seg_lens, *, is_sync: bool,
                remote_lens=None, scale: Optional[float] = None) -> np.ndarray:
    """Output [N, Hq, D] (float64) of one decoding step of one block."""
    q, k_cache, v_cache = _f32(q), _f32(k_cache), _f32(v_cache)
    N, Hq, D = q.shape
    cap, Hkv, _ = k_cache.shape
    seg, lens = _i32(seg_offsets), _i32(seg_lens)
    assert len(seg) == N + 1 and seg[-1] == cap and len(lens) == N
    assert np.all(lens >= 0) and np.all(lens <= np.diff(seg))
    rl = None
    if remote_lens is not None:
        rl = _i32(remote_lens)
        assert len(rl) == N and np.all(rl >= 0) and np.all(rl <= np.diff(seg))
    sc = (1.0 / math.sqrt(D)) if scale is None else float(scale)
    out = np.zeros((N, Hq, D), dtype=np.float64)
    _load().fedattn_oracle_decode(_ptr(q), _ptr(k_cache), _ptr(v_cache), N, Hq, Hkv, D, _ptr(seg),
                                  _ptr(lens), _ptr(rl), sc, int(bool(is_sync)), _ptr(out))
    return out
