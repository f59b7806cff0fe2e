"""Host-side checks that need no GPU: the shared library loads, exports every
symbol the header declares, and validation failures come back as return codes."""
import ctypes
import os
import re

import pytest
import torch

import paper_2511_02647_amd as fa
from paper_2511_02647_amd import build as fabuild

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    fabuild.build(force=False)
    return fa.load()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "fedattn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fedattn_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(lib):
    names = declared_symbols()
    assert set(names) == set(fa.EXPORTS)
    for name in names:
        assert getattr(lib, name) is not None


def test_sync_rule_host_side(lib):
    assert [fa.fedattn_is_sync_block(4, b) for b in range(8)] == [False] * 3 + [True] + [False] * 3 + [True]
    assert [fa.fedattn_is_sync_block(1, b) for b in range(3)] == [True] * 3
    assert not any(fa.fedattn_is_sync_block(0, b) for b in range(8))
    assert [fa.fedattn_is_sync_block(32, b) for b in range(32)].count(True) == 1


def test_params_struct_matches_header(lib):
    assert ctypes.sizeof(fa.fedattn_params) == 32


def test_validation_returns_codes_without_touching_the_gpu(lib):
    ok = fa.make_params(2, 4, 2, 128, 2, torch.bfloat16)
    seg = (ctypes.c_int32 * 3)(0, 4, 8)
    null = ctypes.c_void_p(None)
    call = lambda p, s=seg: lib.fedattn_prefill(ctypes.byref(p), 0, null, null, null, null, s, null, 0, -1, null, 0, null)
    assert call(ok) == fa.FEDATTN_EINVAL and b"NULL" in lib.fedattn_last_error()
    bad = fa.make_params(2, 4, 3, 128, 2, torch.bfloat16)
    assert call(bad) == fa.FEDATTN_EINVAL and b"multiple" in lib.fedattn_last_error()
    bad = fa.make_params(2, 4, 2, 100, 2, torch.bfloat16)
    assert call(bad) == fa.FEDATTN_EINVAL
    bad = fa.make_params(1000, 4, 2, 128, 2, torch.bfloat16)
    assert call(bad) == fa.FEDATTN_EINVAL
    assert call(ok, (ctypes.c_int32 * 3)(1, 4, 8)) == fa.FEDATTN_EINVAL
    assert call(ok, (ctypes.c_int32 * 3)(0, 9, 8)) == fa.FEDATTN_EINVAL
    # an empty problem is a no-op, not an error
    assert call(ok, (ctypes.c_int32 * 3)(0, 0, 0)) == fa.FEDATTN_OK
    assert fa.fedattn_workspace_bytes(ok, fa.FEDATTN_OP_PREFILL, 4096, 0) == 0
    assert fa.fedattn_workspace_bytes(ok, fa.FEDATTN_OP_PREFILL, 4096, 64) > 0
    assert fa.fedattn_workspace_bytes(ok, fa.FEDATTN_OP_DECODE, 4096) > 0


def test_decode_validation_returns_codes_without_touching_the_gpu(lib):
    ok = fa.make_params(2, 4, 2, 128, 2, torch.bfloat16)
    seg = (ctypes.c_int32 * 3)(0, 64, 128)
    lens = (ctypes.c_int32 * 2)(64, 10)
    null = ctypes.c_void_p(None)
    fake = ctypes.c_void_p(0x10000)      # never dereferenced: every call below fails validation first
    for fn in (lib.fedattn_decode_blocks, lib.fedattn_decode_blocks_fused):
        assert fn(ctypes.byref(ok), 0, 2, fake, fake, fake, fake, 1024, 32768, seg, null, null, -1, null, 0, null) == fa.FEDATTN_EINVAL
        assert fn(ctypes.byref(ok), 0, 0, null, null, null, null, 0, 0, seg, lens, null, -1, null, 0, null) == fa.FEDATTN_OK
        bad = (ctypes.c_int32 * 2)(65, 10)   # more valid rows than the segment's capacity
        assert fn(ctypes.byref(ok), 0, 2, fake, fake, fake, fake, 1024, 32768, seg, bad, null, -1, null, 0, null) == fa.FEDATTN_EINVAL
        assert fn(ctypes.byref(ok), 0, 2, fake, fake, fake, fake, 1024, 32768, seg, lens, null, 2, null, 0, null) == fa.FEDATTN_EINVAL
        assert fn(ctypes.byref(ok), 0, 2, fake, fake, fake, fake, 1023, 32768, seg, lens, null, -1, null, 0, null) == fa.FEDATTN_EINVAL
        assert fn(ctypes.byref(ok), 0, 2, fake, fake, fake, fake, 1024, 32768, seg, lens, null, -1, null, 0, null) == fa.FEDATTN_EWORKSPACE
    big = fa.fedattn_workspace_bytes(ok, fa.FEDATTN_OP_DECODE, 128)
    assert lib.fedattn_decode_blocks_fused(ctypes.byref(ok), 0, 70000, fake, fake, fake, fake, 1024, 32768, seg, lens, null,
                                           -1, fake, big, null) == fa.FEDATTN_EINVAL
    assert b"65535" in lib.fedattn_last_error()
