"""fedattn_decode_static (the decode entry point that allocates nothing and works in the
library's built-in scratch array) against fedattn_decode with a caller's workspace: two calls
in a row on one GPU, the second on a smaller problem, local and sync blocks.  Both entry
points run the same kernels, so the outputs must be bit-identical; the oracle bar is checked
as well."""
import gc

import numpy as np
import pytest
import torch

import fedattn_inputs as fi
import oracle
import paper_2511_02647_amd as fa
from gpu_util import check, dev, host, say

pytestmark = pytest.mark.gpu
BF16 = torch.bfloat16


def _case(seed, N, cap, lens, Hq, Hkv, D):
    g = np.random.default_rng(seed)
    mk = lambda *s: fi.round_to_bf16(g.standard_normal(s).astype(np.float32))
    seg = (np.arange(N + 1) * cap).astype(np.int32)
    return seg, np.asarray(lens, dtype=np.int32), mk(N, Hq, D), mk(N * cap, Hkv, D), mk(N * cap, Hkv, D)


def test_decode_static_matches_decode_with_a_workspace():
    Hq, Hkv, D = 8, 2, 128
    cases = [_case(901, 6, 1500, [1500, 1, 700, 1333, 64, 65], Hq, Hkv, D),   # several chunks per segment
             _case(902, 3, 200, [200, 77, 130], Hq, Hkv, D)]                  # smaller problem, same array
    for ci, (seg, lens, q, kc, vc) in enumerate(cases):
        N = len(lens)
        p = fa.make_params(N, Hq, Hkv, D, 2, BF16)
        tq, tk, tv = dev(q, BF16), dev(kc, BF16), dev(vc, BF16)
        ws = torch.empty(fa.fedattn_workspace_bytes(p, fa.FEDATTN_OP_DECODE, int(seg[-1])), dtype=torch.uint8, device="cuda")
        prompt = np.minimum(lens, 100).astype(np.int32)
        for block, rl in [(0, None), (1, None), (1, prompt)]:
            sync = oracle.is_sync_block(2, block)
            want = torch.full_like(tq, float("nan"))
            fa.fedattn_decode(p, block, tq, tk, tv, want, seg, lens, remote_lens=rl, workspace=ws)
            got = torch.full_like(tq, float("nan"))
            say("decode_static call %d block %d (%s) remote=%s" % (ci, block, "sync" if sync else "local", rl is not None))
            gc.collect()       # tensors of earlier tests must not be released while we watch the allocator
            before, reserved = torch.cuda.memory_allocated(), torch.cuda.memory_reserved()
            fa.fedattn_decode_static(p, block, tq, tk, tv, got, seg, lens, remote_lens=rl)
            torch.cuda.synchronize()
            assert torch.cuda.memory_allocated() <= before and torch.cuda.memory_reserved() == reserved
            assert torch.equal(got, want), "static-scratch decode differs from the workspace decode (call %d, block %d)" % (ci, block)
            ref = oracle.decode_step(q, kc, vc, seg, lens, is_sync=sync, remote_lens=rl)
            check(host(got), ref, BF16, "decode_static call %d block %d remote=%s" % (ci, block, rl is not None))


def test_decode_static_rejects_problems_beyond_its_array():
    N, Hq, Hkv, D = 128, 64, 8, 128
    p = fa.make_params(N, Hq, Hkv, D, 1, BF16)
    seg = (np.arange(N + 1) * 64).astype(np.int32)
    assert fa.fedattn_workspace_bytes(p, fa.FEDATTN_OP_DECODE, int(seg[-1])) > fa.FEDATTN_STATIC_SCRATCH_BYTES
    t = torch.zeros(N, Hq, D, dtype=BF16, device="cuda")
    kv = torch.zeros(N * 64, Hkv, D, dtype=BF16, device="cuda")
    with pytest.raises(fa.FedAttnError) as e:
        fa.fedattn_decode_static(p, 0, t, kv, kv, torch.empty_like(t), seg, np.full(N, 64, np.int32))
    assert e.value.status == fa.FEDATTN_EWORKSPACE and "scratch" in str(e.value)
    torch.cuda.synchronize()
