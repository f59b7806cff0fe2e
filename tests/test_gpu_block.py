"""The decoder block around the attention (end-to-end configuration) on the GPU against the
fp64 block oracle: the four element-wise kernels one by one, then whole blocks."""
import numpy as np
import pytest
import torch

import fedattn_inputs as fi
import paper_2511_02647_amd as fa
from paper_2511_02647_amd.block import BlockBuffers, BlockWeights, block_forward
import oracle
from oracle import block as ob
from gpu_util import check, dev, host, say

pytestmark = pytest.mark.gpu
BF16 = torch.bfloat16

ULP = 2.0 ** -8      # spacing of bf16 relative to the value (one unit in the last place, upper bound)


def _bf16_close(got, ref_unrounded, what, slack=1.0):
    """A bf16 result computed in fp32 from exactly known inputs: within one bf16 step of the
    unrounded fp64 value (half a step of rounding + a flip when fp32 arithmetic lands on the
    other side of a rounding boundary)."""
    err = np.abs(got - ref_unrounded)
    tol = slack * ULP * np.abs(ref_unrounded) + 1e-6
    worst = float((err / tol).max())
    print("[parity] %-60s max err / (one bf16 step) = %.3f" % (what, worst), flush=True)
    assert worst <= 1.0, what


def test_rmsnorm_kernel():
    g = np.random.default_rng(1)
    for rows, d in ((37, 2048), (5, 96), (1, 4), (6, 4096), (3, 4100), (2, 8192)):   # in registers up to 4096, two passes beyond
        x = (g.standard_normal((rows, d)) * 3).astype(np.float32)
        tx = torch.from_numpy(x).cuda()
        out = torch.full((rows, d), float("nan"), dtype=BF16, device="cuda")
        say("rmsnorm %dx%d" % (rows, d))
        fa.fedattn_rmsnorm(tx, out)
        torch.cuda.synchronize()
        _bf16_close(host(out), ob.rmsnorm(x), "rmsnorm %dx%d" % (rows, d))


def test_rope_split_kernel():
    g = np.random.default_rng(2)
    for T, Hq, Hkv, D in ((50, 8, 4, 128), (7, 3, 1, 64), (3, 2, 2, 8)):
        qkv = fi.round_to_bf16(g.standard_normal((T, (Hq + 2 * Hkv) * D)).astype(np.float32))
        tq = dev(qkv, BF16)
        q = torch.full((T, Hq, D), float("nan"), dtype=BF16, device="cuda")
        k = torch.full((T, Hkv, D), float("nan"), dtype=BF16, device="cuda")
        v = torch.full((T, Hkv, D), float("nan"), dtype=BF16, device="cuda")
        for pos in (None, g.integers(0, 70000, size=T).astype(np.int32)):
            say("rope T=%d Hq=%d Hkv=%d D=%d pos=%s" % (T, Hq, Hkv, D, "given" if pos is not None else "index"))
            fa.fedattn_rope_split_qkv(tq, None if pos is None else torch.from_numpy(pos).cuda(), q, k, v)
            torch.cuda.synchronize()
            p = np.arange(T) if pos is None else pos
            x64 = qkv.astype(np.float64)
            rq = ob.rope(x64[:, :Hq * D].reshape(T, Hq, D), p)
            rk = ob.rope(x64[:, Hq * D:(Hq + Hkv) * D].reshape(T, Hkv, D), p)
            # the rotation mixes two inputs: allow the step of the larger one
            for got, ref, src, nm in ((host(q), rq, x64[:, :Hq * D].reshape(T, Hq, D), "q"),
                                      (host(k), rk, x64[:, Hq * D:(Hq + Hkv) * D].reshape(T, Hkv, D), "k")):
                mag = np.sqrt(src[..., :D // 2] ** 2 + src[..., D // 2:] ** 2)
                mag = np.concatenate([mag, mag], axis=-1)
                err = np.abs(got - ref)
                worst = float((err / (ULP * mag + 1e-6)).max())
                print("[parity] rope %s D=%d: max err / (one bf16 step of the pair) = %.3f" % (nm, D, worst), flush=True)
                assert worst <= 1.0
            assert np.array_equal(host(v), x64[:, (Hq + Hkv) * D:].reshape(T, Hkv, D)), "v must be copied bit for bit"


def test_swiglu_and_residual_kernels():
    g = np.random.default_rng(3)
    rows, F = 29, 5632
    gu = fi.round_to_bf16((g.standard_normal((rows, 2 * F)) * 3).astype(np.float32))
    out = torch.full((rows, F), float("nan"), dtype=BF16, device="cuda")
    say("swiglu")
    fa.fedattn_swiglu(dev(gu, BF16), out)
    torch.cuda.synchronize()
    ref = ob.swiglu(gu[:, :F].astype(np.float64), gu[:, F:].astype(np.float64))
    _bf16_close(host(out), ref, "swiglu %dx%d" % (rows, F))
    x = g.standard_normal((rows, 2048)).astype(np.float32)
    y = fi.round_to_bf16(g.standard_normal((rows, 2048)).astype(np.float32))
    tx = torch.from_numpy(x).cuda()
    say("residual add")
    fa.fedattn_residual_add(tx, dev(y, BF16))
    torch.cuda.synchronize()
    assert np.array_equal(tx.cpu().numpy(), x + y), "fp32 residual add must be exactly rounded"


def test_residual_add_fused_into_rmsnorm_equals_the_two_kernels():
    g = np.random.default_rng(4)
    for rows, d in ((37, 2048), (5, 96), (6, 4096), (3, 4100), (2, 8192)):     # held in registers / two passes
        x = (g.standard_normal((rows, d)) * 3).astype(np.float32)
        y = fi.round_to_bf16(g.standard_normal((rows, d)).astype(np.float32))
        ty = dev(y, BF16)
        x_two, x_one = torch.from_numpy(x).cuda(), torch.from_numpy(x).cuda()
        h_two = torch.full((rows, d), float("nan"), dtype=BF16, device="cuda")
        h_one = torch.full_like(h_two, float("nan"))
        say("residual add + rmsnorm %dx%d" % (rows, d))
        fa.fedattn_residual_add(x_two, ty)
        fa.fedattn_rmsnorm(x_two, h_two)
        fa.fedattn_residual_add_rmsnorm(x_one, ty, h_one)
        torch.cuda.synchronize()
        assert torch.equal(x_one, x_two) and torch.equal(h_one, h_two), "fused pass differs from the two kernels"
        assert np.array_equal(x_one.cpu().numpy(), x + y)
        _bf16_close(host(h_one), ob.rmsnorm((x + y).astype(np.float64)), "residual add + rmsnorm %dx%d" % (rows, d))


def test_block_stack_with_deferred_updates_equals_block_by_block():
    """A stack whose feed-forward updates are handed on to the next block's first kernel gives the
    residual stream of the stack run block by block, bit for bit."""
    w = fi.workload("cfg5_sparse_sync")
    seg = np.array([0, 100, 228, 420], dtype=np.int32)
    d_model, hidden, T, n_blocks = 512, 704, 420, 3
    p = fa.make_params(3, w.n_q_heads, w.n_kv_heads, w.head_dim, 2, BF16)
    buf = BlockBuffers(p, T, d_model, hidden)
    x0 = torch.from_numpy(fi.hidden_input(w, d_model, total=T).astype(np.float32)).cuda()
    wts = [BlockWeights(*(dev(fi.block_weights(w, b, d_model, hidden)[k], BF16) for k in ("qkv", "o", "gate_up", "down")))
           for b in range(n_blocks)]
    xa = x0.clone()
    for b in range(n_blocks):
        block_forward(p, b, xa, wts[b], seg, buf)
    xb, pending = x0.clone(), None
    say("block stack, updates deferred into the next normalisation")
    for b in range(n_blocks):
        pending = block_forward(p, b, xb, wts[b], seg, buf, pending=pending, defer_update=True)["pending"]
    fa.fedattn_residual_add(xb, pending)
    torch.cuda.synchronize()
    assert torch.equal(xa, xb)


def test_block_op_errors_are_return_codes():
    x = torch.zeros(4, 6, device="cuda")
    with pytest.raises(fa.FedAttnError) as e:
        fa.fedattn_rmsnorm(x, torch.zeros(4, 6, dtype=BF16, device="cuda"))     # d_model not a multiple of 4
    assert e.value.status == fa.FEDATTN_EINVAL


MEAN_FACTOR, MAX_FACTOR = 1.5, 2.0


def _drift_check(got, ref_rounding, ref_exact, what):
    """A block output (or the output of a stack of blocks) against the oracle that rounds to bf16
    wherever the device stores bf16, with the oracle's own rounding drift as the yardstick: the
    distance between that oracle and the one that never rounds is what bf16 storage by itself does
    to the result.  The device differs from the rounding oracle by roundings that fall the other
    way (its sums are fp32-accumulated and its attention carries bf16 weights), i.e. by rounding
    noise of the same origin and size.  Bars: mean-abs <= 1.5 x the drift's (two independent noises
    of equal size differ by sqrt 2 of one; 1.5 leaves 6 % of margin), max-abs <= 2 x the drift's
    (a rounding that falls the other way is a whole bf16 spacing where rounding itself moves a
    value by at most half of one)."""
    err = np.abs(got - ref_rounding)
    drift = np.abs(ref_rounding - ref_exact)
    print("[parity] %-44s device vs rounding oracle max-abs %.3e mean-abs %.3e | rounding vs exact oracle max-abs %.3e "
          "mean-abs %.3e" % (what, err.max(), err.mean(), drift.max(), drift.mean()), flush=True)
    assert err.mean() <= MEAN_FACTOR * drift.mean() and err.max() <= MAX_FACTOR * drift.max(), what


def _run_blocks(w, seg, d_model, hidden, n_blocks, total, keep_for_block):
    """GPU blocks 0..n_blocks-1 on x0, with the oracle teacher-forced block by block."""
    N = len(seg) - 1
    p = fa.make_params(N, w.n_q_heads, w.n_kv_heads, w.head_dim, w.sync_interval, BF16)
    buf = BlockBuffers(p, total, d_model, hidden, chunk_tokens=w.chunk_tokens)
    x0 = fi.hidden_input(w, d_model, total=total)
    x = torch.from_numpy(x0.astype(np.float32)).cuda()
    x_rounding = x0.astype(np.float64)     # the oracle on its own, rounding where the device stores bf16
    x_exact = x0.astype(np.float64)        # the oracle on its own, never rounding
    kw = dict(n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim)
    for b in range(n_blocks):
        wts = fi.block_weights(w, b, d_model, hidden)
        bw = BlockWeights(*(dev(wts[k], BF16) for k in ("qkv", "o", "gate_up", "down")))
        sync = oracle.is_sync_block(w.sync_interval, b)
        flags = keep_for_block(b) if sync else None
        kt = None if flags is None else oracle.expand_keep_chunks(flags, seg, w.chunk_tokens)
        x_in = x.cpu().numpy().astype(np.float64)
        say("block %d (%s%s), %d tokens, d_model %d" % (b, "sync" if sync else "local", ", sparse" if kt is not None else "", total, d_model))
        res = block_forward(p, b, x, bw, seg, buf, keep_chunks=None if flags is None else torch.from_numpy(flags).cuda(),
                            chunk_tokens=w.chunk_tokens if flags is not None else 0)
        torch.cuda.synchronize()
        # gate (i), teacher-forced: the attention of the GPU's own q, k, v, to the attention tolerance
        ref_attn = oracle.attend_block(host(res["q"]), host(res["k"]), host(res["v"]), seg, is_sync=sync, keep_tok=kt)
        check(host(res["attn"]), ref_attn, BF16, "block %d attention on the device's q, k, v" % b)
        # the whole block from the GPU's block input, oracle rounding at the bf16 interfaces
        ref = ob.block_forward(x_in, wts, seg, is_sync=sync, keep_tok=kt, round_fn=fi.round_to_bf16, **kw)
        exact = ob.block_forward(x_in, wts, seg, is_sync=sync, keep_tok=kt, **kw)
        _drift_check(x.cpu().numpy().astype(np.float64), ref["out"], exact["out"], "block %d output, same input:" % b)
        x_rounding = ob.block_forward(x_rounding, wts, seg, is_sync=sync, keep_tok=kt, round_fn=fi.round_to_bf16, **kw)["out"]
        x_exact = ob.block_forward(x_exact, wts, seg, is_sync=sync, keep_tok=kt, **kw)["out"]
    # gate (ii), end to end: both oracles carried through all blocks on their own
    _drift_check(x.cpu().numpy().astype(np.float64), x_rounding, x_exact, "%d blocks end to end:" % n_blocks)


def test_blocks_small_model():
    w = fi.workload("cfg5_sparse_sync")          # 16/4 heads of 128, H = 2, 64-token keep chunks
    seg = np.array([0, 100, 228, 420], dtype=np.int32)
    g = np.random.default_rng(8)
    nch = int(fi.chunk_counts(np.diff(seg), w.chunk_tokens).sum())
    _run_blocks(w, seg, d_model=512, hidden=704, n_blocks=4, total=420,
                keep_for_block=lambda b: (g.random(nch) < 0.5).astype(np.uint8))


def test_blocks_end_to_end_configuration_scaled_down():
    """The end-to-end configuration (d_model 2048, feed-forward 5632, 16/4 heads, H = 2, a quarter
    of the 64-token chunks exchanged) at 16 x 256 tokens, two blocks (one local, one sparse sync)."""
    w = fi.workload("cfg5_sparse_sync")
    seg = (np.arange(17) * 256).astype(np.int32)
    import dataclasses
    small = dataclasses.replace(w, seg_lens=(256,) * 16)
    _run_blocks(w, seg, d_model=2048, hidden=5632, n_blocks=2, total=4096,
                keep_for_block=lambda b: fi.keep_chunks(small, b // w.sync_interval))


@pytest.mark.timeout(900)
def test_cfg5_full_size_blocks_teacher_forced_on_sampled_rows():
    """The end-to-end configuration at its full size (16 x 4096 tokens, d_model 2048, feed-forward
    5632, 16/4 heads, H = 2, a quarter of the 64-token chunks exchanged): the first local block and
    the first sparse sync block, each checked against the oracle from the device's own block input.
    The attention is compared on every tile-boundary row and 4096 random (row, head) pairs of the
    device's q, k, v; the block output on sampled token rows (all heads), for which the oracle
    computes keys and values of all 65 536 tokens and the rest of the block for those rows only."""
    w = fi.workload("cfg5_sparse_sync")
    seg, T, d_model, hidden = w.seg_offsets, w.total_tokens, 2048, 5632
    p = fa.make_params(w.n_participants, w.n_q_heads, w.n_kv_heads, w.head_dim, w.sync_interval, BF16)
    buf = BlockBuffers(p, T, d_model, hidden, chunk_tokens=w.chunk_tokens)
    x = torch.from_numpy(fi.hidden_input(w, d_model).astype(np.float32)).cuda()
    kw = dict(n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim)
    g = fi.stream(fi.DEFAULT_SEED, 97, 0, 5)
    for b in (0, 1):
        wts = fi.block_weights(w, b, d_model, hidden)
        bw = BlockWeights(*(dev(wts[k], BF16) for k in ("qkv", "o", "gate_up", "down")))
        sync = oracle.is_sync_block(w.sync_interval, b)
        flags = fi.keep_chunks(w, b // w.sync_interval) if sync else None
        kt = None if flags is None else oracle.expand_keep_chunks(flags, seg, w.chunk_tokens)
        x_in = x.cpu().numpy()
        say("cfg5 full size, block %d (%s)" % (b, "sparse sync" if sync else "local"))
        res = block_forward(p, b, x, bw, seg, buf, keep_chunks=None if flags is None else torch.from_numpy(flags).cuda(),
                            chunk_tokens=w.chunk_tokens if flags is not None else 0)
        torch.cuda.synchronize()
        assert bool(torch.isfinite(x).all())
        dq, dk, dv = (res[n].float().cpu().numpy() for n in ("q", "k", "v"))
        rows, heads = fi.sample_rows(seg, w.n_q_heads, 4096, fi.DEFAULT_SEED, salt=500 + b)
        ref_attn = oracle.attend_rows(dq, dk, dv, seg, rows, heads, is_sync=sync, keep_tok=kt)
        check(host(res["attn"])[rows, heads], ref_attn, BF16, "cfg5 full size block %d attention (%d rows)" % (b, len(rows)))
        del dq, dk, dv
        # block output on token rows: segment ends, a tile boundary of every participant, random rows
        pick = [int(seg[n]) for n in range(16)] + [int(seg[n + 1]) - 1 for n in range(16)]
        pick += [int(seg[n]) + 64 * int(g.integers(1, 64)) - int(n % 2) for n in range(16)]
        pick += [int(r) for r in g.integers(0, T, size=48)]
        pick = np.array(sorted(set(pick)), dtype=np.int64)
        ref = ob.block_forward_rows(x_in, wts, seg, pick, is_sync=sync, keep_tok=kt, round_fn=fi.round_to_bf16, **kw)
        exact = ob.block_forward_rows(x_in, wts, seg, pick, is_sync=sync, keep_tok=kt, **kw)
        _drift_check(x[torch.from_numpy(pick).cuda()].cpu().numpy().astype(np.float64), ref["out"], exact["out"],
                     "cfg5 full size block %d output (%d rows):" % (b, len(pick)))
        check(host(res["attn"])[pick], ref["attn"], BF16, "cfg5 full size block %d attention from the block input" % b)
