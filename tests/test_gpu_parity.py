"""GPU parity: the HIP path, called through the C ABI, against the fp64 CPU oracle
on the same seeded inputs.  Bar: max-abs 2e-2 and mean-abs 2e-3 for bf16 inputs,
max-abs 1e-5 for fp32 inputs."""
import numpy as np
import pytest
import torch

import fedattn_inputs as fi
import oracle
import paper_2511_02647_amd as fa
from gpu_util import check, decode, dev, host, prefill, say

pytestmark = pytest.mark.gpu
BF16, F32 = torch.bfloat16, torch.float32


def rand_block(seed, total, Hq, Hkv, D, bf16=True, sigma=1.0):
    g = np.random.default_rng(seed)
    mk = lambda *s: (sigma * g.standard_normal(s)).astype(np.float32)
    q, k, v = mk(total, Hq, D), mk(total, Hkv, D), mk(total, Hkv, D)
    if bf16:
        q, k, v = fi.round_to_bf16(q), fi.round_to_bf16(k), fi.round_to_bf16(v)
    return q, k, v


# ----------------------------------------------------------------- config 1
def test_cfg1_tiny_fp32_all_blocks():
    w = fi.workload("cfg1_tiny")
    seg = w.seg_offsets
    blocks = [fi.prefill_block(w, b) for b in range(w.n_blocks)]
    ref = oracle.schedule.run_stack(*zip(*blocks), seg, w.sync_interval)
    for b, (q, k, v) in enumerate(blocks):
        say("cfg1 block %d" % b)
        got = prefill(q, k, v, seg, Hq=2, Hkv=2, D=64, H=w.sync_interval, block=b, dtype=F32)
        check(got, ref[b], F32, "cfg1_tiny fp32 block %d (%s)" % (b, "sync" if b % 2 else "local"))


# ------------------------------------------------- general (ALU) kernel shapes
@pytest.mark.parametrize("dtype,D,Hq,Hkv", [(F32, 64, 4, 2), (F32, 40, 3, 3), (BF16, 32, 4, 1), (F32, 256, 2, 1)])
@pytest.mark.parametrize("causal", [True, False])
def test_general_kernel_shapes(dtype, D, Hq, Hkv, causal):
    seg = np.array([0, 70, 70, 333, 391], dtype=np.int32)
    q, k, v = rand_block(5, 391, Hq, Hkv, D, bf16=dtype == BF16)
    for sync in (0, 1):
        say("general kernel dtype=%s D=%d Hq=%d Hkv=%d causal=%d sync=%d" % (dtype, D, Hq, Hkv, causal, sync))
        got = prefill(q, k, v, seg, Hq=Hq, Hkv=Hkv, D=D, H=0, block=0, dtype=dtype, causal=causal,
                      sync_override=sync)
        ref = oracle.attend_block(q, k, v, seg, is_sync=bool(sync), causal=causal)
        check(got, ref, dtype, "general D=%d %s causal=%d sync=%d" % (D, dtype, causal, sync))


def test_general_kernel_token_granular_keep_list():
    seg = np.array([0, 50, 131, 200], dtype=np.int32)
    q, k, v = rand_block(6, 200, 4, 2, 64, bf16=False)
    flags = (np.random.default_rng(3).random(int(fi.chunk_counts(np.diff(seg), 8).sum())) < 0.5).astype(np.uint8)
    kt = oracle.expand_keep_chunks(flags, seg, 8)
    for causal in (True, False):
        say("general kernel keep-list chunk=8 causal=%d" % causal)
        got = prefill(q, k, v, seg, Hq=4, Hkv=2, D=64, H=1, block=0, dtype=F32, causal=causal,
                      keep_chunks=flags, chunk_tokens=8)
        ref = oracle.attend_block(q, k, v, seg, is_sync=True, causal=causal, keep_tok=kt)
        check(got, ref, F32, "general keep-list chunk=8 causal=%d" % causal)


# ------------------------------------------------------ MFMA kernel, small, full
@pytest.mark.parametrize("Hq,Hkv,D", [(8, 2, 128), (2, 2, 128), (4, 2, 128), (8, 1, 128), (8, 2, 64), (3, 1, 64)])
def test_mfma_prefill_small_full(Hq, Hkv, D):
    seg = np.array([0, 100, 100, 137, 402, 403], dtype=np.int32)   # ragged, empty and 1-token segments
    q, k, v = rand_block(7, 403, Hq, Hkv, D)
    for causal in (True, False):
        for sync in (0, 1):
            say("mfma small Hq=%d Hkv=%d D=%d causal=%d sync=%d" % (Hq, Hkv, D, causal, sync))
            got = prefill(q, k, v, seg, Hq=Hq, Hkv=Hkv, D=D, H=0, block=0, dtype=BF16, causal=causal,
                          sync_override=sync)
            ref = oracle.attend_block(q, k, v, seg, is_sync=bool(sync), causal=causal)
            check(got, ref, BF16, "mfma Hq=%d Hkv=%d D=%d causal=%d sync=%d" % (Hq, Hkv, D, causal, sync))


@pytest.mark.parametrize("N", [65, 100, 128])
def test_many_participants(N):
    """More than 64 participants (up to the maximum of 128): the kernels look their segment up in
    tables that span two registers per lane."""
    g = np.random.default_rng(100 + N)
    lens = g.integers(0, 40, size=N)
    lens[g.integers(0, N, size=5)] = 0            # some empty participants
    lens[N - 1] = 70                              # the last one spans two KV tiles
    seg = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    total = int(seg[-1])
    Hq, Hkv, D = 8, 2, 128
    q, k, v = rand_block(50 + N, total, Hq, Hkv, D)
    for sync in (0, 1):
        say("prefill N=%d sync=%d" % (N, sync))
        got = prefill(q, k, v, seg, Hq=Hq, Hkv=Hkv, D=D, H=0, block=0, dtype=BF16, sync_override=sync)
        check(got, oracle.attend_block(q, k, v, seg, is_sync=bool(sync)), BF16, "prefill N=%d sync=%d" % (N, sync))
    # sparse exchange, token-granular (packed rows) and whole participants dropped
    flags = (g.random(total) < 0.5).astype(np.uint8)
    flags[seg[N // 2]:seg[N // 2 + 10]] = 0
    say("prefill N=%d sparse" % N)
    got = prefill(q, k, v, seg, Hq=Hq, Hkv=Hkv, D=D, H=1, block=0, dtype=BF16, keep_chunks=flags, chunk_tokens=1)
    check(got, oracle.attend_block(q, k, v, seg, is_sync=True, keep_tok=flags), BF16, "prefill N=%d sparse" % N)
    # decode over caches of the same layout (capacity = the segments, every row valid but a few)
    cache_lens = np.maximum(lens - g.integers(0, 3, size=N), 0).astype(np.int32)
    cache_lens[N - 1] = 70
    qd, _, _ = rand_block(60 + N, N, Hq, Hkv, D)
    for sync in (0, 1):
        say("decode N=%d sync=%d" % (N, sync))
        got = decode(qd, k, v, seg, cache_lens, Hq=Hq, Hkv=Hkv, D=D, H=0, block=0, dtype=BF16, sync_override=sync)
        ref = oracle.decode_step(qd, k, v, seg, cache_lens, is_sync=bool(sync))
        check(got, ref, BF16, "decode N=%d sync=%d" % (N, sync))
    # every participant has rows: local blocks merge their chunks inside the streaming kernel
    cache_lens = np.maximum(lens, 1).astype(np.int32)
    cap = np.maximum(lens, 1)
    seg2 = np.concatenate([[0], np.cumsum(cap)]).astype(np.int32)
    _, k2, v2 = rand_block(70 + N, int(seg2[-1]), Hq, Hkv, D)
    say("decode N=%d local, no empty cache" % N)
    got = decode(qd, k2, v2, seg2, cache_lens, Hq=Hq, Hkv=Hkv, D=D, H=0, block=0, dtype=BF16, sync_override=0)
    check(got, oracle.decode_step(qd, k2, v2, seg2, cache_lens, is_sync=False), BF16, "decode N=%d local fused" % N)


def test_mfma_prefill_sync_rule_and_scale():
    seg = np.array([0, 96, 224], dtype=np.int32)
    q, k, v = rand_block(8, 224, 4, 1, 128)
    loc = oracle.attend_block(q, k, v, seg, is_sync=False, scale=0.05)
    glo = oracle.attend_block(q, k, v, seg, is_sync=True, scale=0.05)
    for H, b in [(2, 0), (2, 1), (3, 2), (3, 3), (0, 5), (1, 0)]:
        say("sync rule H=%d block=%d" % (H, b))
        got = prefill(q, k, v, seg, Hq=4, Hkv=1, D=128, H=H, block=b, dtype=BF16, scale=0.05)
        sync = oracle.is_sync_block(H, b)
        assert sync == fa.fedattn_is_sync_block(H, b)
        check(got, glo if sync else loc, BF16, "rule H=%d block=%d -> %s" % (H, b, "sync" if sync else "local"))


@pytest.mark.parametrize("D,scale", [(128, 0.0), (128, 0.3), (64, 0.0), (64, 0.4)])
@pytest.mark.parametrize("trend", ["rising", "falling"])
def test_mfma_prefill_scores_that_keep_outgrowing_the_reference(D, scale, trend):
    """The online softmax keeps a reference value per row and moves it only when a tile's maximum
    has outgrown it by 2^8: random inputs move it once, at the first tile.  Here the scores rise
    over the first 320 keys by about 12 (in log2 units) per 64 keys, so that each of the first tiles
    of a walk moves it (accumulators rescaled mid-walk), or fall at the same rate, so that it never
    moves again and later weights underflow.  With the usual scale (0: 1/sqrt(D); the kernel folds it into Q) and
    with a larger one (applied to the scores in fp32)."""
    Hq, Hkv = 8, 2
    seg = np.array([0, 300, 300, 937, 1200], dtype=np.int32)
    total = int(seg[-1])
    g = np.random.default_rng(40)
    u = g.standard_normal(D)
    u /= np.linalg.norm(u)
    pos = np.arange(total, dtype=np.float64)
    ramp = np.minimum(pos, 320.0) if trend == "rising" else np.maximum(320.0 - pos, 0.0)   # over the first five tiles
    sc = scale if scale else D ** -0.5
    per_key = 12.0 / 64.0 / (sc * np.log2(np.e))          # growth of q.k per key for 12 log2 units per tile
    q = fi.round_to_bf16((u[None, None, :] * 4.0 + 0.3 * g.standard_normal((total, Hq, D))).astype(np.float32))
    k = fi.round_to_bf16((u[None, None, :] * (ramp * per_key / 4.0)[:, None, None]
                          + 0.3 * g.standard_normal((total, Hkv, D))).astype(np.float32))
    v = fi.round_to_bf16(g.standard_normal((total, Hkv, D)).astype(np.float32))
    for causal in (True, False):
        for sync in (0, 1):
            say("growing scores D=%d scale=%g %s causal=%d sync=%d" % (D, scale, trend, causal, sync))
            got = prefill(q, k, v, seg, Hq=Hq, Hkv=Hkv, D=D, H=0, block=0, dtype=BF16, causal=causal,
                          sync_override=sync, scale=scale)
            ref = oracle.attend_block(q, k, v, seg, is_sync=bool(sync), causal=causal, scale=scale if scale else None)
            check(got, ref, BF16, "growing scores D=%d scale=%g %s causal=%d sync=%d" % (D, scale, trend, causal, sync))


@pytest.mark.parametrize("D,Hkv", [(64, 1), (64, 2), (128, 1), (128, 2)])
@pytest.mark.parametrize("scale", [0.0, 0.4])
def test_mfma_prefill_few_long_walks(D, Hkv, scale):
    """A grid of few workgroups whose walks are long (4 x 512 tokens, one or two KV heads, sync block): the
    launch that splits every walk's KV tiles between the two halves of an 8-wave workgroup and merges the
    halves at the end, at both head dimensions, with the folded scale and without; the local block of
    the same layout (short walks, one tile per 4-wave workgroup) beside it.  Every row is checked."""
    Hq = 4 * Hkv
    seg = np.array([0, 512, 1024, 1536, 2048], dtype=np.int32)
    q, k, v = rand_block(17, 2048, Hq, Hkv, D, sigma=0.7)
    for causal in (True, False):
        for sync in (1, 0):
            say("few long walks D=%d Hkv=%d scale=%g causal=%d sync=%d" % (D, Hkv, scale, causal, sync))
            got = prefill(q, k, v, seg, Hq=Hq, Hkv=Hkv, D=D, H=0, block=0, dtype=BF16, causal=causal,
                          sync_override=sync, scale=scale)
            ref = oracle.attend_block(q, k, v, seg, is_sync=bool(sync), causal=causal, scale=scale if scale else None)
            check(got, ref, BF16, "few long walks D=%d Hkv=%d scale=%g causal=%d sync=%d" % (D, Hkv, scale, causal, sync))


@pytest.mark.parametrize("chunk", [64, 128])
def test_mfma_prefill_sparse_exchange(chunk):
    seg = np.array([0, 256, 256, 579, 900, 1001], dtype=np.int32)   # ragged last chunks
    Hq, Hkv, D = 8, 2, 128
    q, k, v = rand_block(9, 1001, Hq, Hkv, D)
    nch = int(fi.chunk_counts(np.diff(seg), chunk).sum())
    g = np.random.default_rng(4)
    for name, flags in [("random", (g.random(nch) < 0.4).astype(np.uint8)),
                        ("none", np.zeros(nch, np.uint8)), ("all", np.ones(nch, np.uint8))]:
        kt = oracle.expand_keep_chunks(flags, seg, chunk)
        for causal in (True, False):
            say("mfma sparse chunk=%d keep=%s causal=%d" % (chunk, name, causal))
            got = prefill(q, k, v, seg, Hq=Hq, Hkv=Hkv, D=D, H=1, block=0, dtype=BF16, causal=causal,
                          keep_chunks=flags, chunk_tokens=chunk)
            ref = oracle.attend_block(q, k, v, seg, is_sync=True, causal=causal, keep_tok=kt)
            check(got, ref, BF16, "sparse chunk=%d keep=%s causal=%d" % (chunk, name, causal))
    # a local block ignores the keep-list
    flags = np.zeros(nch, np.uint8)
    got = prefill(q, k, v, seg, Hq=Hq, Hkv=Hkv, D=D, H=0, block=0, dtype=BF16, keep_chunks=flags, chunk_tokens=chunk)
    check(got, oracle.attend_block(q, k, v, seg, is_sync=False), BF16, "local block with keep-list")


@pytest.mark.parametrize("chunk", [1, 16, 100])
def test_mfma_prefill_keep_lists_finer_than_a_tile(chunk):
    """Keep chunks that are not whole 64-row tiles (down to single tokens): the MFMA path packs
    every participant's kept rows and walks dense tiles of the packed copy."""
    seg = np.array([0, 200, 500, 731, 731, 1000], dtype=np.int32)   # an empty participant, ragged tails
    Hq, Hkv, D = 8, 2, 128
    q, k, v = rand_block(41, 1000, Hq, Hkv, D)
    counts = fi.chunk_counts(np.diff(seg), chunk)
    nch, first = int(counts.sum()), np.concatenate([[0], np.cumsum(counts)])
    g = np.random.default_rng(6 + chunk)
    random_flags = (g.random(nch) < 0.3).astype(np.uint8)
    mixed = random_flags.copy()
    mixed[first[1]:first[2]] = 0      # participant 1 shares nothing
    mixed[first[2]:first[3]] = 1      # participant 2 shares everything
    for name, flags in [("random", random_flags), ("none/all mix", mixed), ("all", np.ones(nch, np.uint8))]:
        kt = oracle.expand_keep_chunks(flags, seg, chunk)
        for causal in (True, False):
            say("mfma packed keep-list chunk=%d keep=%s causal=%d" % (chunk, name, causal))
            got = prefill(q, k, v, seg, Hq=Hq, Hkv=Hkv, D=D, H=1, block=0, dtype=BF16, causal=causal,
                          keep_chunks=flags, chunk_tokens=chunk)
            ref = oracle.attend_block(q, k, v, seg, is_sync=True, causal=causal, keep_tok=kt)
            check(got, ref, BF16, "packed keep-list chunk=%d keep=%s causal=%d" % (chunk, name, causal))


def test_prefill_blocks_batched_equals_per_block():
    w = fi.workload("cfg2_llama8b_prefill")
    seg = np.array([0, 130, 200, 333], dtype=np.int32)
    M, H = 5, 2
    blocks = [fi.prefill_block(w, b, total=333) for b in range(M)]
    p = fa.make_params(3, w.n_q_heads, w.n_kv_heads, w.head_dim, H, BF16)
    tq = torch.stack([dev(b[0], BF16) for b in blocks])
    tk = torch.stack([dev(b[1], BF16) for b in blocks])
    tv = torch.stack([dev(b[2], BF16) for b in blocks])
    out = torch.full_like(tq, float("nan"))
    say("prefill_blocks M=5 H=2")
    fa.fedattn_prefill_blocks(p, 0, M, tq, tk, tv, out, tq[0].numel(), tk[0].numel(), seg)
    torch.cuda.synchronize()
    for b in range(M):
        one = torch.full_like(tq[b], float("nan"))
        fa.fedattn_prefill(p, b, tq[b], tk[b], tv[b], one, seg)
        torch.cuda.synchronize()
        ref = oracle.attend_block(*blocks[b], seg, is_sync=oracle.is_sync_block(H, b))
        check(host(out[b]), ref, BF16, "batched block %d" % b)
        check(host(one), ref, BF16, "per-block launch of block %d" % b)
        # the two launches may split the KV tiles differently (summation order), nothing more
        assert (one.float() - out[b].float()).abs().max().item() <= 2.0 ** -7 * ref.__abs__().max(), \
            "batched launch differs from the per-block launch at block %d" % b


# ------------------------------------- variable sync schedules, exclusion, token-granular exchange
def test_variable_sync_schedules():
    # Theorem 3 / "where to perform global attention": any set of sync blocks; the four
    # placements of the experiments (4 global blocks among M = 8)
    seg = np.array([0, 64, 150, 260], dtype=np.int32)
    M, Hq, Hkv, D = 8, 8, 2, 128
    w = fi.workload("cfg2_llama8b_prefill")
    blocks = [fi.prefill_block(w, b, total=260) for b in range(M)]
    from paper_2511_02647_amd.planning import sync_schedule
    schedules = {name: sync_schedule(name, M, 4) for name in ("shallow-half", "deep-half", "progressive", "regressive")}
    schedules["doubling intervals"] = [b in (0, 1, 3, 7) for b in range(M)]
    refs = {}
    for name, flags in schedules.items():
        for b in range(M):
            sync = bool(flags[b])
            say("schedule %s block %d (%s)" % (name, b, "sync" if sync else "local"))
            got = prefill(*[x[:, :Hq if i == 0 else Hkv] for i, x in enumerate(blocks[b])], seg, Hq=Hq, Hkv=Hkv, D=D,
                          H=4, block=b, dtype=BF16, sync_override=int(sync))
            if (b, sync) not in refs:
                q, k, v = blocks[b]
                refs[(b, sync)] = oracle.attend_block(q[:, :Hq], k[:, :Hkv], v[:, :Hkv], seg, is_sync=sync)
            check(got, refs[(b, sync)], BF16, "%s block %d" % (name, b))


def test_participant_exclusion_and_token_granular_exchange():
    seg = np.array([0, 128, 256, 448], dtype=np.int32)
    Hq, Hkv, D = 8, 2, 128
    q, k, v = rand_block(31, 448, Hq, Hkv, D)
    # pi_n = 0 for participant 1: its rows never reach the others (64-token chunks, MFMA path)
    flags = np.array([1, 1, 0, 0, 1, 1, 1], dtype=np.uint8)
    kt = oracle.expand_keep_chunks(flags, seg, 64)
    say("participant 1 excluded from the aggregation")
    got = prefill(q, k, v, seg, Hq=Hq, Hkv=Hkv, D=D, H=1, block=0, dtype=BF16, keep_chunks=flags, chunk_tokens=64)
    check(got, oracle.attend_block(q, k, v, seg, is_sync=True, keep_tok=kt), BF16, "participant excluded")
    # token-granular random exchange (chunk = 1 token: kept rows packed, MFMA kernel)
    tok = (np.random.default_rng(5).random(448) < 0.3).astype(np.uint8)
    say("token-granular sparse exchange")
    got = prefill(q, k, v, seg, Hq=Hq, Hkv=Hkv, D=D, H=1, block=0, dtype=BF16, keep_chunks=tok, chunk_tokens=1)
    check(got, oracle.attend_block(q, k, v, seg, is_sync=True, keep_tok=tok), BF16, "token-granular exchange")


def test_sparse_local_attention_by_gather():
    # sparse local attention: each participant keeps a sampled subset of its tokens before the
    # local computation; the operator then runs on the gathered (shorter) segments
    seg = np.array([0, 200, 520], dtype=np.int32)
    Hq, Hkv, D = 8, 2, 128
    q, k, v = rand_block(32, 520, Hq, Hkv, D)
    g = np.random.default_rng(6)
    keep = np.sort(np.concatenate([g.choice(200, 120, replace=False), 200 + g.choice(320, 150, replace=False)]))
    seg2 = np.array([0, 120, 270], dtype=np.int32)
    say("sparse local attention (gathered tokens)")
    got = prefill(q[keep], k[keep], v[keep], seg2, Hq=Hq, Hkv=Hkv, D=D, H=0, block=0, dtype=BF16)
    check(got, oracle.attend_block(q[keep], k[keep], v[keep], seg2, is_sync=False), BF16, "sparse local attention")


# ------------------------------------------------------------- full-size configs
def _sampled_check(q, k, v, seg, got, *, is_sync, n_random, what, keep_tok=None, salt=0):
    rows, heads = fi.sample_rows(seg, q.shape[1], n_random, fi.DEFAULT_SEED, salt=salt)
    ref = oracle.attend_rows(q, k, v, seg, rows, heads, is_sync=is_sync, keep_tok=keep_tok)
    check(got[rows, heads], ref, BF16, what + " (%d sampled rows)" % len(rows))


def test_cfg2_full_size():
    w = fi.workload("cfg2_llama8b_prefill")
    seg = w.seg_offsets
    for b in (0, 3):
        q, k, v = fi.prefill_block(w, b)
        say("cfg2 block %d" % b)
        got = prefill(q, k, v, seg, Hq=w.n_q_heads, Hkv=w.n_kv_heads, D=w.head_dim, H=w.sync_interval,
                      block=b, dtype=BF16)
        sync = oracle.is_sync_block(w.sync_interval, b)
        assert sync == (b == 3)
        _sampled_check(q, k, v, seg, got, is_sync=sync, n_random=4096, what="cfg2 block %d" % b, salt=b)


def test_cfg3_full_size_sync_interval_sweep():
    """Every H of the sweep gets its own sample: all tile-boundary rows plus 4096 random (row, head)
    pairs per (block, H); launches of the same kind of block must also agree bit for bit."""
    w = fi.workload("cfg3_hetero_prefill")
    seg = w.seg_offsets
    for b in (0, 31):
        q, k, v = fi.prefill_block(w, b)
        tq, tk, tv = dev(q, BF16), dev(k, BF16), dev(v, BF16)
        results = {}
        for H in (1, 4, 8, 32):
            sync = oracle.is_sync_block(H, b)
            say("cfg3 block %d H=%d (%s)" % (b, H, "sync" if sync else "local"))
            p = fa.make_params(w.n_participants, w.n_q_heads, w.n_kv_heads, w.head_dim, H, BF16)
            out = torch.full_like(tq, float("nan"))
            fa.fedattn_prefill(p, b, tq, tk, tv, out, seg)
            torch.cuda.synchronize()
            if (b, sync) in results:     # same block, same kind of block: identical output
                assert torch.equal(results[(b, sync)], out)
            results[(b, sync)] = out
            _sampled_check(q, k, v, seg, host(out), is_sync=sync, n_random=4096,
                           what="cfg3 block %d H=%d %s" % (b, H, "sync" if sync else "local"), salt=10 + 100 * H + b)
        del tq, tk, tv, results


def test_cfg5_sparse_sync_full_size():
    w = fi.workload("cfg5_sparse_sync")
    seg = w.seg_offsets
    for b in (0, 1):
        q, k, v = fi.prefill_block(w, b)
        sync = oracle.is_sync_block(w.sync_interval, b)
        flags = fi.keep_chunks(w, b // w.sync_interval)
        kt = oracle.expand_keep_chunks(flags, seg, w.chunk_tokens)
        say("cfg5 block %d (%s)" % (b, "sparse sync" if sync else "local"))
        got = prefill(q, k, v, seg, Hq=w.n_q_heads, Hkv=w.n_kv_heads, D=w.head_dim, H=w.sync_interval,
                      block=b, dtype=BF16, keep_chunks=flags, chunk_tokens=w.chunk_tokens)
        _sampled_check(q, k, v, seg, got, is_sync=sync, n_random=4096, keep_tok=kt,
                       what="cfg5 block %d" % b, salt=20 + b)


@pytest.mark.parametrize("case", range(24))
def test_random_shapes(case):
    """Seeded random layouts: participants, ragged and empty segments, head grouping, head
    dimension, causal or not, local / sync / sparse sync, and a decoding step on the same layout."""
    g = np.random.default_rng(7000 + case)
    N = int(g.integers(1, 12))
    lens = g.integers(0, 300, size=N)
    if g.random() < 0.5:
        lens[g.integers(0, N)] = 0
    if lens.sum() == 0:
        lens[0] = 17
    seg = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    total = int(seg[-1])
    D = int(g.choice([64, 128]))
    Hkv = int(g.choice([1, 2, 3]))
    Hq = Hkv * int(g.choice([1, 2, 4, 8]))
    causal = bool(g.random() < 0.7)
    scale = float(g.choice([0.0, 0.05, 0.3]))
    q, k, v = rand_block(8000 + case, total, Hq, Hkv, D, sigma=float(g.choice([0.5, 1.0])))
    for sync in (0, 1):
        say("random case %d: N=%d total=%d Hq=%d Hkv=%d D=%d causal=%d sync=%d" % (case, N, total, Hq, Hkv, D, causal, sync))
        got = prefill(q, k, v, seg, Hq=Hq, Hkv=Hkv, D=D, H=0, block=0, dtype=BF16, causal=causal, sync_override=sync, scale=scale)
        ref = oracle.attend_block(q, k, v, seg, is_sync=bool(sync), causal=causal, scale=scale if scale else None)
        check(got, ref, BF16, "random case %d sync=%d" % (case, sync))
    chunk = int(g.choice([1, 7, 64, 128]))
    nch = int(fi.chunk_counts(np.diff(seg), chunk).sum())
    flags = (g.random(nch) < g.choice([0.1, 0.5, 0.9])).astype(np.uint8)
    say("random case %d: sparse sync, chunk %d" % (case, chunk))
    got = prefill(q, k, v, seg, Hq=Hq, Hkv=Hkv, D=D, H=1, block=0, dtype=BF16, causal=causal, keep_chunks=flags, chunk_tokens=chunk)
    ref = oracle.attend_block(q, k, v, seg, is_sync=True, causal=causal, keep_tok=oracle.expand_keep_chunks(flags, seg, chunk))
    check(got, ref, BF16, "random case %d sparse chunk=%d" % (case, chunk))
    # decoding step over the same buffers as caches
    cache_lens = np.array([int(g.integers(0, l + 1)) for l in lens], dtype=np.int32)
    prompt = np.minimum(cache_lens, g.integers(0, 300, size=N)).astype(np.int32)
    qd, _, _ = rand_block(9000 + case, N, Hq, Hkv, D)
    for sync, rl in [(0, None), (1, None), (1, prompt)]:
        say("random case %d: decode sync=%d remote=%s" % (case, sync, rl is not None))
        got = decode(qd, k, v, seg, cache_lens, Hq=Hq, Hkv=Hkv, D=D, H=0, block=0, dtype=BF16, remote_lens=rl, sync_override=sync)
        ref = oracle.decode_step(qd, k, v, seg, cache_lens, is_sync=bool(sync), remote_lens=rl)
        check(got, ref, BF16, "random case %d decode sync=%d remote=%s" % (case, sync, rl is not None))


@pytest.mark.parametrize("case", range(16))
def test_random_mid_size_layouts(case):
    """Seeded random layouts of up to 8 participants x 2600 tokens, checked on sampled rows: these
    sizes reach every launch shape of the MFMA kernel (paired and one-tile workgroups, 4-wave and
    8-wave split-KV workgroups), whole-tile and finer keep chunks, and decoding with chunked caches."""
    g = np.random.default_rng(31000 + case)
    N = int(g.integers(1, 9))
    hi = int(g.choice([200, 700, 1500, 2600]))
    lens = g.integers(0, hi, size=N)
    if g.random() < 0.3:
        lens[g.integers(0, N)] = 0
    if g.random() < 0.3:
        lens[:] = (lens // 64) * 64
    if lens.sum() == 0:
        lens[0] = 65
    seg = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    total = int(seg[-1])
    D = int(g.choice([64, 128]))
    Hkv = int(g.choice([1, 2, 4, 8]))
    Hq = Hkv * int(g.choice([1, 2, 4]))
    causal = bool(g.random() < 0.75)
    q, k, v = rand_block(32000 + case, total, Hq, Hkv, D)
    rows, heads = fi.sample_rows(seg, Hq, 96, fi.DEFAULT_SEED, salt=300 + case)
    for sync in (0, 1):
        say("mid-size case %d: lens=%s Hq=%d Hkv=%d D=%d causal=%d sync=%d" % (case, lens.tolist(), Hq, Hkv, D, causal, sync))
        got = prefill(q, k, v, seg, Hq=Hq, Hkv=Hkv, D=D, H=0, block=0, dtype=BF16, causal=causal, sync_override=sync)
        ref = oracle.attend_rows(q, k, v, seg, rows, heads, is_sync=bool(sync), causal=causal)
        check(got[rows, heads], ref, BF16, "mid-size case %d sync=%d" % (case, sync))
    chunk = int(g.choice([1, 5, 16, 64, 128, 192]))
    nch = int(fi.chunk_counts(np.diff(seg), chunk).sum())
    flags = (g.random(nch) < g.choice([0.05, 0.25, 0.5, 0.95])).astype(np.uint8)
    say("mid-size case %d: sparse sync, chunk %d" % (case, chunk))
    got = prefill(q, k, v, seg, Hq=Hq, Hkv=Hkv, D=D, H=1, block=0, dtype=BF16, causal=causal, keep_chunks=flags, chunk_tokens=chunk)
    ref = oracle.attend_rows(q, k, v, seg, rows, heads, is_sync=True, causal=causal,
                             keep_tok=oracle.expand_keep_chunks(flags, seg, chunk))
    check(got[rows, heads], ref, BF16, "mid-size case %d sparse chunk=%d" % (case, chunk))
    cache_lens = np.array([int(g.integers(0, l + 1)) for l in lens], dtype=np.int32)
    if g.random() < 0.5:
        cache_lens = np.maximum(cache_lens, np.minimum(lens, 1)).astype(np.int32)   # no empty cache where there is room
    prompt = np.minimum(cache_lens, g.integers(0, hi, size=N)).astype(np.int32)
    qd, _, _ = rand_block(33000 + case, N, Hq, Hkv, D)
    for sync, rl in [(0, None), (1, None), (1, prompt)]:
        say("mid-size case %d: decode sync=%d remote=%s" % (case, sync, rl is not None))
        got = decode(qd, k, v, seg, cache_lens, Hq=Hq, Hkv=Hkv, D=D, H=0, block=0, dtype=BF16, remote_lens=rl, sync_override=sync)
        ref = oracle.decode_step(qd, k, v, seg, cache_lens, is_sync=bool(sync), remote_lens=rl)
        check(got, ref, BF16, "mid-size case %d decode sync=%d remote=%s" % (case, sync, rl is not None))


def test_more_than_65535_query_tiles():
    """2.1 million tokens in 128 ragged segments, bidirectional local block with 32-row query
    tiles: 65 664 query tiles in one launch (tile indices beyond 16 bits)."""
    N, seglen, Hq, Hkv, D = 128, 16400, 4, 1, 64
    total = N * seglen
    seg = (np.arange(N + 1) * seglen).astype(np.int32)
    g = torch.Generator(device="cuda")
    g.manual_seed(78)
    q = torch.randn(total, Hq, D, generator=g, device="cuda", dtype=BF16)
    k = torch.randn(total, Hkv, D, generator=g, device="cuda", dtype=BF16)
    v = torch.randn(total, Hkv, D, generator=g, device="cuda", dtype=BF16)
    out = torch.full_like(q, float("nan"))
    p = fa.make_params(N, Hq, Hkv, D, 0, BF16, causal=False)
    say("prefill local, bidirectional, 65664 query tiles")
    fa.fedattn_prefill(p, 0, q, k, v, out, seg, sync_override=0)
    torch.cuda.synchronize()
    rng = np.random.default_rng(10)
    for n in (0, 64, 127):
        sl = slice(int(seg[n]), int(seg[n + 1]))
        rows = np.concatenate([[0, 31, 32, seglen - 17, seglen - 16, seglen - 1], rng.integers(0, seglen, size=18)]).astype(np.int32)
        heads = rng.integers(0, Hq, size=rows.shape[0]).astype(np.int32)
        ref = oracle.attend_rows(host(q[sl]), host(k[sl]), host(v[sl]), [0, seglen], rows, heads, is_sync=False, causal=False)
        check(host(out[sl])[rows, heads], ref, BF16, "65664 query tiles, participant %d" % n)
    assert bool(torch.isfinite(out.float()).all()), "rows never written"


def test_offsets_beyond_32_bits():
    """One million tokens, 128 participants: byte offsets into q, k, v, out and the caches pass
    2^32 (q/out 8.6 GB, k/v 4.3 GB each).  Inputs of this size are drawn on the device; the
    oracle gets host copies of the segments and heads it checks."""
    N, seglen, Hq, Hkv, D = 128, 8192, 32, 16, 128
    total = N * seglen
    seg = (np.arange(N + 1) * seglen).astype(np.int32)
    g = torch.Generator(device="cuda")
    g.manual_seed(77)
    q = torch.randn(total, Hq, D, generator=g, device="cuda", dtype=BF16)
    k = torch.randn(total, Hkv, D, generator=g, device="cuda", dtype=BF16)
    v = torch.randn(total, Hkv, D, generator=g, device="cuda", dtype=BF16)
    out = torch.full_like(q, float("nan"))
    p = fa.make_params(N, Hq, Hkv, D, 0, BF16)
    say("prefill local, 2^20 tokens")
    fa.fedattn_prefill(p, 0, q, k, v, out, seg, sync_override=0)
    torch.cuda.synchronize()
    rng = np.random.default_rng(9)
    for n in (0, 63, 127):
        sl = slice(int(seg[n]), int(seg[n + 1]))
        rows = np.concatenate([[0, 1, 63, 64, seglen - 2, seglen - 1], rng.integers(0, seglen, size=26)]).astype(np.int32)
        heads = rng.integers(0, Hq, size=rows.shape[0]).astype(np.int32)
        ref = oracle.attend_rows(host(q[sl]), host(k[sl]), host(v[sl]), [0, seglen], rows, heads, is_sync=False)
        check(host(out[sl])[rows, heads], ref, BF16, "2^20 tokens, local block, participant %d" % n)
    del out

    # decode over the same buffers as caches
    lens = rng.integers(seglen - 200, seglen, size=N, endpoint=True).astype(np.int32)
    qd = torch.randn(N, Hq, D, generator=g, device="cuda", dtype=BF16)
    od = torch.full_like(qd, float("nan"))
    ws = torch.empty(fa.fedattn_workspace_bytes(p, fa.FEDATTN_OP_DECODE, total), dtype=torch.uint8, device="cuda")
    say("decode local, caches of 2^20 rows")
    fa.fedattn_decode(p, 0, qd, k, v, od, seg, lens, sync_override=0, workspace=ws)
    torch.cuda.synchronize()
    for n in (0, 127):
        sl = slice(int(seg[n]), int(seg[n + 1]))
        ref = oracle.decode_step(host(qd[n:n + 1]), host(k[sl]), host(v[sl]), [0, seglen], lens[n:n + 1], is_sync=False)
        check(host(od[n:n + 1]), ref, BF16, "2^20 cache rows, local decode, participant %d" % n)
    say("decode sync, caches of 2^20 rows")
    od.fill_(float("nan"))
    fa.fedattn_decode(p, 0, qd, k, v, od, seg, lens, sync_override=1, workspace=ws)
    torch.cuda.synchronize()
    G = Hq // Hkv
    for h in (0, Hq - 1):
        kv = h // G
        ref = oracle.decode_step(host(qd[:, h:h + 1]), host(k[:, kv:kv + 1]), host(v[:, kv:kv + 1]), seg, lens, is_sync=True)
        check(host(od[:, h:h + 1]), ref, BF16, "2^20 cache rows, sync decode, head %d" % h)


@pytest.mark.parametrize("case", range(24))
def test_random_shapes_with_score_ramps(case):
    """Seeded random layouts as above, with softmax scales on both sides of 1/sqrt(D) (the MFMA kernel folds
    scales up to there into its Q operand) and, in three cases of four, scores that rise, fall or peak along
    the sequence by 6 to 14 (log2 units) per 64 keys, so that the reference of the online softmax moves in
    the middle of walks; dense local and sync blocks, or a sparse sync block."""
    g = np.random.default_rng(52000 + case)
    N = int(g.integers(1, 10))
    lens = g.integers(0, int(g.choice([40, 200, 700, 1500])), size=N)
    if lens.sum() == 0:
        lens[0] = 33
    seg = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    total = int(seg[-1])
    D = int(g.choice([64, 128]))
    Hkv = int(g.choice([1, 2, 4]))
    Hq = Hkv * int(g.choice([1, 2, 4, 8]))
    causal = bool(g.random() < 0.7)
    dflt = D ** -0.5
    scale = float(g.choice([0.0, dflt * 0.5, dflt * 0.999, dflt * 1.001, dflt * 2.0]))
    sigma = float(g.choice([0.5, 1.0]))
    mk = lambda *s: (sigma * g.standard_normal(s)).astype(np.float32)
    q, k, v = mk(total, Hq, D), mk(total, Hkv, D), mk(total, Hkv, D)
    mode = int(g.integers(0, 4))
    if mode:
        u = g.standard_normal(D)
        u /= np.linalg.norm(u)
        sc = scale if scale else dflt
        per_key = float(g.uniform(6, 14)) / 64.0 / (sc * np.log2(np.e))
        pos = np.arange(total, dtype=np.float64)
        span = float(g.choice([128, 320]))
        ramp = {1: np.minimum(pos, span), 2: np.maximum(span - pos, 0.0),
                3: np.maximum(span - np.abs(pos - total / 2), 0.0)}[mode]
        q = q * 0.3 + (u[None, None, :] * 4.0).astype(np.float32)
        k = k * 0.3 + (u[None, None, :] * (ramp * per_key / 4.0)[:, None, None]).astype(np.float32)
    q, k, v = fi.round_to_bf16(q), fi.round_to_bf16(k), fi.round_to_bf16(v)
    sparse = g.random() < 0.3
    flags, chunk = None, 0
    if sparse:
        chunk = int(g.choice([1, 16, 64]))
        flags = (g.random(int(fi.chunk_counts(np.diff(seg), chunk).sum())) < 0.5).astype(np.uint8)
    for sync in ((1,) if sparse else (0, 1)):
        say("ramp case %d: N=%d total=%d Hq=%d Hkv=%d D=%d causal=%d scale=%.4f mode=%d sparse=%d sync=%d"
            % (case, N, total, Hq, Hkv, D, causal, scale, mode, sparse, sync))
        got = prefill(q, k, v, seg, Hq=Hq, Hkv=Hkv, D=D, H=0, block=0, dtype=BF16, causal=causal, sync_override=sync,
                      scale=scale, keep_chunks=flags, chunk_tokens=chunk)
        ref = oracle.attend_block(q, k, v, seg, is_sync=bool(sync), causal=causal, scale=scale if scale else None,
                                  keep_tok=oracle.expand_keep_chunks(flags, seg, chunk) if sparse else None)
        check(got, ref, BF16, "ramp case %d sync=%d" % (case, sync))


# --------------------------------------------------------------------- decode
@pytest.mark.parametrize("N,Hq,Hkv,D,dtype", [(3, 8, 2, 128, BF16), (1, 4, 1, 128, BF16), (20, 8, 2, 128, BF16),
                                              (5, 6, 3, 64, BF16), (3, 4, 2, 64, F32), (2, 2, 1, 40, BF16)])
def test_decode_small(N, Hq, Hkv, D, dtype):
    cap = 300
    g = np.random.default_rng(11)
    seg = (np.arange(N + 1) * cap).astype(np.int32)
    lens = g.integers(1, cap, size=N, endpoint=True).astype(np.int32)
    lens[0] = cap
    if N > 2:
        lens[1] = 0          # a participant with an empty cache
    prompt = np.minimum(lens, g.integers(0, cap, size=N)).astype(np.int32)
    q, _, _ = rand_block(12, N, Hq, Hkv, D, bf16=dtype == BF16)
    _, kc, vc = rand_block(13, N * cap, Hq, Hkv, D, bf16=dtype == BF16)
    for sync, rl in [(0, None), (1, None), (1, prompt)]:
        say("decode N=%d Hq=%d Hkv=%d D=%d %s sync=%d remote=%s" % (N, Hq, Hkv, D, dtype, sync, rl is not None))
        got = decode(q, kc, vc, seg, lens, Hq=Hq, Hkv=Hkv, D=D, H=0, block=0, dtype=dtype,
                     remote_lens=rl, sync_override=sync)
        ref = oracle.decode_step(q, kc, vc, seg, lens, is_sync=bool(sync), remote_lens=rl)
        check(got, ref, dtype, "decode N=%d D=%d sync=%d remote=%s" % (N, D, sync, rl is not None))


def test_cfg4_decode_full_size():
    """All 16 x 32 output rows at decoding steps {0, 1, 127, 255} of blocks {0, 3, 16, 31} (local: 0, 16;
    sync: 3, 31) plus eight seeded random (step, block) pairs; sync blocks under both readings of
    what the other participants' caches show (everything cached / the prompt only)."""
    w = fi.workload("cfg4_decode")
    seg = w.seg_offsets
    prompt = np.full(w.n_participants, 1024, dtype=np.int32)
    cases = [(b, s) for b in (0, 3, 16, 31) for s in (0, 1, 127, 255)]
    g = fi.stream(fi.DEFAULT_SEED, 98, 0, 5)
    cases += [(int(b), int(s)) for b, s in zip(g.integers(0, w.n_blocks, size=8), g.integers(0, w.decode_steps, size=8))]
    p = fa.make_params(w.n_participants, w.n_q_heads, w.n_kv_heads, w.head_dim, w.sync_interval, BF16)
    ws = torch.empty(fa.fedattn_workspace_bytes(p, fa.FEDATTN_OP_DECODE, int(seg[-1])), dtype=torch.uint8, device="cuda")
    for b in sorted(set(c[0] for c in cases)):
        kc, vc = fi.decode_cache_block(w, b)
        tk, tv = dev(kc, BF16), dev(vc, BF16)
        sync = oracle.is_sync_block(w.sync_interval, b)
        for step in sorted(set(c[1] for c in cases if c[0] == b)):
            lens = prompt + step + 1
            q = fi.decode_query(w, step, b)
            tq = dev(q, BF16)
            for rl in ([None, prompt] if sync else [None]):
                say("cfg4 block %d step %d remote=%s" % (b, step, rl is not None))
                out = torch.full_like(tq, float("nan"))
                fa.fedattn_decode(p, b, tq, tk, tv, out, seg, lens, remote_lens=rl, workspace=ws)
                torch.cuda.synchronize()
                ref = oracle.decode_step(q, kc, vc, seg, lens, is_sync=sync, remote_lens=rl)
                check(host(out), ref, BF16, "cfg4 block %d step %d %s" % (b, step, "prompt-only remote" if rl is not None else "all cached"))
        del tk, tv


def test_decode_local_chunk_merge_in_kernel_with_dirty_workspace():
    """Local blocks merge a segment's chunks inside the streaming kernel, counting chunks in
    through the workspace: whatever the workspace held before must not matter, and it must be
    reusable call after call (1, 2 and many chunks per segment)."""
    N, Hq, Hkv, D, cap = 3, 8, 2, 128, 1000
    seg = (np.arange(N + 1) * cap).astype(np.int32)
    lens = np.array([1000, 64, 513], dtype=np.int32)
    p = fa.make_params(N, Hq, Hkv, D, 0, BF16)
    nbytes = fa.fedattn_workspace_bytes(p, fa.FEDATTN_OP_DECODE, N * cap)
    ws = torch.full((nbytes,), 0xFF, dtype=torch.uint8, device="cuda")
    _, kc, vc = rand_block(31, N * cap, Hq, Hkv, D, bf16=True)
    tk, tv = dev(kc, BF16), dev(vc, BF16)
    for rep in range(3):
        q, _, _ = rand_block(32 + rep, N, Hq, Hkv, D, bf16=True)
        tq = dev(q, BF16)
        out = torch.full_like(tq, float("nan"))
        say("decode local, dirty workspace, call %d" % rep)
        fa.fedattn_decode(p, 0, tq, tk, tv, out, seg, lens, sync_override=0, workspace=ws)
        torch.cuda.synchronize()
        ref = oracle.decode_step(q, kc, vc, seg, lens, is_sync=False)
        check(host(out), ref, BF16, "decode local in-kernel merge, call %d" % rep)


@pytest.mark.parametrize("N,Hkv,G,cap,n_lens", [(16, 8, 4, 1280, 1152), (2, 2, 4, 4096, 4000)])
def test_decode_local_merge_is_reproducible_over_alternating_inputs(N, Hkv, G, cap, n_lens):
    """The in-kernel merge hands partials from workgroup to workgroup through the workspace.  Launch
    after launch over the same workspace, alternating between two sets of queries and caches: every
    result must equal, bit for bit, the first result of its input (the merge sums the chunks in a
    fixed order, so the result does not depend on which workgroup arrives last; a partial read
    stale would be the other input's).  Shapes: the decode workload's (2 chunks per segment) and
    two long segments (64 chunks per segment); single launches and blocks sharing a launch in
    their own workspace slices.  Stops at the first mismatch."""
    Hq, D, M = Hkv * G, 128, 6
    seg = (np.arange(N + 1) * cap).astype(np.int32)
    lens = np.full(N, n_lens, dtype=np.int32)
    lens[-1] = n_lens - 37
    p = fa.make_params(N, Hq, Hkv, D, 0, BF16)
    g = torch.Generator(device="cuda")
    g.manual_seed(91)
    sets = []
    for i in range(2):
        sets.append((torch.randn(M, N, Hq, D, generator=g, device="cuda", dtype=BF16),
                     torch.randn(M, N * cap, Hkv, D, generator=g, device="cuda", dtype=BF16),
                     torch.randn(M, N * cap, Hkv, D, generator=g, device="cuda", dtype=BF16)))
    one = fa.fedattn_workspace_bytes(p, fa.FEDATTN_OP_DECODE, N * cap)
    slice_bytes = (one + 255) // 256 * 256
    ws = torch.full((one + (M - 1) * slice_bytes,), 0xFF, dtype=torch.uint8, device="cuda")
    # the oracle on one block of the first input, so that "the first result" is a checked one
    q0, k0, v0 = (host(t[0]) for t in sets[0])
    first = [None, None]
    first_fused = [None, None]
    for it in range(200):
        i = it & 1
        tq, tk, tv = sets[i]
        out = torch.full_like(tq[0], float("nan"))
        fa.fedattn_decode(p, 0, tq[0], tk[0], tv[0], out, seg, lens, sync_override=0, workspace=ws)
        fused = torch.full_like(tq, float("nan"))
        fa.fedattn_decode_blocks_fused(p, 0, M, tq, tk, tv, fused, tq[0].numel(), tk[0].numel(), seg, lens,
                                       sync_override=0, workspace=ws)
        torch.cuda.synchronize()
        if first[i] is None:
            say("decode local, alternating inputs, N=%d chunks over %d rows: first results" % (N, n_lens))
            first[i], first_fused[i] = out, fused
            assert torch.equal(fused[0], out), "blocks sharing a launch differ from the single launch"
            if i == 0:
                check(host(out), oracle.decode_step(q0, k0, v0, seg, lens, is_sync=False), BF16,
                      "decode local, N=%d, %d rows" % (N, n_lens))
            continue
        assert torch.equal(out, first[i]), "launch %d (input %d) differs from the first result of its input" % (it, i)
        assert torch.equal(fused, first_fused[i]), "fused launch %d (input %d) differs from its first result" % (it, i)


def test_decode_blocks_equals_per_block_calls():
    N, Hq, Hkv, D, cap, M, H = 4, 8, 2, 128, 200, 4, 2
    seg = (np.arange(N + 1) * cap).astype(np.int32)
    lens = np.array([200, 150, 1, 77], dtype=np.int32)
    g = np.random.default_rng(21)
    mk = lambda *s: fi.round_to_bf16(g.standard_normal(s).astype(np.float32))
    q, kc, vc = mk(M, N, Hq, D), mk(M, N * cap, Hkv, D), mk(M, N * cap, Hkv, D)
    tq, tk, tv = dev(q, BF16), dev(kc, BF16), dev(vc, BF16)
    p = fa.make_params(N, Hq, Hkv, D, H, BF16)
    ws = torch.empty(fa.fedattn_workspace_bytes(p, fa.FEDATTN_OP_DECODE, N * cap), dtype=torch.uint8, device="cuda")
    out = torch.full_like(tq, float("nan"))
    say("decode_blocks M=4 H=2")
    fa.fedattn_decode_blocks(p, 0, M, tq, tk, tv, out, tq[0].numel(), tk[0].numel(), seg, lens, workspace=ws)
    torch.cuda.synchronize()
    for b in range(M):
        one = torch.full_like(tq[b], float("nan"))
        fa.fedattn_decode(p, b, tq[b], tk[b], tv[b], one, seg, lens, workspace=ws)
        torch.cuda.synchronize()
        assert torch.equal(one, out[b]), "decode_blocks differs from fedattn_decode at block %d" % b
        ref = oracle.decode_step(q[b], kc[b], vc[b], seg, lens, is_sync=oracle.is_sync_block(H, b))
        check(host(out[b]), ref, BF16, "decode_blocks block %d" % b)


@pytest.mark.parametrize("lens", [[200, 150, 1, 77], [130, 0, 64, 200]])
def test_decode_blocks_fused_equals_decode_blocks(lens):
    """Blocks of one kind sharing launches (every block in flight in its own workspace slice):
    bit-equal to one launch per block, whatever the number of slices the workspace holds; with
    and without empty caches (chunks merged in the streaming kernel / by the combine kernel)."""
    N, Hq, Hkv, D, cap, M, H = 4, 8, 2, 128, 200, 9, 4
    seg = (np.arange(N + 1) * cap).astype(np.int32)
    lens = np.array(lens, dtype=np.int32)
    g = np.random.default_rng(22)
    mk = lambda *s: fi.round_to_bf16(g.standard_normal(s).astype(np.float32))
    q, kc, vc = mk(M, N, Hq, D), mk(M, N * cap, Hkv, D), mk(M, N * cap, Hkv, D)
    tq, tk, tv = dev(q, BF16), dev(kc, BF16), dev(vc, BF16)
    p = fa.make_params(N, Hq, Hkv, D, H, BF16)
    one = fa.fedattn_workspace_bytes(p, fa.FEDATTN_OP_DECODE, N * cap)
    slice_bytes = (one + 255) // 256 * 256
    ws1 = torch.empty(one, dtype=torch.uint8, device="cuda")
    prompt = np.minimum(lens, 100).astype(np.int32)
    for override, rl in [(-1, None), (-1, prompt), (0, None), (1, None)]:
        ref = torch.full_like(tq, float("nan"))
        fa.fedattn_decode_blocks(p, 0, M, tq, tk, tv, ref, tq[0].numel(), tk[0].numel(), seg, lens, remote_lens=rl,
                                 sync_override=override, workspace=ws1)
        torch.cuda.synchronize()
        for n_slices in (1, 3, 9):
            ws = torch.full((one + (n_slices - 1) * slice_bytes,), 0xFF, dtype=torch.uint8, device="cuda")
            out = torch.full_like(tq, float("nan"))
            say("decode_blocks_fused lens=%s override=%d remote=%s slices=%d" % (lens.tolist(), override, rl is not None, n_slices))
            fa.fedattn_decode_blocks_fused(p, 0, M, tq, tk, tv, out, tq[0].numel(), tk[0].numel(), seg, lens,
                                           remote_lens=rl, sync_override=override, workspace=ws)
            torch.cuda.synchronize()
            assert torch.equal(out, ref), "fused decode differs (override %d, %d slices)" % (override, n_slices)
    b = 3
    check(host(ref[b]), oracle.decode_step(q[b], kc[b], vc[b], seg, lens, is_sync=True), BF16, "decode block 3 (forced sync)")


# ------------------------------------------------------------------ aggregate
def test_hip_graph_replays_match_eager():
    """A sequence of the library's launches (aggregate, local and sync prefill, sparse prefill with
    its list kernels, a decoding step over several blocks) captured in a HIP graph: every replay,
    with eager work and synchronisations in between, must reproduce the eager results bit for bit."""
    N, Hq, Hkv, D, M, H = 3, 8, 2, 128, 4, 2
    seg = np.array([0, 100, 260, 420], dtype=np.int32)
    total = 420
    g = np.random.default_rng(81)
    mk = lambda *s: fi.round_to_bf16(g.standard_normal(s).astype(np.float32))
    q, k, v = dev(mk(M, total, Hq, D), BF16), dev(mk(M, total, Hkv, D), BF16), dev(mk(M, total, Hkv, D), BF16)
    p = fa.make_params(N, Hq, Hkv, D, H, BF16)
    out = torch.zeros_like(q)
    out_sparse = torch.zeros_like(q[0])
    kg, vg = torch.empty_like(k[0]), torch.empty_like(v[0])
    flags = torch.from_numpy((g.random(total) < 0.4).astype(np.uint8)).cuda()
    ws_p = torch.empty(fa.fedattn_workspace_bytes(p, fa.FEDATTN_OP_PREFILL, total, 1), dtype=torch.uint8, device="cuda")
    lens = np.array([100, 130, 160], dtype=np.int32)
    qd = dev(mk(M, N, Hq, D), BF16)
    od = torch.zeros_like(qd)
    ws_d = torch.empty(fa.fedattn_workspace_bytes(p, fa.FEDATTN_OP_DECODE, total), dtype=torch.uint8, device="cuda")

    def sequence():
        for b in range(M):
            kk, vv = k[b], v[b]
            if fa.fedattn_is_sync_block(H, b):
                fa.fedattn_aggregate_kv(p, [k[b][seg[i]:seg[i + 1]] for i in range(N)],
                                        [v[b][seg[i]:seg[i + 1]] for i in range(N)], seg, kg, vg)
                kk, vv = kg, vg
            fa.fedattn_prefill(p, b, q[b], kk, vv, out[b], seg)
        fa.fedattn_prefill(p, 1, q[1], k[1], v[1], out_sparse, seg, keep_chunks=flags, chunk_tokens=1, workspace=ws_p)
        fa.fedattn_decode_blocks(p, 0, M, qd, k, v, od, qd[0].numel(), k[0].numel(), seg, lens, workspace=ws_d)

    say("graph: eager reference")
    sequence()
    torch.cuda.synchronize()
    ref = [out.clone(), out_sparse.clone(), od.clone()]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            sequence()
    torch.cuda.synchronize()
    for rep in range(4):
        for t in (out, out_sparse, od):
            t.fill_(float("nan"))
        ws_d.fill_(0xAB)                      # eager work between the replays, on the workspace too
        torch.cuda.synchronize()
        say("graph: replay %d" % rep)
        graph.replay()
        torch.cuda.synchronize()
        for got, want, name in zip((out, out_sparse, od), ref, ("prefill", "sparse prefill", "decode")):
            assert torch.equal(got, want), "graph replay %d: %s differs from the eager run" % (rep, name)


@pytest.mark.parametrize("dtype", [BF16, F32])
def test_prefill_sync_local_kv_in_place_and_through_a_copy(dtype):
    """Phase II in one call from the participants' own K/V: read in place when they lie back to back
    in participant order, aggregated into the workspace first when they do not; both bit-equal to
    fedattn_aggregate_kv + fedattn_prefill, dense and under sparse exchange."""
    seg = np.array([0, 100, 100, 260, 420], dtype=np.int32)
    N, Hq, Hkv, D = 4, 8, 2, 128 if dtype == BF16 else 64
    q, k, v = rand_block(91, 420, Hq, Hkv, D, bf16=dtype == BF16)
    p = fa.make_params(N, Hq, Hkv, D, 3, dtype)
    tq, tk, tv = dev(q, dtype), dev(k, dtype), dev(v, dtype)
    flags = (np.random.default_rng(92).random(int(fi.chunk_counts(np.diff(seg), 16).sum())) < 0.4).astype(np.uint8)
    tflags = torch.from_numpy(flags).cuda()
    kt = oracle.expand_keep_chunks(flags, seg, 16)
    views_k = [tk[seg[n]:seg[n + 1]] for n in range(N)]
    views_v = [tv[seg[n]:seg[n + 1]] for n in range(N)]

    def apart(views):
        """The participants' matrices in reverse order, one row of padding between them, inside one
        allocation: never back to back in participant order, whatever the allocator does."""
        pool = torch.zeros(420 + N, Hkv, D, dtype=dtype, device="cuda")
        out, at = [None] * N, 0
        for n in reversed(range(N)):
            rows = views[n].shape[0]
            if rows:
                pool[at:at + rows].copy_(views[n])
                out[n] = pool[at:at + rows]
            at += rows + 1
        return out

    apart_k, apart_v = apart(views_k), apart(views_v)
    ws_pre = torch.empty(max(16, fa.fedattn_workspace_bytes(p, fa.FEDATTN_OP_PREFILL, 420, 16)), dtype=torch.uint8, device="cuda")
    ws_all = torch.empty(fa.fedattn_workspace_bytes(p, fa.FEDATTN_OP_PREFILL_SYNC_LOCAL_KV, 420, 16), dtype=torch.uint8, device="cuda")
    for sparse in (False, True):
        kc, ct = (tflags, 16) if sparse else (None, 0)
        want = torch.full_like(tq, float("nan"))
        fa.fedattn_prefill(p, 0, tq, tk, tv, want, seg, keep_chunks=kc, chunk_tokens=ct, sync_override=1, workspace=ws_pre)
        torch.cuda.synchronize()
        ref = oracle.attend_block(q, k, v, seg, is_sync=True, keep_tok=kt if sparse else None)
        check(host(want), ref, dtype, "sync block via fedattn_prefill, sparse=%d" % sparse)
        for name, kl, vl, ws in [("in place", views_k, views_v, ws_pre if sparse else None), ("copied", apart_k, apart_v, ws_all)]:
            say("prefill_sync_local_kv %s %s sparse=%d" % (dtype, name, sparse))
            got = torch.full_like(tq, float("nan"))
            fa.fedattn_prefill_sync_local_kv(p, tq, kl, vl, got, seg, keep_chunks=kc, chunk_tokens=ct, workspace=ws)
            torch.cuda.synchronize()
            assert torch.equal(got, want), "Phase II from local K/V (%s, sparse=%d) differs" % (name, sparse)
    with pytest.raises(fa.FedAttnError) as e:     # matrices apart and nowhere to aggregate them
        fa.fedattn_prefill_sync_local_kv(p, tq, apart_k, apart_v, torch.empty_like(tq), seg)
    assert e.value.status == fa.FEDATTN_EWORKSPACE
    torch.cuda.synchronize()


@pytest.mark.parametrize("dtype", [BF16, F32])
def test_aggregate_kv_bit_exact(dtype):
    seg = np.array([0, 77, 77, 300, 1325], dtype=np.int32)
    Hkv, D = 8, 128
    _, k, v = rand_block(14, 1325, Hkv, Hkv, D, bf16=dtype == BF16)
    kl = [k[seg[n]:seg[n + 1]] for n in range(4)]
    vl = [v[seg[n]:seg[n + 1]] for n in range(4)]
    Kref, Vref = oracle.aggregate_kv(kl, vl, seg)
    p = fa.make_params(4, Hkv, Hkv, D, 1, dtype)
    tkl = [dev(x, dtype) if x.shape[0] else None for x in kl]
    tvl = [dev(x, dtype) if x.shape[0] else None for x in vl]
    Kg = torch.full((1325, Hkv, D), float("nan"), dtype=dtype, device="cuda")
    Vg = torch.full_like(Kg, float("nan"))
    say("aggregate_kv %s" % dtype)
    fa.fedattn_aggregate_kv(p, tkl, tvl, seg, Kg, Vg)
    torch.cuda.synchronize()
    assert np.array_equal(Kg.float().cpu().numpy(), Kref) and np.array_equal(Vg.float().cpu().numpy(), Vref)


# --------------------------------------------------------------- error paths
def test_errors_are_return_codes():
    p = fa.make_params(2, 4, 2, 128, 1, BF16)
    t = torch.zeros(64 * 4 * 128 + 8, dtype=BF16, device="cuda")
    q = t[:64 * 4 * 128].view(64, 4, 128)
    kv = torch.zeros(64, 2, 128, dtype=BF16, device="cuda")
    out = torch.zeros_like(q)
    with pytest.raises(fa.FedAttnError) as e:
        fa.fedattn_prefill(p, 0, t[1:1 + 64 * 4 * 128].view(64, 4, 128), kv, kv, out, [0, 32, 64])
    assert e.value.status == fa.FEDATTN_EINVAL
    with pytest.raises(fa.FedAttnError) as e:
        fa.fedattn_prefill(p, 0, q, kv, kv, out, [0, 40, 32])
    assert e.value.status == fa.FEDATTN_EINVAL
    flags = torch.ones(2, dtype=torch.uint8, device="cuda")
    with pytest.raises(fa.FedAttnError) as e:
        fa.fedattn_prefill(p, 0, q, kv, kv, out, [0, 32, 64], keep_chunks=flags, chunk_tokens=64)
    assert e.value.status == fa.FEDATTN_EWORKSPACE
    with pytest.raises(fa.FedAttnError) as e:
        fa.fedattn_decode(p, 0, q[:2], kv, kv, out[:2], [0, 32, 64], [33, 1],
                          workspace=torch.empty(1 << 20, dtype=torch.uint8, device="cuda"))
    assert e.value.status == fa.FEDATTN_EINVAL
    with pytest.raises(fa.FedAttnError) as e:
        fa.fedattn_decode(p, 0, q[:2], kv, kv, out[:2], [0, 32, 64], [32, 1])
    assert e.value.status == fa.FEDATTN_EWORKSPACE
    torch.cuda.synchronize()
