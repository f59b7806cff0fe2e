"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these tests needs a GPU.  Each pin compares the oracle with something
that is not the oracle: a library attention routine (torch SDPA in fp64), closed
forms, printed values, or brute force over the dense visibility matrix.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import fedattn_inputs as fi
import oracle
from oracle import dense
from oracle.aggregate import aggregate_kv, aggregate_kv_by_definition

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rand_qkv(seed, total, Hq, Hkv, D, sigma=1.0):
    g = np.random.default_rng(seed)
    q = (sigma * g.standard_normal((total, Hq, D))).astype(np.float32)
    k = (sigma * g.standard_normal((total, Hkv, D))).astype(np.float32)
    v = g.standard_normal((total, Hkv, D)).astype(np.float32)
    return q, k, v


def sdpa(q, k, v, causal=True, mask=None):
    """Library attention in fp64: torch scaled_dot_product_attention, MHA/GQA by
    repeating KV heads.  q [L,Hq,D] -> out [L,Hq,D]."""
    tq = torch.from_numpy(np.asarray(q, dtype=np.float64)).permute(1, 0, 2)
    tk = torch.from_numpy(np.asarray(k, dtype=np.float64)).permute(1, 0, 2)
    tv = torch.from_numpy(np.asarray(v, dtype=np.float64)).permute(1, 0, 2)
    rep = tq.shape[0] // tk.shape[0]
    tk = tk.repeat_interleave(rep, dim=0)
    tv = tv.repeat_interleave(rep, dim=0)
    if mask is not None:
        o = F.scaled_dot_product_attention(tq, tk, tv, attn_mask=torch.from_numpy(mask))
    else:
        o = F.scaled_dot_product_attention(tq, tk, tv, is_causal=causal)
    return o.permute(1, 0, 2).numpy()


# ---------------------------------------------------------------- sync rule
def test_sync_rule_follows_algorithm_1():
    # enumerate rounds t and local forwards h as the algorithm does; block m = Ht + h
    for H in (1, 2, 3, 4, 8):
        for T in (1, 2, 5):
            M = H * T
            expect = np.zeros(M, dtype=bool)
            for t in range(T):
                for h in range(1, H + 1):
                    if h == H:
                        expect[H * t + h - 1] = True
            got = np.array([oracle.is_sync_block(H, b) for b in range(M)])
            assert np.array_equal(got, expect)
    # H = M: exactly the last block synchronises
    assert [oracle.is_sync_block(32, b) for b in range(32)] == [False] * 31 + [True]
    # never
    assert not any(oracle.is_sync_block(0, b) for b in range(16))
    assert not any(oracle.is_sync_block(-1, b) for b in range(16))


def test_sync_fraction_matches_printed_values():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "sync_interval_tradeoff.txt"))
            if l.strip() and not l.startswith("#")]
    M = 12 * 5 * 7 * 8
    frac = lambda H: Fraction(sum(oracle.is_sync_block(H, b) for b in range(M)), M)
    for h0, h1, red, err in rows:
        h0, h1 = int(h0), int(h1)
        assert frac(h0) - frac(h1) == Fraction(red)
        assert 1 - frac(h1) == Fraction(err)


# ------------------------------------------------- reduction to library attention
@pytest.mark.parametrize("Hq,Hkv,D", [(2, 2, 64), (4, 2, 32), (8, 2, 16)])
def test_sync_block_is_centralized_causal_attention(Hq, Hkv, D):
    # H = 1: every block attends over the whole global sequence (CenAttn)
    seg = [0, 7, 7, 20, 33]
    q, k, v = rand_qkv(1, 33, Hq, Hkv, D)
    got = oracle.attend_block(q, k, v, seg, is_sync=True)
    np.testing.assert_allclose(got, sdpa(q, k, v), rtol=0, atol=1e-12)


def test_single_participant_is_centralized_attention():
    q, k, v = rand_qkv(2, 29, 4, 2, 32)
    ref = sdpa(q, k, v)
    for is_sync in (False, True):
        got = oracle.attend_block(q, k, v, [0, 29], is_sync=is_sync)
        np.testing.assert_allclose(got, ref, rtol=0, atol=1e-12)


def test_local_block_is_independent_attention_per_participant():
    seg = [0, 5, 18, 19, 40]
    q, k, v = rand_qkv(3, 40, 4, 2, 32)
    got = oracle.attend_block(q, k, v, seg, is_sync=False)
    for n in range(len(seg) - 1):
        s, e = seg[n], seg[n + 1]
        np.testing.assert_allclose(got[s:e], sdpa(q[s:e], k[s:e], v[s:e]), rtol=0, atol=1e-12)


def test_bidirectional_variant_matches_library():
    seg = [0, 6, 16]
    q, k, v = rand_qkv(4, 16, 2, 2, 16)
    got = oracle.attend_block(q, k, v, seg, is_sync=True, causal=False)
    np.testing.assert_allclose(got, sdpa(q, k, v, causal=False), rtol=0, atol=1e-12)
    got = oracle.attend_block(q, k, v, seg, is_sync=False, causal=False)
    np.testing.assert_allclose(got[:6], sdpa(q[:6], k[:6], v[:6], causal=False), rtol=0, atol=1e-12)
    np.testing.assert_allclose(got[6:], sdpa(q[6:], k[6:], v[6:], causal=False), rtol=0, atol=1e-12)


def test_printed_mask_condition_contradicts_the_prose():
    # The case condition as printed (key j visible iff i <= j) gives row 0 all L
    # keys and is not causal attention; the reading j <= i is the one that
    # reproduces the library's causal attention (checked above).
    q, k, v = rand_qkv(5, 12, 1, 1, 8)
    idx = np.arange(12)
    printed = idx[:, None] <= idx[None, :]
    wrong = sdpa(q, k, v, mask=printed)
    right = oracle.attend_block(q, k, v, [0, 12], is_sync=True)
    assert np.abs(wrong - right).max() > 1e-3
    np.testing.assert_allclose(right[0, 0], v[0, 0].astype(np.float64), atol=1e-15)


# ------------------------------------------------------------- closed forms
def test_zero_queries_give_running_mean_of_values():
    seg = np.array([0, 9, 21, 30])
    q, k, v = rand_qkv(6, 30, 2, 1, 8)
    q[:] = 0
    v64 = v.astype(np.float64)
    loc = oracle.attend_block(q, k, v, seg, is_sync=False)
    glo = oracle.attend_block(q, k, v, seg, is_sync=True)
    csum = np.cumsum(v64[:, 0, :], axis=0)
    for i in range(30):
        n = np.searchsorted(seg, i, side="right") - 1
        s = seg[n]
        mean_glo = csum[i] / (i + 1)
        mean_loc = (csum[i] - (csum[s - 1] if s > 0 else 0)) / (i - s + 1)
        for h in range(2):
            np.testing.assert_allclose(glo[i, h], mean_glo, atol=1e-13)
            np.testing.assert_allclose(loc[i, h], mean_loc, atol=1e-13)


def test_dominant_key_selects_its_value():
    seg = [0, 10, 20]
    q, k, v = rand_qkv(7, 20, 1, 1, 16)
    q[:] = 0
    k[:] = 0
    q[:, 0, 0] = 200.0
    k[3, 0, 0] = 200.0     # key 3 (participant 0) dominates wherever it is visible
    k[12, 0, 0] = 100.0    # key 12 (participant 1) is next
    glo = oracle.attend_block(q, k, v, seg, is_sync=True)
    loc = oracle.attend_block(q, k, v, seg, is_sync=False)
    for i in range(3, 20):
        np.testing.assert_allclose(glo[i, 0], v[3, 0], atol=1e-9)
    for i in range(3, 10):
        np.testing.assert_allclose(loc[i, 0], v[3, 0], atol=1e-9)
    for i in range(12, 20):          # key 3 is remote: invisible in a local block
        np.testing.assert_allclose(loc[i, 0], v[12, 0], atol=1e-9)


def test_first_row_of_a_segment_sees_only_itself_in_local_blocks():
    seg = [0, 4, 11, 12]
    q, k, v = rand_qkv(8, 12, 2, 2, 8)
    loc = oracle.attend_block(q, k, v, seg, is_sync=False)
    for s in (0, 4, 11):
        np.testing.assert_array_equal(loc[s], v[s].astype(np.float64))


def test_softmax_shift_invariance():
    # adding the same vector u to every key shifts all scores of a row equally
    seg = [0, 8, 24]
    q, k, v = rand_qkv(9, 24, 2, 1, 16)
    u = np.random.default_rng(0).standard_normal(16).astype(np.float32)
    a = oracle.attend_block(q, k, v, seg, is_sync=True)
    b = oracle.attend_block(q, k + u, v, seg, is_sync=True)
    np.testing.assert_allclose(a, b, atol=1e-6)  # k+u rounds in float32


def test_explicit_scale_is_applied_to_scores():
    q, k, v = rand_qkv(10, 10, 1, 1, 16)
    a = oracle.attend_block(q, k, v, [0, 10], is_sync=True, scale=0.7)
    b = oracle.attend_block(q * np.float32(2.0), k, v, [0, 10], is_sync=True, scale=0.35)
    np.testing.assert_allclose(a, b, atol=1e-13)
    c = oracle.attend_block((q.astype(np.float64) * 0.7 * 4.0).astype(np.float32), k, v, [0, 10],
                            is_sync=True)  # default scale 1/sqrt(16) = 1/4
    np.testing.assert_allclose(a, c, atol=1e-5)


# ------------------------------------------------------- probabilities (rows)
def test_rows_are_probability_distributions_with_exact_zeros():
    seg = np.array([0, 6, 6, 15, 22])
    q, k, v = rand_qkv(11, 22, 2, 1, 8)
    rows = np.repeat(np.arange(22), 2).astype(np.int32)
    heads = np.tile(np.arange(2), 22).astype(np.int32)
    for is_sync in (False, True):
        _, p = oracle.attend_rows(q, k, v, seg, rows, heads, is_sync=is_sync, return_prob=True)
        assert np.all(p >= 0)
        np.testing.assert_allclose(p.sum(axis=1), 1.0, atol=1e-14)
        for r, i in enumerate(rows):
            n = np.searchsorted(seg, i, side="right") - 1
            lo = 0 if is_sync else seg[n]
            assert np.all(p[r, :lo] == 0) and np.all(p[r, i + 1:] == 0)
            assert np.count_nonzero(p[r]) == i - lo + 1


# ------------------------------------------------------------- brute force
@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("is_sync", [True, False])
def test_rowwise_equals_brute_force(is_sync, causal):
    seg = [0, 13, 13, 30, 41]
    q, k, v = rand_qkv(12, 41, 4, 2, 16)
    keep = (np.random.default_rng(1).random(41) < 0.4).astype(np.uint8)
    for kt in (None, keep):
        a = oracle.attend_block(q, k, v, seg, is_sync=is_sync, causal=causal, keep_tok=kt)
        b, _ = dense.attention(q, k, v, seg, is_sync=is_sync, causal=causal, keep_tok=kt)
        np.testing.assert_allclose(a, b, atol=1e-13)


def test_tiny_workload_both_routes_and_schedule():
    w = fi.workload("cfg1_tiny")
    seg = w.seg_offsets
    qs, ks, vs = zip(*[fi.prefill_block(w, b) for b in range(w.n_blocks)])
    outs = oracle.schedule.run_stack(qs, ks, vs, seg, w.sync_interval)
    for b in range(w.n_blocks):
        sync = oracle.is_sync_block(w.sync_interval, b)
        assert sync == (b in (1, 3))
        uni = oracle.attend_block(qs[b], ks[b], vs[b], seg, is_sync=sync)
        bf, _ = dense.attention(qs[b], ks[b], vs[b], seg, is_sync=sync)
        np.testing.assert_allclose(outs[b], uni, atol=1e-13)
        np.testing.assert_allclose(outs[b], bf, atol=1e-13)


def test_gqa_equals_mha_with_repeated_kv_heads():
    seg = [0, 10, 25]
    q, k, v = rand_qkv(13, 25, 8, 2, 16)
    a = oracle.attend_block(q, k, v, seg, is_sync=True)
    b = oracle.attend_block(q, np.repeat(k, 4, axis=1), np.repeat(v, 4, axis=1), seg, is_sync=True)
    np.testing.assert_array_equal(a, b)
    # and head h really reads KV head h // 4: zero all but KV head 1
    k2, v2 = k.copy(), v.copy()
    v2[:, 0] = 0
    c = oracle.attend_block(q, k2, v2, seg, is_sync=True)
    assert np.all(c[:, :4] == 0) and np.array_equal(c[:, 4:], a[:, 4:])


# ------------------------------------------------------------- schedule
def test_schedule_limits():
    seg = [0, 9, 20]
    M = 5
    blocks = [rand_qkv(20 + b, 20, 2, 1, 8) for b in range(M)]
    qs, ks, vs = zip(*blocks)
    cen = [sdpa(*blocks[b]) for b in range(M)]
    loc = [np.concatenate([sdpa(q[:9], k[:9], v[:9]), sdpa(q[9:], k[9:], v[9:])]) for q, k, v in blocks]
    # H = 1: centralized attention in every block
    for o, r in zip(oracle.schedule.run_stack(qs, ks, vs, seg, 1), cen):
        np.testing.assert_allclose(o, r, atol=1e-12)
    # never synchronise: fully local attention in every block
    for o, r in zip(oracle.schedule.run_stack(qs, ks, vs, seg, 0), loc):
        np.testing.assert_allclose(o, r, atol=1e-12)
    # H = 2 with M = 5: blocks 2 and 4 (1-based) are global, the rest local
    outs = oracle.schedule.run_stack(qs, ks, vs, seg, 2)
    for b in range(M):
        np.testing.assert_allclose(outs[b], cen[b] if b in (1, 3) else loc[b], atol=1e-12)


# ------------------------------------------------------------- aggregation
def test_aggregation_is_the_selection_matrix_sum():
    seg = [0, 3, 3, 8, 12]
    g = np.random.default_rng(14)
    K = g.standard_normal((12, 2, 4)).astype(np.float32)
    V = g.standard_normal((12, 2, 4)).astype(np.float32)
    kl = [K[seg[n]:seg[n + 1]] for n in range(4)]
    vl = [V[seg[n]:seg[n + 1]] for n in range(4)]
    Ka, Va = aggregate_kv(kl, vl, seg)
    assert np.array_equal(Ka, K) and np.array_equal(Va, V)       # X = sum Pi_n Pi_n^T X
    Kd, Vd = aggregate_kv_by_definition(kl, vl, seg)
    assert np.array_equal(Kd, K.astype(np.float64)) and np.array_equal(Vd, V.astype(np.float64))


# ------------------------------------------------------- sparse KV exchange
def test_sparse_exchange_limits():
    seg = [0, 16, 40, 56]
    q, k, v = rand_qkv(15, 56, 4, 2, 16)
    none = oracle.expand_keep_chunks(np.zeros(2 + 3 + 2, dtype=np.uint8), seg, 8)
    full = oracle.expand_keep_chunks(np.ones(2 + 3 + 2, dtype=np.uint8), seg, 8)
    loc = oracle.attend_block(q, k, v, seg, is_sync=False)
    glo = oracle.attend_block(q, k, v, seg, is_sync=True)
    # every remote participant excluded: the sync block degenerates to a local one
    np.testing.assert_array_equal(oracle.attend_block(q, k, v, seg, is_sync=True, keep_tok=none), loc)
    # everything sent: dense sync
    np.testing.assert_array_equal(oracle.attend_block(q, k, v, seg, is_sync=True, keep_tok=full), glo)
    # excluding participant 1 only: equals attention over the sequence with its rows
    # removed, for the queries of the other participants
    flags = np.array([1, 1, 0, 0, 0, 1, 1], dtype=np.uint8)
    kt = oracle.expand_keep_chunks(flags, seg, 8)
    got = oracle.attend_block(q, k, v, seg, is_sync=True, keep_tok=kt)
    sel = np.r_[0:16, 40:56]
    ref = sdpa(q[sel], k[sel], v[sel])
    np.testing.assert_allclose(got[sel], ref, atol=1e-12)
    # participant 1 itself still attends to all of its own rows
    sel1 = np.r_[0:40]
    np.testing.assert_allclose(got[16:40], sdpa(q[sel1], k[sel1], v[sel1])[16:40], atol=1e-12)


@pytest.mark.parametrize("causal", [True, False])
def test_sparse_exchange_matches_library_attention_with_an_explicit_mask(causal):
    """Sparse KV exchange (own rows complete, a remote row visible only if its flag is set;
    adaptive KV aggregation of Section V), causal and bidirectional, against library attention
    under a visibility matrix written out here token by token, independently of the oracle."""
    seg = [0, 11, 11, 30, 47]
    L, Hq, Hkv, D = 47, 4, 2, 16
    q, k, v = rand_qkv(16, L, Hq, Hkv, D)
    g = np.random.default_rng(17)
    keep = (g.random(L) < 0.4).astype(np.uint8)
    keep[30:47] = 0                    # the last participant shares nothing, yet sees itself
    owner = np.zeros(L, dtype=np.int64)
    for n in range(len(seg) - 1):
        owner[seg[n]:seg[n + 1]] = n
    mask = np.zeros((L, L), dtype=bool)
    for i in range(L):
        for j in range(L):
            if causal and j > i:
                continue
            mask[i, j] = owner[i] == owner[j] or keep[j] == 1
    got = oracle.attend_block(q, k, v, seg, is_sync=True, causal=causal, keep_tok=keep)
    np.testing.assert_allclose(got, sdpa(q, k, v, mask=mask), atol=1e-12)
    # and the mask does bind: the dense sync block differs
    assert np.abs(got - oracle.attend_block(q, k, v, seg, is_sync=True, causal=causal)).max() > 1e-3


def test_chunk_expansion_ragged_tail():
    seg = [0, 10, 10, 27]
    flags = np.array([1, 0, 0, 1, 1], dtype=np.uint8)   # 2 chunks, 0 chunks, 3 chunks of 8
    kt = oracle.expand_keep_chunks(flags, seg, 8)
    expect = np.zeros(27, dtype=np.uint8)
    expect[0:8] = 1
    expect[18:27] = 1
    assert np.array_equal(kt, expect)


# ---------------------------------------------------- local-vs-global deviation
def test_deviation_vanishes_when_remote_scores_are_very_negative():
    seg = [0, 12, 24]
    q, k, v = rand_qkv(16, 24, 1, 1, 8)
    # one extra coordinate: +c on own segment's keys/queries pairing, so that a
    # remote pair scores -c*c lower than a local one
    c = 40.0
    qx = np.concatenate([q, np.zeros((24, 1, 2), np.float32)], axis=2)
    kx = np.concatenate([k, np.zeros((24, 1, 2), np.float32)], axis=2)
    qx[:12, 0, 8] = c
    kx[:12, 0, 8] = c
    qx[12:, 0, 9] = c
    kx[12:, 0, 9] = c
    vx = np.concatenate([v, np.zeros((24, 1, 2), np.float32)], axis=2)
    loc = oracle.attend_block(qx, kx, vx, seg, is_sync=False)
    glo = oracle.attend_block(qx, kx, vx, seg, is_sync=True)
    assert np.linalg.norm(loc - glo) < 1e-12
    # without the separation the deviation is positive for the later participant
    loc0 = oracle.attend_block(q, k, v, seg, is_sync=False)
    glo0 = oracle.attend_block(q, k, v, seg, is_sync=True)
    assert np.linalg.norm(loc0[12:] - glo0[12:]) > 1e-3
    assert np.linalg.norm(loc0[:12] - glo0[:12]) == 0.0     # first participant sees no one else


# ------------------------------------------------------------------ decode
def test_decode_single_participant_equals_last_prefill_row():
    P, steps = 9, 4
    q, k, v = rand_qkv(17, P + steps, 4, 2, 16)
    full = sdpa(q, k, v)
    for s in range(steps):
        n_valid = P + s + 1
        got = oracle.decode_step(q[n_valid - 1][None], k, v, [0, P + steps], [n_valid], is_sync=False)
        np.testing.assert_allclose(got[0], full[n_valid - 1], atol=1e-12)
        got = oracle.decode_step(q[n_valid - 1][None], k, v, [0, P + steps], [n_valid], is_sync=True)
        np.testing.assert_allclose(got[0], full[n_valid - 1], atol=1e-12)


def test_decode_visibility_and_brute_force():
    N, cap, Hq, Hkv, D = 3, 10, 4, 2, 16
    g = np.random.default_rng(18)
    q = g.standard_normal((N, Hq, D)).astype(np.float32)
    kc = g.standard_normal((N * cap, Hkv, D)).astype(np.float32)
    vc = g.standard_normal((N * cap, Hkv, D)).astype(np.float32)
    seg = np.arange(N + 1) * cap
    lens = np.array([7, 10, 4])
    prompt = np.array([5, 6, 2])
    # local: participant n over its own valid rows == library attention on that slice
    loc = oracle.decode_step(q, kc, vc, seg, lens, is_sync=False)
    for n in range(N):
        sl = slice(seg[n], seg[n] + lens[n])
        ref = sdpa(q[n][None], kc[sl], vc[sl], causal=False)
        np.testing.assert_allclose(loc[n], ref[0], atol=1e-12)
    # sync, everyone's valid rows
    glo = oracle.decode_step(q, kc, vc, seg, lens, is_sync=True)
    idx = np.concatenate([np.arange(seg[m], seg[m] + lens[m]) for m in range(N)])
    for n in range(N):
        ref = sdpa(q[n][None], kc[idx], vc[idx], causal=False)
        np.testing.assert_allclose(glo[n], ref[0], atol=1e-12)
    # sync, remote participants expose their prompt rows only
    glo2 = oracle.decode_step(q, kc, vc, seg, lens, is_sync=True, remote_lens=prompt)
    for n in range(N):
        idx = np.concatenate([np.arange(seg[m], seg[m] + (lens[m] if m == n else prompt[m]))
                              for m in range(N)])
        ref = sdpa(q[n][None], kc[idx], vc[idx], causal=False)
        np.testing.assert_allclose(glo2[n], ref[0], atol=1e-12)
    for kw in (dict(is_sync=False), dict(is_sync=True), dict(is_sync=True, remote_lens=prompt)):
        np.testing.assert_allclose(oracle.decode_step(q, kc, vc, seg, lens, **kw),
                                   dense.decode(q, kc, vc, seg, lens, **kw), atol=1e-13)


def test_empty_segments_and_empty_key_sets():
    q, k, v = rand_qkv(19, 6, 1, 1, 4)
    out = oracle.attend_block(q, k, v, [0, 0, 6, 6], is_sync=True)
    np.testing.assert_allclose(out, sdpa(q, k, v), atol=1e-13)
    # decode with an empty cache for one participant gives zeros there
    o = oracle.decode_step(q[:2], k, v, [0, 3, 6], [0, 2], is_sync=False)
    assert np.all(o[0] == 0) and np.any(o[1] != 0)


# --------------------------------------------------------------- generators
def test_inputs_are_reproducible_and_bf16_exact():
    w = fi.workload("cfg2_llama8b_prefill")
    q1, k1, v1 = fi.prefill_block(w, 3, total=64)
    q2, _, _ = fi.prefill_block(w, 3, total=64)
    assert np.array_equal(q1, q2)
    assert not np.any(q1.view(np.uint32) & 0xFFFF)
    t = torch.from_numpy(q1.copy())
    assert torch.equal(t.to(torch.bfloat16).to(torch.float32), t)
    x = np.random.default_rng(0).standard_normal(10000).astype(np.float32)
    assert np.array_equal(fi.round_to_bf16(x), torch.from_numpy(x).to(torch.bfloat16).float().numpy())
    assert abs(float(q1.std()) - 0.5) < 0.01
    w3 = fi.workload("cfg3_hetero_prefill")
    assert len(w3.seg_lens) == 8 and all(1024 <= l <= 3072 for l in w3.seg_lens)
    kc = fi.keep_chunks(fi.workload("cfg5_sparse_sync"), 0)
    assert kc.shape == (16 * 64,) and np.all(kc.reshape(16, 64).sum(axis=1) == 16)
